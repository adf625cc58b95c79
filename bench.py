#!/usr/bin/env python3
"""Benchmark of the DHSA prefill hot path on one MI355X.

One step = one pass of the whole path (pool -> S_c -> rank/budget -> sparse
attention) over one synthetic layer of the 128K / 6.25 %-density workload
("c3": L=131072, 32 query heads, 8 kv heads, d=128, bf16, N_b=8192).  Inputs
are resident in HBM before the timed region.  Prints ONE JSON line.

The step is issued as dhsa_route + dhsa_sparse_prefill (exactly what
dhsa_prefill enqueues) so that HIP events on the same stream can bracket the
attention kernel inside the timed region.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
# HBM bytes of the attention step on c3 (all k_attn_mfma launches of one step), from the rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE runs summarised in profiles/attn_mfma_c3_counters.md and
# profiles/attn_mfma_c3_blocks_counters.md (counter KiB x the copy-kernel factors 2.0 / 1.0 of
# profiles/counter_calibration.md), keyed by B_r.  The K/V gather asks the L2 for 220 GB (row form) /
# 146 GB (row blocks of 128); 46 % / 56 % of the requests hit.
MEASURED_TRAFFIC_C3 = {0: {"fetch_bytes": 1.189e11, "write_bytes": 1.074e9},
                       128: {"fetch_bytes": 6.20e10, "write_bytes": 1.074e9}}
PAPER_CONTEXT = {"what": "paper Tab. 11, DHSA 6.25% @128K, LLaMA-3.1-8B bf16, attention kernel only",
                 "ms_per_layer": 214.5, "hardware": "RTX 3090"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3", help="c1..c5 (the metric is quoted on c3)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--B_r", type=int, default=0,
                    help="0 (default, the headline): per-row budgets on the dynamic chunks; > 0: time Alg. 1 as "
                         "printed with row blocks of this many rows instead")
    ap.add_argument("--no-block-form", action="store_true",
                    help="skip the extra measurement of Alg. 1 as printed (row blocks of 128 rows)")
    ap.add_argument("--no-decode", action="store_true", help="skip the decoding-step timing")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (whole kv-head groups would shard across GPUs without any exchange); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import dhsa_inputs
    import paper_2510_24606_amd as dhsa

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dhsa.lib()   # fail loudly if the HIP library is missing

    w = dhsa_inputs.make(args.workload)
    Q, K, V = (t.cuda() for t in (w.Q, w.K, w.V))
    O = torch.empty_like(Q)

    def measure(B_r):
        """W warm-up steps, then K timed steps of route + sparse attention: (ms/step, attention ms, wall ms)."""
        prob = dhsa.problem(Q, K, w.B, w.N_b, B_r=B_r)
        plan, ws = dhsa.alloc(prob, w.B)
        torch.cuda.synchronize()

        def step(ev=None):
            dhsa.dhsa_route(prob, Q, K, w.B, plan, ws)
            if ev is not None:
                ev[0].record()
            dhsa.dhsa_sparse_prefill(prob, Q, K, V, w.B, plan, O)
            if ev is not None:
                ev[1].record()

        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(args.steps)]
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for k in range(args.steps):
            step(evs[k])
        e1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / args.steps
        ms = e0.elapsed_time(e1) / args.steps
        return ms, float(np.mean([a.elapsed_time(b) for a, b in evs])), wall, plan

    ms_per_step, attn_ms, wall_ms, plan_main = measure(args.B_r)
    route_ms = ms_per_step - attn_ms

    def attended_pairs(B_r, plan):
        """(row, key) pairs the attention step computes on, all heads.  Row form: H_q sum_i min(N_b, i+1).
        Row-block form: counted exactly from the plan -- per block and listed chunk (first `t` tokens of
        chunk k, from b0 = B[k]) row i attends min(max(i + 1 - b0, 0), t) of them (the causal mask inside
        the block's own range is taken off, not just the listed size)."""
        if B_r == 0:
            return float(w.pairs_per_head()) * w.H_q
        P = dhsa.parse_plan(plan.cpu().numpy())
        Bk, RB = P["B"].astype(np.int64), P["RB"].astype(np.int64)
        ent, cnt = P["entries"], P["count"]
        live = np.arange(ent.shape[2])[None, None, :] < cnt[:, :, None]
        k = np.where(live, ent[..., 0] & ((1 << dhsa.POS_SHIFT) - 1), 0).astype(np.int64)
        t = np.where(live, ent[..., 1], 0).astype(np.int64)
        b0 = Bk[k]
        r0, r1 = RB[:-1][None, :, None], RB[1:][None, :, None]
        a = np.maximum(r0, b0)                                    # first row that sees a token of the chunk
        n1 = np.maximum(0, np.minimum(r1 - 1, b0 + t - 1) - a + 1)    # rows that see a growing part of it
        n2 = np.maximum(0, r1 - 1 - np.maximum(a - 1, b0 + t - 1))    # rows that see all t
        tot = np.where(a < r1, n1 * (a + 1 - b0) + n1 * (n1 - 1) // 2 + n2 * t, 0)
        return float(tot.sum())

    flops = 4.0 * w.D * attended_pairs(args.B_r, plan_main)      # selected (row, key) pairs only
    achieved = flops / (attn_ms * 1e-3) / 1e12
    out = {
        "metric": "DHSA prefill ms/layer @128K, 6.25% density; % of MFMA bf16 peak"
                  + (f" [Alg. 1 row blocks, B_r={args.B_r}]" if args.B_r else ""),
        "value": round(ms_per_step, 4), "unit": "ms/layer",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: L={w.L} H_q={w.H_q} H_kv={w.H_kv} d={w.D} N_b={w.N_b} "
                               f"N_c={w.N_c} {w.dtype}, one layer, batch 1",
                   "density": w.N_b / w.L},
        "stages_ms": {"route(pool+S_c+select)": round(route_ms, 4), "sparse_attention": round(attn_ms, 4),
                      "host_wall_per_step": round(wall_ms, 4)},
        "pct_of_bf16_mfma_peak": round(100.0 * achieved / PEAK_BF16_TFLOPS, 3),
        "roofline": {"bound": "mfma",
                     "kernel": "k_attn_mfma (launches: row tiles of > 64 rows, then row tiles of <= 64 rows)",
                     "achieved": round(achieved, 3),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 5),
                     "flop_per_launch": flops,
                     "traffic": (sum(MEASURED_TRAFFIC_C3[args.B_r].values())
                                 if args.workload == "c3" and args.B_r in MEASURED_TRAFFIC_C3 else None),
                     "traffic_detail": (MEASURED_TRAFFIC_C3[args.B_r]
                                        if args.workload == "c3" and args.B_r in MEASURED_TRAFFIC_C3 else None)},
        "paper_context": PAPER_CONTEXT,
    }
    if not args.no_block_form and args.B_r == 0:
        # Alg. 1 as printed on the same tensors: row blocks of B_r rows, one list of N_b keys per block,
        # causal mask per token.  B_r = 128 is the paper's tile height (App. C); with B_r = 256 two row
        # tiles share one list and, running side by side, find each other's K / V rows in the L2.
        for B_r, key in ((128, "alg1_block_form"), (256, "alg1_block_form_Br256")):
            ms_b, attn_b, _, plan_b = measure(B_r)
            fl_b = 4.0 * w.D * attended_pairs(B_r, plan_b)
            out[key] = {"B_r": B_r, "ms_per_layer": round(ms_b, 4), "sparse_attention_ms": round(attn_b, 4),
                        "route_ms": round(ms_b - attn_b, 4), "flop_attended_pairs": fl_b,
                        "achieved_tflops": round(fl_b / (attn_b * 1e-3) / 1e12, 3),
                        "frac_of_bf16_mfma_peak": round(fl_b / (attn_b * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 5)}
            del plan_b
    # what the matrix unit alone sustains on this chip (same instruction as the attention kernel):
    # with operands that never change, and with random operands (the chip then clocks down to stay
    # inside its power limit, as it does on real attention data)
    tf_c, mhz_c = dhsa.dhsa_mfma_probe(False)
    tf_r, mhz_r = dhsa.dhsa_mfma_probe(True)
    out["mfma_microkernel"] = {"constant_operands_tflops": round(tf_c, 1), "constant_operands_shader_mhz": round(mhz_c),
                               "random_operands_tflops": round(tf_r, 1), "random_operands_shader_mhz": round(mhz_r),
                               "attention_vs_random_operand_rate": round(achieved / tf_r, 4)}

    if not args.no_decode:
        # one decoding step for the newest token at the workload's full context (same tensors as caches):
        # steady state = the pooled keys of the closed chunks are kept from the step before; cold = every
        # chunk pooled anew.  HBM-bound: the selected K and V rows of every query head are read once.
        prob_d = dhsa.problem(Q, K, w.B, w.N_b, B_r=args.B_r)
        ws_d = dhsa.alloc_decode(prob_d, w.N_c, w.L)

        O_row = torch.empty((w.H_q, w.D), dtype=Q.dtype, device=Q.device)

        def time_decode(kc_valid, n):
            for _ in range(3):
                dhsa.dhsa_decode_step(prob_d, Q, K, V, w.B, ws_d, w.N_c, w.L, kc_valid, out=O_row)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(n):
                dhsa.dhsa_decode_step(prob_d, Q, K, V, w.B, ws_d, w.N_c, w.L, kc_valid, out=O_row)
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / n

        cold_ms = time_decode(0, 20)
        steady_ms = time_decode(w.N_c - 1, 100)
        esz = 2 if w.dtype == "bf16" else 4
        kv_bytes = 2.0 * w.H_q * min(w.N_b, w.L) * w.D * esz            # selected K and V rows, per query head
        kc_bytes = 8.0 * w.H_kv * w.N_c * w.D                             # pooled keys (fp64), read by the scores
        out["decode_step"] = {"ms_steady": round(steady_ms, 4), "ms_cold": round(cold_ms, 4),
                              "algorithmic_hbm_bytes": kv_bytes + kc_bytes,
                              "achieved_GBps": round((kv_bytes + kc_bytes) / (steady_ms * 1e-3) / 1e9, 1),
                              "frac_of_hbm_peak": round((kv_bytes + kc_bytes) / (steady_ms * 1e-3) / 8e12, 4),
                              "note": "newest token of the same sequence; steady = pooled keys of closed chunks reused"}

    if not args.no_cpu_baseline:
        import oracle
        Qf, Kf, Vf = w.f32("Q"), w.f32("K"), w.f32("V")
        nb = min(w.N_b, w.L)

        def run(n):
            rows = dhsa_inputs.sample_rows(w, n, seed=1)
            t = time.perf_counter()
            oracle.prefill_rows(Qf, Kf, Vf, w.B, w.N_b, rows)
            dt = time.perf_counter() - t
            pairs = int(np.minimum(rows + 1, nb).sum())
            return dt, pairs, len(rows)

        dt, pairs, n = run(48)                                # calibration
        if dt < args.cpu_seconds / 2:
            n2 = int(min(w.L, max(48, n * args.cpu_seconds / max(dt, 1e-3))))
            dt, pairs, n = run(n2)
        full_ms = dt * 1e3 * w.pairs_per_head() / pairs        # rows are independent: scale by selected pairs
        if "decode_step" in out and args.B_r == 0:
            t = time.perf_counter()
            oracle.decode_row(Qf, Kf, Vf, w.B, w.N_b)
            out["decode_step"]["cpu_oracle_ms"] = round((time.perf_counter() - t) * 1e3, 1)
        out["cpu_baseline"] = {"value": round(full_ms, 1), "unit": "ms/layer", "cores": oracle.num_threads(),
                               "kind": "oracle",
                               "sample": f"{n} stratified rows x {w.H_q} heads incl. routing of their chunks, "
                                         f"{dt:.1f} s measured, extrapolated by selected (row,key) pairs"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
