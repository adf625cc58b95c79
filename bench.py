#!/usr/bin/env python3
"""Benchmark of the DHSA prefill hot path on one MI355X.

One step = one pass of the whole path (pool -> S_c -> rank/budget -> sparse
attention) over one synthetic layer of the 128K / 6.25 %-density workload
("c3": L=131072, 32 query heads, 8 kv heads, d=128, bf16, N_b=8192).  Inputs
are resident in HBM before the timed region.  Prints ONE JSON line.

The step is issued as dhsa_route + dhsa_sparse_prefill (exactly what
dhsa_prefill enqueues) so that HIP events on the same stream can bracket the
attention kernels inside the timed region.  Outside the timed region the line
also gets: the time of every stage and of every attention launch with its share
of the FLOP (dhsa_prefill_stage_times), the same figures for the other
workloads, near-tie counts and the error against the oracle on sampled rows,
Alg. 1 as printed (row blocks), one decoding step, the matrix unit alone, and
the oracle timed on the host cores.

Other modes (they print plain lines and exit): --calibrate-counters (a 1 GiB copy,
to price rocprofv3's FETCH_SIZE / WRITE_SIZE), --extras (boundary finalisation
and the recall diagnostic at c3 size).
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "attn_mfma_traffic.json")
KERNEL_SOURCES = ("paper_2510_24606_amd/csrc/attn_mfma.hip", "paper_2510_24606_amd/csrc/dhsa_internal.h")
PAPER_CONTEXT = {"what": "paper Tab. 11, DHSA 6.25% @128K, LLaMA-3.1-8B bf16, attention kernel only",
                 "ms_per_layer": 214.5, "hardware": "RTX 3090"}
ROW_CLASSES = (("rows_gt64", "attn_rows_gt64"), ("rows_33_64", "attn_rows_33_64"), ("rows_le32", "attn_rows_le32"))


def kernel_source_hash() -> str:
    """Identifies the attention kernel the counters in profiles/ were taken with: a hash of its source
    without // comments and blank lines (a reworded comment does not make the counters stale)."""
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "r") as f:
            for line in f:
                code = line.split("//", 1)[0].rstrip()
                if code.strip():
                    h.update(code.encode() + b"\n")
    return h.hexdigest()[:16]


def measured_traffic(workload: str, B_r: int):
    """HBM bytes of one attention step from the rocprofv3 --pmc runs recorded in profiles/ (FETCH_SIZE /
    WRITE_SIZE x the copy-kernel factors), or None when the kernel source has changed since."""
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        return None
    if rec.get("kernel_source_sha256_16") != kernel_source_hash():
        return None
    return rec.get("entries", {}).get(f"{workload}:B_r={B_r}")


def calibrate_counters() -> int:
    import torch
    a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()   # 1 GiB
    b = torch.empty_like(a)
    torch.cuda.synchronize()
    for _ in range(3):
        b.copy_(a)          # reads 1 GiB, writes 1 GiB per launch
    torch.cuda.synchronize()
    print("copied 1 GiB three times (1 048 576 KiB read and written per launch)")
    return 0


def extras() -> int:
    """Boundary finalisation (threshold + NMS over L = 131072 seeded scores) and the recall diagnostic."""
    import numpy as np
    import torch
    import dhsa_inputs
    import paper_2510_24606_amd as dhsa

    L = 131072

    def peaked_scores(seed):
        rng = np.random.default_rng(seed)
        p = 0.2 * rng.random(L)
        at = np.cumsum(rng.integers(20, 80, size=L // 20 + 2))
        at = at[at < L]
        p[at] += 0.5 + 0.3 * rng.random(len(at))
        for d in (-1, 1):
            ok = (at + d >= 0) & (at + d < L)
            p[at[ok] + d] += 0.3
        return p.astype(np.float32)

    for kind, W in (("peaks", 8), ("peaks", 64), ("noise", 8), ("noise", 64)):
        p = peaked_scores(7) if kind == "peaks" else np.random.default_rng(7).random(L).astype(np.float32)
        tau = 0.4 if kind == "peaks" else 0.5
        pd = torch.from_numpy(p).cuda()
        dhsa.dhsa_finalize_boundaries(pd, tau, W)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        B = dhsa.dhsa_finalize_boundaries(pd, tau, W)
        e1.record(); torch.cuda.synchronize()
        print(f"finalize_boundaries {kind} L={L} tau={tau} W={W}: N_c={len(B) - 1}, {e0.elapsed_time(e1):.3f} ms "
              f"(incl. the copy of B to the host)", flush=True)
    w = dhsa_inputs.make("c3")
    Q, K = w.Q.cuda(), w.K.cuda()
    prob = dhsa.problem(Q, K, w.B, w.N_b)
    plan, ws = dhsa.alloc(prob, w.B)
    dhsa.dhsa_route(prob, Q, K, w.B, plan, ws)
    rows = dhsa_inputs.sample_rows(w, 48)
    dhsa.dhsa_recall_rows(prob, Q, K, w.B, plan, 5, rows)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    hits, size = dhsa.dhsa_recall_rows(prob, Q, K, w.B, plan, 5, rows)
    e1.record(); torch.cuda.synchronize()
    rec = (hits.cpu().numpy() / size.cpu().numpy()).mean()
    print(f"recall_rows c3 head 5, {len(rows)} rows: mean recall {rec:.4f}, {e0.elapsed_time(e1):.3f} ms", flush=True)
    return 0


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
                    help="skip the extra measurement of Alg. 1 as printed (row blocks of 128 / 256 rows)")
    ap.add_argument("--no-decode", action="store_true", help="skip the decoding-step timing")
    ap.add_argument("--no-other-workloads", action="store_true", help="skip the short runs of the other workloads")
    ap.add_argument("--no-parity-report", action="store_true",
                    help="skip near-tie counts and the error against the oracle on sampled rows")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--calibrate-counters", action="store_true", help="only copy 1 GiB three times, then exit")
    ap.add_argument("--extras", action="store_true", help="only time boundary finalisation and recall, then exit")
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
    if args.calibrate_counters:
        return calibrate_counters()
    if args.extras:
        return extras()

    def load(name):
        w = dhsa_inputs.make(name)
        Q, K, V = (t.cuda() for t in (w.Q, w.K, w.V))
        return w, Q, K, V, torch.empty_like(Q)

    def measure(w, Q, K, V, O, B_r, steps, warmup):
        """`warmup` untimed steps, then `steps` timed steps of route + sparse attention:
        (ms/step, attention ms, host wall ms, plan, workspace, problem)."""
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

        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for k in range(steps):
            step(evs[k])
        e1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / steps
        ms = e0.elapsed_time(e1) / steps
        return ms, float(np.mean([a.elapsed_time(b) for a, b in evs])), wall, plan, ws, prob

    def attended_pairs_by_class(w, B_r, plan):
        """(row, key) pairs the attention step computes on, all heads, split by the height class of the row
        tile (the three attention launches).  Row form: row i attends min(N_b, i + 1) keys.  Row-block form:
        counted exactly from the plan -- per block and listed chunk (first `t` tokens of chunk k, from
        b0 = B[k]) row i attends min(max(i + 1 - b0, 0), t) of them (the causal mask inside the block's own
        range is taken off, not just the listed size)."""
        P = dhsa.parse_plan(plan.cpu().numpy())
        tiles = P["tiles"]
        order = np.argsort(tiles[:, 1], kind="stable")
        nrows = np.empty(len(tiles), dtype=np.int64)
        nrows[order] = np.r_[tiles[order][1:, 1], w.L] - tiles[order][:, 1]
        launch_of_tile = np.where(nrows > 64, 0, np.where(nrows > 32, 1, 2))
        if B_r == 0:
            per_row = np.minimum(np.arange(1, w.L + 1, dtype=np.int64), min(w.N_b, w.L))
            csum = np.r_[0, np.cumsum(per_row)]
            per_tile = (csum[tiles[:, 1] + nrows] - csum[tiles[:, 1]]) * w.H_q
        else:
            Bk, RB = P["B"].astype(np.int64), P["RB"].astype(np.int64)
            ent, cnt = P["entries"], P["count"]
            live = np.arange(ent.shape[2])[None, None, :] < cnt[:, :, None]
            k = np.where(live, ent[..., 0] & ((1 << dhsa.POS_SHIFT) - 1), 0).astype(np.int64)
            t = np.where(live, ent[..., 1], 0).astype(np.int64)
            b0 = Bk[k]
            per_tile = np.zeros(len(tiles), dtype=np.int64)
            for ti in range(len(tiles)):                      # a block has one tile per 128 rows
                blk, r0 = int(tiles[ti, 0]), int(tiles[ti, 1])
                r1 = r0 + int(nrows[ti])
                bb, tt = b0[:, blk, :], t[:, blk, :]
                a = np.maximum(r0, bb)                        # first row of the tile that sees a token of the chunk
                n1 = np.maximum(0, np.minimum(r1 - 1, bb + tt - 1) - a + 1)    # rows that see a growing part of it
                n2 = np.maximum(0, r1 - 1 - np.maximum(a - 1, bb + tt - 1))    # rows that see all t
                per_tile[ti] = np.where(a < r1, n1 * (a + 1 - bb) + n1 * (n1 - 1) // 2 + n2 * tt, 0).sum()
        return [float(per_tile[launch_of_tile == c].sum()) for c in range(3)], [int((launch_of_tile == c).sum())
                                                                                 for c in range(3)]

    def stage_report(w, Q, K, V, O, prob, plan, ws, B_r, reps=5):
        """Per-stage and per-attention-launch milliseconds (median of `reps` passes with events between the
        kernels), the FLOP of each launch and its fraction of the bf16 MFMA peak."""
        runs = [dhsa.dhsa_prefill_stage_times(prob, Q, K, V, w.B, O, plan, ws) for _ in range(reps + 1)][1:]
        med = {k: float(np.median([r[k] for r in runs])) for k in dhsa.STAGES}
        pairs, ntiles = attended_pairs_by_class(w, B_r, plan)
        launches = {}
        for c, (label, stage) in enumerate(ROW_CLASSES):
            fl = 4.0 * w.D * pairs[c]
            launches[label] = {"tiles_per_head": ntiles[c], "flop": fl, "ms": round(med[stage], 4),
                               "frac_of_bf16_mfma_peak": (round(fl / (med[stage] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 5)
                                                          if med[stage] > 0 and w.dtype == "bf16" else None)}
        stages = {"t_setup": round(med["setup"], 4), "t_pool": round(med["pool"], 4), "t_sc": round(med["scores"], 4),
                  "t_select": round(med["select"], 4),
                  "t_attn": round(med["attn_rows_gt64"] + med["attn_rows_33_64"] + med["attn_rows_le32"], 4),
                  "t_total": round(med["total"], 4)}
        return stages, launches, sum(pairs)

    def parity_report(w, O, prob, plan, n_rows=24):
        """Near-tie groups (query groups whose cut-off score gap is <= 1e-5, from the oracle's fp64 scores)
        and max |O - oracle| on a stratified row sample, with the mask of those rows compared exactly."""
        import oracle
        Qf, Kf, Vf = w.f32("Q"), w.f32("K"), w.f32("V")
        G = w.H_q // w.H_kv
        nb = min(w.N_b, w.L)
        Qc, Kc = oracle.pool(Qf, w.B), oracle.pool(Kf, w.B)
        near = sum(int((oracle.plan_head(Qc[h], Kc[h // G], w.B, nb)[2] <= 1e-5).sum()) for h in range(w.H_q))
        rows = dhsa_inputs.sample_rows(w, n_rows, seed=3)
        O_ref, I_ref, cnt_ref = oracle.prefill_rows(Qf, Kf, Vf, w.B, w.N_b, rows)
        got = O[:, torch.from_numpy(rows).cuda()].float().cpu().numpy().astype(np.float64)
        mask_ok = True
        for h in range(w.H_q):
            idx, cnt = dhsa.dhsa_plan_expand_rows(prob, plan, h, rows)
            mask_ok &= bool(np.array_equal(idx.cpu().numpy(), I_ref[h][:, :idx.shape[1]])
                            and np.array_equal(cnt.cpu().numpy(), cnt_ref[h]))
        return {"near_tie_groups_le_1e-5": near, "query_groups": w.N_c * w.H_q, "sampled_rows": int(len(rows)),
                "mask_exact_on_sample": mask_ok, "max_abs_err_vs_oracle": float(np.abs(got - O_ref).max())}

    w, Q, K, V, O = load(args.workload)
    ms_per_step, attn_ms, wall_ms, plan_main, ws_main, prob_main = measure(w, Q, K, V, O, args.B_r, args.steps,
                                                                           args.warmup)
    route_ms = ms_per_step - attn_ms
    stages, launches, pairs_total = stage_report(w, Q, K, V, O, prob_main, plan_main, ws_main, args.B_r)
    flops = 4.0 * w.D * pairs_total                              # selected (row, key) pairs only
    achieved = flops / (attn_ms * 1e-3) / 1e12
    traffic = measured_traffic(args.workload, args.B_r)
    out = {
        "metric": f"DHSA prefill ms/layer @{w.L // 1024}K, {100.0 * w.N_b / w.L:.4g}% density; % of MFMA bf16 peak"
                  + (f" [Alg. 1 row blocks, B_r={args.B_r}]" if args.B_r else ""),
        "value": round(ms_per_step, 4), "unit": "ms/layer",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: L={w.L} H_q={w.H_q} H_kv={w.H_kv} d={w.D} N_b={w.N_b} "
                               f"N_c={w.N_c} {w.dtype}, one layer, batch 1",
                   "density": w.N_b / w.L},
        "stages_ms": {"route(pool+S_c+select)": round(route_ms, 4), "sparse_attention": round(attn_ms, 4),
                      "host_wall_per_step": round(wall_ms, 4), **stages},
        "pct_of_bf16_mfma_peak": round(100.0 * achieved / PEAK_BF16_TFLOPS, 3),
        "roofline": {"bound": "mfma",
                     "kernel": "k_attn_mfma (one launch per height class of the row tiles: > 64 rows, 33..64, <= 32)",
                     "achieved": round(achieved, 3),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 5),
                     "flop_per_launch": flops, "launches": launches,
                     "traffic": (traffic["fetch_bytes"] + traffic["write_bytes"]) if traffic else None,
                     "traffic_detail": traffic},
        "paper_context": PAPER_CONTEXT,
    }
    if not args.no_parity_report and args.B_r == 0:
        out["parity_report"] = parity_report(w, O, prob_main, plan_main)
    if not args.no_block_form and args.B_r == 0:
        # Alg. 1 as printed on the same tensors: row blocks of B_r rows, one list of N_b keys per block,
        # causal mask per token.  B_r = 128 is the paper's tile height (App. C); with B_r = 256 two row
        # tiles share one list and, running side by side, find each other's K / V rows in the L2.
        for B_r, key in ((128, "alg1_block_form"), (256, "alg1_block_form_Br256")):
            ms_b, attn_b, _, plan_b, ws_b, prob_b = measure(w, Q, K, V, O, B_r, max(3, args.steps // 2), 2)
            pairs_b, _ = attended_pairs_by_class(w, B_r, plan_b)
            fl_b = 4.0 * w.D * sum(pairs_b)
            out[key] = {"B_r": B_r, "ms_per_layer": round(ms_b, 4), "sparse_attention_ms": round(attn_b, 4),
                        "route_ms": round(ms_b - attn_b, 4), "flop_attended_pairs": fl_b,
                        "achieved_tflops": round(fl_b / (attn_b * 1e-3) / 1e12, 3),
                        "frac_of_bf16_mfma_peak": round(fl_b / (attn_b * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 5)}
            del plan_b, ws_b
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
        del ws_d

    cpu_inputs = (w.f32("Q"), w.f32("K"), w.f32("V"), w) if not args.no_cpu_baseline else None
    del plan_main, ws_main

    if not args.no_other_workloads and args.workload == "c3" and args.B_r == 0:
        # the other configurations, a few steps each (same launch configuration, same code path)
        del Q, K, V, O
        torch.cuda.empty_cache()
        others = {}
        for name in ("c1", "c2", "c4", "c5"):
            wo, Qo, Ko, Vo, Oo = load(name)
            ms_o, attn_o, _, plan_o, ws_o, prob_o = measure(wo, Qo, Ko, Vo, Oo, 0, 5, 2)
            st_o, la_o, pairs_o = stage_report(wo, Qo, Ko, Vo, Oo, prob_o, plan_o, ws_o, 0)
            fl_o = 4.0 * wo.D * pairs_o
            rec = {"workload": f"L={wo.L} H_q={wo.H_q} H_kv={wo.H_kv} d={wo.D} N_b={wo.N_b} N_c={wo.N_c} {wo.dtype}",
                   "ms_per_layer": round(ms_o, 4), "route_ms": round(ms_o - attn_o, 4),
                   "sparse_attention_ms": round(attn_o, 4), "stages_ms": st_o, "launches": la_o,
                   "achieved_tflops": round(fl_o / (attn_o * 1e-3) / 1e12, 3),
                   "frac_of_bf16_mfma_peak": (round(fl_o / (attn_o * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 5)
                                              if wo.dtype == "bf16" else None)}
            if not args.no_parity_report:
                rec["parity_report"] = parity_report(wo, Oo, prob_o, plan_o)
            others[name] = rec
            del wo, Qo, Ko, Vo, Oo, plan_o, ws_o
            torch.cuda.empty_cache()
        out["other_workloads"] = others

    if not args.no_cpu_baseline:
        import oracle
        Qf, Kf, Vf, w = cpu_inputs
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
