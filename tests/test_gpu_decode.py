"""One decoding step (dhsa_decode_step, through the C ABI) against the CPU oracle:
the newest token's selected keys bit-exact, its output row within the attention
tolerances (1e-4 fp32, 2e-2 bf16).  The oracle is the prefill path's row L - 1."""
import numpy as np
import pytest
import torch

import dhsa_inputs
import oracle
import paper_2510_24606_amd as dhsa

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}

CASES = [
    # name, overrides, B_r
    ("c1", dict(), 0),                                                   # fp32, D = 64, G = 4
    ("c1", dict(L=777, N_b=5000), 0),                                    # N_b > L: every token
    ("c1", dict(L=1536, D=128, N_b=300, lens=("uniform", 1, 9)), 0),     # fp32, D = 128, tiny chunks
    ("c2", dict(L=6000, H_q=8, H_kv=2, N_b=384), 0),                     # bf16, D = 128
    ("c3", dict(L=4096, H_q=4, H_kv=4, D=64, N_b=256), 0),               # bf16, D = 64
    ("c5", dict(L=6144, H_q=7, H_kv=1, N_b=768), 0),                     # G = 7, chunks up to 256
    ("c4", dict(L=10007, H_q=8, H_kv=8, N_b=313), 0),                    # odd L, geometric lens
    ("c3", dict(L=3000, H_q=2, H_kv=1, N_b=700, lens=("fixed", 3000)), 0),    # one chunk
    ("c3", dict(L=2048, H_q=2, H_kv=2, N_b=100, lens=("fixed", 1)), 0),       # one-token chunks
    ("c3", dict(L=8192, H_q=2, H_kv=1, N_b=600, lens=("fixed", 1)), 0),       # N_c = 8192, > 256 plan entries
    ("c3", dict(L=8192, H_q=8, H_kv=2, N_b=512), 128),                   # Alg. 1 row blocks
    ("c1", dict(L=1000, N_b=100), 48),                                   # row blocks, fp32, ragged open block
    ("c2", dict(L=5000, H_q=6, H_kv=3, N_b=1), 0),                       # a budget of one key
]


def open_group_start(w, B_r):
    return ((w.L - 1) // B_r) * B_r if B_r else int(w.B[-2])


def oracle_row(w, B_r, pooling=0, L=None, B=None):
    L = w.L if L is None else L
    B = w.B if B is None else B
    return oracle.decode_row(w.f32("Q")[:, :L], w.f32("K")[:, :L], w.f32("V")[:, :L], B, w.N_b, B_r=B_r,
                             pooling=pooling)


def check(w, O_row, idx, cnt, O_ref, I_ref, cnt_ref):
    np.testing.assert_array_equal(cnt.cpu().numpy(), cnt_ref)
    cap = idx.shape[1]
    np.testing.assert_array_equal(idx.cpu().numpy(), I_ref[:, :cap])
    assert (I_ref[:, cap:] == -1).all()
    got = O_row.float().cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    err = np.abs(got - O_ref).max()
    assert err <= TOL[w.dtype], f"max |O_row - oracle| = {err}"
    return err


@pytest.mark.parametrize("name,kw,B_r", CASES, ids=[f"{n}-Br{b}-{i}" for i, (n, _, b) in enumerate(CASES)])
def test_decode_step_parity(name, kw, B_r):
    w = dhsa_inputs.make(name, **kw)
    print(f"\n[{name} {kw} B_r={B_r}] L={w.L} N_c={w.N_c} N_b={w.N_b} dtype={w.dtype}", flush=True)
    Q, K, V = (t.cuda() for t in (w.Q, w.K, w.V))
    # the queries below the open query group play no part: poison them
    Q[:, :open_group_start(w, B_r)] = float("nan")
    prob = dhsa.problem(Q, K, w.B, w.N_b, B_r=B_r)
    ws = dhsa.alloc_decode(prob, w.N_c, w.L)
    O_row, idx, cnt = dhsa.dhsa_decode_step(prob, Q, K, V, w.B, ws, w.N_c, w.L, 0, want_idx=True)
    torch.cuda.synchronize()
    O_ref, I_ref, cnt_ref = oracle_row(w, B_r)
    err = check(w, O_row, idx, cnt, O_ref, I_ref, cnt_ref)
    # without the optional outputs, and with larger caps: the same row, bit for bit
    ws2 = dhsa.alloc_decode(prob, min(w.N_c + 7, 8192), w.L + 1000)
    O2 = dhsa.dhsa_decode_step(prob, Q, K, V, w.B, ws2, min(w.N_c + 7, 8192), w.L + 1000, 0)
    torch.cuda.synchronize()
    assert torch.equal(O2.view(torch.int16 if w.dtype == "bf16" else torch.int32),
                       O_row.view(torch.int16 if w.dtype == "bf16" else torch.int32))
    print(f"   keys exact on {w.H_q} heads ({int(cnt_ref[0])} each); max |O_row - oracle| = {err:.3e}", flush=True)


def test_decode_equals_the_prefill_row():
    """The step's output is the prefill path's last row (same selection, same keys; the two
    attention kernels differ in arithmetic only)."""
    w = dhsa_inputs.make("c3", L=8192, H_q=8, H_kv=2, N_b=512)
    Q, K, V = (t.cuda() for t in (w.Q, w.K, w.V))
    prob = dhsa.problem(Q, K, w.B, w.N_b)
    plan, ws = dhsa.alloc(prob, w.B)
    O = torch.empty_like(Q)
    dhsa.dhsa_prefill(prob, Q, K, V, w.B, O, plan, ws)
    wsd = dhsa.alloc_decode(prob, w.N_c, w.L)
    O_row, idx, cnt = dhsa.dhsa_decode_step(prob, Q, K, V, w.B, wsd, w.N_c, w.L, 0, want_idx=True)
    torch.cuda.synchronize()
    rows = np.array([w.L - 1], dtype=np.int64)
    for h in range(w.H_q):
        I_p, c_p = dhsa.dhsa_plan_expand_rows(prob, plan, h, rows)
        assert torch.equal(I_p[0], idx[h]) and int(c_p[0]) == int(cnt[h])
    assert (O[:, -1].float() - O_row.float()).abs().max().item() <= 2e-2


@pytest.mark.parametrize("B_r,pooling", [(0, 0), (32, 0), (0, 1)], ids=["chunks", "row_blocks", "mean_pooling"])
def test_generation_loop_reuses_the_pooled_keys(B_r, pooling):
    """40 steps over growing caches: a new token joins the open chunk or starts a chunk; the pooled
    keys of closed chunks are reused (kc_valid = N_c - 1).  Every step is checked against the oracle
    and is bit-identical to a step that pools everything anew."""
    L0, steps = 2500, 40
    w = dhsa_inputs.make("c3", L=L0 + steps, H_q=8, H_kv=2, N_b=300, lens=("uniform", 8, 40))
    rng = np.random.default_rng(5)
    Q, K, V = (t.cuda() for t in (w.Q, w.K, w.V))      # caches with room for every step
    B = [int(b) for b in w.B if b < L0] + [L0]          # boundaries of the first L0 tokens
    N_c_cap, L_cap = len(B) + steps, L0 + steps
    ws = ws_cold = None
    worst = 0.0
    bits = torch.int16
    for t in range(steps):
        L = L0 + t + 1
        if rng.random() < 0.3:
            B = B + [L]             # the new token starts a chunk
        else:
            B = B[:-1] + [L]        # ... or joins the open one
        Bt = np.asarray(B, dtype=np.int32)
        Qv, Kv, Vv = Q[:, :L], K[:, :L], V[:, :L]
        prob = dhsa.problem(Qv, Kv, Bt, w.N_b, B_r=B_r, pooling=pooling, V=Vv)
        if ws is None:
            ws = dhsa.alloc_decode(prob, N_c_cap, L_cap)
            ws_cold = dhsa.alloc_decode(prob, N_c_cap, L_cap)
        N_c = len(B) - 1
        O_row, idx, cnt = dhsa.dhsa_decode_step(prob, Qv, Kv, Vv, Bt, ws, N_c_cap, L_cap,
                                                0 if t == 0 else N_c - 1, want_idx=True)
        ws_cold.zero_()
        O_c, idx_c, cnt_c = dhsa.dhsa_decode_step(prob, Qv, Kv, Vv, Bt, ws_cold, N_c_cap, L_cap, 0, want_idx=True)
        torch.cuda.synchronize()
        assert torch.equal(O_row.view(bits), O_c.view(bits)) and torch.equal(idx, idx_c) and torch.equal(cnt, cnt_c)
        O_ref, I_ref, cnt_ref = oracle_row(w, B_r, pooling, L=L, B=Bt)
        worst = max(worst, check(w, O_row, idx, cnt, O_ref, I_ref, cnt_ref))
    print(f"\n   {steps} steps, N_c {len(w.B) - 1} -> {len(B) - 1}; max |O_row - oracle| = {worst:.3e}", flush=True)


@pytest.mark.parametrize("name", ["c3", "c4"])
def test_full_size_decode_step(name):
    """The step at the full context length of the workload (131072 / 100000 tokens)."""
    w = dhsa_inputs.make(name)
    Q, K, V = (t.cuda() for t in (w.Q, w.K, w.V))
    for B_r in (0, 128):
        prob = dhsa.problem(Q, K, w.B, w.N_b, B_r=B_r)
        ws = dhsa.alloc_decode(prob, w.N_c, w.L)
        O_row, idx, cnt = dhsa.dhsa_decode_step(prob, Q, K, V, w.B, ws, w.N_c, w.L, 0, want_idx=True)
        torch.cuda.synchronize()
        O_ref, I_ref, cnt_ref = oracle_row(w, B_r)
        err = check(w, O_row, idx, cnt, O_ref, I_ref, cnt_ref)
        print(f"\n   {name} B_r={B_r}: keys exact on {w.H_q} heads; max |O_row - oracle| = {err:.3e}", flush=True)
