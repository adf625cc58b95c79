"""Parity of the HIP boundary finalisation (threshold + non-maximum suppression) with the CPU oracle:
integer result, bit-exact.  Scores are seeded and synthetic (the predictor network is not part of this
build): smooth noise with peaks, plain noise, heavily tied scores, and monotone ramps (the slowest case
for the round-based kernel: one chunk end per round)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_24606_amd as dhsa

pytestmark = pytest.mark.gpu


def scores(kind, L, seed):
    rng = np.random.default_rng(seed)
    if kind == "noise":
        return rng.random(L).astype(np.float32)
    if kind == "peaks":      # a low noise floor with a sharp peak every ~50 tokens, like a detector's output
        p = 0.2 * rng.random(L)
        at = np.cumsum(rng.integers(20, 80, size=L // 20 + 2))
        at = at[at < L]
        p[at] += 0.5 + 0.3 * rng.random(len(at))
        for d in (-1, 1):    # shoulders next to each peak
            ok = (at + d >= 0) & (at + d < L)
            p[at[ok] + d] += 0.3
        return p.astype(np.float32)
    if kind == "tied":
        return (np.round(rng.random(L) * 6) / 6).astype(np.float32)
    if kind == "ramp_up":
        return np.linspace(0.01, 0.99, L).astype(np.float32)
    if kind == "ramp_down":
        return np.linspace(0.99, 0.01, L).astype(np.float32)
    raise ValueError(kind)


CASES = [("noise", 1, 0.5, 0), ("noise", 2, 0.5, 8), ("noise", 777, 0.3, 8), ("noise", 131072, 0.5, 8),
         ("noise", 131072, 0.9, 64), ("noise", 100000, 0.0, 1), ("peaks", 131072, 0.4, 8), ("peaks", 32768, 0.4, 64),
         ("tied", 50000, 0.4, 8), ("tied", 4097, 0.0, 64), ("ramp_up", 20000, 0.2, 8), ("ramp_down", 20000, 0.2, 64),
         ("noise", 5000, 2.0, 8), ("noise", 5000, -1.0, 5000)]


@pytest.mark.parametrize("kind,L,tau,W", CASES, ids=[f"{k}-L{L}-t{t}-W{W}" for k, L, t, W in CASES])
def test_finalize_boundaries_parity(kind, L, tau, W):
    p = scores(kind, L, 1234 + L + W)
    if kind == "noise" and L == 777:
        p[::5] = np.nan          # NaN scores never exceed the threshold
    want = oracle.finalize_boundaries(p, tau, W)
    got = dhsa.dhsa_finalize_boundaries(torch.from_numpy(p).cuda(), tau, W)
    print(f"\n[{kind} L={L} tau={tau} W={W}] N_c = {len(want) - 1}", flush=True)
    np.testing.assert_array_equal(got, want)


def test_boundaries_feed_the_path():
    """Scores -> boundaries on the GPU -> the prefill path on those boundaries, against the oracle end to end."""
    import dhsa_inputs
    w = dhsa_inputs.make("c3", L=8192, H_q=4, H_kv=2, N_b=512)
    p = scores("peaks", w.L, 99)
    B = dhsa.dhsa_finalize_boundaries(torch.from_numpy(p).cuda(), 0.4, 8)
    np.testing.assert_array_equal(B, oracle.finalize_boundaries(p, 0.4, 8))
    Q, K, V = (t.cuda() for t in (w.Q, w.K, w.V))
    O = torch.empty_like(Q)
    prob = dhsa.problem(Q, K, B, w.N_b)
    plan, ws = dhsa.alloc(prob, B)
    dhsa.dhsa_prefill(prob, Q, K, V, B, O, plan, ws)
    torch.cuda.synchronize()
    rows = np.arange(0, w.L, 7, dtype=np.int64)
    O_ref, I_ref, cnt_ref = oracle.prefill_rows(w.f32("Q"), w.f32("K"), w.f32("V"), B, w.N_b, rows)
    for h in range(w.H_q):
        idx, cnt = dhsa.dhsa_plan_expand_rows(prob, plan, h, rows)
        np.testing.assert_array_equal(idx.cpu().numpy(), I_ref[h])
        np.testing.assert_array_equal(cnt.cpu().numpy(), cnt_ref[h])
    err = np.abs(O[:, torch.from_numpy(rows).cuda()].float().cpu().numpy().astype(np.float64) - O_ref).max()
    assert err <= 2e-2, err
