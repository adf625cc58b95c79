"""The mask the attention kernels APPLY, pinned key by key (Alg. 2's mask; Alg. 1's index sets).

The plan is routed with the workload's real Q and K.  Attention is then run on
that plan with Q = 0 and V[j, d] = [j mod D = d]: every attended key gets weight
exactly 1 / |I_i| (all logits are 0), so O[i, d] * |I_i| is the number of
attended keys of row i in residue class d.  One key wrongly attended or dropped
changes an integer count of about |I_i| / D by one, far above the rounding of a
bf16 output (2^-9 relative, counts stay below 256), so the comparison with the
oracle's index sets is exact.
"""
import numpy as np
import pytest
import torch

import dhsa_inputs
import oracle
import paper_2510_24606_amd as dhsa

pytestmark = pytest.mark.gpu


def gpu_counts(w, B_r, rows):
    """O of `rows` for every head from a plan routed with the real Q, attended with Q = 0 and one-hot V."""
    Q, K = w.Q.cuda(), w.K.cuda()
    prob = dhsa.problem(Q, K, w.B, w.N_b, B_r=B_r)
    plan, ws = dhsa.alloc(prob, w.B)
    dhsa.dhsa_route(prob, Q, K, w.B, plan, ws)
    Q0 = torch.zeros_like(Q)
    V1 = torch.zeros_like(K)
    j = torch.arange(w.L, device="cuda")
    V1[:, j, j % w.D] = 1.0
    O = torch.full_like(Q, float("nan"))
    dhsa.dhsa_sparse_prefill(prob, Q0, K, V1, w.B, plan, O)
    torch.cuda.synchronize()
    return O[:, torch.from_numpy(rows).cuda()].float().cpu().numpy().astype(np.float64)


def oracle_counts(w, B_r, rows):
    """(per-residue counts [H_q, n, D], set sizes [H_q, n]) of the keys each row attends, from the oracle."""
    Qf, Kf = w.f32("Q"), w.f32("K")
    n = len(rows)
    if B_r == 0:
        I, cnt = oracle.route_rows(Qf, Kf, w.B, w.N_b, rows)
        keep = np.arange(I.shape[2])[None, None, :] < cnt[:, :, None]
    else:
        blocks, inv = np.unique(rows // B_r, return_inverse=True)
        Ib, cb = oracle.route_blocks(Qf, Kf, w.B, B_r, w.N_b, blocks)
        I, cnt = Ib[:, inv], cb[:, inv]
        # Alg. 2: row i attends the listed keys at or below i
        keep = (np.arange(I.shape[2])[None, None, :] < cnt[:, :, None]) & (I <= rows[None, :, None])
    H = I.shape[0]
    flat = (np.arange(H)[:, None, None] * n + np.arange(n)[None, :, None]) * w.D + (I % w.D)
    counts = np.bincount(flat[keep], minlength=H * n * w.D).reshape(H, n, w.D)
    return counts, keep.sum(2)


def check(w, B_r, rows):
    want, size = oracle_counts(w, B_r, rows)
    assert want.max() < 256                      # bf16 rounding of O stays below half a count
    got = gpu_counts(w, B_r, rows) * size[:, :, None]
    assert np.isfinite(got).all()
    np.testing.assert_array_equal(np.rint(got).astype(np.int64), want)
    assert np.abs(got - np.rint(got)).max() < 0.26
    return int(size.sum())


ALL_ROWS = [
    # both launch classes of the bf16 kernel (row tiles above and below 64 rows), ragged tails
    ("c3", dict(L=8192, H_q=8, H_kv=2, N_b=512), 0),
    ("c3", dict(L=8192, H_q=8, H_kv=2, N_b=512), 128),
    # geometric chunk lengths 8..512: row tiles of every size, several tiles per chunk
    ("c4", dict(L=10007, H_q=8, H_kv=8, N_b=313), 0),
    ("c4", dict(L=10007, H_q=8, H_kv=8, N_b=313), 100),
    # more than 256 plan entries per query group (several entry batches in the kernel)
    ("c2", dict(L=5000, H_q=6, H_kv=3, N_b=4000, lens=("uniform", 4, 12)), 0),
    ("c2", dict(L=5000, H_q=6, H_kv=3, N_b=4000, lens=("uniform", 4, 12)), 128),
    # D = 64, and the fp32 kernel
    ("c3", dict(L=4096, H_q=4, H_kv=4, D=64, N_b=256), 0),
    ("c1", dict(), 0),
    ("c1", dict(), 32),
]


@pytest.mark.parametrize("name,kw,B_r", ALL_ROWS, ids=[f"{n}-{i}-Br{b}" for i, (n, _, b) in enumerate(ALL_ROWS)])
def test_applied_mask_every_row(name, kw, B_r):
    w = dhsa_inputs.make(name, **kw)
    pairs = check(w, B_r, np.arange(w.L, dtype=np.int64))
    print(f"\n[{name} {kw} B_r={B_r}] applied mask exact on {w.L} rows x {w.H_q} heads ({pairs} attended pairs)",
          flush=True)


@pytest.mark.parametrize("name,B_r", [("c3", 0), ("c3", 128), ("c4", 0)])
def test_applied_mask_full_size_sample(name, B_r):
    """The bench configuration itself: sampled rows of every head at full size."""
    w = dhsa_inputs.make(name)
    rows = dhsa_inputs.sample_rows(w, 192)
    pairs = check(w, B_r, rows)
    print(f"\n[{name} full size B_r={B_r}] applied mask exact on {len(rows)} rows x {w.H_q} heads "
          f"({pairs} attended pairs)", flush=True)
