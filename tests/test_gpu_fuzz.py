"""Seeded random small problems through the C ABI against the oracle, every row: shapes, chunk laws,
budgets, head groupings, both dtypes, both head sizes, the row form and the row-block form, both
chunk representations; each also runs the recall diagnostic on a few rows and one decoding step for
its newest token.  Integer results bit-exact, outputs within the tolerance of the dtype."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_24606_amd as dhsa

pytestmark = pytest.mark.gpu

TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2}


def draw_case(seed):
    rng = np.random.default_rng(9000 + seed)
    L = int(rng.choice([1, 2, 31, 33, 64, 65, 127, 129, 200, 513, 1000, 1777, 2500]))
    law = rng.integers(0, 4)
    if law == 0:
        lens_hi = int(rng.integers(1, 8))
    elif law == 1:
        lens_hi = int(rng.integers(8, 70))
    elif law == 2:
        lens_hi = int(rng.integers(70, 300))
    else:
        lens_hi = L + 5                                   # often a single chunk
    B = [0]
    while B[-1] < L:
        B.append(min(L, B[-1] + int(rng.integers(1, lens_hi + 1))))
    B = np.asarray(B, dtype=np.int32)
    H_kv = int(rng.choice([1, 2, 3]))
    G = int(rng.choice([1, 2, 4, 7]))
    D = int(rng.choice([64, 128]))
    dtype = torch.bfloat16 if rng.random() < 0.7 else torch.float32
    N_b = int(rng.choice([1, 2, 17, 64, 100, 257, L, L + 9]))
    B_r = int(rng.choice([0, 0, 1, 16, 32, 50, 128, 200]))
    pooling = int(rng.random() < 0.25)
    scale = float(rng.choice([0.0, 0.0, 0.3]))
    g = torch.Generator().manual_seed(1234 + seed)
    Q = torch.randn((H_kv * G, L, D), generator=g).to(dtype)
    K = torch.randn((H_kv, L, D), generator=g).to(dtype)
    V = torch.randn((H_kv, L, D), generator=g).to(dtype)
    return dict(L=L, B=B, H_kv=H_kv, G=G, D=D, dtype=dtype, N_b=N_b, B_r=B_r, pooling=pooling, scale=scale,
                Q=Q, K=K, V=V)


@pytest.mark.parametrize("seed", range(48))
def test_random_small_problem(seed):
    c = draw_case(seed)
    print(f"\n[seed {seed}] L={c['L']} N_c={len(c['B']) - 1} H={c['H_kv'] * c['G']}/{c['H_kv']} D={c['D']} "
          f"{c['dtype']} N_b={c['N_b']} B_r={c['B_r']} pooling={c['pooling']} scale={c['scale']}", flush=True)
    Q, K, V = (c[k].cuda() for k in "QKV")
    O = torch.full_like(Q, float("nan"))
    prob = dhsa.problem(Q, K, c["B"], c["N_b"], c["scale"], B_r=c["B_r"], pooling=c["pooling"])
    plan, ws = dhsa.alloc(prob, c["B"])
    dhsa.dhsa_prefill(prob, Q, K, V, c["B"], O, plan, ws)
    torch.cuda.synchronize()
    Qf, Kf, Vf = (c[k].float().numpy() for k in "QKV")
    rows = np.arange(c["L"], dtype=np.int64)
    sc = c["scale"] if c["scale"] > 0 else None
    if c["B_r"]:
        O_ref, I_ref, cnt_ref = oracle.prefill_rows_blocks(Qf, Kf, Vf, c["B"], c["B_r"], c["N_b"], rows, scale=sc,
                                                           pooling=c["pooling"])
    else:
        O_ref, I_ref, cnt_ref = oracle.prefill_rows(Qf, Kf, Vf, c["B"], c["N_b"], rows, scale=sc, pooling=c["pooling"])
    for h in range(Q.shape[0]):
        idx, cnt = dhsa.dhsa_plan_expand_rows(prob, plan, h, rows)
        np.testing.assert_array_equal(cnt.cpu().numpy(), cnt_ref[h])
        cap = idx.shape[1]
        np.testing.assert_array_equal(idx.cpu().numpy(), I_ref[h][:, :cap])
    got = O.float().cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    err = np.abs(got - O_ref).max()
    assert err <= TOL[c["dtype"]], err
    # the recall diagnostic on a few rows of the last head
    rr = rows[:: max(1, c["L"] // 7)]
    hits, size = dhsa.dhsa_recall_rows(prob, Q, K, c["B"], plan, Q.shape[0] - 1, rr)
    torch.cuda.synchronize()
    h_ref, s_ref = oracle.recall_rows(Qf, Kf, c["B"], c["N_b"], Q.shape[0] - 1, rr, B_r=c["B_r"], pooling=c["pooling"])
    np.testing.assert_array_equal(hits.cpu().numpy(), h_ref)
    np.testing.assert_array_equal(size.cpu().numpy(), s_ref)
    # one decoding step for the newest token: the last row of the same problem
    wsd = dhsa.alloc_decode(prob, len(c["B"]) - 1, c["L"])
    O_row, idx_d, cnt_d = dhsa.dhsa_decode_step(prob, Q, K, V, c["B"], wsd, len(c["B"]) - 1, c["L"], 0, want_idx=True)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(cnt_d.cpu().numpy(), cnt_ref[:, -1])
    np.testing.assert_array_equal(idx_d.cpu().numpy(), I_ref[:, -1, :idx_d.shape[1]])
    err_d = np.abs(O_row.float().cpu().numpy().astype(np.float64) - O_ref[:, -1]).max()
    assert err_d <= TOL[c["dtype"]], err_d
