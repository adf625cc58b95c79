"""Parity for the ablation variants of App. D: plain average pooling ("without robust chunk
representation"), fixed-size chunks ("without dynamic chunking"), and both together (conventional
block-sparse attention) -- through the same entry points, against the oracle run in the same mode."""
import numpy as np
import pytest
import torch

import dhsa_inputs
import oracle
import paper_2510_24606_amd as dhsa

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}

CASES = [
    # workload, overrides, B_r, what
    ("c1", dict(L=1500, N_b=200), 0, "mean pooling, dynamic chunks, fp32"),
    ("c3", dict(L=8192, H_q=8, H_kv=2, N_b=512), 0, "mean pooling, dynamic chunks"),
    ("c4", dict(L=10007, H_q=8, H_kv=4, N_b=313), 0, "mean pooling, geometric chunk lengths"),
    ("c3", dict(L=8192, H_q=8, H_kv=2, N_b=512, lens=("fixed", 64)), 0, "block-sparse: fixed chunks of 64 + mean pooling"),
    ("c2", dict(L=6000, H_q=8, H_kv=2, N_b=384), 128, "mean pooling, row blocks of 128"),
    ("c3", dict(L=8192, H_q=4, H_kv=2, N_b=512, lens=("fixed", 128)), 128, "block-sparse in the row-block form"),
]


@pytest.mark.parametrize("name,kw,B_r,what", CASES, ids=[f"{n}-Br{b}-{i}" for i, (n, _, b, _) in enumerate(CASES)])
def test_mean_pooling_and_fixed_chunks(name, kw, B_r, what):
    w = dhsa_inputs.make(name, **kw)
    print(f"\n[{what}] L={w.L} N_c={w.N_c} N_b={w.N_b} dtype={w.dtype}", flush=True)
    Q, K, V = (t.cuda() for t in (w.Q, w.K, w.V))
    O = torch.full_like(Q, float("nan"))
    prob = dhsa.problem(Q, K, w.B, w.N_b, B_r=B_r, pooling=dhsa.DHSA_POOL_MEAN)
    plan, ws = dhsa.alloc(prob, w.B)
    dhsa.dhsa_prefill(prob, Q, K, V, w.B, O, plan, ws)
    torch.cuda.synchronize()
    rows = np.arange(w.L, dtype=np.int64)
    if B_r:
        O_ref, I_ref, cnt_ref = oracle.prefill_rows_blocks(w.f32("Q"), w.f32("K"), w.f32("V"), w.B, B_r, w.N_b, rows,
                                                           pooling=1)
        Qp_ref = oracle.pool_blocks_mean(w.f32("Q"), B_r)
    else:
        O_ref, I_ref, cnt_ref = oracle.prefill_rows(w.f32("Q"), w.f32("K"), w.f32("V"), w.B, w.N_b, rows, pooling=1)
        Qp_ref = oracle.pool_mean(w.f32("Q"), w.B)
    Qp, Kp, _ = dhsa.dhsa_debug_routing(prob, w.B, ws, want_Sc=False)
    np.testing.assert_allclose(Qp.cpu().numpy(), Qp_ref, rtol=1e-14, atol=1e-14)
    np.testing.assert_allclose(Kp.cpu().numpy(), oracle.pool_mean(w.f32("K"), w.B), rtol=1e-14, atol=1e-14)
    for h in range(w.H_q):
        idx, cnt = dhsa.dhsa_plan_expand_rows(prob, plan, h, rows)
        np.testing.assert_array_equal(cnt.cpu().numpy(), cnt_ref[h])
        cap = idx.shape[1]
        np.testing.assert_array_equal(idx.cpu().numpy(), I_ref[h][:, :cap])
    got = O.float().cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    err = np.abs(got - O_ref).max()
    print(f"   lists exact on all {w.L} rows x {w.H_q} heads; max |O - oracle| = {err:.3e}", flush=True)
    assert err <= TOL[w.dtype]


def test_fixed_chunks_with_either_pooling_select_the_same_keys():
    """App. D: with uniform chunks the two representations differ by one common factor, so the
    selected sets (hence the outputs) are identical."""
    w = dhsa_inputs.make("c3", L=8192, H_q=4, H_kv=2, N_b=512, lens=("fixed", 64))
    Q, K, V = (t.cuda() for t in (w.Q, w.K, w.V))
    outs = []
    for pooling in (dhsa.DHSA_POOL_ROBUST, dhsa.DHSA_POOL_MEAN):
        O = torch.empty_like(Q)
        prob = dhsa.problem(Q, K, w.B, w.N_b, pooling=pooling)
        plan, ws = dhsa.alloc(prob, w.B)
        dhsa.dhsa_prefill(prob, Q, K, V, w.B, O, plan, ws)
        torch.cuda.synchronize()
        outs.append(O)
    assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16))


# ----------------------------------------------------------------------------
# Recall of the routed sets against exact top-k attention (integer counts, bit-exact)
# ----------------------------------------------------------------------------
RECALL_CASES = [
    ("c1", dict(L=1500, N_b=200), 0, 0),
    ("c2", dict(L=4000, H_q=4, H_kv=2, N_b=384), 0, 0),
    ("c3", dict(L=4096, H_q=4, H_kv=2, N_b=512), 0, 1),                       # plain average pooling
    ("c3", dict(L=4096, H_q=4, H_kv=2, N_b=512), 128, 0),                     # row blocks
    ("c3", dict(L=2048, H_q=2, H_kv=2, D=64, N_b=100, lens=("fixed", 1)), 0, 0),   # one-token chunks: recall 1
]


@pytest.mark.parametrize("name,kw,B_r,pooling", RECALL_CASES,
                         ids=[f"{n}-Br{b}-p{p}-{i}" for i, (n, _, b, p) in enumerate(RECALL_CASES)])
def test_recall_rows_parity(name, kw, B_r, pooling):
    w = dhsa_inputs.make(name, **kw)
    Q, K = w.Q.cuda(), w.K.cuda()
    prob = dhsa.problem(Q, K, w.B, w.N_b, B_r=B_r, pooling=pooling)
    plan, ws = dhsa.alloc(prob, w.B)
    dhsa.dhsa_route(prob, Q, K, w.B, plan, ws)
    rows = np.arange(0, w.L, 3, dtype=np.int64)
    for head in (0, w.H_q - 1):
        hits, size = dhsa.dhsa_recall_rows(prob, Q, K, w.B, plan, head, rows)
        torch.cuda.synchronize()
        h_ref, s_ref = oracle.recall_rows(w.f32("Q"), w.f32("K"), w.B, w.N_b, head, rows, B_r=B_r, pooling=pooling)
        np.testing.assert_array_equal(size.cpu().numpy(), s_ref)
        np.testing.assert_array_equal(hits.cpu().numpy(), h_ref)
        rec = hits.cpu().numpy() / np.maximum(size.cpu().numpy(), 1)
        print(f"\n[{name} B_r={B_r} pooling={pooling} head {head}] mean recall over {len(rows)} rows = {rec.mean():.4f}",
              flush=True)
        if kw.get("lens") == ("fixed", 1):
            assert (hits == size).all()


def test_recall_rows_full_size_sample():
    w = dhsa_inputs.make("c3")
    Q, K = w.Q.cuda(), w.K.cuda()
    prob = dhsa.problem(Q, K, w.B, w.N_b)
    plan, ws = dhsa.alloc(prob, w.B)
    dhsa.dhsa_route(prob, Q, K, w.B, plan, ws)
    rows = dhsa_inputs.sample_rows(w, 48)
    hits, size = dhsa.dhsa_recall_rows(prob, Q, K, w.B, plan, 5, rows)
    torch.cuda.synchronize()
    h_ref, s_ref = oracle.recall_rows(w.f32("Q"), w.f32("K"), w.B, w.N_b, 5, rows)
    np.testing.assert_array_equal(size.cpu().numpy(), s_ref)
    np.testing.assert_array_equal(hits.cpu().numpy(), h_ref)
    print(f"\n[c3 head 5] mean recall over {len(rows)} sampled rows = "
          f"{(hits.cpu().numpy() / size.cpu().numpy()).mean():.4f}", flush=True)
