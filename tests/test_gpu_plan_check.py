"""A plan that was routed for another problem of equal size must not be used silently:
the kernels compare the plan's header with the problem and leave the outputs untouched,
dhsa_plan_check reports the mismatch to the host.  Also the two small inspection calls
dhsa_prefill_stage_times and dhsa_debug_scores."""
import numpy as np
import pytest
import torch

import dhsa_inputs
import paper_2510_24606_amd as dhsa

pytestmark = pytest.mark.gpu


def setup(name="c3", **kw):
    w = dhsa_inputs.make(name, **kw)
    Q, K, V = (t.cuda() for t in (w.Q, w.K, w.V))
    return w, Q, K, V


def attend_with_foreign_plan(w, Q, K, V, prob_route, B_route, prob_use, B_use):
    plan, ws = dhsa.alloc(prob_route, B_route)
    dhsa.dhsa_route(prob_route, Q, K, B_route, plan, ws)
    assert dhsa.dhsa_plan_bytes(prob_use, B_use) == plan.numel(), "the case must pass the host's size check"
    dhsa.dhsa_plan_check(prob_route, B_route, plan)            # its own problem: fine
    with pytest.raises(dhsa.DhsaError) as e:
        dhsa.dhsa_plan_check(prob_use, B_use, plan)
    assert e.value.code == 8
    O = torch.full_like(Q, 3.0)
    dhsa.dhsa_sparse_prefill(prob_use, Q, K, V, B_use, plan, O)    # enqueued: the host cannot see the mismatch
    torch.cuda.synchronize()
    assert (O == 3.0).all(), "a foreign plan must leave O untouched"
    rows = np.arange(0, w.L, 97, dtype=np.int64)
    hits, size = dhsa.dhsa_recall_rows(prob_route, Q, K, B_route, plan, 0, rows)
    torch.cuda.synchronize()
    assert (size.cpu().numpy() == np.minimum(prob_route.N_b, rows + 1)).all()
    # and the right plan still works
    dhsa.dhsa_sparse_prefill(prob_route, Q, K, V, B_route, plan, O)
    torch.cuda.synchronize()
    assert not (O == 3.0).all() and torch.isfinite(O.float()).all()


@pytest.mark.parametrize("name,kw", [("c3", dict(L=4096, H_q=4, H_kv=2, N_b=256)), ("c1", dict(L=1024, N_b=128))])
def test_plan_of_another_representation(name, kw):
    w, Q, K, V = setup(name, **kw)
    attend_with_foreign_plan(w, Q, K, V, dhsa.problem(Q, K, w.B, w.N_b, pooling=dhsa.DHSA_POOL_ROBUST), w.B,
                             dhsa.problem(Q, K, w.B, w.N_b, pooling=dhsa.DHSA_POOL_MEAN), w.B)


def test_plan_of_other_boundaries_with_the_same_lengths():
    w, Q, K, V = setup("c3", L=4096, H_q=4, H_kv=2, N_b=256)
    B2 = np.r_[0, np.cumsum(np.diff(w.B)[::-1])].astype(np.int32)      # the same chunk lengths in reverse order
    assert not np.array_equal(B2, w.B)
    prob = dhsa.problem(Q, K, w.B, w.N_b)
    attend_with_foreign_plan(w, Q, K, V, prob, w.B, dhsa.problem(Q, K, B2, w.N_b), B2)


def test_plan_of_another_budget():
    w, Q, K, V = setup("c3", L=4096, H_q=4, H_kv=2, N_b=256)
    for nb2 in (255, 257, 250, 260):
        p1, p2 = dhsa.problem(Q, K, w.B, w.N_b), dhsa.problem(Q, K, w.B, nb2)
        if dhsa.dhsa_plan_bytes(p1, w.B) == dhsa.dhsa_plan_bytes(p2, w.B):
            attend_with_foreign_plan(w, Q, K, V, p1, w.B, p2, w.B)
            return
    pytest.skip("no nearby budget gives a plan of the same size")


def test_stage_times_and_debug_scores():
    w, Q, K, V = setup("c3", L=8192, H_q=8, H_kv=2, N_b=512)
    prob = dhsa.problem(Q, K, w.B, w.N_b)
    plan, ws = dhsa.alloc(prob, w.B)
    O1, O2 = torch.empty_like(Q), torch.empty_like(Q)
    dhsa.dhsa_prefill(prob, Q, K, V, w.B, O1, plan, ws)
    t = dhsa.dhsa_prefill_stage_times(prob, Q, K, V, w.B, O2, plan, ws)
    torch.cuda.synchronize()
    assert torch.equal(O1.view(torch.int16), O2.view(torch.int16))
    assert set(t) == set(dhsa.STAGES) and all(v >= 0.0 for v in t.values())
    parts = sum(v for k, v in t.items() if k != "total")
    assert t["pool"] > 0 and t["scores"] > 0 and t["select"] > 0 and t["attn_rows_gt64"] > 0
    assert abs(parts - t["total"]) <= 0.02 * t["total"] + 0.01
    _, _, Sc = dhsa.dhsa_debug_routing(prob, w.B, ws)
    Sc2 = dhsa.dhsa_debug_scores(prob, w.B, ws)
    tri = np.tril(np.ones((w.N_c, w.N_c), dtype=bool))
    np.testing.assert_array_equal(Sc.cpu().numpy()[:, tri], Sc2.cpu().numpy()[:, tri])
