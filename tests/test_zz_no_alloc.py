"""dhsa_prefill_static (routing scratch in the library's static device array, for
callers that cannot allocate) against dhsa_prefill, through the C ABI.

Both run the same kernels on the same inputs, so the plan must be equal word by
word and O bit for bit.  Two calls in a row share the static array: the second
is a smaller problem whose scratch overlaps what the first call left behind.
"""
import numpy as np
import pytest
import torch

import dhsa_inputs
import paper_2510_24606_amd as dhsa

pytestmark = pytest.mark.gpu


def both_ways(name, B_r=0, **kw):
    w = dhsa_inputs.make(name, **kw)
    Q, K, V = (t.cuda() for t in (w.Q, w.K, w.V))
    prob = dhsa.problem(Q, K, w.B, w.N_b, B_r=B_r)
    assert dhsa.dhsa_workspace_bytes(prob, w.B) <= dhsa.dhsa_static_scratch_bytes()
    plan_a, ws = dhsa.alloc(prob, w.B)
    plan_a.zero_()
    plan_b = torch.zeros_like(plan_a)
    O_a = torch.full_like(Q, float("nan"))
    O_b = torch.full_like(Q, float("nan"))
    dhsa.dhsa_prefill(prob, Q, K, V, w.B, O_a, plan_a, ws)
    dhsa.dhsa_prefill_static(prob, Q, K, V, w.B, O_b, plan_b)
    torch.cuda.synchronize()
    pa, pb = dhsa.parse_plan(plan_a.cpu().numpy()), dhsa.parse_plan(plan_b.cpu().numpy())
    for key in ("B", "RB", "count", "tiles"):
        np.testing.assert_array_equal(pa[key], pb[key], err_msg=f"{name}: plan part {key}")
    live = np.arange(pa["stride"])[None, None, :] < pa["count"][:, :, None]
    np.testing.assert_array_equal(pa["entries"][live], pb["entries"][live], err_msg=f"{name}: plan entries")
    assert not torch.isnan(O_b.float()).any()
    assert torch.equal(O_a.view(torch.int16 if Q.dtype == torch.bfloat16 else torch.int32),
                       O_b.view(torch.int16 if Q.dtype == torch.bfloat16 else torch.int32)), f"{name}: O differs"


def test_static_scratch_two_calls_in_a_row():
    # a bf16 problem with > 960 boundaries (two argument blocks), then a smaller fp32 one, then row blocks
    both_ways("c2", L=16384, H_q=4, H_kv=2, N_b=1024, lens=("uniform", 8, 24))
    both_ways("c1", L=1536, N_b=192)
    both_ways("c3", B_r=128, L=4096, H_q=8, H_kv=2, N_b=512)


def test_static_scratch_limit():
    """A problem whose routing scratch exceeds the static array is rejected before any launch."""
    # 64 query heads x 8192 one-token chunks: S_c alone would be 64 * 8192 * 8192 * 8 bytes
    L = 8192
    Qb = torch.zeros((64, L, 64), dtype=torch.float32, device="cuda")
    Kb = torch.zeros((1, L, 64), dtype=torch.float32, device="cuda")
    B = np.arange(L + 1, dtype=np.int32)
    prob = dhsa.problem(Qb, Kb, B, 16)
    assert dhsa.dhsa_workspace_bytes(prob, B) > dhsa.dhsa_static_scratch_bytes()
    plan = torch.zeros(max(dhsa.dhsa_plan_bytes(prob, B), 256), dtype=torch.uint8, device="cuda")
    O = torch.full_like(Qb, 7.0)
    with pytest.raises(dhsa.DhsaError) as e:
        dhsa.dhsa_prefill_static(prob, Qb, Kb, Kb, B, O, plan)
    assert e.value.code == 6
    torch.cuda.synchronize()
    assert (O == 7.0).all() and (plan == 0).all()
