"""Parity of the HIP path (through the C ABI) with the CPU oracle.

Bars (from the benchmark spec): routing mask bit-exact; attention output
max-abs error <= 1e-4 for fp32 inputs and <= 2e-2 for bf16 inputs.  Routing
scores are fp64 on both sides; groups whose cut-off score gap is below 1e-5
are counted and reported (none is expected to mismatch).
"""
import numpy as np
import pytest
import torch

import dhsa_inputs
import oracle
import paper_2510_24606_amd as dhsa

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def run_gpu(w, scale=0.0):
    Q, K, V = (t.cuda() for t in (w.Q, w.K, w.V))
    O = torch.full_like(Q, float("nan"))
    prob = dhsa.problem(Q, K, w.B, w.N_b, scale)
    plan, ws = dhsa.alloc(prob, w.B)
    dhsa.dhsa_prefill(prob, Q, K, V, w.B, O, plan, ws)
    torch.cuda.synchronize()
    return dict(prob=prob, plan=plan, ws=ws, O=O, Q=Q, K=K, V=V)


def check_mask_rows(w, g, rows, I_ref, cnt_ref):
    for h in range(w.H_q):
        idx, cnt = dhsa.dhsa_plan_expand_rows(g["prob"], g["plan"], h, rows)
        np.testing.assert_array_equal(cnt.cpu().numpy(), cnt_ref[h], err_msg=f"head {h} counts")
        cap = idx.shape[1]                       # min(N_b, L)
        np.testing.assert_array_equal(idx.cpu().numpy(), I_ref[h][:, :cap], err_msg=f"head {h} index sets")
        assert (I_ref[h][:, cap:] == -1).all()


def check_plan_all_chunks(w, g):
    """Every (head, query chunk): the plan lists exactly the chunks some row
    takes a token from, with the oracle's walk state; returns near-tie counts."""
    plan = dhsa.parse_plan(g["plan"].cpu().numpy())
    assert plan["N_c"] == w.N_c and plan["L"] == w.L and plan["N_b"] == min(w.N_b, w.L)
    np.testing.assert_array_equal(plan["B"], w.B)
    Qc = oracle.pool(w.f32("Q"), w.B)
    Kc = oracle.pool(w.f32("K"), w.B)
    G = w.H_q // w.H_kv
    near = 0
    lens = np.diff(w.B)
    for h in range(w.H_q):
        rem, pos, gap = oracle.plan_head(Qc[h], Kc[h // G], w.B, min(w.N_b, w.L))
        near += int((gap <= 1e-5).sum())
        need = ((pos < 2) & (rem > 0)) | ((pos == 2) & (rem > 1))
        cnt = plan["count"][h]
        np.testing.assert_array_equal(cnt, need.sum(1), err_msg=f"head {h}: entries per chunk")
        for l in range(w.N_c):
            e = plan["entries"][h, l, :cnt[l]]
            ks = np.nonzero(need[l])[0]
            np.testing.assert_array_equal(e[:, 0] & ((1 << dhsa.POS_SHIFT) - 1), ks)
            np.testing.assert_array_equal(e[:, 0] >> dhsa.POS_SHIFT, pos[l, ks])
            np.testing.assert_array_equal(e[:, 1], rem[l, ks])
    # tile table: rows of one chunk, <= 128 each, covering [0, L); listed by class (more than 96 rows,
    # 65..96, 33..64, at most 32), each class by row; the first T_big have more than 64 rows
    t = plan["tiles"]
    order = np.argsort(t[:, 1], kind="stable")
    nrows_t = np.empty(len(t), dtype=np.int64)
    nrows_t[order] = np.r_[t[order][1:, 1], w.L] - t[order][:, 1]
    cls = np.where(nrows_t > 96, 0, np.where(nrows_t > 64, 1, np.where(nrows_t > 32, 2, 3)))
    assert (np.diff(cls) >= 0).all() and (cls < 2).sum() == plan["T_big"]
    for c in range(4):
        assert (np.diff(t[cls == c, 1]) > 0).all()
    t = t[order]
    assert t[0, 1] == 0
    ends = np.r_[t[1:, 1], w.L]
    assert ((ends - t[:, 1]) <= 128).all() and ((ends - t[:, 1]) > 0).all()
    assert (w.B[t[:, 0]] <= t[:, 1]).all() and (ends <= w.B[t[:, 0] + 1]).all()
    del lens
    return near


def check_outputs(w, g, rows, O_ref):
    got = g["O"][:, torch.from_numpy(rows).cuda()].float().cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    err = np.abs(got - O_ref).max()
    assert err <= TOL[w.dtype], f"max |O - oracle| = {err}"
    return err


SMALL = [
    # name, overrides  -- sizes the oracle does in seconds, several row tiles and ragged tails
    ("c1", dict()),                                                   # the full small config
    ("c1", dict(L=1000, N_b=1)),
    ("c1", dict(L=777, N_b=5000)),                                    # N_b > L: dense causal
    ("c1", dict(L=1536, D=128, N_b=300, lens=("uniform", 1, 9))),     # tiny chunks, several entry batches
    ("c2", dict(L=6000, H_q=8, H_kv=2, N_b=384)),
    ("c3", dict(L=8192, H_q=8, H_kv=2, N_b=512)),
    ("c4", dict(L=10007, H_q=8, H_kv=8, N_b=313)),                    # odd L, geometric lens up to 512
    ("c5", dict(L=6144, H_q=7, H_kv=1, N_b=768)),                     # G = 7, chunks up to 256
    ("c3", dict(L=4096, H_q=4, H_kv=4, D=64, N_b=256)),               # bf16 with D = 64
    ("c2", dict(L=5000, H_q=6, H_kv=3, N_b=4000, lens=("uniform", 4, 12))),   # > 256 plan entries per chunk
    ("c3", dict(L=3000, H_q=2, H_kv=1, N_b=700, lens=("fixed", 3000))),       # one chunk
    ("c3", dict(L=2048, H_q=2, H_kv=2, N_b=100, lens=("fixed", 1))),          # one-token chunks
    ("c3", dict(L=8192, H_q=2, H_kv=1, N_b=64, lens=("fixed", 1))),           # N_c = 8192, the chunk-count limit
]


@pytest.mark.parametrize("name,kw", SMALL, ids=[f"{n}-{i}" for i, (n, _) in enumerate(SMALL)])
def test_small_full_parity(name, kw):
    w = dhsa_inputs.make(name, **kw)
    print(f"\n[{name} {kw}] L={w.L} N_c={w.N_c} N_b={w.N_b} dtype={w.dtype}", flush=True)
    g = run_gpu(w)
    rows = np.arange(w.L, dtype=np.int64)
    O_ref, I_ref, cnt_ref = oracle.prefill_rows(w.f32("Q"), w.f32("K"), w.f32("V"), w.B, w.N_b, rows)
    # stage-wise: pooled vectors and chunk scores
    Qc, Kc, Sc = dhsa.dhsa_debug_routing(g["prob"], w.B, g["ws"])
    Qc_ref, Kc_ref = oracle.pool(w.f32("Q"), w.B), oracle.pool(w.f32("K"), w.B)
    np.testing.assert_allclose(Qc.cpu().numpy(), Qc_ref, rtol=1e-14, atol=1e-14)
    np.testing.assert_allclose(Kc.cpu().numpy(), Kc_ref, rtol=1e-14, atol=1e-14)
    Sc_ref = oracle.scores(Qc_ref, Kc_ref)
    tri = np.tril(np.ones((w.N_c, w.N_c), dtype=bool))
    np.testing.assert_allclose(Sc.cpu().numpy()[:, tri], Sc_ref[:, tri], rtol=1e-12, atol=1e-11)
    # mask: every row, every head, bit-exact; and the compact plan itself
    check_mask_rows(w, g, rows, I_ref, cnt_ref)
    near = check_plan_all_chunks(w, g)
    err = check_outputs(w, g, rows, O_ref)
    print(f"   mask exact on all {w.L} rows x {w.H_q} heads; near-tie groups (<=1e-5): {near}; "
          f"max |O - oracle| = {err:.3e}", flush=True)


def test_row_tiles_at_the_edges_of_the_height_classes():
    """Chunks whose last row tile has exactly 1, 16, 17, 31, 32, 33, 63, 64, 65, 95, 96, 97, 127, 128 rows
    (alone and behind one or two full tiles): every wave arrangement of the attention kernels at the edge
    of its range, all rows compared."""
    rem = [1, 16, 17, 31, 32, 33, 48, 63, 64, 65, 80, 95, 96, 97, 112, 127, 128]
    lens = [r + 128 * f for f in (0, 1, 2) for r in rem]
    rng = np.random.default_rng(5)
    rng.shuffle(lens)
    B = np.r_[0, np.cumsum(lens)].astype(np.int32)
    L = int(B[-1])
    for D, N_b in ((128, 700), (64, 90)):
        w = dhsa_inputs.make("c2", L=L, H_q=4, H_kv=2, D=D, N_b=N_b, lens=("fixed", 1))
        w.B = B                                       # iid rows: nothing in Q, K, V depends on the boundaries
        w.Q, w.K, w.V = (t.clone() for t in (w.Q, w.K, w.V))
        g = run_gpu(w)
        rows = np.arange(L, dtype=np.int64)
        O_ref, I_ref, cnt_ref = oracle.prefill_rows(w.f32("Q"), w.f32("K"), w.f32("V"), w.B, w.N_b, rows)
        check_mask_rows(w, g, rows, I_ref, cnt_ref)
        check_plan_all_chunks(w, g)
        err = check_outputs(w, g, rows, O_ref)
        plan = dhsa.parse_plan(g["plan"].cpu().numpy())
        assert all(c > 0 for c in plan["T_cls"])      # all four height classes occur
        print(f"   D={D}: {len(lens)} chunks, tiles per class {plan['T_cls']}, max |O - oracle| = {err:.3e}", flush=True)


def plans_equal(a, b):
    """Compare the defined words of two plans (slots past `count` are unspecified)."""
    pa, pb = dhsa.parse_plan(a.cpu().numpy()), dhsa.parse_plan(b.cpu().numpy())
    for k in ("H_q", "N_c", "N_b", "stride", "L", "T1", "T_big"):
        if pa[k] != pb[k]:
            return False
    if not (np.array_equal(pa["B"], pb["B"]) and np.array_equal(pa["count"], pb["count"])
            and np.array_equal(pa["tiles"], pb["tiles"])):
        return False
    live = np.arange(pa["stride"])[None, None, :] < pa["count"][:, :, None]
    return np.array_equal(pa["entries"][live], pb["entries"][live])


def test_route_then_sparse_prefill_equals_prefill_and_is_deterministic():
    w = dhsa_inputs.make("c3", L=8192, H_q=8, H_kv=2, N_b=512)
    g1 = run_gpu(w)
    g2 = run_gpu(w)
    assert plans_equal(g1["plan"], g2["plan"])
    assert torch.equal(g1["O"].view(torch.int16), g2["O"].view(torch.int16))
    plan, ws = dhsa.alloc(g1["prob"], w.B)
    dhsa.dhsa_route(g1["prob"], g1["Q"], g1["K"], w.B, plan, ws)
    O = torch.zeros_like(g1["Q"])
    dhsa.dhsa_sparse_prefill(g1["prob"], g1["Q"], g1["K"], g1["V"], w.B, plan, O)
    dhsa.dhsa_sparse_prefill(g1["prob"], g1["Q"], g1["K"], g1["V"], w.B, plan, O)   # the plan is reusable
    torch.cuda.synchronize()
    assert plans_equal(plan, g1["plan"])
    assert torch.equal(O.view(torch.int16), g1["O"].view(torch.int16))


def test_work_is_enqueued_on_the_callers_stream():
    """The whole path on a side stream (default priority) gives the same bits as on the default stream,
    and events recorded on that stream bracket it."""
    w = dhsa_inputs.make("c3", L=8192, H_q=8, H_kv=2, N_b=512)
    g = run_gpu(w)
    side = torch.cuda.Stream()
    Q, K, V = g["Q"], g["K"], g["V"]
    O = torch.zeros_like(Q)
    plan, ws = dhsa.alloc(g["prob"], w.B)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        dhsa.dhsa_prefill(g["prob"], Q, K, V, w.B, O, plan, ws)
        e1.record()
    side.synchronize()
    assert e0.elapsed_time(e1) > 0.0
    assert plans_equal(plan, g["plan"])
    assert torch.equal(O.view(torch.int16), g["O"].view(torch.int16))


def test_strided_inputs_and_explicit_scale():
    w = dhsa_inputs.make("c2", L=3000, H_q=4, H_kv=2, N_b=256)
    big_q = torch.zeros((4, 3000, 256), dtype=torch.bfloat16, device="cuda")
    big_kv = torch.zeros((2, 3000, 384), dtype=torch.bfloat16, device="cuda")
    Q = big_q[:, :, 128:]; Q.copy_(w.Q.cuda())
    K = big_kv[:, :, :128]; K.copy_(w.K.cuda())
    V = big_kv[:, :, 256:]; V.copy_(w.V.cuda())
    O = torch.zeros((4, 3000, 128), dtype=torch.bfloat16, device="cuda")
    prob = dhsa.problem(Q, K, w.B, w.N_b, 0.05)
    plan, ws = dhsa.alloc(prob, w.B)
    dhsa.dhsa_prefill(prob, Q, K, V, w.B, O, plan, ws)
    torch.cuda.synchronize()
    rows = np.arange(w.L, dtype=np.int64)
    O_ref, I_ref, cnt_ref = oracle.prefill_rows(w.f32("Q"), w.f32("K"), w.f32("V"), w.B, w.N_b, rows, scale=0.05)
    g = dict(prob=prob, plan=plan, O=O)
    check_mask_rows(w, g, rows, I_ref, cnt_ref)
    check_outputs(w, g, rows, O_ref)


def test_peaky_softmax_moves_the_exponent_reference():
    """Logits spread over +-50 (scale 1 instead of 1/sqrt(d)): the probabilities of
    later key blocks exceed those of the first block by far more than 2^20, so the
    kernel has to move its exponent reference and rescale (several times per row)."""
    for name, kw in (("c2", dict(L=6000, H_q=8, H_kv=2, N_b=384)), ("c3", dict(L=4096, H_q=4, H_kv=2, N_b=512))):
        w = dhsa_inputs.make(name, **kw)
        g = run_gpu(w, scale=1.0)
        rows = np.arange(w.L, dtype=np.int64)
        O_ref, _, _ = oracle.prefill_rows(w.f32("Q"), w.f32("K"), w.f32("V"), w.B, w.N_b, rows, scale=1.0)
        got = g["O"].float().cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all()
        err = np.abs(got - O_ref).max()
        # near one-hot rows return single value vectors, |O| up to ~4.5 here: rounding O to bf16
        # costs up to |O| * 2^-8 (half an ulp), rounding the probabilities another |O| * 2^-9
        tol = np.abs(O_ref).max() * (2.0 ** -8 + 2.0 ** -9) * 1.05
        # The 2e-2 bar of the other tests is an absolute one for outputs of unit scale; here the bound
        # above is ~2.8e-2 because |O| is ~4.5.  Relative to the row's own magnitude the error meets
        # the same bar: asserted too, and both figures are printed.
        rel = (np.abs(got - O_ref).max(axis=2) / np.maximum(np.abs(O_ref).max(axis=2), 1.0)).max()
        over = int((np.abs(got - O_ref).max(axis=2) > TOL["bf16"]).sum())
        print(f"   {name}: peaky softmax max |O - oracle| = {err:.3e} (bound {tol:.3e}); {over} of "
              f"{got.shape[0] * got.shape[1]} rows above 2e-2 absolute; max error relative to max(|O_row|, 1) = "
              f"{rel:.3e}", flush=True)
        assert err <= tol
        assert rel <= TOL["bf16"]


FULL = ["c2", "c3", "c4", "c5"]


@pytest.mark.parametrize("name", FULL)
def test_full_size_sampled_parity(name):
    """The five configs at full size, in the launch configuration the bench
    times: mask bit-exact on a stratified row sample (and, through the compact
    plan, on every row of every head); outputs within tolerance on the sample."""
    w = dhsa_inputs.make(name)
    print(f"\n[{name}] L={w.L} N_c={w.N_c} N_b={w.N_b}", flush=True)
    g = run_gpu(w)
    rows = dhsa_inputs.sample_rows(w, 192)
    O_ref, I_ref, cnt_ref = oracle.prefill_rows(w.f32("Q"), w.f32("K"), w.f32("V"), w.B, w.N_b, rows)
    print("   oracle rows done", flush=True)
    check_mask_rows(w, g, rows, I_ref, cnt_ref)
    near = check_plan_all_chunks(w, g)
    err = check_outputs(w, g, rows, O_ref)
    print(f"   mask exact (sample of {len(rows)} rows + plan of all chunks); near-tie groups (<=1e-5): {near}; "
          f"max |O - oracle| = {err:.3e}", flush=True)


@pytest.mark.gpu
def test_mfma_probe_reports_plausible_rates():
    """The matrix-unit probe: constant operands reach the neighbourhood of the published 2.5 PFLOP/s,
    random operands (power-limited) stay below that and above a third of it; clocks are sane."""
    tf_c, mhz_c = dhsa.dhsa_mfma_probe(False, 50000)
    tf_r, mhz_r = dhsa.dhsa_mfma_probe(True, 50000)
    assert 1200.0 < tf_c < 2600.0, tf_c
    assert 800.0 < tf_r <= tf_c * 1.02, (tf_r, tf_c)
    assert 500.0 < mhz_r < 2600.0 and 500.0 < mhz_c < 2600.0, (mhz_c, mhz_r)


def _short_best_workload(tied: bool, seed: int):
    """Many 8-token chunks whose keys share a strong direction with every query, and few
    128-token chunks of weak noise: the best-ranked chunks are all short, so far more chunks
    hold the budget than the mean chunk length suggests.  With `tied`, only 180 short chunks
    keep their keys; every other key is zero, so all other chunk scores tie at exactly 0."""
    rng = np.random.default_rng([dhsa_inputs.BASE_SEED, 77, seed])
    lens = np.r_[np.full(1100, 8), np.full(200, 128)]
    rng.shuffle(lens)
    B = np.r_[0, np.cumsum(lens)].astype(np.int32)
    L, D, H_q, H_kv = int(B[-1]), 64, 2, 1
    u = np.full(D, 3.0 / np.sqrt(D), dtype=np.float32)
    Q = (0.1 * rng.standard_normal((H_q, L, D))).astype(np.float32) + u
    K = (0.1 * rng.standard_normal((H_kv, L, D))).astype(np.float32)
    V = rng.standard_normal((H_kv, L, D)).astype(np.float32)
    short = np.repeat(lens == 8, lens)
    K[:, short] += 2.0 * u
    if tied:
        keep = rng.choice(np.nonzero(lens == 8)[0], size=180, replace=False)
        live = np.repeat(np.isin(np.arange(len(lens)), keep), lens)
        K[:, ~live] = 0.0
    return dhsa_inputs.Workload(name="short_best", L=L, H_q=H_q, H_kv=H_kv, D=D, N_b=3000, dtype="f32", B=B,
                                Q=torch.from_numpy(Q), K=torch.from_numpy(K), V=torch.from_numpy(V), seed=seed)


@pytest.mark.parametrize("tied", [False, True], ids=["distinct", "tied_at_zero"])
@pytest.mark.parametrize("B_r", [0, 128])
def test_best_chunks_much_shorter_than_the_mean(tied, B_r):
    """The ranking is first sorted over a short candidate list sized from the mean chunk
    length; here that list never holds the budget (and, with ties, the longer list cannot be
    cut either), so the plan must come out of the second, longer sort."""
    w = _short_best_workload(tied, seed=1 + int(tied))
    print(f"\n[short-best tied={tied} B_r={B_r}] L={w.L} N_c={w.N_c} N_b={w.N_b}", flush=True)
    Q, K, V = (t.cuda() for t in (w.Q, w.K, w.V))
    O = torch.full_like(Q, float("nan"))
    prob = dhsa.problem(Q, K, w.B, w.N_b, B_r=B_r)
    plan, ws = dhsa.alloc(prob, w.B)
    dhsa.dhsa_prefill(prob, Q, K, V, w.B, O, plan, ws)
    torch.cuda.synchronize()
    g = dict(prob=prob, plan=plan, ws=ws, O=O)
    rows = np.unique(np.r_[np.arange(0, w.L, 37), w.B[1:] - 1, w.L - 1]).astype(np.int64)
    if B_r:
        O_ref, I_ref, cnt_ref = oracle.prefill_rows_blocks(w.f32("Q"), w.f32("K"), w.f32("V"), w.B, B_r, w.N_b,
                                                           rows)
    else:
        O_ref, I_ref, cnt_ref = oracle.prefill_rows(w.f32("Q"), w.f32("K"), w.f32("V"), w.B, w.N_b, rows)
        check_plan_all_chunks(w, g)
    check_mask_rows(w, g, rows, I_ref, cnt_ref)
    err = check_outputs(w, g, rows, O_ref)
    print(f"   mask exact on {len(rows)} rows x {w.H_q} heads; max |O - oracle| = {err:.3e}", flush=True)
