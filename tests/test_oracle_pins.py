"""Pins for the CPU oracle: closed forms, hand-worked values, library special
cases and brute force, chosen so that a dropped term, a wrong sign or index or
a transposed operand in oracle/dhsa_oracle.c fails at least one of them.

Citations are to the paper (arXiv 2510.24606): Sec. 3.1 (hierarchical sparsity
prediction), Sec. 3.3 Eq. 4 (robust chunk representation), Alg. 1 (sparsity
prediction), Alg. 2 / Alg. 3 (SDPA and tiled online-softmax backends), App. D
ablation paragraph (fixed blocks => block-sparse scores up to the factor B).
"""
import json
import math
import os

import numpy as np
import pytest
import torch
from hypothesis import given, settings, strategies as st

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def rand_boundaries(rng, L, lo, hi):
    out = [0]
    while out[-1] < L:
        out.append(min(L, out[-1] + int(rng.integers(lo, hi + 1))))
    return np.asarray(out, dtype=np.int32)


# ----------------------------------------------------------------------------
# hand-worked example (tests/golden/hand_example.json)
# ----------------------------------------------------------------------------
def _ev(x):
    if isinstance(x, str):
        return eval(x, {"sqrt2": math.sqrt(2.0), "exp": math.exp, "p0": 1 / (1 + math.exp(-2 * math.sqrt(2.0)))})
    return float(x)


@pytest.fixture(scope="module")
def hand():
    with open(os.path.join(HERE, "golden", "hand_example.json")) as f:
        return json.load(f)


def test_hand_pooling_and_scores(hand):
    B = np.array(hand["B"], dtype=np.int32)
    Q = np.array(hand["Q"], dtype=np.float32)[None]
    K = np.array(hand["K"], dtype=np.float32)[None]
    Qc = oracle.pool(Q, B)
    Kc = oracle.pool(K, B)
    np.testing.assert_allclose(Qc[0], [[_ev(v) for v in r] for r in hand["Qc"]], rtol=0, atol=1e-15)
    np.testing.assert_allclose(Kc[0], [[_ev(v) for v in r] for r in hand["Kc"]], rtol=0, atol=1e-15)
    Sc = oracle.scores(Qc, Kc)
    np.testing.assert_allclose(Sc[0], [[_ev(v) for v in r] for r in hand["Sc"]], rtol=0, atol=1e-14)


def test_hand_ranking_selection_attention(hand):
    B = np.array(hand["B"], dtype=np.int32)
    Q = np.array(hand["Q"], dtype=np.float32)[None]
    K = np.array(hand["K"], dtype=np.float32)[None]
    V = np.array(hand["V"], dtype=np.float32)[None]
    Sc = oracle.scores(oracle.pool(Q, B), oracle.pool(K, B))[0]
    for l, want in hand["rank_row_chunk"].items():
        assert oracle.rank(Sc[int(l)]).tolist() == want
    rows = np.arange(7)
    for nb, key in ((3, "I_Nb3"), (2, "I_Nb2")):
        I, cnt = oracle.route_rows(Q, K, B, nb, rows)
        for i in range(7):
            assert I[0, i, :cnt[0, i]].tolist() == hand[key][str(i)], (nb, i)
            # the same sets from the token-pair formulation
        I2, cnt2 = oracle.select_pairs(Sc, B, nb)
        np.testing.assert_array_equal(I[0], I2)
        np.testing.assert_array_equal(cnt[0], cnt2)
    O, I, cnt = oracle.prefill_rows(Q, K, V, B, 3, np.array([1]))
    p0 = _ev(hand["attn_row1_Nb3"]["p0"])
    np.testing.assert_allclose(O[0, 0], [p0, 1 - p0], rtol=0, atol=1e-15)


# ----------------------------------------------------------------------------
# pooling (Eq. 4)
# ----------------------------------------------------------------------------
def test_pool_one_token_chunks_is_identity():
    rng = np.random.default_rng(0)
    X = rng.standard_normal((2, 17, 8)).astype(np.float32)
    B = np.arange(18, dtype=np.int32)
    np.testing.assert_array_equal(oracle.pool(X, B), X.astype(np.float64))


def test_pool_constant_chunk_scales_by_sqrt_len():
    # a chunk of len copies of x pools to sqrt(len) * x
    B = np.array([0, 4, 13, 14, 30], dtype=np.int32)
    x = np.array([1.5, -2.0, 0.25], dtype=np.float32)
    X = np.tile(x, (1, 30, 1)).astype(np.float32)
    got = oracle.pool(X, B)[0]
    for k in range(4):
        n = B[k + 1] - B[k]
        np.testing.assert_allclose(got[k], math.sqrt(n) * x.astype(np.float64), rtol=1e-15)


def test_pool_matches_reduceat():
    rng = np.random.default_rng(1)
    L = 301
    B = rand_boundaries(rng, L, 1, 40)
    X = rng.standard_normal((3, L, 16)).astype(np.float32)
    want = np.add.reduceat(X.astype(np.float64), B[:-1], axis=1) / np.sqrt(np.diff(B))[None, :, None]
    np.testing.assert_allclose(oracle.pool(X, B), want, rtol=1e-14, atol=1e-14)


# ----------------------------------------------------------------------------
# chunk similarity
# ----------------------------------------------------------------------------
def test_scores_one_token_chunks_equal_token_scores():
    rng = np.random.default_rng(2)
    L, D = 33, 8
    Q = rng.standard_normal((4, L, D)).astype(np.float32)
    K = rng.standard_normal((2, L, D)).astype(np.float32)
    B = np.arange(L + 1, dtype=np.int32)
    Sc = oracle.scores(oracle.pool(Q, B), oracle.pool(K, B))
    for h in range(4):
        want = Q[h].astype(np.float64) @ K[h // 2].astype(np.float64).T   # GQA: kv head = h // G
        np.testing.assert_allclose(Sc[h], want, rtol=1e-13, atol=1e-13)
    # not symmetric: a transposed operand would fail here
    assert not np.allclose(Sc[0], Sc[0].T)


def test_scores_double_sum_identity():
    # S_c[l,k] = (len_l len_k)^(-1/2) sum_{i in l} sum_{j in k} q_i . k_j   (linearity of Eq. 4)
    rng = np.random.default_rng(3)
    L, D = 97, 4
    B = rand_boundaries(rng, L, 1, 20)
    Q = rng.standard_normal((1, L, D)).astype(np.float32)
    K = rng.standard_normal((1, L, D)).astype(np.float32)
    Sc = oracle.scores(oracle.pool(Q, B), oracle.pool(K, B))[0]
    P = Q[0].astype(np.float64) @ K[0].astype(np.float64).T
    N_c = len(B) - 1
    for l in range(N_c):
        for k in range(N_c):
            want = P[B[l]:B[l + 1], B[k]:B[k + 1]].sum() / math.sqrt((B[l + 1] - B[l]) * (B[k + 1] - B[k]))
            assert abs(Sc[l, k] - want) < 1e-12


def test_scores_uniform_chunks_are_block_mean_similarity_times_block():
    # App. D: with b_k = k*Bsz, S_c = Bsz * (mean-pooled block similarity)
    rng = np.random.default_rng(4)
    Bsz, n, D = 8, 6, 5
    L = Bsz * n
    Q = rng.standard_normal((1, L, D)).astype(np.float32)
    K = rng.standard_normal((1, L, D)).astype(np.float32)
    B = np.arange(0, L + 1, Bsz, dtype=np.int32)
    Sc = oracle.scores(oracle.pool(Q, B), oracle.pool(K, B))[0]
    qm = Q[0].astype(np.float64).reshape(n, Bsz, D).mean(1)
    km = K[0].astype(np.float64).reshape(n, Bsz, D).mean(1)
    np.testing.assert_allclose(Sc, Bsz * (qm @ km.T), rtol=1e-13, atol=1e-13)


# ----------------------------------------------------------------------------
# ranking
# ----------------------------------------------------------------------------
def test_rank_matches_stable_argsort_with_ties():
    rng = np.random.default_rng(5)
    for _ in range(20):
        n = int(rng.integers(1, 60))
        s = rng.integers(-3, 4, size=n).astype(np.float64)       # many ties
        s[rng.random(n) < 0.2] *= -0.0                            # signed zeros tie with each other
        want = np.argsort(-s, kind="stable")
        np.testing.assert_array_equal(oracle.rank(s), want)


def test_rank_signed_zero_is_a_tie():
    assert oracle.rank(np.array([-0.0, 0.0, -0.0])).tolist() == [0, 1, 2]
    assert oracle.rank(np.array([0.0, -0.0, 1.0])).tolist() == [2, 0, 1]


# ----------------------------------------------------------------------------
# selection (Alg. 1 with q_max = i + 1)
# ----------------------------------------------------------------------------
def py_select_from_sentence(Sc_h, B, N_b, i):
    """Sec. 3.1 Step 2 read literally at token level: every causal key j <= i
    carries its chunk's score; keep the N_b best, ties to the lower key index."""
    c = np.searchsorted(B, np.arange(int(B[-1])), side="right") - 1
    keys = sorted(range(i + 1), key=lambda j: (-Sc_h[c[i], c[j]], j))
    return sorted(keys[:N_b])


def test_select_single_chunk_closed_form():
    B = np.array([0, 50], dtype=np.int32)
    pi = np.array([0], dtype=np.int32)
    for nb in (1, 7, 50, 80):
        for i in (0, 5, 6, 7, 49):
            assert oracle.select(pi, B, i + 1, nb).tolist() == list(range(min(nb, i + 1)))


@settings(max_examples=60, deadline=None)
@given(st.integers(0, 10**6), st.integers(2, 64), st.integers(1, 70), st.integers(1, 9), st.booleans())
def test_select_equals_token_pair_bruteforce(seed, L, N_b, maxlen, ties):
    rng = np.random.default_rng(seed)
    B = rand_boundaries(rng, L, 1, maxlen)
    N_c = len(B) - 1
    if ties:
        Sc = rng.integers(-2, 3, size=(N_c, N_c)).astype(np.float64)
    else:
        Sc = rng.standard_normal((N_c, N_c))
    I2, cnt2 = oracle.select_pairs(Sc, B, N_b)
    for i in range(L):
        l = int(np.searchsorted(B, i, side="right") - 1)
        I = oracle.select(oracle.rank(Sc[l]), B, i + 1, N_b)
        want = py_select_from_sentence(Sc, B, N_b, i)
        assert I.tolist() == want
        assert I2[i, :cnt2[i]].tolist() == want
        assert (I2[i, cnt2[i]:] == -1).all()


def test_select_invariants_nestedness_and_scale_invariance():
    rng = np.random.default_rng(7)
    L, D = 400, 16
    B = rand_boundaries(rng, L, 3, 40)
    Q = rng.standard_normal((2, L, D)).astype(np.float32)
    K = rng.standard_normal((1, L, D)).astype(np.float32)
    rows = np.arange(L)
    prev = None
    for nb in (1, 17, 64, 399, 400, 1000):
        I, cnt = oracle.route_rows(Q, K, B, nb, rows)
        for h in range(2):
            for i in range(L):
                sel = I[h, i, :cnt[h, i]]
                assert cnt[h, i] == min(nb, i + 1)                 # exact budget
                assert (sel <= i).all() and (sel >= 0).all()       # causal
                assert (np.diff(sel) > 0).all()                    # ascending, unique
                # union of whole chunks, at most one truncated chunk prefix, clipped own chunk
                l = np.searchsorted(B, i, side="right") - 1
                partial = 0
                for k in range(l):
                    n_in = int(((sel >= B[k]) & (sel < B[k + 1])).sum())
                    if 0 < n_in < B[k + 1] - B[k]:
                        partial += 1
                        assert (sel[(sel >= B[k]) & (sel < B[k + 1])] == np.arange(B[k], B[k] + n_in)).all()
                own = sel[sel >= B[l]]
                assert (own == np.arange(B[l], B[l] + len(own))).all()   # a prefix of the own chunk
                assert partial + (0 < len(own) < i + 1 - B[l]) <= 1
                if prev is not None:
                    assert set(prev[0][h, i, :prev[1][h, i]]) <= set(sel)   # nested in N_b
        prev = (I, cnt)
    # routing scores are unscaled inner products: Q -> 4Q (exact in fp) changes no set
    I1, c1 = oracle.route_rows(Q, K, B, 64, rows)
    I2, c2 = oracle.route_rows(4.0 * Q, K, B, 64, rows)
    np.testing.assert_array_equal(I1, I2)
    # N_b >= L: every row takes all its causal keys
    I, cnt = oracle.route_rows(Q, K, B, L, rows)
    for i in (0, 1, L // 2, L - 1):
        assert I[0, i, :cnt[0, i]].tolist() == list(range(i + 1))


@settings(max_examples=40, deadline=None)
@given(st.integers(0, 10**6), st.integers(2, 120), st.integers(1, 130), st.integers(1, 30))
def test_chunk_walk_rule_reproduces_rows(seed, L, N_b, maxlen):
    """The chunk-level walk state (before[k], pos[k]) determines every row's set:
    row i with v = i+1-b_l visible tokens of its own chunk takes, from chunk k,
    the first clamp(N_b - before[k] - [pos=2]*v, 0, len_eff) tokens."""
    rng = np.random.default_rng(seed)
    B = rand_boundaries(rng, L, 1, maxlen)
    N_c = len(B) - 1
    Sc = rng.integers(-3, 4, size=(N_c, N_c)).astype(np.float64)
    for l in range(N_c):
        pi = oracle.rank(Sc[l])
        before, pos = oracle.chunk_walk(pi, B, l)
        assert (pos[l + 1:] == 3).all() and pos[l] == 1
        for i in range(B[l], B[l + 1]):
            v = i + 1 - B[l]
            got = []
            for k in range(l + 1):
                len_eff = v if k == l else B[k + 1] - B[k]
                room = N_b - before[k] - (v if pos[k] == 2 else 0)
                take = max(0, min(len_eff, room))
                got.extend(range(B[k], B[k] + take))
            assert got == oracle.select(pi, B, i + 1, N_b).tolist()


# ----------------------------------------------------------------------------
# attention (Alg. 2, Alg. 3)
# ----------------------------------------------------------------------------
def test_attention_dense_special_case_matches_sdpa():
    # N_b >= L: the path is exact dense causal attention (library routine on CPU)
    rng = np.random.default_rng(8)
    L, D, H_q, H_kv = 130, 16, 4, 2
    B = rand_boundaries(rng, L, 2, 30)
    Q = rng.standard_normal((H_q, L, D)).astype(np.float32)
    K = rng.standard_normal((H_kv, L, D)).astype(np.float32)
    V = rng.standard_normal((H_kv, L, D)).astype(np.float32)
    O, I, cnt = oracle.prefill_rows(Q, K, V, B, L + 5, np.arange(L))
    tq = torch.from_numpy(Q).double()[None]
    tk = torch.from_numpy(K).double().repeat_interleave(H_q // H_kv, 0)[None]
    tv = torch.from_numpy(V).double().repeat_interleave(H_q // H_kv, 0)[None]
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].numpy()
    np.testing.assert_allclose(O, want, rtol=1e-12, atol=1e-12)


def test_attention_sparse_rows_match_plain_softmax_formula():
    rng = np.random.default_rng(9)
    L, D = 90, 8
    Kg = rng.standard_normal((L, D)).astype(np.float32)
    Vg = rng.standard_normal((L, D)).astype(np.float32)
    q = rng.standard_normal(D).astype(np.float32)
    i = 70
    I = np.sort(rng.choice(i + 1, size=20, replace=False)).astype(np.int32)
    s = (Kg[I].astype(np.float64) @ q.astype(np.float64)) * 0.37
    p = np.exp(s - s.max()); p /= p.sum()
    np.testing.assert_allclose(oracle.attend_row(q, Kg, Vg, I, i, 0.37), p @ Vg[I].astype(np.float64), rtol=1e-13)
    # keys above the row are masked by absolute position (Alg. 2's mask)
    I2 = np.concatenate([I, [75, 80]]).astype(np.int32)
    np.testing.assert_allclose(oracle.attend_row(q, Kg, Vg, I2, i, 0.37), p @ Vg[I].astype(np.float64), rtol=1e-13)


def test_attention_closed_forms():
    rng = np.random.default_rng(10)
    L, D = 40, 4
    Q = rng.standard_normal((1, L, D)).astype(np.float32)
    K = rng.standard_normal((1, L, D)).astype(np.float32)
    V = rng.standard_normal((1, L, D)).astype(np.float32)
    B = np.array([0, 7, 19, 40], dtype=np.int32)
    rows = np.arange(L)
    # one key per row: the output is that key's value vector
    O, I, cnt = oracle.prefill_rows(Q, K, V, B, 1, rows)
    for i in range(L):
        np.testing.assert_array_equal(O[0, i], V[0, I[0, i, 0]].astype(np.float64))
    # probabilities sum to one: constant V comes back unchanged
    Vc = np.ones_like(V) * 2.5
    O, _, _ = oracle.prefill_rows(Q, K, Vc, B, 9, rows)
    np.testing.assert_allclose(O, 2.5, rtol=1e-14)
    # equal keys: uniform weights, output = mean of the selected values
    K0 = np.zeros_like(K)
    O, I, cnt = oracle.prefill_rows(Q, K0, V, B, 5, rows)
    for i in range(L):
        np.testing.assert_allclose(O[0, i], V[0, I[0, i, :cnt[0, i]]].astype(np.float64).mean(0), rtol=1e-13, atol=1e-15)
    # the attention logits carry the scale, the routing scores do not
    O1, I1, _ = oracle.prefill_rows(Q, K, V, B, 9, rows, scale=1.0)
    O2, I2, _ = oracle.prefill_rows(Q, K, V, B, 9, rows, scale=0.25)
    np.testing.assert_array_equal(I1, I2)
    assert np.abs(O1 - O2).max() > 1e-3


def test_tiled_online_softmax_equals_masked_softmax():
    # Alg. 3 == Alg. 2 on a row block that shares one index list, incl. keys
    # above early rows of the block (masked by absolute position) and a ragged last tile
    rng = np.random.default_rng(11)
    L, D = 200, 8
    Qh = rng.standard_normal((L, D)).astype(np.float32)
    Kg = rng.standard_normal((L, D)).astype(np.float32)
    Vg = rng.standard_normal((L, D)).astype(np.float32)
    q_s, q_e = 128, 160
    I = np.sort(rng.choice(q_e, size=77, replace=False)).astype(np.int32)
    I[0] = 0
    for B_c in (1, 16, 77, 128):
        O3 = oracle.attend_block_tiled(Qh, Kg, Vg, I, q_s, q_e, 0.5, B_c)
        for u in range(q_e - q_s):
            want = oracle.attend_row(Qh[q_s + u], Kg, Vg, I, q_s + u, 0.5)
            np.testing.assert_allclose(O3[u], want, rtol=1e-12, atol=1e-14)


# ----------------------------------------------------------------------------
# plan_head: chunk-level state and near-tie accounting
# ----------------------------------------------------------------------------
def test_plan_head_matches_chunk_walk_and_flags_planted_near_tie():
    rng = np.random.default_rng(12)
    L, D, N_b = 600, 8, 100
    B = rand_boundaries(rng, L, 5, 30)
    N_c = len(B) - 1
    Qc = rng.standard_normal((N_c, D))
    Kc = rng.standard_normal((N_c, D))
    rem, pos, gap = oracle.plan_head(Qc, Kc, B, N_b)
    Sc = oracle.scores(Qc[None], Kc[None])[0]
    for l in (0, 1, N_c // 2, N_c - 1):
        before, p = oracle.chunk_walk(oracle.rank(Sc[l]), B, l)
        np.testing.assert_array_equal(pos[l], p)
        vis = p != 3
        np.testing.assert_array_equal(rem[l][vis], N_b - before[vis])
    assert (gap > 0).all()
    # duplicate a key chunk vector: wherever both copies sit at the cut-off the gap is exactly 0
    Kc2 = Kc.copy()
    Kc2[3] = Kc2[2]
    _, _, gap2 = oracle.plan_head(Qc, Kc2, B, 40)
    Sc2 = oracle.scores(Qc[None], Kc2[None])[0]
    hits = 0
    for l in range(4, N_c):
        pi = [k for k in oracle.rank(Sc2[l]) if k <= l]
        r = pi.index(2)
        assert pi[r + 1] == 3                                    # tie -> lower id first
        before, p = oracle.chunk_walk(oracle.rank(Sc2[l]), B, l)
        at_cut = before[2] < 40 and not (before[3] + (B[4] - B[3]) + (B[l + 1] - B[l]) <= 40)
        if at_cut:
            assert gap2[l] == 0.0
            hits += 1
    assert hits > 0


# ----------------------------------------------------------------------------
# Alg. 1 as printed (fixed row blocks): hand-worked example, closed forms, brute force
# ----------------------------------------------------------------------------
def _evb(x):
    if isinstance(x, str):
        return eval(x, {"sqrt2": math.sqrt(2.0), "sqrt3": math.sqrt(3.0), "a": math.exp(-3 * math.sqrt(2.0))})
    return float(x)


@pytest.fixture(scope="module")
def hand_blocks():
    with open(os.path.join(HERE, "golden", "hand_example_blocks.json")) as f:
        return json.load(f)


def test_hand_blocks(hand_blocks):
    hb = hand_blocks
    B = np.array(hb["B"], dtype=np.int32)
    B_r = hb["B_r"]
    Q = np.array(hb["Q"], dtype=np.float32)[None]
    K = np.array(hb["K"], dtype=np.float32)[None]
    V = np.array(hb["V"], dtype=np.float32)[None]
    Qb = oracle.pool_blocks(Q, B_r)
    np.testing.assert_allclose(Qb[0], [[_evb(v) for v in r] for r in hb["Qb"]], rtol=0, atol=1e-15)
    Kc = oracle.pool(K, B)
    Sb = Qb[0] @ Kc[0].T
    np.testing.assert_allclose(Sb, [[_evb(v) for v in r] for r in hb["Sb"]], rtol=0, atol=1e-14)
    for i, want in hb["rank_block"].items():
        assert oracle.rank(Sb[int(i)]).tolist() == want
    blocks = np.arange(3)
    for nb, key in ((3, "I_Nb3"), (2, "I_Nb2"), (1, "I_Nb1")):
        I, cnt = oracle.route_blocks(Q, K, B, B_r, nb, blocks)
        I2, cnt2 = oracle.select_pairs_blocks(Sb, B, B_r, nb)
        for i in range(3):
            assert I[0, i, :cnt[0, i]].tolist() == hb[key][str(i)], (nb, i)
            q_max = min((i + 1) * B_r, 7)
            assert oracle.select_block(Qb[0, i], Kc[0], B, q_max, nb).tolist() == hb[key][str(i)]
        np.testing.assert_array_equal(I[0], I2)
        np.testing.assert_array_equal(cnt[0], cnt2)
    for nb, key in ((3, "O_Nb3"), (1, "O_Nb1")):
        rows = np.array(sorted(int(r) for r in hb[key]))
        O, _, _ = oracle.prefill_rows_blocks(Q, K, V, B, B_r, nb, rows)
        for t, r in enumerate(rows):
            np.testing.assert_allclose(O[0, t], [_evb(v) for v in hb[key][str(r)]], rtol=0, atol=1e-15)


def test_pool_blocks_is_scaled_mean_with_a_ragged_last_block():
    rng = np.random.default_rng(7)
    X = rng.standard_normal((3, 37, 4)).astype(np.float32)
    for B_r in (1, 5, 8, 37, 64):
        got = oracle.pool_blocks(X, B_r)
        starts = np.arange(0, 37, B_r)
        for i, s in enumerate(starts):
            e = min(s + B_r, 37)
            want = math.sqrt(B_r) * X[:, s:e].astype(np.float64).mean(axis=1)
            np.testing.assert_allclose(got[:, i], want, rtol=1e-14, atol=1e-15)
    # B_r = 1: the block representation is the row itself
    np.testing.assert_allclose(oracle.pool_blocks(X, 1), X.astype(np.float64), rtol=0, atol=0)


@settings(max_examples=60, deadline=None)
@given(st.integers(0, 10**6), st.integers(2, 48), st.integers(1, 9), st.integers(1, 12), st.integers(1, 50),
       st.booleans())
def test_block_selection_equals_token_level_brute_force(seed, L, B_r, hi, N_b, tied):
    rng = np.random.default_rng(seed)
    B = rand_boundaries(rng, L, 1, hi)
    N_c = len(B) - 1
    H_q, H_kv, D = 2, 1, 4
    Q = rng.standard_normal((H_q, L, D)).astype(np.float32)
    K = rng.standard_normal((H_kv, L, D)).astype(np.float32)
    if tied:   # equal chunk scores: quantise so that ties occur
        Q = np.round(Q); K = np.round(K)
    N_r = (L + B_r - 1) // B_r
    I, cnt = oracle.route_blocks(Q, K, B, B_r, N_b, np.arange(N_r))
    Qb, Kc = oracle.pool_blocks(Q, B_r), oracle.pool(K, B)
    for h in range(H_q):
        Sb = np.stack([Qb[h, i] @ Kc[0].T for i in range(N_r)])
        # the oracle's own score routine sums in index order: use it so that ties are identical
        Sb = np.stack([_score_row(Qb[h, i], Kc[0]) for i in range(N_r)])
        I2, cnt2 = oracle.select_pairs_blocks(Sb, B, B_r, N_b)
        np.testing.assert_array_equal(I[h], I2)
        np.testing.assert_array_equal(cnt[h], cnt2)
        for i in range(N_r):
            q_max = min((i + 1) * B_r, L)
            assert cnt[h, i] == min(N_b, q_max)
            sel = I[h, i, :cnt[h, i]]
            assert np.all(np.diff(sel) > 0) and sel[-1] < q_max
        # the per-chunk take counts reproduce the lists (each listed chunk contributes its first tokens)
        take, _ = oracle.plan_blocks_head(Qb[h], Kc[0], B, B_r, N_b)
        for i in range(N_r):
            rebuilt = np.concatenate([np.arange(B[k], B[k] + take[i, k]) for k in range(N_c)]) if N_c else []
            np.testing.assert_array_equal(rebuilt, I[h, i, :cnt[h, i]])


def _score_row(q, Kc):
    import ctypes as C
    q = np.ascontiguousarray(q, dtype=np.float64); Kc = np.ascontiguousarray(Kc, dtype=np.float64)
    out = np.empty(Kc.shape[0], dtype=np.float64)
    oracle.lib().dhsa_oracle_score_row(q.ctypes.data_as(C.POINTER(C.c_double)), Kc.ctypes.data_as(C.POINTER(C.c_double)),
                                       Kc.shape[0], Kc.shape[1], out.ctypes.data_as(C.POINTER(C.c_double)))
    return out


def test_blocks_that_coincide_with_chunks_reduce_to_the_row_form():
    """With every chunk exactly one row block, sqrt(B_r) AvgPool is Eq. 4, so S_c is the same matrix and the
    list of row block i is the per-row list of the block's LAST row (q_max = block end = i_last + 1)."""
    rng = np.random.default_rng(11)
    B_r, N_r, D = 6, 9, 8
    L = B_r * N_r
    B = np.arange(0, L + 1, B_r, dtype=np.int32)
    Q = rng.standard_normal((2, L, D)).astype(np.float32)
    K = rng.standard_normal((1, L, D)).astype(np.float32)
    np.testing.assert_allclose(oracle.pool_blocks(Q, B_r), oracle.pool(Q, B), rtol=1e-15, atol=1e-15)
    for N_b in (1, 5, 17, 60):
        Ib, cb = oracle.route_blocks(Q, K, B, B_r, N_b, np.arange(N_r))
        last = np.arange(B_r - 1, L, B_r)
        Ir, cr = oracle.route_rows(Q, K, B, N_b, last)
        np.testing.assert_array_equal(cb, cr)
        np.testing.assert_array_equal(Ib, Ir)


def _swap_gap(S_row, B, q_max, N_b):
    """Near-tie gap of one row block from its definition, by trial: the smallest |score gap| over pairs
    of adjacently ranked visible chunks whose exchange changes the block's list (Alg. 1 walk, written out)."""
    order = [int(k) for k in oracle.rank(S_row) if B[k] < q_max]

    def takes(seq):
        room, out = N_b, {}
        for k in seq:
            t = max(0, min(room, min(int(B[k + 1]), q_max) - int(B[k])))
            out[k] = t
            room -= min(int(B[k + 1]), q_max) - int(B[k])
        return out

    base = takes(order)
    gap = math.inf
    for r in range(len(order) - 1):
        sw = order[:r] + [order[r + 1], order[r]] + order[r + 2:]
        if takes(sw) != base:
            gap = min(gap, abs(float(S_row[order[r]]) - float(S_row[order[r + 1]])))
    return gap


def test_block_form_cut_gap_by_trial_and_with_planted_ties():
    """cut_gap of plan_blocks_head (the near-tie count of the row-block form, Alg. 1's Argsort tie rule):
    equal to the gap found by exchanging adjacent ranks one pair at a time; exactly 0 where two identical
    key-chunk vectors sit at a block's cut-off and positive elsewhere; never below the row form's gap
    when the blocks coincide with the chunks (the block's list is its last row's list)."""
    rng = np.random.default_rng(21)
    L, D, B_r, N_b = 420, 8, 12, 45
    B = rand_boundaries(rng, L, 3, 20)
    N_c = len(B) - 1
    Q = rng.standard_normal((1, L, D)).astype(np.float32)
    Kc = rng.standard_normal((N_c, D))
    Qb = oracle.pool_blocks(Q, B_r)[0]
    N_r = Qb.shape[0]
    take, gap = oracle.plan_blocks_head(Qb, Kc, B, B_r, N_b)
    finite = 0
    for i in range(N_r):
        q_max = min((i + 1) * B_r, L)
        want = _swap_gap(_score_row(Qb[i], Kc), B, q_max, N_b)
        assert gap[i] == want, (i, gap[i], want)
        finite += math.isfinite(want)
    assert finite > N_r // 2 and (gap > 0).all()
    assert math.isinf(gap[0]) and take[0].sum() == min(N_b, B_r)     # the first block takes all it sees: no cut-off
    # plant a duplicate: chunks 2 and 3 get the same vector, so they are always adjacent in the ranking
    Kc2 = Kc.copy()
    Kc2[3] = Kc2[2]
    take2, gap2 = oracle.plan_blocks_head(Qb, Kc2, B, B_r, N_b)
    zeros = 0
    for i in range(N_r):
        q_max = min((i + 1) * B_r, L)
        S_row = _score_row(Qb[i], Kc2)
        assert gap2[i] == _swap_gap(S_row, B, q_max, N_b)
        if B[3] < q_max:
            pi = [int(k) for k in oracle.rank(S_row) if B[k] < q_max]
            assert pi[pi.index(2) + 1] == 3                                # tie -> lower id first
            len2, len3 = (min(int(B[k + 1]), q_max) - int(B[k]) for k in (2, 3))
            at_cut = take2[i, 2] > 0 and not (take2[i, 2] == len2 and take2[i, 3] == len3)
            assert (gap2[i] == 0.0) == at_cut
            zeros += at_cut
        else:
            assert gap2[i] > 0
    assert zeros > 0
    # blocks that coincide with the chunks: the pairs that matter to the block's (= last row's) list are
    # among those that matter to some row of the chunk
    B_u = np.arange(0, 40 * B_r + 1, B_r, dtype=np.int32)
    Qu = rng.standard_normal((40, D))
    Ku = rng.standard_normal((40, D))
    Ku[7] = Ku[6]
    zeros = 0
    for nb in (7, 30, 100):
        _, _, gap_rows = oracle.plan_head(Qu, Ku, B_u, nb)
        _, gap_blocks = oracle.plan_blocks_head(Qu, Ku, B_u, B_r, nb)
        assert (gap_blocks >= gap_rows).all()
        zeros += int((gap_blocks == 0).sum())
    assert zeros > 0


def test_block_form_with_a_budget_of_everything_is_dense_causal_attention():
    rng = np.random.default_rng(13)
    H_q, H_kv, L, D, B_r = 4, 2, 45, 8, 7
    B = rand_boundaries(rng, L, 2, 9)
    Q = rng.standard_normal((H_q, L, D)).astype(np.float32)
    K = rng.standard_normal((H_kv, L, D)).astype(np.float32)
    V = rng.standard_normal((H_kv, L, D)).astype(np.float32)
    rows = np.arange(L)
    O, I, cnt = oracle.prefill_rows_blocks(Q, K, V, B, B_r, L + 3, rows)
    for i in rows:
        q_max = min((i // B_r + 1) * B_r, L)
        assert cnt[0, i] == q_max and I[0, i, :q_max].tolist() == list(range(q_max))
    q, k, v = (torch.from_numpy(x.astype(np.float64)) for x in (Q, K, V))
    k = k.repeat_interleave(H_q // H_kv, 0); v = v.repeat_interleave(H_q // H_kv, 0)
    want = torch.nn.functional.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0].numpy()
    np.testing.assert_allclose(O, want, rtol=1e-12, atol=1e-12)


def test_block_form_alg3_equals_alg2_and_rows_without_a_visible_key_are_zero():
    L, D, B_r, N_b = 40, 8, 8, 3
    scale = 1.0 / math.sqrt(D)
    saw_empty = 0
    for seed in range(6):
        rng = np.random.default_rng(100 + seed)
        B = rand_boundaries(rng, L, 1, 6)
        Q = rng.standard_normal((1, L, D)).astype(np.float32)
        K = rng.standard_normal((1, L, D)).astype(np.float32)
        V = rng.standard_normal((1, L, D)).astype(np.float32)
        rows = np.arange(L)
        O, I, cnt = oracle.prefill_rows_blocks(Q, K, V, B, B_r, N_b, rows)
        for blk in range(L // B_r):
            q_s, q_e = blk * B_r, (blk + 1) * B_r
            sel = I[0, q_s, :cnt[0, q_s]]
            for B_c in (1, 2, 64):
                O3 = oracle.attend_block_tiled(Q[0], K[0], V[0], sel, q_s, q_e, scale, B_c)
                np.testing.assert_allclose(O3, O[0, q_s:q_e], rtol=1e-12, atol=1e-13)
            for i in range(q_s, q_e):
                if sel[0] > i:      # the row precedes every key of its block's list
                    saw_empty += 1
                    assert np.all(O[0, i] == 0.0)
                else:
                    assert np.any(O[0, i] != 0.0)
    assert saw_empty > 0


# ----------------------------------------------------------------------------
# Boundary finalisation: threshold + greedy non-maximum suppression
# (Sec. 3.2 "Inference Pipeline"; App. "Inference of the Boundary Predictor")
# ----------------------------------------------------------------------------
def test_finalize_boundaries_hand_example():
    # candidates above 0.5: positions 1 (.9), 2 (.8), 4 (.95), 6 (.6), 7 (.6), 9 (.7); visiting order 4, 1, 2, 9, 6, 7
    p = np.array([0.1, 0.9, 0.8, 0.2, 0.95, 0.1, 0.6, 0.6, 0.05, 0.7], dtype=np.float32)
    # W = 1: 4 kept (removes 3, 5); 1 kept (removes 0, 2); 9 kept (removes 8); 6 kept before 7 (tie: lower
    # position first) and removes it.  Chunk ends 1, 4, 6, 9 -> half-open boundaries 2, 5, 7, 10 (= L)
    assert oracle.finalize_boundaries(p, 0.5, 1).tolist() == [0, 2, 5, 7, 10]
    # W = 0: nothing is suppressed, every candidate is a chunk end
    assert oracle.finalize_boundaries(p, 0.5, 0).tolist() == [0, 2, 3, 5, 7, 8, 10]
    # W = 2: 4 removes 2..6; 1 kept; 9 removes 7, 8  -> ends 1, 4, 9
    assert oracle.finalize_boundaries(p, 0.5, 2).tolist() == [0, 2, 5, 10]
    # the threshold is strict, and nothing above it leaves one chunk
    assert oracle.finalize_boundaries(p, 0.95, 3).tolist() == [0, 10]
    assert oracle.finalize_boundaries(p, 0.9, 3).tolist() == [0, 5, 10]


def _kept_by_repeated_argmax(p, tau, W):
    """Independent statement of the same greedy: repeatedly take the best remaining candidate (first
    occurrence of the maximum = lowest position) and blank its neighbourhood."""
    s = np.where(p.astype(np.float64) > tau, p.astype(np.float64), -np.inf)
    kept = []
    while np.isfinite(s).any():
        i = int(np.argmax(s))
        kept.append(i)
        s[max(0, i - W):i + W + 1] = -np.inf
    return np.array(sorted(kept), dtype=np.int64)


@settings(max_examples=150, deadline=None)
@given(st.integers(0, 10**6), st.integers(1, 400), st.integers(0, 70), st.floats(0.0, 1.0), st.booleans())
def test_finalize_boundaries_equals_repeated_argmax_and_is_a_maximal_spaced_set(seed, L, W, tau, tied):
    rng = np.random.default_rng(seed)
    p = rng.random(L).astype(np.float32)
    if tied:
        p = np.round(p * 8) / 8          # many equal scores
    B = oracle.finalize_boundaries(p, tau, W)
    kept = _kept_by_repeated_argmax(p, tau, W)
    assert B.tolist() == [0] + [int(i) + 1 for i in sorted(set(kept.tolist()) | {L - 1})]
    assert B[0] == 0 and B[-1] == L and np.all(np.diff(B) > 0)
    cand = np.nonzero(p.astype(np.float64) > tau)[0]
    assert set(kept.tolist()) <= set(cand.tolist())
    if len(kept) > 1:
        assert np.all(np.diff(kept) > W)                   # kept ends are more than W apart
    for j in cand:                                          # every other candidate lies within W of a kept, better one
        if j in kept:
            continue
        near = kept[np.abs(kept - j) <= W]
        assert any((p[i] > p[j]) or (p[i] == p[j] and i < j) for i in near), (j, near)


def test_finalize_boundaries_special_cases():
    rng = np.random.default_rng(5)
    p = rng.random(1000).astype(np.float32)
    # a strictly increasing transform of the scores (and of the threshold) changes nothing
    np.testing.assert_array_equal(oracle.finalize_boundaries(p, 0.3, 8), oracle.finalize_boundaries(p * 2, 0.6, 8))
    # an isolated strict local maximum above the threshold is always a chunk end
    B = oracle.finalize_boundaries(p, 0.3, 8)
    for i in range(8, 991):
        w = np.r_[p[i - 8:i], p[i + 1:i + 9]]
        if p[i] > 0.3 and np.all(p[i] > w):
            assert (i + 1) in B
    # scores that rise along the sequence: the greedy walks from the end in steps of W + 1
    q = np.linspace(0.5, 1.0, 100).astype(np.float32)
    assert oracle.finalize_boundaries(q, 0.0, 9).tolist() == [0] + list(range(10, 101, 10))
    # NaN scores never exceed the threshold
    q2 = q.copy(); q2[::2] = np.nan
    assert (oracle.finalize_boundaries(q2, 0.0, 0)[1:-1] - 1).tolist() == list(range(1, 99, 2))


# ----------------------------------------------------------------------------
# The ablation "without robust chunk representation": plain average pooling (App. D)
# ----------------------------------------------------------------------------
def test_mean_pooling_closed_form_and_its_relation_to_eq4():
    rng = np.random.default_rng(23)
    L, D = 90, 6
    B = rand_boundaries(rng, L, 1, 11)
    X = rng.standard_normal((2, L, D)).astype(np.float32)
    lens = np.diff(B).astype(np.float64)
    want = np.add.reduceat(X.astype(np.float64), B[:-1], axis=1) / lens[None, :, None]
    np.testing.assert_allclose(oracle.pool_mean(X, B), want, rtol=1e-14, atol=1e-15)
    # Eq. 4 is sqrt(len) times the plain average, so S_c(mean)[l, k] = S_c(Eq. 4)[l, k] / sqrt(len_l len_k)
    np.testing.assert_allclose(oracle.pool(X, B), want * np.sqrt(lens)[None, :, None], rtol=1e-14, atol=1e-15)
    # row blocks: the plain average drops the sqrt(B_r) factor
    np.testing.assert_allclose(oracle.pool_blocks_mean(X, 7) * math.sqrt(7.0), oracle.pool_blocks(X, 7),
                                rtol=1e-14, atol=1e-15)


def test_mean_pooling_selects_like_eq4_on_equal_chunks_and_differently_on_unequal_ones():
    rng = np.random.default_rng(29)
    H_q, H_kv, D = 2, 1, 8
    # equal chunk lengths: the two representations differ by one common factor, rankings and sets agree (App. D)
    L = 96
    B = np.arange(0, L + 1, 8, dtype=np.int32)
    Q = rng.standard_normal((H_q, L, D)).astype(np.float32)
    K = rng.standard_normal((H_kv, L, D)).astype(np.float32)
    V = rng.standard_normal((H_kv, L, D)).astype(np.float32)
    rows = np.arange(L)
    for N_b in (3, 20):
        I0, c0 = oracle.route_rows(Q, K, B, N_b, rows, pooling=0)
        I1, c1 = oracle.route_rows(Q, K, B, N_b, rows, pooling=1)
        np.testing.assert_array_equal(I0, I1)
        np.testing.assert_array_equal(c0, c1)
        Ib0, _ = oracle.route_blocks(Q, K, B, 16, N_b, np.arange(6), pooling=0)
        Ib1, _ = oracle.route_blocks(Q, K, B, 16, N_b, np.arange(6), pooling=1)
        np.testing.assert_array_equal(Ib0, Ib1)
    # unequal lengths: the mean favours short chunks less than Eq. 4 favours long ones -- the sets differ somewhere,
    # and the mean-pooled sets are exactly the walk over rankings of the mean-pooled scores
    B2 = rand_boundaries(rng, L, 1, 20)
    I0, _ = oracle.route_rows(Q, K, B2, 10, rows, pooling=0)
    I1, c1 = oracle.route_rows(Q, K, B2, 10, rows, pooling=1)
    assert (I0 != I1).any()
    Qm, Km = oracle.pool_mean(Q, B2), oracle.pool_mean(K, B2)
    Sm = oracle.scores(Qm, Km)
    for h in range(H_q):
        for i in rows:
            l = int(np.searchsorted(B2, i, side="right") - 1)
            want = oracle.select(oracle.rank(Sm[h, l]), B2, i + 1, 10)
            assert I1[h, i, :c1[h, i]].tolist() == want.tolist()
    O1, _, _ = oracle.prefill_rows(Q, K, V, B2, 10, rows, pooling=1)
    for i in (0, 17, 95):
        np.testing.assert_allclose(O1[1, i], oracle.attend_row(Q[1, i], K[0], V[0], I1[1, i, :c1[1, i]], i, 1 / math.sqrt(D)),
                                   rtol=1e-13, atol=1e-14)


# ----------------------------------------------------------------------------
# Recall against exact top-k attention (App. "Theoretical Analysis", Setup and Notation)
# ----------------------------------------------------------------------------
def test_recall_row_hand_example_and_brute_force():
    # one row, logits 3, 1, 3, 2, 0 for keys 0..4 (q = [1], keys are the logits); top-2 = {0, 2} (tie of 3s)
    q = np.array([1.0], dtype=np.float32)
    Kg = np.array([[3.0], [1.0], [3.0], [2.0], [0.0]], dtype=np.float32)
    assert oracle.recall_row(q, Kg, 4, np.array([0, 2]), 2) == (2, 2)
    assert oracle.recall_row(q, Kg, 4, np.array([1, 4]), 2) == (0, 2)
    assert oracle.recall_row(q, Kg, 4, np.array([2, 3, 4]), 2) == (1, 2)
    # top-1 with equal best logits: the lower index wins
    assert oracle.recall_row(q, Kg, 4, np.array([2]), 1) == (0, 1)
    assert oracle.recall_row(q, Kg, 4, np.array([0]), 1) == (1, 1)
    # the budget is clipped to the causal length: row 1 sees keys 0, 1 only
    assert oracle.recall_row(q, Kg, 1, np.array([0, 1]), 4) == (2, 2)
    rng = np.random.default_rng(31)
    for _ in range(20):
        L, D = int(rng.integers(5, 60)), 4
        q = np.round(rng.standard_normal(D) * 2).astype(np.float32)      # integer-valued: ties occur
        Kg = np.round(rng.standard_normal((L, D)) * 2).astype(np.float32)
        i = int(rng.integers(0, L)); k = int(rng.integers(1, L + 3))
        I_hat = np.sort(rng.choice(i + 1, size=int(rng.integers(1, i + 2)), replace=False)).astype(np.int32)
        logits = Kg[:i + 1].astype(np.float64) @ q.astype(np.float64)
        top = set(np.argsort(-logits, kind="stable")[:min(k, i + 1)].tolist())
        assert oracle.recall_row(q, Kg, i, I_hat, k) == (len(top & set(I_hat.tolist())), min(k, i + 1))


def test_recall_of_routed_sets_special_cases():
    rng = np.random.default_rng(37)
    H_q, H_kv, L, D = 2, 1, 120, 8
    B = rand_boundaries(rng, L, 2, 12)
    Q = rng.standard_normal((H_q, L, D)).astype(np.float32)
    K = rng.standard_normal((H_kv, L, D)).astype(np.float32)
    rows = np.arange(L)
    # a budget of everything: both sets are all causal keys, recall 1
    hits, size = oracle.recall_rows(Q, K, B, L, 0, rows)
    np.testing.assert_array_equal(hits, rows + 1); np.testing.assert_array_equal(size, rows + 1)
    # one-token chunks: chunk scores ARE the token logits, so the routed set is exactly top-k: recall 1
    B1 = np.arange(L + 1, dtype=np.int32)
    hits, size = oracle.recall_rows(Q, K, B1, 9, 1, rows)
    np.testing.assert_array_equal(hits, size)
    np.testing.assert_array_equal(size, np.minimum(9, rows + 1))
    # general chunks: recall below 1 somewhere, and equal to an explicit set intersection
    hits, size = oracle.recall_rows(Q, K, B, 10, 1, rows)
    assert (hits < size).any() and (hits <= size).all()
    I, cnt = oracle.route_rows(Q, K, B, 10, rows)
    for i in (5, 60, 119):
        logits = K[0, :i + 1].astype(np.float64) @ Q[1, i].astype(np.float64)
        top = set(np.argsort(-logits, kind="stable")[:min(10, i + 1)].tolist())
        assert hits[i] == len(top & set(I[1, i, :cnt[1, i]].tolist()))
    # row-block form: keys of the block's list above the row do not count as retained
    hb, sb = oracle.recall_rows(Q, K, B, 10, 0, rows, B_r=16)
    Ib, cb = oracle.route_blocks(Q, K, B, 16, 10, rows // 16)
    for i in (3, 40, 119):
        logits = K[0, :i + 1].astype(np.float64) @ Q[0, i].astype(np.float64)
        top = set(np.argsort(-logits, kind="stable")[:min(10, i + 1)].tolist())
        vis = [j for j in Ib[0, i, :cb[0, i]].tolist() if j <= i]
        assert hb[i] == len(top & set(vis)) and sb[i] == min(10, i + 1)


# ----------------------------------------------------------------------------
# One decoding step (Sec. 3.4, the remark on decoding): the newest token's row
# ----------------------------------------------------------------------------
def test_decode_row_special_cases():
    rng = np.random.default_rng(41)
    H_q, H_kv, L, D = 4, 2, 90, 8
    B = rand_boundaries(rng, L, 2, 12)
    Q = rng.standard_normal((H_q, L, D)).astype(np.float32)
    K = rng.standard_normal((H_kv, L, D)).astype(np.float32)
    V = rng.standard_normal((H_kv, L, D)).astype(np.float32)
    scale = 1.0 / np.sqrt(D)

    def dense_last(keys, h):
        s = (K[h // 2, keys].astype(np.float64) @ Q[h, L - 1].astype(np.float64)) * scale
        p = np.exp(s - s.max())
        return (p / p.sum()) @ V[h // 2, keys].astype(np.float64)

    # a budget of everything: the newest token attends to every token, itself included
    for B_r in (0, 16):
        O, I, cnt = oracle.decode_row(Q, K, V, B, L + 5, B_r=B_r)
        assert (cnt == L).all() and (I[:, :L] == np.arange(L)).all()
        for h in range(H_q):
            np.testing.assert_allclose(O[h], dense_last(np.arange(L), h), rtol=1e-12, atol=1e-12)
    # one-token chunks: the chunk scores are the token logits q_{L-1} . k_j, so the step keeps the
    # N_b largest of them (equal logits: lower index) -- an argsort written out here
    B1 = np.arange(L + 1, dtype=np.int32)
    N_b = 7
    O, I, cnt = oracle.decode_row(Q, K, V, B1, N_b)
    for h in range(H_q):
        logits = K[h // 2].astype(np.float64) @ Q[h, L - 1].astype(np.float64)
        top = np.sort(np.argsort(-logits, kind="stable")[:N_b])
        assert cnt[h] == N_b and (I[h, :N_b] == top).all()
        np.testing.assert_allclose(O[h], dense_last(top, h), rtol=1e-12, atol=1e-12)
    # the queries of earlier chunks play no part in the step
    Q2 = Q.copy()
    Q2[:, :B[-2]] = 123.0
    O_a, I_a, _ = oracle.decode_row(Q, K, V, B, 20)
    O_b, I_b, _ = oracle.decode_row(Q2, K, V, B, 20)
    assert (I_a == I_b).all() and (O_a == O_b).all()
    # ... while the other queries of the open chunk do (Eq. 4 pools the chunk's queries); looked for
    # over a few draws, since one perturbation need not move a key across the cut-off
    moved = False
    for seed in range(10):
        r2 = np.random.default_rng(seed)
        if B[-1] - B[-2] < 2:
            break
        Q3 = Q.copy()
        Q3[:, B[-2]:L - 1] = 5.0 * r2.standard_normal((H_q, L - 1 - B[-2], D)).astype(np.float32)
        _, I_c, _ = oracle.decode_row(Q3, K, V, B, 20)
        moved = moved or not (I_c == I_a).all()
    assert moved or B[-1] - B[-2] < 2
