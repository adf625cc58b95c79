"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, sizes buffers sanely and rejects bad
arguments before any device call."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2510_24606_amd as dhsa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(dhsa.LIB_PATH):
        from paper_2510_24606_amd import build
        build.build()
    return dhsa.lib()


def header_symbols():
    text = open(os.path.join(ROOT, "include", "dhsa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dhsa_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = header_symbols()
    assert set(names) == set(dhsa.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    assert dhsa.dhsa_version() >= 100


def mk(L=1000, H_q=4, H_kv=2, D=128, N_c=10, N_b=64, dtype=dhsa.DHSA_BF16, **kw):
    return dhsa.dhsa_problem(L=L, H_q=H_q, H_kv=H_kv, D=D, N_c=N_c, N_b=N_b, dtype=dtype, **kw)


def bounds(L=1000, N_c=10):
    return np.linspace(0, L, N_c + 1).astype(np.int32)


def test_sizes(lib):
    B = bounds()
    p = mk()
    pb, wb = dhsa.dhsa_plan_bytes(p, B), dhsa.dhsa_workspace_bytes(p, B)
    # workspace: pooled Q, K and S_c in fp64
    assert wb >= 8 * (4 * 10 * 128 + 2 * 10 * 128 + 4 * 10 * 10)
    # plan: header + B + counts + entries (stride <= N_c) + tiles
    assert 64 + 4 * 11 + 4 * 40 <= pb <= 4 * (16 + 12 + 40 + 4 * 10 * 10 * 2 + 2 * 10 + 64 + 16)
    # a tighter budget needs no more plan than a looser one
    assert dhsa.dhsa_plan_bytes(mk(N_b=8), B) <= pb
    # chunks longer than a row tile get several tiles
    B2 = np.array([0, 1000], dtype=np.int32)
    assert dhsa.dhsa_plan_bytes(mk(N_c=1), B2) > 0
    # row-block form: the plan holds N_r = ceil(L / B_r) lists per head, the workspace S_c of N_r x N_c
    pr = mk(B_r=100)
    assert dhsa.dhsa_plan_bytes(pr, B) > 0
    assert dhsa.dhsa_workspace_bytes(pr, B) >= 8 * (4 * 10 * 128 + 2 * 10 * 128 + 4 * 10 * 10)
    assert dhsa.dhsa_workspace_bytes(mk(B_r=10), B) >= 8 * (4 * 100 * 128 + 2 * 10 * 128 + 4 * 100 * 10)


def test_plan_size_follows_the_documented_layout(lib):
    """Plan words = header 32 | B | counts | entries [H_q][N_c][stride][2] | tiles, where stride =
    min(N_c, n + 2) and n = how many of the shortest chunks have lengths summing to less than N_b
    (recomputed here with a sort; the library counts lengths, and sorts only for very long chunks)."""
    rng = np.random.default_rng(3)
    al = lambda x, a: (x + a - 1) // a * a
    for case in range(40):
        N_c = int(rng.integers(1, 300))
        hi = 70000 if case % 8 == 7 else int(rng.integers(1, 400))       # some chunks past the counting range
        lens = rng.integers(1, hi + 1, size=N_c)
        if case % 8 == 7:
            lens[rng.integers(0, N_c)] = 70000
        B = np.r_[0, np.cumsum(lens)].astype(np.int32)
        L = int(B[-1])
        N_b = int(rng.integers(1, max(2, L)))
        H_q = 4
        p = mk(L=L, H_q=H_q, H_kv=2, N_c=N_c, N_b=N_b)
        srt = np.sort(lens)
        acc, n = 0, 0
        while n < N_c and acc + srt[n] < N_b:
            acc += int(srt[n]); n += 1
        stride = min(N_c, n + 2)
        T1 = int(((lens + 127) // 128).sum())
        off_count = al(32 + N_c + 1, 4)
        off_entries = al(off_count + H_q * N_c, 4)
        off_tiles = al(off_entries + H_q * N_c * stride * 2, 4)
        words = al(off_tiles + 2 * T1, 64)
        assert dhsa.dhsa_plan_bytes(p, B) == 4 * words, (case, N_c, N_b, stride)


@pytest.mark.parametrize("kw,code", [
    (dict(dtype=7), 5),
    (dict(L=0), 2),
    (dict(H_q=5), 2),            # H_q % H_kv != 0
    (dict(D=96), 2),
    (dict(N_c=0), 2),
    (dict(N_c=9000, L=20000), 2),  # above the chunk limit
    (dict(N_b=0), 4),
    (dict(scale=-1.0), 2),
    (dict(q_stride_l=100), 2),   # row stride shorter than D
    (dict(q_stride_l=132), 9),   # 264-byte rows break 16-byte alignment
    (dict(B_r=-1), 2),           # row-block size below 0
    (dict(pooling=2), 2),        # unknown chunk representation
])
def test_bad_problems_are_rejected_on_the_host(lib, kw, code):
    p = mk(**kw)
    B = bounds(L=max(p.L, 1), N_c=max(p.N_c, 1))
    assert dhsa.dhsa_plan_bytes(p, B) == 0 and dhsa.dhsa_workspace_bytes(p, B) == 0
    rc = lib.dhsa_route(C.byref(p), 16, 16, B.ctypes.data_as(C.POINTER(C.c_int32)), 16, 1 << 30, 16, 1 << 30, None)
    assert rc == code, lib.dhsa_status_string(rc)


def test_bad_boundaries_and_buffers(lib):
    p = mk()
    bp = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
    for bad in (np.r_[1, bounds()[1:]], np.r_[bounds()[:-1], 999], np.r_[0, 100, 100, bounds()[3:]],
                np.r_[0, 200, 100, bounds()[3:]]):
        bad = bad.astype(np.int32)
        assert lib.dhsa_route(C.byref(p), 16, 16, bp(bad), 16, 1 << 30, 16, 1 << 30, None) == 3
        assert lib.dhsa_prefill(C.byref(p), 16, 16, 16, bp(bad), 16, 16, 1 << 30, 16, 1 << 30, None) == 3
    B = bounds()
    assert lib.dhsa_route(C.byref(p), None, 16, bp(B), 16, 1 << 30, 16, 1 << 30, None) == 1      # NULL
    assert lib.dhsa_route(C.byref(p), 16, 16, None, 16, 1 << 30, 16, 1 << 30, None) == 1
    assert lib.dhsa_route(C.byref(p), 16, 24, bp(B), 16, 1 << 30, 16, 1 << 30, None) == 9        # misaligned
    assert lib.dhsa_route(C.byref(p), 16, 16, bp(B), 16, 8, 16, 1 << 30, None) == 6              # plan too small
    assert lib.dhsa_route(C.byref(p), 16, 16, bp(B), 16, 1 << 30, 16, 8, None) == 6              # ws too small
    assert lib.dhsa_sparse_prefill(C.byref(p), 16, 16, 16, bp(B), 16, 8, 16, None) == 8          # plan too small
    assert lib.dhsa_prefill(C.byref(p), 16, 16, None, bp(B), 16, 16, 1 << 30, 16, 1 << 30, None) == 1
    for s in range(10):
        assert len(lib.dhsa_status_string(s)) > 1


def test_static_scratch_plan_check_and_stage_times_reject_bad_arguments_on_the_host(lib):
    p, B = mk(), bounds()
    bp = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
    assert dhsa.dhsa_static_scratch_bytes() == 64 << 20
    # dhsa_prefill_static: NULL, misaligned, plan too small, and a problem beyond the static scratch
    assert lib.dhsa_prefill_static(C.byref(p), 16, 16, None, bp(B), 16, 16, 1 << 30, None) == 1
    assert lib.dhsa_prefill_static(C.byref(p), 16, 16, 16, bp(B), 24, 16, 1 << 30, None) == 9
    assert lib.dhsa_prefill_static(C.byref(p), 16, 16, 16, bp(B), 16, 16, 8, None) == 6
    big_B = np.arange(8193, dtype=np.int32)
    big = mk(L=8192, H_q=64, H_kv=1, D=64, N_c=8192, N_b=16, dtype=dhsa.DHSA_F32)
    assert dhsa.dhsa_workspace_bytes(big, big_B) > dhsa.dhsa_static_scratch_bytes()
    assert lib.dhsa_prefill_static(C.byref(big), 16, 16, 16, bp(big_B), 16, 16, 1 << 40, None) == 6
    bad = np.r_[0, 200, 100, bounds()[3:]].astype(np.int32)
    assert lib.dhsa_prefill_static(C.byref(p), 16, 16, 16, bp(bad), 16, 16, 1 << 30, None) == 3
    # dhsa_plan_check
    assert lib.dhsa_plan_check(C.byref(p), bp(B), None, 1 << 30, None) == 1
    assert lib.dhsa_plan_check(C.byref(p), bp(B), 24, 1 << 30, None) == 9
    assert lib.dhsa_plan_check(C.byref(p), bp(B), 16, 8, None) == 8
    assert lib.dhsa_plan_check(C.byref(mk(N_b=0)), bp(B), 16, 1 << 30, None) == 4
    # dhsa_prefill_stage_times
    ms = (C.c_float * 8)()
    assert lib.dhsa_prefill_stage_times(C.byref(p), 16, 16, 16, bp(B), 16, 16, 1 << 30, 16, 1 << 30, None, None) == 1
    assert lib.dhsa_prefill_stage_times(C.byref(p), 16, 16, 16, bp(B), 16, 16, 8, 16, 1 << 30, ms, None) == 6
    assert lib.dhsa_prefill_stage_times(C.byref(mk(D=96)), 16, 16, 16, bp(B), 16, 16, 1 << 30, 16, 1 << 30, ms, None) == 2
    # dhsa_debug_scores
    assert lib.dhsa_debug_scores(C.byref(p), bp(B), 16, 1 << 30, None, None) == 1
    assert lib.dhsa_debug_scores(C.byref(p), bp(B), 16, 8, 16, None) == 6


def test_mfma_probe_rejects_bad_arguments_on_the_host(lib):
    import ctypes as C
    tf = C.c_double(0.0)
    need = lib.dhsa_mfma_probe_scratch_bytes()
    assert need >= 512 * 256 * 4
    fake = C.c_void_p(256)   # never dereferenced: every call below fails validation first (1 NULL, 2 SHAPE, 6 WORKSPACE)
    assert lib.dhsa_mfma_probe(0, 100, None, need, C.byref(tf), None, None) == 1
    assert lib.dhsa_mfma_probe(0, 100, fake, need, None, None, None) == 1
    assert lib.dhsa_mfma_probe(0, 0, fake, need, C.byref(tf), None, None) == 2
    assert lib.dhsa_mfma_probe(0, 1 << 23, fake, need, C.byref(tf), None, None) == 2
    assert lib.dhsa_mfma_probe(0, 100, fake, need - 1, C.byref(tf), None, None) == 6


def test_finalize_boundaries_rejects_bad_arguments_on_the_host(lib):
    import ctypes as C
    fake = C.c_void_p(256)   # never dereferenced: every call below fails validation first (1 NULL, 2 SHAPE, 6 WORKSPACE)
    need = lib.dhsa_finalize_boundaries_workspace_bytes(1000)
    assert need >= 1000 and lib.dhsa_finalize_boundaries_workspace_bytes(0) == 0
    f = lib.dhsa_finalize_boundaries
    assert f(None, 1000, 0.5, 8, fake, fake, fake, need, None) == 1
    assert f(fake, 1000, 0.5, 8, None, fake, fake, need, None) == 1
    assert f(fake, 0, 0.5, 8, fake, fake, fake, need, None) == 2
    assert f(fake, 1000, 0.5, -1, fake, fake, fake, need, None) == 2
    assert f(fake, 1000, float("nan"), 8, fake, fake, fake, need, None) == 2
    assert f(fake, 1000, 0.5, 8, fake, fake, fake, need - 1, None) == 6


def test_recall_rows_rejects_bad_arguments_on_the_host(lib):
    import ctypes as C
    B = bounds()
    p = mk()
    fake = C.c_void_p(256)   # never dereferenced: every call below fails validation first
    rows = (C.c_int64 * 2)(3, 999)
    bad_rows = (C.c_int64 * 2)(3, 1000)
    Bp = B.ctypes.data_as(C.POINTER(C.c_int32))
    pb = dhsa.dhsa_plan_bytes(p, B)
    need = lib.dhsa_recall_workspace_bytes(C.byref(p), 2)
    assert need >= 2 * 1000 * 8
    f = lib.dhsa_recall_rows
    ok_args = [C.byref(p), fake, fake, Bp, fake, pb, 0, rows, 2, fake, fake, need, fake, fake, None]
    def call(**kw):
        a = list(ok_args)
        for k, v in kw.items():
            a[int(k[1:])] = v
        return f(*a)
    assert call(a1=None) == 1                    # Q
    assert call(a13=None) == 1                   # size_dev
    assert call(a6=4) == 2                       # head out of range
    assert call(a7=bad_rows) == 2                # a row beyond L
    assert call(a5=pb - 4) == 8                  # plan too small
    assert call(a11=need - 8) == 6               # workspace too small


def test_decode_step_rejects_bad_arguments_on_the_host(lib):
    import ctypes as C
    B = bounds()
    p = mk()
    fake = C.c_void_p(256)   # never dereferenced: every call below fails validation first
    Bp = B.ctypes.data_as(C.POINTER(C.c_int32))
    need = lib.dhsa_decode_workspace_bytes(C.byref(p), 16, 2000)
    # pooled keys [H_kv][N_c_cap][D] fp64 + slice states [H_q][ceil(N_b / 128)][D + 2] fp32 at least
    assert need >= 2 * 16 * 128 * 8 + 4 * 1 * 130 * 4
    assert lib.dhsa_decode_workspace_bytes(C.byref(p), 0, 2000) == 0
    assert lib.dhsa_decode_workspace_bytes(C.byref(p), 8193, 2000) == 0
    assert lib.dhsa_decode_workspace_bytes(C.byref(p), 16, 0) == 0
    assert lib.dhsa_decode_workspace_bytes(C.byref(mk(D=96)), 16, 2000) == 0
    # a larger budget or cap never shrinks the workspace
    assert lib.dhsa_decode_workspace_bytes(C.byref(mk(N_b=4096)), 16, 100000) > need
    f = lib.dhsa_decode_step
    ok_args = [C.byref(p), fake, fake, fake, Bp, 16, 2000, 0, fake, None, None, fake, need, None]
    def call(**kw):
        a = list(ok_args)
        for k, v in kw.items():
            a[int(k[1:])] = v
        return f(*a)
    assert call(a1=None) == 1                    # Q
    assert call(a8=None) == 1                    # O_row
    assert call(a11=None) == 1                   # workspace
    assert call(a5=9) == 2                       # N_c_cap below N_c = 10
    assert call(a6=999) == 2                     # L_cap below L = 1000
    assert call(a7=10) == 2                      # kc_valid = N_c: the open chunk must be pooled
    assert call(a7=-1) == 2
    assert call(a12=need - 1) == 6               # workspace too small
    assert call(a3=C.c_void_p(264)) == 9         # V not 16-byte aligned
    bad = B.copy(); bad[3] = bad[2]
    assert call(a4=bad.ctypes.data_as(C.POINTER(C.c_int32))) == 3


def test_no_oracle_in_the_product_path():
    """The product package must not import, load or call the oracle."""
    pkg = os.path.join(ROOT, "paper_2510_24606_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
