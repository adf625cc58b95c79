"""ctypes binding of the DHSA CPU oracle (oracle/dhsa_oracle.c).

TEST INFRASTRUCTURE: only tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg may import this package.  It never touches the HIP library.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dhsa_oracle.c")
_LIB = os.path.join(_HERE, "libdhsa_oracle.so")
_lib: Optional[C.CDLL] = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, -O2, OpenMP over independent rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-fvisibility=hidden",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
    return _lib


def _p(a: np.ndarray, ty):
    return a.ctypes.data_as(C.POINTER(ty))


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def num_threads() -> int:
    return int(lib().dhsa_oracle_num_threads())


def pool(X: np.ndarray, B: np.ndarray) -> np.ndarray:
    """Eq. 4 chunk representations of X [H, L, D] -> [H, N_c, D] (fp64)."""
    X = _f32(X); B = _i32(B)
    H, L, D = X.shape
    N_c = B.shape[0] - 1
    out = np.empty((H, N_c, D), dtype=np.float64)
    rc = lib().dhsa_oracle_pool(_p(X, C.c_float), H, C.c_int64(L), D, _p(B, C.c_int32), N_c, _p(out, C.c_double))
    assert rc == 0
    return out


def pool_mean(X: np.ndarray, B: np.ndarray) -> np.ndarray:
    """Plain average pooling of X [H, L, D] over the chunks (the ablation without Eq. 4's factor)."""
    X = _f32(X); B = _i32(B)
    H, L, D = X.shape
    N_c = B.shape[0] - 1
    out = np.empty((H, N_c, D), dtype=np.float64)
    rc = lib().dhsa_oracle_pool_mean(_p(X, C.c_float), H, C.c_int64(L), D, _p(B, C.c_int32), N_c, _p(out, C.c_double))
    assert rc == 0
    return out


def scores(Qc: np.ndarray, Kc: np.ndarray) -> np.ndarray:
    """S_c[h] = Q_c[h] K_c[h // G]^T, full [H_q, N_c, N_c] (fp64)."""
    Qc = _f64(Qc); Kc = _f64(Kc)
    H_q, N_c, D = Qc.shape
    H_kv = Kc.shape[0]
    out = np.empty((H_q, N_c, N_c), dtype=np.float64)
    rc = lib().dhsa_oracle_scores(_p(Qc, C.c_double), _p(Kc, C.c_double), H_q, H_kv, N_c, D, _p(out, C.c_double))
    assert rc == 0
    return out


def rank(S_row: np.ndarray) -> np.ndarray:
    """Chunk ids by score descending, equal scores by ascending id."""
    S_row = _f64(S_row)
    n = S_row.shape[0]
    pi = np.empty(n, dtype=np.int32)
    rc = lib().dhsa_oracle_rank(_p(S_row, C.c_double), n, _p(pi, C.c_int32))
    assert rc == 0
    return pi


def select(pi: np.ndarray, B: np.ndarray, q_max: int, N_b: int) -> np.ndarray:
    """Alg. 1 walk for one ranking and one causal limit q_max; ascending indices."""
    pi = _i32(pi); B = _i32(B)
    out = np.empty(N_b, dtype=np.int32)
    n = lib().dhsa_oracle_select(_p(pi, C.c_int32), _p(B, C.c_int32), B.shape[0] - 1, C.c_int64(q_max), N_b,
                                 _p(out, C.c_int32))
    assert n >= 0
    return out[:n].copy()


def select_pairs(Sc_h: np.ndarray, B: np.ndarray, N_b: int) -> Tuple[np.ndarray, np.ndarray]:
    """Token-pair form of the selection for one head (tiny L): (I [L, N_b], cnt [L])."""
    Sc_h = _f64(Sc_h); B = _i32(B)
    N_c = B.shape[0] - 1
    L = int(B[-1])
    I = np.empty((L, N_b), dtype=np.int32)
    cnt = np.empty(L, dtype=np.int32)
    rc = lib().dhsa_oracle_select_pairs(_p(Sc_h, C.c_double), _p(B, C.c_int32), N_c, N_b, _p(I, C.c_int32),
                                        _p(cnt, C.c_int32))
    assert rc == 0
    return I, cnt


def attend_row(q, Kg, Vg, I, i: int, scale: float) -> np.ndarray:
    """Alg. 2 for one query row i of one head over the index list I."""
    q = _f32(q); Kg = _f32(Kg); Vg = _f32(Vg); I = _i32(I)
    D = q.shape[0]
    o = np.empty(D, dtype=np.float64)
    rc = lib().dhsa_oracle_attend_row(_p(q, C.c_float), _p(Kg, C.c_float), _p(Vg, C.c_float), _p(I, C.c_int32),
                                      I.shape[0], C.c_int64(i), D, C.c_double(scale), _p(o, C.c_double))
    assert rc == 0
    return o


def attend_block_tiled(Qh, Kg, Vg, I, q_s: int, q_e: int, scale: float, B_c: int) -> np.ndarray:
    """Alg. 3 for the row block [q_s, q_e) of one head sharing the index list I."""
    Qh = _f32(Qh); Kg = _f32(Kg); Vg = _f32(Vg); I = _i32(I)
    D = Qh.shape[1]
    O = np.empty((q_e - q_s, D), dtype=np.float64)
    rc = lib().dhsa_oracle_attend_block_tiled(_p(Qh, C.c_float), _p(Kg, C.c_float), _p(Vg, C.c_float),
                                              _p(I, C.c_int32), I.shape[0], C.c_int64(q_s), C.c_int64(q_e), D,
                                              C.c_double(scale), B_c, _p(O, C.c_double))
    assert rc == 0
    return O


def chunk_walk(pi: np.ndarray, B: np.ndarray, l: int) -> Tuple[np.ndarray, np.ndarray]:
    pi = _i32(pi); B = _i32(B)
    N_c = B.shape[0] - 1
    before = np.empty(N_c, dtype=np.int32)
    pos = np.empty(N_c, dtype=np.int8)
    rc = lib().dhsa_oracle_chunk_walk(_p(pi, C.c_int32), _p(B, C.c_int32), N_c, l, _p(before, C.c_int32),
                                      _p(pos, C.c_int8))
    assert rc == 0
    return before, pos


def route_rows(Q, K, B, N_b: int, rows, pooling: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Index sets of the given rows for every query head: (I [H_q, n, N_b] (-1 padded), cnt [H_q, n])."""
    Q = _f32(Q); K = _f32(K); B = _i32(B)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    H_q, L, D = Q.shape
    H_kv = K.shape[0]
    n = rows.shape[0]
    I = np.empty((H_q, n, N_b), dtype=np.int32)
    cnt = np.empty((H_q, n), dtype=np.int32)
    rc = lib().dhsa_oracle_route_rows(_p(Q, C.c_float), _p(K, C.c_float), H_q, H_kv, C.c_int64(L), D,
                                      _p(B, C.c_int32), B.shape[0] - 1, N_b, int(pooling), _p(rows, C.c_int64), n,
                                      _p(I, C.c_int32), _p(cnt, C.c_int32))
    assert rc == 0
    return I, cnt


def prefill_rows(Q, K, V, B, N_b: int, rows, scale: Optional[float] = None, pooling: int = 0):
    """The whole path on the given rows: (O [H_q, n, D] fp64, I, cnt)."""
    Q = _f32(Q); K = _f32(K); V = _f32(V); B = _i32(B)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    H_q, L, D = Q.shape
    H_kv = K.shape[0]
    n = rows.shape[0]
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    O = np.empty((H_q, n, D), dtype=np.float64)
    I = np.empty((H_q, n, N_b), dtype=np.int32)
    cnt = np.empty((H_q, n), dtype=np.int32)
    rc = lib().dhsa_oracle_prefill_rows(_p(Q, C.c_float), _p(K, C.c_float), _p(V, C.c_float), H_q, H_kv,
                                        C.c_int64(L), D, _p(B, C.c_int32), B.shape[0] - 1, N_b, int(pooling),
                                        C.c_double(scale), _p(rows, C.c_int64), n, _p(O, C.c_double),
                                        _p(I, C.c_int32), _p(cnt, C.c_int32))
    assert rc == 0
    return O, I, cnt


def plan_head(Qc_h, Kc_g, B, N_b: int):
    """Chunk-level walk state of one query head: (rem [N_c, N_c], pos [N_c, N_c], cut_gap [N_c])."""
    Qc_h = _f64(Qc_h); Kc_g = _f64(Kc_g); B = _i32(B)
    N_c, D = Qc_h.shape
    rem = np.empty((N_c, N_c), dtype=np.int32)
    pos = np.empty((N_c, N_c), dtype=np.int8)
    gap = np.empty(N_c, dtype=np.float64)
    rc = lib().dhsa_oracle_plan_head(_p(Qc_h, C.c_double), _p(Kc_g, C.c_double), _p(B, C.c_int32), N_c, D, N_b,
                                     _p(rem, C.c_int32), _p(pos, C.c_int8), _p(gap, C.c_double))
    assert rc == 0
    return rem, pos, gap


# ---- Alg. 1 as printed: fixed row blocks ----

def pool_blocks(X: np.ndarray, B_r: int) -> np.ndarray:
    """Row-block query representations sqrt(B_r) * AvgPool of X [H, L, D] -> [H, N_r, D] (fp64)."""
    X = _f32(X)
    H, L, D = X.shape
    N_r = (L + B_r - 1) // B_r
    out = np.empty((H, N_r, D), dtype=np.float64)
    rc = lib().dhsa_oracle_pool_blocks(_p(X, C.c_float), H, C.c_int64(L), D, B_r, _p(out, C.c_double))
    assert rc == 0
    return out


def select_block(q_i, Kc_g, B, q_max: int, N_b: int) -> np.ndarray:
    """Alg. 1 for one row block: scores against every key chunk, stable ranking, walk with q_max."""
    q_i = _f64(q_i); Kc_g = _f64(Kc_g); B = _i32(B)
    N_c, D = Kc_g.shape
    out = np.empty(N_b, dtype=np.int32)
    n = lib().dhsa_oracle_select_block(_p(q_i, C.c_double), _p(Kc_g, C.c_double), _p(B, C.c_int32), N_c, D,
                                       C.c_int64(q_max), N_b, _p(out, C.c_int32))
    assert n >= 0
    return out[:n].copy()


def select_pairs_blocks(Sb_h, B, B_r: int, N_b: int) -> Tuple[np.ndarray, np.ndarray]:
    """Token-level form of the block selection for one head (tiny L): (I [N_r, N_b], cnt [N_r])."""
    Sb_h = _f64(Sb_h); B = _i32(B)
    N_c = B.shape[0] - 1
    L = int(B[-1])
    N_r = (L + B_r - 1) // B_r
    assert Sb_h.shape == (N_r, N_c)
    I = np.empty((N_r, N_b), dtype=np.int32)
    cnt = np.empty(N_r, dtype=np.int32)
    rc = lib().dhsa_oracle_select_pairs_blocks(_p(Sb_h, C.c_double), _p(B, C.c_int32), N_c, B_r, N_b,
                                               _p(I, C.c_int32), _p(cnt, C.c_int32))
    assert rc == 0
    return I, cnt


def pool_blocks_mean(X: np.ndarray, B_r: int) -> np.ndarray:
    """Plain average of every row block of X [H, L, D] -> [H, N_r, D] (fp64)."""
    X = _f32(X)
    H, L, D = X.shape
    N_r = (L + B_r - 1) // B_r
    out = np.empty((H, N_r, D), dtype=np.float64)
    rc = lib().dhsa_oracle_pool_blocks_mean(_p(X, C.c_float), H, C.c_int64(L), D, B_r, _p(out, C.c_double))
    assert rc == 0
    return out


def route_blocks(Q, K, B, B_r: int, N_b: int, blocks, pooling: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Index lists of the given row blocks for every query head: (I [H_q, n, N_b] (-1 padded), cnt [H_q, n])."""
    Q = _f32(Q); K = _f32(K); B = _i32(B)
    blocks = np.ascontiguousarray(blocks, dtype=np.int64)
    H_q, L, D = Q.shape
    H_kv = K.shape[0]
    n = blocks.shape[0]
    I = np.empty((H_q, n, N_b), dtype=np.int32)
    cnt = np.empty((H_q, n), dtype=np.int32)
    rc = lib().dhsa_oracle_route_blocks(_p(Q, C.c_float), _p(K, C.c_float), H_q, H_kv, C.c_int64(L), D,
                                        _p(B, C.c_int32), B.shape[0] - 1, B_r, N_b, int(pooling),
                                        _p(blocks, C.c_int64), n, _p(I, C.c_int32), _p(cnt, C.c_int32))
    assert rc == 0
    return I, cnt


def prefill_rows_blocks(Q, K, V, B, B_r: int, N_b: int, rows, scale: Optional[float] = None, pooling: int = 0):
    """The block-form path on the given rows: (O [H_q, n, D] fp64, I of each row's block, cnt)."""
    Q = _f32(Q); K = _f32(K); V = _f32(V); B = _i32(B)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    H_q, L, D = Q.shape
    H_kv = K.shape[0]
    n = rows.shape[0]
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    O = np.empty((H_q, n, D), dtype=np.float64)
    I = np.empty((H_q, n, N_b), dtype=np.int32)
    cnt = np.empty((H_q, n), dtype=np.int32)
    rc = lib().dhsa_oracle_prefill_rows_blocks(_p(Q, C.c_float), _p(K, C.c_float), _p(V, C.c_float), H_q, H_kv,
                                               C.c_int64(L), D, _p(B, C.c_int32), B.shape[0] - 1, B_r, N_b,
                                               int(pooling), C.c_double(scale), _p(rows, C.c_int64), n, _p(O, C.c_double),
                                               _p(I, C.c_int32), _p(cnt, C.c_int32))
    assert rc == 0
    return O, I, cnt


def plan_blocks_head(Qb_h, Kc_g, B, B_r: int, N_b: int):
    """Per row block of one head: tokens listed per key chunk (take [N_r, N_c]) and cut_gap [N_r]."""
    Qb_h = _f64(Qb_h); Kc_g = _f64(Kc_g); B = _i32(B)
    N_r, D = Qb_h.shape
    N_c = B.shape[0] - 1
    take = np.empty((N_r, N_c), dtype=np.int32)
    gap = np.empty(N_r, dtype=np.float64)
    rc = lib().dhsa_oracle_plan_blocks_head(_p(Qb_h, C.c_double), _p(Kc_g, C.c_double), _p(B, C.c_int32), N_c, D,
                                            B_r, N_b, _p(take, C.c_int32), _p(gap, C.c_double))
    assert rc == 0
    return take, gap


# ---- boundary finalisation (threshold + NMS) ----

def finalize_boundaries(p, tau: float, W: int) -> np.ndarray:
    """Boundary scores p [L] (position i = end of a chunk) -> boundaries B [N_c + 1] (half-open, 0 ... L)."""
    p = _f32(p)
    L = p.shape[0]
    B = np.empty(L + 1, dtype=np.int32)
    lib().dhsa_oracle_finalize_boundaries.restype = C.c_int64
    n_c = lib().dhsa_oracle_finalize_boundaries(_p(p, C.c_float), C.c_int64(L), C.c_double(tau), int(W),
                                                _p(B, C.c_int32))
    assert n_c >= 1
    return B[:n_c + 1].copy()


# ---- recall against exact top-k attention ----

def recall_row(q, Kg, i: int, I_hat, k_top: int) -> Tuple[int, int]:
    """(|I* n I_hat|, |I*|) for one row: I* = the min(k_top, i+1) keys j <= i with the largest logits."""
    q = _f32(q); Kg = _f32(Kg); I_hat = _i32(I_hat)
    hits, size = C.c_int32(0), C.c_int32(0)
    rc = lib().dhsa_oracle_recall_row(_p(q, C.c_float), _p(Kg, C.c_float), C.c_int64(i), q.shape[0],
                                      _p(I_hat, C.c_int32), I_hat.shape[0], int(k_top), C.byref(hits), C.byref(size))
    assert rc == 0
    return hits.value, size.value


def recall_rows(Q, K, B, N_b: int, head: int, rows, B_r: int = 0, pooling: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Recall counts of the routed sets of `rows` of one query head: (hits [n], size [n])."""
    Q = _f32(Q); K = _f32(K); B = _i32(B)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    H_q, L, D = Q.shape
    n = rows.shape[0]
    hits = np.empty(n, dtype=np.int32); size = np.empty(n, dtype=np.int32)
    rc = lib().dhsa_oracle_recall_rows(_p(Q, C.c_float), _p(K, C.c_float), H_q, K.shape[0], C.c_int64(L), D,
                                       _p(B, C.c_int32), B.shape[0] - 1, int(B_r), int(N_b), int(pooling), int(head),
                                       _p(rows, C.c_int64), n, _p(hits, C.c_int32), _p(size, C.c_int32))
    assert rc == 0
    return hits, size


def decode_row(Q, K, V, B, N_b: int, B_r: int = 0, scale: Optional[float] = None, pooling: int = 0):
    """The newest token of a sequence of L tokens, i.e. one decoding step with the keys restricted
    by the same mechanism (Sec. 3.4, the remark on decoding): row L - 1 of the path above, its
    query group being the open chunk (B_r = 0) or the open row block (B_r > 0).
    Returns (O [H_q, D] fp64, I [H_q, N_b] (-1 padded), cnt [H_q])."""
    L = np.asarray(Q).shape[1]
    rows = np.array([L - 1], dtype=np.int64)
    if B_r:
        O, I, cnt = prefill_rows_blocks(Q, K, V, B, B_r, N_b, rows, scale, pooling)
    else:
        O, I, cnt = prefill_rows(Q, K, V, B, N_b, rows, scale, pooling)
    return O[:, 0], I[:, 0], cnt[:, 0]
