"""Python binding of libdhsa (include/dhsa.h): argument marshalling only.

Every step of the DHSA prefill path runs in the HIP kernels of libdhsa.so;
torch is used for device memory and the current stream.  There is no CPU
fallback: without the built library (or without a GPU for the compute calls)
these functions raise.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdhsa.so")

DHSA_F32, DHSA_BF16 = 0, 1
DHSA_POOL_ROBUST, DHSA_POOL_MEAN = 0, 1
PLAN_MAGIC = 0x41534844
POS_SHIFT = 28

EXPORTS = ["dhsa_plan_bytes", "dhsa_workspace_bytes", "dhsa_route", "dhsa_sparse_prefill", "dhsa_prefill",
           "dhsa_prefill_static", "dhsa_static_scratch_bytes", "dhsa_plan_check", "dhsa_prefill_stage_times",
           "dhsa_debug_scores",
           "dhsa_plan_expand_rows", "dhsa_debug_routing", "dhsa_mfma_probe", "dhsa_mfma_probe_scratch_bytes",
           "dhsa_finalize_boundaries", "dhsa_finalize_boundaries_workspace_bytes",
           "dhsa_recall_rows", "dhsa_recall_workspace_bytes",
           "dhsa_decode_step", "dhsa_decode_workspace_bytes",
           "dhsa_status_string", "dhsa_version"]


class dhsa_problem(C.Structure):
    _fields_ = [("L", C.c_int64), ("H_q", C.c_int32), ("H_kv", C.c_int32), ("D", C.c_int32),
                ("N_c", C.c_int32), ("N_b", C.c_int32), ("dtype", C.c_int32), ("scale", C.c_float),
                ("q_stride_h", C.c_int64), ("q_stride_l", C.c_int64),
                ("k_stride_h", C.c_int64), ("k_stride_l", C.c_int64),
                ("v_stride_h", C.c_int64), ("v_stride_l", C.c_int64),
                ("o_stride_h", C.c_int64), ("o_stride_l", C.c_int64),
                ("B_r", C.c_int32), ("pooling", C.c_int32)]


class DhsaError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libdhsa status {code}: {msg}")
        self.code = code


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    """Load libdhsa.so (build it with paper_2510_24606_amd.build first)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built: run `python -m paper_2510_24606_amd.build`")
        l = C.CDLL(LIB_PATH)
        P = C.POINTER(dhsa_problem)
        i32p, i64p, vp = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.c_void_p
        l.dhsa_plan_bytes.argtypes = [P, i32p]; l.dhsa_plan_bytes.restype = C.c_size_t
        l.dhsa_workspace_bytes.argtypes = [P, i32p]; l.dhsa_workspace_bytes.restype = C.c_size_t
        l.dhsa_route.argtypes = [P, vp, vp, i32p, vp, C.c_size_t, vp, C.c_size_t, vp]
        l.dhsa_route.restype = C.c_int
        l.dhsa_sparse_prefill.argtypes = [P, vp, vp, vp, i32p, vp, C.c_size_t, vp, vp]
        l.dhsa_sparse_prefill.restype = C.c_int
        l.dhsa_prefill.argtypes = [P, vp, vp, vp, i32p, vp, vp, C.c_size_t, vp, C.c_size_t, vp]
        l.dhsa_prefill.restype = C.c_int
        l.dhsa_prefill_static.argtypes = [P, vp, vp, vp, i32p, vp, vp, C.c_size_t, vp]
        l.dhsa_prefill_static.restype = C.c_int
        l.dhsa_static_scratch_bytes.argtypes = []; l.dhsa_static_scratch_bytes.restype = C.c_size_t
        l.dhsa_plan_check.argtypes = [P, i32p, vp, C.c_size_t, vp]; l.dhsa_plan_check.restype = C.c_int
        l.dhsa_prefill_stage_times.argtypes = [P, vp, vp, vp, i32p, vp, vp, C.c_size_t, vp, C.c_size_t,
                                               C.POINTER(C.c_float), vp]
        l.dhsa_prefill_stage_times.restype = C.c_int
        l.dhsa_debug_scores.argtypes = [P, i32p, vp, C.c_size_t, vp, vp]; l.dhsa_debug_scores.restype = C.c_int
        l.dhsa_plan_expand_rows.argtypes = [P, vp, C.c_size_t, C.c_int32, i64p, C.c_int32, vp, vp, C.c_int32, vp, vp]
        l.dhsa_plan_expand_rows.restype = C.c_int
        l.dhsa_debug_routing.argtypes = [P, i32p, vp, C.c_size_t, vp, vp, vp, vp]
        l.dhsa_debug_routing.restype = C.c_int
        l.dhsa_mfma_probe.argtypes = [C.c_int, C.c_int, vp, C.c_size_t, C.POINTER(C.c_double), C.POINTER(C.c_double), vp]
        l.dhsa_mfma_probe.restype = C.c_int
        l.dhsa_mfma_probe_scratch_bytes.argtypes = []; l.dhsa_mfma_probe_scratch_bytes.restype = C.c_size_t
        l.dhsa_finalize_boundaries.argtypes = [vp, C.c_int64, C.c_float, C.c_int32, vp, vp, vp, C.c_size_t, vp]
        l.dhsa_finalize_boundaries.restype = C.c_int
        l.dhsa_finalize_boundaries_workspace_bytes.argtypes = [C.c_int64]
        l.dhsa_finalize_boundaries_workspace_bytes.restype = C.c_size_t
        l.dhsa_recall_rows.argtypes = [P, vp, vp, i32p, vp, C.c_size_t, C.c_int32, i64p, C.c_int32, vp, vp, C.c_size_t,
                                       vp, vp, vp]
        l.dhsa_recall_rows.restype = C.c_int
        l.dhsa_recall_workspace_bytes.argtypes = [P, C.c_int32]; l.dhsa_recall_workspace_bytes.restype = C.c_size_t
        l.dhsa_decode_step.argtypes = [P, vp, vp, vp, i32p, C.c_int32, C.c_int64, C.c_int32, vp, vp, vp, vp,
                                       C.c_size_t, vp]
        l.dhsa_decode_step.restype = C.c_int
        l.dhsa_decode_workspace_bytes.argtypes = [P, C.c_int32, C.c_int64]
        l.dhsa_decode_workspace_bytes.restype = C.c_size_t
        l.dhsa_status_string.argtypes = [C.c_int]; l.dhsa_status_string.restype = C.c_char_p
        l.dhsa_version.argtypes = []; l.dhsa_version.restype = C.c_int
        _lib = l
    return _lib


def _check(code: int) -> None:
    if code != 0:
        raise DhsaError(code, lib().dhsa_status_string(code).decode())


def _b(B) -> np.ndarray:
    return np.ascontiguousarray(B, dtype=np.int32)


def _bp(B: np.ndarray):
    return B.ctypes.data_as(C.POINTER(C.c_int32))


def _stream() -> int:
    import torch
    return int(torch.cuda.current_stream().cuda_stream)


def problem(Q, K, B, N_b: int, scale: float = 0.0, B_r: int = 0, pooling: int = 0, V=None) -> dhsa_problem:
    """Describe Q [H_q, L, D] and K [H_kv, L, D] (torch tensors, last dim contiguous).
    B_r > 0 selects Alg. 1 as printed (row blocks of B_r rows, one index list per block).
    V (same shape as K) is only needed when its strides differ from a contiguous [H_kv, L, D]."""
    import torch
    H_q, L, D = Q.shape
    H_kv = K.shape[0]
    dt = {torch.float32: DHSA_F32, torch.bfloat16: DHSA_BF16}.get(Q.dtype, -1)
    return dhsa_problem(L=L, H_q=H_q, H_kv=H_kv, D=D, N_c=len(B) - 1, N_b=N_b, dtype=dt, scale=scale,
                        q_stride_h=Q.stride(0), q_stride_l=Q.stride(1),
                        k_stride_h=K.stride(0), k_stride_l=K.stride(1),
                        v_stride_h=0 if V is None else V.stride(0), v_stride_l=0 if V is None else V.stride(1),
                        B_r=B_r, pooling=pooling)


def dhsa_plan_bytes(prob: dhsa_problem, B) -> int:
    B = _b(B)
    return int(lib().dhsa_plan_bytes(C.byref(prob), _bp(B)))


def dhsa_workspace_bytes(prob: dhsa_problem, B) -> int:
    B = _b(B)
    return int(lib().dhsa_workspace_bytes(C.byref(prob), _bp(B)))


def alloc(prob: dhsa_problem, B, device="cuda"):
    """(plan, workspace) as uint8 device tensors of the sizes the library asks for."""
    import torch
    pb, wb = dhsa_plan_bytes(prob, B), dhsa_workspace_bytes(prob, B)
    if pb == 0 or wb == 0:
        # let the library name the reason
        _check(lib().dhsa_route(C.byref(prob), 16, 16, _bp(_b(B)), 16, 0, 16, 0, None) or 6)
    return (torch.empty(pb, dtype=torch.uint8, device=device), torch.empty(wb, dtype=torch.uint8, device=device))


def dhsa_route(prob, Q, K, B, plan, ws) -> None:
    B = _b(B)
    _check(lib().dhsa_route(C.byref(prob), Q.data_ptr(), K.data_ptr(), _bp(B), plan.data_ptr(), plan.numel(),
                            ws.data_ptr(), ws.numel(), _stream()))


def _with_vo(prob: dhsa_problem, V, O) -> dhsa_problem:
    p = dhsa_problem.from_buffer_copy(prob)
    p.v_stride_h, p.v_stride_l = V.stride(0), V.stride(1)
    p.o_stride_h, p.o_stride_l = O.stride(0), O.stride(1)
    return p


def dhsa_sparse_prefill(prob, Q, K, V, B, plan, O) -> None:
    B = _b(B)
    p = _with_vo(prob, V, O)
    _check(lib().dhsa_sparse_prefill(C.byref(p), Q.data_ptr(), K.data_ptr(), V.data_ptr(), _bp(B),
                                     plan.data_ptr(), plan.numel(), O.data_ptr(), _stream()))


def dhsa_prefill(prob, Q, K, V, B, O, plan, ws) -> None:
    B = _b(B)
    p = _with_vo(prob, V, O)
    _check(lib().dhsa_prefill(C.byref(p), Q.data_ptr(), K.data_ptr(), V.data_ptr(), _bp(B), O.data_ptr(),
                              plan.data_ptr(), plan.numel(), ws.data_ptr(), ws.numel(), _stream()))


def dhsa_prefill_static(prob, Q, K, V, B, O, plan) -> None:
    """dhsa_prefill with the routing scratch in the library's static device array (no workspace)."""
    B = _b(B)
    p = _with_vo(prob, V, O)
    _check(lib().dhsa_prefill_static(C.byref(p), Q.data_ptr(), K.data_ptr(), V.data_ptr(), _bp(B), O.data_ptr(),
                                     plan.data_ptr(), plan.numel(), _stream()))


def dhsa_plan_check(prob, B, plan) -> None:
    """Raises DhsaError (code 8) unless `plan` was routed for this problem and these boundaries.  Waits for the stream."""
    B = _b(B)
    _check(lib().dhsa_plan_check(C.byref(prob), _bp(B), plan.data_ptr(), plan.numel(), _stream()))


STAGES = ("setup", "pool", "scores", "select", "attn_rows_gt64", "attn_rows_33_64", "attn_rows_le32", "total")


def dhsa_prefill_stage_times(prob, Q, K, V, B, O, plan, ws) -> dict:
    """One pass of the whole path with events between its kernels: {stage: ms}.  Blocks."""
    B = _b(B)
    p = _with_vo(prob, V, O)
    ms = (C.c_float * 8)()
    _check(lib().dhsa_prefill_stage_times(C.byref(p), Q.data_ptr(), K.data_ptr(), V.data_ptr(), _bp(B), O.data_ptr(),
                                          plan.data_ptr(), plan.numel(), ws.data_ptr(), ws.numel(), ms, _stream()))
    return dict(zip(STAGES, (float(x) for x in ms)))


def dhsa_debug_scores(prob, B, ws):
    """S_c [H_q, N_q, N_c] fp64 (entries of chunks a query group cannot see are zero here)."""
    import torch
    B = _b(B)
    Sc = torch.zeros((prob.H_q, n_query_groups(prob), prob.N_c), dtype=torch.float64, device=ws.device)
    _check(lib().dhsa_debug_scores(C.byref(prob), _bp(B), ws.data_ptr(), ws.numel(), Sc.data_ptr(), _stream()))
    return Sc


def dhsa_static_scratch_bytes() -> int:
    return int(lib().dhsa_static_scratch_bytes())


def dhsa_plan_expand_rows(prob, plan, head: int, rows) -> Tuple["torch.Tensor", "torch.Tensor"]:
    """Index sets of `rows` (host int64) for one head: (idx [n, cap] int32 ascending, -1 padded; cnt [n])."""
    import torch
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    n = rows.shape[0]
    cap = int(min(prob.N_b, prob.L))
    idx = torch.empty((n, cap), dtype=torch.int32, device=plan.device)
    cnt = torch.empty(n, dtype=torch.int32, device=plan.device)
    scratch = torch.empty(max(n, 1), dtype=torch.int64, device=plan.device)
    _check(lib().dhsa_plan_expand_rows(C.byref(prob), plan.data_ptr(), plan.numel(), head,
                                       rows.ctypes.data_as(C.POINTER(C.c_int64)), n, scratch.data_ptr(),
                                       idx.data_ptr(), cap, cnt.data_ptr(), _stream()))
    return idx, cnt


def n_query_groups(prob) -> int:
    """Query groups of the routing: the chunks, or the row blocks when B_r > 0."""
    return (prob.L + prob.B_r - 1) // prob.B_r if prob.B_r > 0 else prob.N_c


def dhsa_debug_routing(prob, B, ws, want_Sc: bool = True):
    """(Q_c, K_c, S_c) fp64 device tensors copied out of a workspace dhsa_route filled."""
    import torch
    B = _b(B)
    dev = ws.device
    N_q = n_query_groups(prob)
    Qc = torch.empty((prob.H_q, N_q, prob.D), dtype=torch.float64, device=dev)
    Kc = torch.empty((prob.H_kv, prob.N_c, prob.D), dtype=torch.float64, device=dev)
    Sc = torch.zeros((prob.H_q, N_q, prob.N_c), dtype=torch.float64, device=dev) if want_Sc else None
    _check(lib().dhsa_debug_routing(C.byref(prob), _bp(B), ws.data_ptr(), ws.numel(), Qc.data_ptr(), Kc.data_ptr(),
                                    Sc.data_ptr() if want_Sc else None, _stream()))
    return Qc, Kc, Sc


def dhsa_mfma_probe(random_operands: bool, iters: int = 100000):
    """(TFLOP/s, shader MHz) of the bf16 MFMA alone on the whole chip; blocks until measured."""
    import torch
    L = lib()
    n = int(L.dhsa_mfma_probe_scratch_bytes())
    scratch = torch.empty(n, dtype=torch.uint8, device="cuda")
    tf, mhz = C.c_double(0.0), C.c_double(0.0)
    _check(L.dhsa_mfma_probe(int(bool(random_operands)), int(iters), scratch.data_ptr(), n, C.byref(tf), C.byref(mhz),
                             _stream()))
    return tf.value, mhz.value


def dhsa_finalize_boundaries(scores, threshold: float, window: int) -> np.ndarray:
    """Boundary scores [L] (fp32 device tensor; position i = end of a chunk) -> boundaries B as a host
    int32 array [N_c + 1] (0 ... L).  Synchronises the stream to bring B to the host."""
    import torch
    L = int(scores.shape[0])
    n = int(lib().dhsa_finalize_boundaries_workspace_bytes(L))
    ws = torch.empty(max(n, 1), dtype=torch.uint8, device=scores.device)
    B = torch.empty(L + 1, dtype=torch.int32, device=scores.device)
    N_c = torch.zeros(1, dtype=torch.int32, device=scores.device)
    _check(lib().dhsa_finalize_boundaries(scores.data_ptr(), L, float(threshold), int(window), B.data_ptr(),
                                          N_c.data_ptr(), ws.data_ptr(), ws.numel(), _stream()))
    torch.cuda.synchronize()
    return B[:int(N_c.item()) + 1].cpu().numpy()


def dhsa_recall_rows(prob, Q, K, B, plan, head: int, rows) -> Tuple["torch.Tensor", "torch.Tensor"]:
    """Recall counts of the routed sets of `rows` (host int64) of one head against exact top-k
    attention: (hits [n], size [n]) int32 device tensors; recall = hits / size."""
    import torch
    B = _b(B)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    n = rows.shape[0]
    nb = int(lib().dhsa_recall_workspace_bytes(C.byref(prob), n))
    ws = torch.empty(max(nb, 256), dtype=torch.uint8, device=plan.device)
    scratch = torch.empty(max(n, 1), dtype=torch.int64, device=plan.device)
    hits = torch.empty(n, dtype=torch.int32, device=plan.device)
    size = torch.empty(n, dtype=torch.int32, device=plan.device)
    _check(lib().dhsa_recall_rows(C.byref(prob), Q.data_ptr(), K.data_ptr(), _bp(B), plan.data_ptr(), plan.numel(),
                                  head, rows.ctypes.data_as(C.POINTER(C.c_int64)), n, scratch.data_ptr(),
                                  ws.data_ptr(), ws.numel(), hits.data_ptr(), size.data_ptr(), _stream()))
    return hits, size


def dhsa_decode_workspace_bytes(prob: dhsa_problem, N_c_cap: int, L_cap: int) -> int:
    return int(lib().dhsa_decode_workspace_bytes(C.byref(prob), N_c_cap, L_cap))


def alloc_decode(prob: dhsa_problem, N_c_cap: int, L_cap: int, device="cuda"):
    """Workspace of the decoding step (it keeps the pooled keys between steps)."""
    import torch
    n = dhsa_decode_workspace_bytes(prob, N_c_cap, L_cap)
    if n == 0:
        raise DhsaError(2, "problem or caps rejected by dhsa_decode_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def dhsa_decode_step(prob, Q, K, V, B, ws, N_c_cap: int, L_cap: int, kc_valid: int = 0, want_idx: bool = False,
                     out=None):
    """One decoding step for the newest token (row L - 1): O_row [H_q, D] in the input dtype (written
    into `out` if given); with want_idx also (idx [H_q, min(N_b, L)] int32 ascending, cnt [H_q] int32)."""
    import torch
    B = _b(B)
    O_row = out if out is not None else torch.empty((prob.H_q, prob.D), dtype=Q.dtype, device=Q.device)
    idx = cnt = None
    if want_idx:
        idx = torch.empty((prob.H_q, min(prob.N_b, prob.L)), dtype=torch.int32, device=Q.device)
        cnt = torch.empty(prob.H_q, dtype=torch.int32, device=Q.device)
    _check(lib().dhsa_decode_step(C.byref(prob), Q.data_ptr(), K.data_ptr(), V.data_ptr(), _bp(B), N_c_cap, L_cap,
                                  kc_valid, O_row.data_ptr(), idx.data_ptr() if want_idx else None,
                                  cnt.data_ptr() if want_idx else None, ws.data_ptr(), ws.numel(), _stream()))
    return (O_row, idx, cnt) if want_idx else O_row


def dhsa_version() -> int:
    return int(lib().dhsa_version())


def parse_plan(plan_host: np.ndarray) -> dict:
    """Split a plan (int32 words copied to the host) into its documented parts."""
    w = plan_host.view(np.int32)
    assert w[0] == PLAN_MAGIC, "not a DHSA plan"
    H_q, N_c, N_b, stride, L, T1 = (int(x) for x in (w[2], w[3], w[4], w[5], w[6], w[7]))
    oB, oC, oE, oT = (int(x) for x in w[8:12])
    oRB, N_q, B_r = int(w[13]), int(w[14]), int(w[15])
    return dict(H_q=H_q, N_c=N_c, N_b=N_b, stride=stride, L=L, T1=T1, T_big=int(w[12]), N_q=N_q, B_r=B_r,
                pooling=int(w[16]), b_sum=int(w[17]), H_kv=int(w[18]), D=int(w[19]), T_cls=[int(x) for x in w[20:24]],
                B=w[oB:oB + N_c + 1], RB=w[oRB:oRB + N_q + 1],
                count=w[oC:oC + H_q * N_q].reshape(H_q, N_q),
                entries=w[oE:oE + H_q * N_q * stride * 2].reshape(H_q, N_q, stride, 2),
                tiles=w[oT:oT + 2 * T1].reshape(T1, 2))
