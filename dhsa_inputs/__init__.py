"""Seeded synthetic workloads for the DHSA prefill path.

This module only draws random numbers and arranges them into tensors: it holds
none of the method's arithmetic (no pooling, scoring, selection or attention),
so both the CPU oracle's tests and the HIP path's tests/bench may import it.

Every workload is one attention layer, batch 1, laid out [H, L, D] (D
contiguous), with one boundary array shared by all heads.  The five named
workloads stand in for the attention shapes, context lengths and token
densities the paper measures on (LLaMA-3.1-8B / Qwen2.5 prompts from
needle-retrieval and long-context QA suites); none of those suites' items are
reproduced, only shapes and statistical structure.

Values are drawn in fp32; where a workload's dtype is bf16 they are rounded
(round-to-nearest-even) once here, and both sides consume the rounded arrays.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, Optional

import numpy as np
import torch

BASE_SEED = 251024606


@dataclasses.dataclass
class Workload:
    name: str
    L: int
    H_q: int
    H_kv: int
    D: int
    N_b: int
    dtype: str                 # "f32" | "bf16"
    B: np.ndarray              # int32 [N_c+1], 0 = B[0] < ... < B[N_c] = L
    Q: torch.Tensor            # [H_q, L, D]  (torch.float32 or torch.bfloat16, CPU)
    K: torch.Tensor            # [H_kv, L, D]
    V: torch.Tensor            # [H_kv, L, D]
    seed: int

    @property
    def N_c(self) -> int:
        return int(self.B.shape[0] - 1)

    def f32(self, which: str) -> np.ndarray:
        """The tensor's exact values as a float32 numpy array (what the oracle reads)."""
        t = getattr(self, which)
        return t.to(torch.float32).contiguous().numpy()

    def pairs_per_head(self) -> int:
        """Number of selected (row, key) pairs per head: sum_i min(N_b, i+1)."""
        nb = min(self.N_b, self.L)
        return self.L * nb - nb * (nb - 1) // 2


# name -> (L, H_q, H_kv, D, dtype, N_b, chunk-length law, structure)
SPECS: Dict[str, dict] = {
    "c1": dict(L=2048, H_q=4, H_kv=1, D=64, dtype="f32", N_b=256,
               lens=("uniform", 16, 64), structure="iid"),
    "c2": dict(L=32768, H_q=32, H_kv=8, D=128, dtype="bf16", N_b=2048,
               lens=("uniform", 32, 128), structure="needles"),
    "c3": dict(L=131072, H_q=32, H_kv=8, D=128, dtype="bf16", N_b=8192,
               lens=("uniform", 32, 128), structure="mixture"),
    "c4": dict(L=100000, H_q=32, H_kv=8, D=128, dtype="bf16", N_b=3125,
               lens=("geometric", 64, 8, 512), structure="loud_chunks"),
    "c5": dict(L=65536, H_q=28, H_kv=4, D=128, dtype="bf16", N_b=8192,
               lens=("uniform", 16, 256), structure="lowrank"),
}
ORDER = ["c1", "c2", "c3", "c4", "c5"]


def draw_boundaries(rng: np.random.Generator, L: int, law: tuple) -> np.ndarray:
    """Chunk lengths drawn iid from `law` until L is covered; the last boundary
    is clipped to L, so the last chunk may be shorter than the law's minimum."""
    out = [0]
    pos = 0
    while pos < L:
        n = max(64, (L - pos) // 8)
        if law[0] == "uniform":
            lens = rng.integers(law[1], law[2] + 1, size=n)
        elif law[0] == "geometric":
            lens = np.clip(rng.geometric(1.0 / law[1], size=n), law[2], law[3])
        elif law[0] == "fixed":
            lens = np.full(n, law[1])
        else:
            raise ValueError(law)
        for x in lens:
            pos += int(x)
            out.append(min(pos, L))
            if pos >= L:
                break
    return np.asarray(out, dtype=np.int32)


def _normal(seed_seq: np.random.SeedSequence, shape) -> np.ndarray:
    """[H, ...] standard normals, one child stream per leading index (head)."""
    H = shape[0]
    kids = seed_seq.spawn(H)
    out = np.empty(shape, dtype=np.float32)

    def fill(h):
        np.random.default_rng(kids[h]).standard_normal(out=out[h], dtype=np.float32)

    if out[0].size >= (1 << 20):
        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(fill, range(H)))
    else:
        for h in range(H):
            fill(h)
    return out


def make(name: str, *, L: Optional[int] = None, H_q: Optional[int] = None,
         H_kv: Optional[int] = None, D: Optional[int] = None, N_b: Optional[int] = None,
         dtype: Optional[str] = None, lens: Optional[tuple] = None,
         seed: Optional[int] = None) -> Workload:
    """Build workload `name` ("c1".."c5"); keyword overrides give reduced-size
    variants with the same statistical structure (used by the parity tests)."""
    spec = dict(SPECS[name])
    for k, v in dict(L=L, H_q=H_q, H_kv=H_kv, D=D, N_b=N_b, dtype=dtype, lens=lens).items():
        if v is not None:
            spec[k] = v
    L, H_q, H_kv, D = spec["L"], spec["H_q"], spec["H_kv"], spec["D"]
    assert H_q % H_kv == 0
    G = H_q // H_kv
    if seed is None:
        seed = BASE_SEED + ORDER.index(name)
    root = np.random.SeedSequence(seed)
    s_b, s_q, s_k, s_v, s_x = root.spawn(5)
    B = draw_boundaries(np.random.default_rng(s_b), L, spec["lens"])
    N_c = B.shape[0] - 1
    Q = _normal(s_q, (H_q, L, D))
    K = _normal(s_k, (H_kv, L, D))
    V = _normal(s_v, (H_kv, L, D))
    rx = np.random.default_rng(s_x)
    st = spec["structure"]
    if st == "iid":
        pass
    elif st == "needles":
        # Planted key chunks aligned with a later query row's direction: every
        # key of the chunk is shifted so that its dot product with that query
        # rises by three standard deviations (sigma = sqrt(D) for N(0,1) data).
        n_needles = min(64, max(1, N_c // 4))
        hi = max(1, int(N_c * 0.9))
        for g in range(H_kv):
            ids = rx.choice(hi, size=min(n_needles, hi), replace=False)
            for c in ids:
                end = int(B[c + 1])
                i_star = int(rx.integers(end, L)) if end < L else L - 1
                h_star = g * G + int(rx.integers(0, G))
                q = Q[h_star, i_star]
                nq = float(np.linalg.norm(q))
                K[g, B[c]:B[c + 1]] += (3.0 * np.sqrt(D) / (nq * nq)) * q
    elif st == "mixture":
        # Keys of a chunk share one of 256 cluster centres (N(0,1) entries),
        # within-chunk spread 0.3.
        for g in range(H_kv):
            mu = rx.standard_normal((256, D), dtype=np.float32)
            comp = rx.integers(0, 256, size=N_c)
            per_tok = np.repeat(comp, np.diff(B))
            K[g] *= np.float32(0.3)
            K[g] += mu[per_tok]
    elif st == "loud_chunks":
        for g in range(H_kv):
            loud = rx.random(N_c) < 0.01
            for c in np.nonzero(loud)[0]:
                K[g, B[c]:B[c + 1]] *= np.float32(4.0)
    elif st == "lowrank":
        Z = rx.standard_normal((L, 8), dtype=np.float32)
        for g in range(H_kv):
            W = rx.standard_normal((8, D), dtype=np.float32)
            K[g] += np.float32(0.5 / np.sqrt(8.0)) * (Z @ W)
    else:
        raise ValueError(st)

    tq, tk, tv = (torch.from_numpy(a) for a in (Q, K, V))
    if spec["dtype"] == "bf16":
        tq, tk, tv = (t.to(torch.bfloat16) for t in (tq, tk, tv))
    elif spec["dtype"] != "f32":
        raise ValueError(spec["dtype"])
    return Workload(name=name, L=L, H_q=H_q, H_kv=H_kv, D=D, N_b=spec["N_b"],
                    dtype=spec["dtype"], B=B, Q=tq, K=tk, V=tv, seed=seed)


def sample_rows(w: Workload, n: int, seed: int = 0) -> np.ndarray:
    """A stratified sample of query rows: the first rows, the rows around the
    budget N_b, the first and last rows of some random chunks, the last row,
    and uniformly random rows; sorted, unique."""
    rng = np.random.default_rng([w.seed, seed, 7])
    L, nb = w.L, w.N_b
    rows = {0, 1, 2, 3, L - 1, nb - 1, nb, nb + 1}
    ch = rng.integers(0, w.N_c, size=min(32, w.N_c))
    for c in ch:
        rows.add(int(w.B[c]))
        rows.add(int(w.B[c + 1]) - 1)
    rows = {r for r in rows if 0 <= r < L}
    target = min(max(n, len(rows)), L)
    while len(rows) < target:
        for x in rng.integers(0, L, size=n):
            if len(rows) >= target:
                break
            rows.add(int(x))
    return np.array(sorted(rows), dtype=np.int64)
