#!/usr/bin/env python3
"""Timing of the two entry points beside the hot path on c3-sized inputs: boundary
finalisation (threshold + non-maximum suppression over L = 131072 seeded scores) and the recall
diagnostic (48 sampled rows of one head).  Prints one line per case; used for the rocprofv3
summary under profiles/."""
from __future__ import annotations

import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def peaked_scores(L: int, seed: int):
    """A low noise floor with a sharp peak (and shoulders) every 20-80 tokens."""
    import numpy as np
    rng = np.random.default_rng(seed)
    p = 0.2 * rng.random(L)
    at = np.cumsum(rng.integers(20, 80, size=L // 20 + 2))
    at = at[at < L]
    p[at] += 0.5 + 0.3 * rng.random(len(at))
    for d in (-1, 1):
        ok = (at + d >= 0) & (at + d < L)
        p[at[ok] + d] += 0.3
    return p.astype(np.float32)


def main() -> int:
    import numpy as np
    import torch
    import dhsa_inputs
    import paper_2510_24606_amd as dhsa

    L = 131072
    for kind, W in (("peaks", 8), ("peaks", 64), ("noise", 8), ("noise", 64)):
        p = peaked_scores(L, 7) if kind == "peaks" else np.random.default_rng(7).random(L).astype(np.float32)
        tau = 0.4 if kind == "peaks" else 0.5
        pd = torch.from_numpy(p).cuda()
        dhsa.dhsa_finalize_boundaries(pd, tau, W)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        B = dhsa.dhsa_finalize_boundaries(pd, tau, W)
        e1.record(); torch.cuda.synchronize()
        print(f"finalize_boundaries {kind} L={L} tau={tau} W={W}: N_c={len(B) - 1}, {e0.elapsed_time(e1):.3f} ms "
              f"(incl. the copy of B to the host)", flush=True)

    w = dhsa_inputs.make("c3")
    Q, K = w.Q.cuda(), w.K.cuda()
    prob = dhsa.problem(Q, K, w.B, w.N_b)
    plan, ws = dhsa.alloc(prob, w.B)
    dhsa.dhsa_route(prob, Q, K, w.B, plan, ws)
    rows = dhsa_inputs.sample_rows(w, 48)
    dhsa.dhsa_recall_rows(prob, Q, K, w.B, plan, 5, rows)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    hits, size = dhsa.dhsa_recall_rows(prob, Q, K, w.B, plan, 5, rows)
    e1.record(); torch.cuda.synchronize()
    rec = (hits.cpu().numpy() / size.cpu().numpy()).mean()
    print(f"recall_rows c3 head 5, {len(rows)} rows: mean recall {rec:.4f}, {e0.elapsed_time(e1):.3f} ms", flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
