"""The seeded workload generator: shapes, determinism, boundary laws."""
import numpy as np
import torch

import dhsa_inputs


def test_c1_shape_and_determinism():
    a = dhsa_inputs.make("c1")
    b = dhsa_inputs.make("c1")
    assert a.Q.shape == (4, 2048, 64) and a.K.shape == (1, 2048, 64) and a.V.shape == (1, 2048, 64)
    assert a.Q.dtype == torch.float32 and a.N_b == 256
    assert torch.equal(a.Q, b.Q) and torch.equal(a.K, b.K) and np.array_equal(a.B, b.B)
    lens = np.diff(a.B)
    assert a.B[0] == 0 and a.B[-1] == 2048 and (lens > 0).all()
    assert lens[:-1].min() >= 16 and lens.max() <= 64
    assert a.pairs_per_head() == 491648


def test_reduced_variants_keep_structure():
    for name, kw in (("c2", dict(L=3000, H_q=4, H_kv=2, N_b=200)),
                     ("c3", dict(L=4096, H_q=4, H_kv=2, N_b=256)),
                     ("c4", dict(L=5000, H_q=4, H_kv=2, N_b=160)),
                     ("c5", dict(L=4096, H_q=7, H_kv=1, N_b=512))):
        w = dhsa_inputs.make(name, **kw)
        assert w.Q.dtype == torch.bfloat16 and w.Q.shape == (kw["H_q"], kw["L"], 128)
        assert w.B[-1] == kw["L"] and (np.diff(w.B) > 0).all()
        assert torch.isfinite(w.K.float()).all()
    w = dhsa_inputs.make("c4", L=100000, H_q=1, H_kv=1)
    lens = np.diff(w.B)
    assert lens[:-1].min() >= 8 and lens.max() <= 512 and 40 < lens.mean() < 90


def test_sample_rows_cover_the_edges():
    w = dhsa_inputs.make("c1")
    rows = dhsa_inputs.sample_rows(w, 64)
    assert rows[0] == 0 and rows[-1] == w.L - 1 and len(np.unique(rows)) == len(rows)
    for r in (w.N_b - 1, w.N_b, w.N_b + 1):
        assert r in rows
