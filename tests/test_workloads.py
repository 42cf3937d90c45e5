"""Seeded workload generators: reproducible, shaped like the paper's mixes."""
import numpy as np

import sgmv_workloads as wl


def test_reproducible_from_seed():
    a, b = wl.tiny(seed=0), wl.tiny(seed=0)
    assert np.array_equal(a.x, b.x) and np.array_equal(a.A[3], b.A[3]) and np.array_equal(a.y0, b.y0)
    c = wl.tiny(seed=1)
    assert not np.array_equal(a.x, c.x)


def test_tiny_shape():
    w = wl.tiny()
    assert (w.h_in, w.h_out, w.r, w.n_tokens, w.n_segs) == (256, 256, 8, 8, 4)
    assert w.seg_starts.tolist() == [0, 1, 4, 6, 8]
    assert w.A[0].shape == (1, 256, 8) and w.B[0].shape == (1, 8, 256)


def test_segments_from_ids():
    s, ids = wl.segments_from_ids([3, 1, 3, 0, 1, 3])
    assert s.tolist() == [0, 1, 3, 6] and ids.tolist() == [0, 1, 3]
    s, ids = wl.segments_from_ids([])
    assert s.tolist() == [0] and len(ids) == 0


def test_popularity_mixes():
    d = wl.popularity("distinct", batch=16, h_in=64, r=8, num_layers=1)
    assert d.n_segs == 16 and d.max_seg_len == 1
    i = wl.popularity("identical", batch=16, h_in=64, r=8, num_layers=1)
    assert i.n_segs == 1 and i.max_seg_len == 16
    u = wl.popularity("uniform", batch=64, h_in=64, r=8, num_layers=1, seed=0)
    assert 25 <= u.n_segs <= 55 and u.n_tokens == 64          # E[n] ~ 40.6
    s = wl.popularity("skewed", batch=64, h_in=64, r=8, num_layers=1, seed=0)
    assert 5 <= s.n_segs <= 30 and s.max_seg_len >= 12        # head adapter ~ 42 %
    up = wl.popularity("uniform_paper", batch=64, h_in=64, r=8, num_layers=1)
    assert up.n_segs == 8 and up.max_seg_len == 8             # ceil(sqrt(64)) models
    sp = wl.popularity("skewed_paper", batch=64, h_in=64, r=8, num_layers=1)
    lens = np.diff(sp.seg_starts)
    assert lens.sum() == 64 and np.all(np.diff(lens) <= 0) and lens[0] in (21, 22)


def test_zipf_and_geometric():
    p = wl.zipf_probabilities(64, 1.5)
    assert abs(p.sum() - 1) < 1e-12 and 0.40 < p[0] < 0.45
    c = wl.geometric_counts(64, 1.5)
    assert c.sum() == 64 and c[0] / c[1] == 1.5 or abs(c[0] / c[1] - 1.5) < 0.2


def test_prefill_lengths():
    w = wl.prefill(h_in=64, h_out=64, r=16, seed=0)
    lens = np.diff(w.seg_starts)
    assert w.n_segs == 8 and lens.min() >= 128 and lens.max() <= 1024


def test_weight_statistics():
    w = wl.decode_distinct(batch=2, h_in=4096, r=16, num_layers=1)
    A = w.A[0].view(np.float16).astype(np.float64)
    B = w.B[0].view(np.float16).astype(np.float64)
    assert abs(A.std() - 1 / 64) < 1e-3 and abs(B.std() - 0.25) < 5e-3
