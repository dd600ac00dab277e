"""Host-side checks of the seeded input generators (no GPU, no optimizer arithmetic): the recipe both sides are fed
from must be deterministic, have the stated distributions and shapes, and hold the five configurations."""
import numpy as np
import pytest

from paper_1911_09030_amd import workloads as wl


def test_configurations():
    c = wl.WORKLOADS
    assert (c["c1"].d, c["c1"].W, c["c1"].H, c["c1"].T) == (1 << 20, 4, 4, 64)
    assert (c["c2"].d, c["c2"].W, c["c2"].H, c["c2"].a_dist) == (25_000_000, 8, 8, "loguniform")
    assert (c["c3"].d, c["c3"].kind, c["c3"].H_sweep) == (100_000_000, "explicit", (1, 4, 16, 64))
    assert (c["c4"].rows, c["c4"].row_len, c["c4"].k, c["c4"].d) == (800_000, 512, 8192, 800_000 * 512)
    assert c["c4"].dense_blocks == ((2048, 8192),) * 4
    assert (c["c5"].d, c["c5"].W, c["c5"].H, c["c5"].eta, c["c5"].eps) == (400_000_000, 8, 16, 0.05, 1e-2)
    for w in c.values():
        assert w.T % w.H == 0 and w.d % 4 == 0


def test_generators_are_deterministic_and_in_range():
    d = 200_000
    a = wl.curvature(d, 7)
    assert a.dtype == np.float32 and np.array_equal(a, wl.curvature(d, 7)) and not np.array_equal(a, wl.curvature(d, 8))
    assert a.min() >= 0.1 and a.max() <= 10.0 and abs(a.mean() - 5.05) < 0.05
    al = wl.curvature(d, 7, "loguniform")
    assert al.min() >= 1e-3 * (1 - 1e-6) and al.max() <= 1e2 * (1 + 1e-6)
    assert abs(np.log10(al).mean() - (-0.5)) < 0.02                     # uniform exponent on [-3, 2]
    xs = wl.optimum(d, 7)
    assert abs(xs.mean()) < 0.01 and abs(xs.std() - 1) < 0.01
    off = wl.offsets(d, 3, 7, 0.1)
    assert off.shape == (3, d) and abs(off.std() - 0.1) < 0.001
    sg = wl.sigma(d, 7)
    assert sg.min() >= 1e-4 * (1 - 1e-6) and sg.max() <= 1.0 and abs(np.log10(sg).mean() - (-2.0)) < 0.02
    G = wl.explicit_gradients(1000, 4, 7, 3, sg[:1000])
    assert G.shape == (4, 1000) and G.dtype == np.float32
    assert np.array_equal(G, wl.explicit_gradients(1000, 4, 7, 3, sg[:1000]))
    assert not np.array_equal(G, wl.explicit_gradients(1000, 4, 7, 4, sg[:1000]))
    # a prefix of a longer draw is the shorter draw: column slices of a workload are consistent
    assert np.array_equal(wl.curvature(1000, 7), a[:1000]) and np.array_equal(wl.optimum(1000, 7), xs[:1000])


def test_zipf_rows_are_distinct_and_head_heavy():
    rows, k = 50_000, 2000
    z = wl.ZipfRows(rows, 1.1)
    rng = np.random.default_rng(1)
    r = z.draw(k, rng)
    assert r.dtype == np.int32 and r.shape == (k,) and len(set(r.tolist())) == k
    assert r.min() >= 0 and r.max() < rows
    # P(rank 1) = 1 / sum_r r^-1.1: check the inverse-CDF table against the closed form and a sample
    p1 = 1.0 / np.sum(np.arange(1, rows + 1, dtype=np.float64) ** -1.1)
    assert abs(z.cdf[0] - p1) < 1e-12 and abs(z.cdf[-1] - 1.0) < 1e-12
    hits = sum(0 in z.draw(50, rng).tolist() for _ in range(400))
    assert hits > 300                                                  # 1 - (1 - p1)^50 is about 0.998 for these sizes
    with pytest.raises(ValueError):
        z.draw(rows + 1, rng)
    idx, vals = wl.sparse_step(z, 3, 100, 8, 5, 2)
    assert idx.shape == (3, 100) and vals.shape == (3, 100, 8) and vals.dtype == np.float32
    assert all(len(set(idx[w].tolist())) == 100 for w in range(3))
    idx2, _ = wl.sparse_step(z, 3, 100, 8, 5, 2, with_vals=False)
    assert np.array_equal(idx, idx2)


def test_column_sample_covers_ends_and_whole_groups():
    for d in (4000, 4003, 8):
        cols = wl.column_sample(d, 16, seed=3)
        assert cols.dtype == np.int64 and np.all(np.diff(cols) > 0) and cols[0] == 0 and cols[-1] == d - 1
        g = cols[cols < (d // 4) * 4].reshape(-1, 4)
        assert np.all(g[:, 0] % 4 == 0) and np.all(g == g[:, :1] + np.arange(4))
        if d % 4:
            assert np.array_equal(cols[-(d % 4):], np.arange((d // 4) * 4, d))
