"""laa_sync_static, the averaging that allocates nothing (its scratch is a static device array of the library),
against laa_sync through the C ABI: bit for bit, on two calls in a row, the second on a smaller table."""
import numpy as np
import pytest

from paper_1911_09030_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_1911_09030_amd import binding
    binding.lib()
    return binding


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _period(B, W, rows, row_len, k, H, seed):
    """Two handles take the same sparse steps; one averages with laa_sync, the other with laa_sync_static."""
    import torch
    print(f"sync_static W={W} rows={rows} row_len={row_len} k={k} H={H}", flush=True)
    d = rows * row_len
    zipf = wl.ZipfRows(rows, 1.1)
    x0 = dev(np.random.default_rng(seed).standard_normal(d).astype(np.float32))
    ref = B.LocalAdaAlter(d, W, H, 0.5, 1.0); ref.init_state(x0)
    sta = B.LocalAdaAlter(d, W, H, 0.5, 1.0); sta.init_state(x0)
    n_dirty = []
    for period in range(2):
        for t in range(1, H + 1):
            idx, vals = wl.sparse_step(zipf, W, k, row_len, seed, period * H + t)
            di, dv = dev(idx), dev(vals)
            ref.local_step_sparse(di, dv, row_len); sta.local_step_sparse(di, dv, row_len)
        n_dirty.append(ref.dirty_rows().size)
        ref.sync(); sta.sync_static()
        torch.cuda.synchronize()
        assert sta.counters() == ref.counters() == ((period + 1) * H, 0)
        assert torch.equal(sta.x, ref.x) and torch.equal(sta.acc, ref.acc) and torch.equal(sta.snap, ref.snap), period
        assert sta.dirty_rows().size == 0
    # consensus on every row after the averaging
    assert all(torch.equal(sta.x[0], sta.x[w]) for w in range(1, W)) and torch.equal(sta.acc[0], sta.snap)
    return n_dirty


def test_sync_static_equals_sync_twice_second_call_smaller(B):
    import torch
    big = _period(B, 8, 6000, 64, 400, 3, seed=101)
    small = _period(B, 4, 500, 16, 30, 2, seed=102)       # fewer rows, shorter list: stale entries of the first call remain
    assert min(big) > max(small) > 0
    # a dense averaging needs no scratch: same path as laa_sync, lazy replicas included
    W, H, d = 4, 2, 4 * 64 * 7 + 8
    rng = np.random.default_rng(103)
    ref = B.LocalAdaAlter(d, W, H, 0.5, 1.0); ref.set_lazy_replicas(True); ref.init_state()
    sta = B.LocalAdaAlter(d, W, H, 0.5, 1.0); sta.set_lazy_replicas(True); sta.init_state()
    for t in range(2 * H):
        G = dev(rng.standard_normal((W, d)).astype(np.float32))
        ref.local_step_dense(G); sta.local_step_dense(G)
        if (t + 1) % H == 0:
            ref.sync(); sta.sync_static()
    sta.sync_static()                                          # nothing pending: a no-op
    ref.materialize(); sta.materialize()
    torch.cuda.synchronize()
    assert torch.equal(sta.x, ref.x) and torch.equal(sta.acc, ref.acc) and torch.equal(sta.snap, ref.snap)


def test_sync_static_rejects_tables_beyond_its_scratch(B):
    import torch
    rows, row_len = (1 << 20) + 1, 4
    g = B.LocalAdaAlter(rows * row_len, 1, 2, 0.5, 1.0); g.init_state()
    idx = torch.tensor([[0, rows - 1]], dtype=torch.int32, device="cuda:0")
    vals = torch.ones((1, 2, row_len), device="cuda:0")
    g.local_step_sparse(idx, vals, row_len)
    with pytest.raises(B.LaaError) as ei:
        g.sync_static()
    assert ei.value.code == B.EINVAL and "1048576" in str(ei.value)
    assert g.counters() == (1, 1)                              # nothing was enqueued, nothing changed
    g.sync()                                                   # the allocating call takes any size
    assert g.counters() == (1, 0) and g.dirty_rows().size == 0
    ok = B.LocalAdaAlter((1 << 20) * row_len, 1, 2, 0.5, 1.0); ok.init_state()      # exactly the maximum
    ok.local_step_sparse(torch.tensor([[5, (1 << 20) - 1]], dtype=torch.int32, device="cuda:0"), vals, row_len)
    ok.sync_static()
    torch.cuda.synchronize()
    x = ok.x.view(1 << 20, row_len)
    assert bool(torch.allclose(x[5], torch.full((row_len,), -0.5 / 2.0 ** 0.5, device="cuda:0"), rtol=1e-6))
    assert bool((x[(1 << 20) - 1] != 0).all()) and bool((x[6] == 0).all())
    assert float(ok.snap.view(-1, row_len)[5, 0]) == 2.0
