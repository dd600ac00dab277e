"""GPU parity tests: the HIP path, called through the C-ABI, against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

import oracle
from oracle import Oracle
from paper_1911_09030_amd import workloads as wl
import parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_1911_09030_amd import binding
    binding.lib()            # raises if liblaa.so is missing: no fallback
    return binding


def dev(a, dtype=None):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to("cuda:0")


def host(t):
    import torch
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()


def say(*a):
    print(*a, flush=True)


# many thread blocks (64 threads x 4 coordinates each) plus a ragged tail
D_SMALL = 4 * (256 * 9 + 37)


def test_philox_words_bit_exact(B):
    rng = np.random.default_rng(0)
    cases = [([0, 0, 0, 0], [0, 0]), ([0xFFFFFFFF] * 4, [0xFFFFFFFF] * 2)]
    cases += [(rng.integers(0, 2**32, 4, dtype=np.uint64).tolist(), rng.integers(0, 2**32, 2, dtype=np.uint64).tolist())
              for _ in range(20)]
    for ctr, key in cases:
        assert np.array_equal(B.debug_philox(ctr, key), oracle.philox4x32_10(ctr, key)), (ctr, key)


@pytest.mark.parametrize("W,H,d", [(4, 4, D_SMALL), (8, 8, D_SMALL), (1, 3, 4 * 300), (2, 2, 4 * 1000),
                                   (3, 5, 4 * 777), (5, 2, 4 * 513), (16, 4, 4 * 2049), (12, 3, 4 * 700),
                                   (4, 4, 4 * 256 * 3 + 3), (8, 2, 1023), (2, 4, 1), (64, 2, 4 * 130), (7, 50, 4 * 64)])
def test_dense_explicit_one_step_and_full_run(B, W, H, d):
    """Same gradient bits on both sides: <= 1e-6 after one step, <= 1e-5 after T steps with syncs."""
    say(f"dense explicit W={W} H={H} d={d}")
    T = 4 * H
    rng = np.random.default_rng(1000 + W * 31 + H)
    x0 = rng.standard_normal(d).astype(np.float32)
    sig = np.power(10.0, rng.uniform(-3, 1, d)).astype(np.float32)
    o = Oracle(d, W, H, 0.5, 1.0); o.init_state(x0)
    g = B.LocalAdaAlter(d, W, H, 0.5, 1.0); g.init_state(dev(x0))
    sc = parity.Scale(o)
    for t in range(1, T + 1):
        G = (rng.standard_normal((W, d)).astype(np.float32) * sig[None, :])
        o.local_step_dense(G)
        g.local_step_dense(dev(G))
        sc.update(o)
        if t == 1:
            parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, parity.ONE_STEP, what="one step", scale=sc)
        if t % H == 0:
            o.sync(); g.sync()
        assert g.counters() == (o.t, o.steps_since_sync)
    e = parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, parity.FULL_RUN, what=f"after {T} steps",
                            scale=sc)
    say("   rel err x/acc/snap", e)


@pytest.mark.parametrize("eta,eps,b0", [(0.5, 0.0, 1.0), (0.05, 1e-3, 0.5), (2.0, 10.0, 3.0), (-0.1, 1.0, 1.0),
                                        (1e-3, 1e-2, 1.0)])
def test_hyperparameters(B, eta, eps, b0):
    """Step size, epsilon and b0 away from the defaults (eps = 0 leaves sqrt(B2) alone under the root; a negative
    step size is ascent; b0 < 1 is outside the theorem's assumption but inside the algorithm)."""
    W, H, d = 4, 3, 4 * 64 * 3 + 8
    rng = np.random.default_rng(97)
    x0 = rng.standard_normal(d).astype(np.float32)
    o = Oracle(d, W, H, eta, eps, b0); o.init_state(x0)
    g = B.LocalAdaAlter(d, W, H, eta, eps, b0=b0); g.set_lazy_replicas(True); g.init_state(dev(x0))
    sc = parity.Scale(o)
    for t in range(1, 3 * H + 2):
        G = rng.standard_normal((W, d)).astype(np.float32)
        o.step_dense(G); g.step_dense(dev(G)); sc.update(o)
        if t == 1:
            parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, parity.ONE_STEP, what="one step", scale=sc,
                                floor_b=1e-3 * b0 * b0)
    g.materialize()
    parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, parity.FULL_RUN, what=f"eta={eta} eps={eps} b0={b0}",
                        scale=sc, floor_b=1e-3 * b0 * b0)


def test_unaligned_buffers_take_scalar_path(B):
    import torch
    W, H, d = 4, 2, 4 * 500
    rng = np.random.default_rng(5)
    buf = torch.empty(2 * W * d + d + 16, dtype=torch.float32, device="cuda:0")
    x = buf[1:1 + W * d].view(W, d)                    # 4-byte but not 16-byte aligned
    acc = buf[1 + W * d:1 + 2 * W * d].view(W, d)
    snap = buf[1 + 2 * W * d:1 + 2 * W * d + d]
    o = Oracle(d, W, H, 0.3, 0.5); o.init_state()
    g = B.LocalAdaAlter(d, W, H, 0.3, 0.5, x=x, acc=acc, snap=snap); g.init_state()
    sc = parity.Scale(o)
    for t in range(1, 5):
        G = rng.standard_normal((W, d)).astype(np.float32)
        o.local_step_dense(G); sc.update(o)
        if t % H == 0:
            o.sync()
        g.step_dense(dev(G))
    parity.assert_state(host(x), host(acc), host(snap), o, parity.FULL_RUN, what="unaligned", scale=sc)


@pytest.mark.parametrize("W,d,pitch", [(8, D_SMALL, D_SMALL + 64), (4, 4 * 300, 4 * 300 + 8), (3, 1001, 1003), (2, 4096, 4096 + 1024)])
def test_pitched_rows(B, W, d, pitch):
    """Rows `pitch` elements apart (dense, generator with stored offsets, fused sync, sparse): same results."""
    import torch
    H = 3
    rng = np.random.default_rng(17)
    x0 = rng.standard_normal(d).astype(np.float32)
    o = Oracle(d, W, H, 0.5, 1.0); o.init_state(x0)
    p = pitch
    xbuf = torch.full((W, p), 7.0, device="cuda:0"); accbuf = torch.full((W, p), 7.0, device="cuda:0")
    g = B.LocalAdaAlter(d, W, H, 0.5, 1.0, x=xbuf[:, :d], acc=accbuf[:, :d], pitch=p); g.init_state(dev(x0))
    assert g.pitch >= d and g.x.stride(0) == g.pitch
    sc = parity.Scale(o)
    for t in range(1, 2 * H + 1):                      # explicit gradients, fused sync
        G = rng.standard_normal((W, d)).astype(np.float32)
        o.local_step_dense(G); sc.update(o)
        if t % H == 0:
            o.sync()
        g.step_dense(g.rows(dev(G)))
    parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, parity.FULL_RUN, what="pitched dense", scale=sc)
    a = rng.uniform(0.1, 10, d).astype(np.float32); xs = rng.standard_normal(d).astype(np.float32)
    off = (0.1 * rng.standard_normal((W, d))).astype(np.float32)
    o.set_generator(oracle.GEN_QUADRATIC, 5, a, xs, off, oracle.OFF_ARRAY, 0.1, 0.1)
    g.set_generator(B.GEN_QUADRATIC, 5, dev(a), dev(xs), g.rows(dev(off)), B.OFF_ARRAY, 0.1, 0.1)
    for t in range(H + 1):                             # generator with stored offsets, separate sync
        G_ref = o.gradient(o.t + 1)
        G_gpu = host(g.generate_gradient())
        assert np.max(np.abs(G_gpu - G_ref) / _gen_scale(a, o.x, xs, 0.1, 0.1)) <= 1e-6
        o.local_step_gen(); g.local_step_gen()
        if o.steps_since_sync == H:
            o.sync(); g.sync()
    parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, 1e-5, floor_x=1.0, what="pitched generator")
    if d % 16 == 0 and g.pitch % 4 == 0:               # sparse rows of 16
        o.sync(); g.sync()
        rows = d // 16
        sc = parity.Scale(o)
        for t in range(H):
            idx = np.stack([rng.permutation(rows)[:min(rows, 20)] for _ in range(W)]).astype(np.int32)
            vals = rng.standard_normal((W, idx.shape[1], 16)).astype(np.float32)
            o.local_step_sparse(idx, vals, 16); g.local_step_sparse(dev(idx), dev(vals), 16); sc.update(o)
        assert np.array_equal(g.dirty_rows(), o.dirty_rows())
        o.sync(); g.sync()
        parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, 1e-5, floor_x=1.0, what="pitched sparse", scale=sc)
    # the padding between rows is never written, and arrays with another pitch are refused
    if g.pitch != d:
        assert bool((xbuf[:, d:] == 7.0).all()) and bool((accbuf[:, d:] == 7.0).all())
        with pytest.raises(ValueError):
            g.step_dense(dev(np.zeros((W, d), np.float32)))


@pytest.mark.parametrize("hold_gaps", [False, True])
def test_spread_buffers_layout(B, hold_gaps):
    """binding.spread_buffers: 2W + 3 arrays a fixed distance apart, usable as the state; with hold_gaps the
    gaps are part of one ordinary allocation, otherwise only the arrays are mapped (laa_spread_alloc)."""
    import torch
    W, d, rd, H = 4, 4 * 300, 4 * 1000, 2
    free0 = torch.cuda.mem_get_info()[0]
    backing, x, acc, snap, a, xs, pitch = B.spread_buffers(d, W, rd, hold_gaps=hold_gaps)
    assert x.shape == (W, d) and x.stride(0) == pitch and acc.stride(0) == pitch and pitch >= rd
    assert [t.data_ptr() - x.data_ptr() for t in (acc, snap, a, xs)] == [4 * pitch * k for k in (W, 2 * W, 2 * W + 1, 2 * W + 2)]
    if hold_gaps:
        assert pitch == rd and backing.numel() == (2 * W + 3) * rd
        backing.fill_(7.0)
    else:
        assert pitch * 4 % (2 << 20) == 0 and backing.n_arrays == 2 * W + 3
    rng = np.random.default_rng(31)
    an = rng.uniform(0.1, 10, d).astype(np.float32); xn = rng.standard_normal(d).astype(np.float32)
    a.copy_(torch.from_numpy(an)); xs.copy_(torch.from_numpy(xn))
    g = B.LocalAdaAlter(d, W, H, 0.5, 1.0, x=x, acc=acc, snap=snap, pitch=pitch); g.set_lazy_replicas(True); g.init_state()
    g.set_generator(B.GEN_QUADRATIC, 1, a, xs, None, B.OFF_PHILOX, 0.1, 0.1)
    o = Oracle(d, W, H, 0.5, 1.0); o.init_state()
    o.set_generator(oracle.GEN_QUADRATIC, 1, an, xn, None, oracle.OFF_PHILOX, 0.1, 0.1)
    for _ in range(2 * H + 1):
        o.step_gen(); g.step_gen()
    parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, 1e-5, floor_x=1.0, what="spread buffers")
    if hold_gaps:
        full = backing.view(2 * W + 3, rd)
        assert bool((full[:, d:] == 7.0).all()), "the gaps between the arrays were written"
    else:
        del g, x, acc, snap, a, xs
        backing.close()
        assert backing.base is None
        with pytest.raises(B.LaaError):
            B._check(B.lib().laa_spread_free(B.C.c_void_p(12345 << 21)))       # not one of ours
    with pytest.raises(ValueError):
        B.spread_buffers(d, W, d - 4)


def test_pool_and_measured_placement(B):
    """binding.Pool (laa_pool_create / trim / free) and placement.tune: arrays at offsets of a chunked pool, the step
    timed on candidate placements, the chunks of the winner kept and the rest released; results as with ordinary
    tensors, bit for bit."""
    import torch
    from paper_1911_09030_amd import placement
    W, d, H = 4, 4 * 64 * 33, 3
    chunk = 2 << 20
    free0 = torch.cuda.mem_get_info()[0]
    pool = B.Pool(40 * chunk, chunk_bytes=chunk)
    assert pool.nbytes == 40 * chunk and pool.chunk_bytes == chunk
    assert free0 - torch.cuda.mem_get_info()[0] >= 40 * chunk
    timed = []

    def measure(mats, vecs, pitch):
        m = placement.quadratic_step_timer(d, W, 0.5, 1.0, 5, B.OFF_PHILOX, 0.1, 0.1)(mats, vecs, pitch)
        timed.append(m)
        return m

    best = placement.tune(pool, d, W, 2, 3, measure, n_random=6, seed=1, refine=2)
    assert best.tried == len(timed) - 3 and best.tried > 16 + 6 and best.ms > 0 and best.pitch >= d and best.pitch % 1024 == 0
    spans = sorted(best.ranges(d, W))
    assert all(a + n <= b for (a, n), (b, _) in zip(spans, spans[1:])), "arrays overlap"
    (x, acc), (snap, a, xs) = placement.views(pool, d, W, best)
    pool.trim(best.ranges(d, W))
    kept = {c for o, n in best.ranges(d, W) for c in range(4 * o // chunk, (4 * (o + n) - 1) // chunk + 1)}
    assert free0 - torch.cuda.mem_get_info()[0] < (len(kept) + 2) * chunk + (64 << 20)      # the rest went back
    rng = np.random.default_rng(37)
    an = rng.uniform(0.1, 10, d).astype(np.float32); xn = rng.standard_normal(d).astype(np.float32)
    a.copy_(torch.from_numpy(an)); xs.copy_(torch.from_numpy(xn))
    g = B.LocalAdaAlter(d, W, H, 0.5, 1.0, x=x, acc=acc, snap=snap, pitch=best.pitch); g.set_lazy_replicas(True); g.init_state()
    g.set_generator(B.GEN_QUADRATIC, 5, a, xs, None, B.OFF_PHILOX, 0.1, 0.1)
    r = B.LocalAdaAlter(d, W, H, 0.5, 1.0); r.set_lazy_replicas(True); r.init_state()
    r.set_generator(B.GEN_QUADRATIC, 5, dev(an), dev(xn), None, B.OFF_PHILOX, 0.1, 0.1)
    for _ in range(2 * H + 1):
        g.step_gen(); r.step_gen()
    torch.cuda.synchronize()
    assert torch.equal(g.x, r.x) and torch.equal(g.acc, r.acc) and torch.equal(g.snap, r.snap)
    with pytest.raises(B.LaaError):
        pool.trim([(0, pool.nbytes // 4 + 1)])                       # outside the pool
    with pytest.raises(ValueError):
        pool.tensor(pool.nbytes // 4 - 10, (64,))
    with pytest.raises(B.LaaError):
        B._check(B.lib().laa_pool_free(B.C.c_void_p(12345 << 21)))   # not one of ours
    del g, x, acc, snap, a, xs
    pool.close()
    assert pool.base is None
    with pytest.raises(ValueError):
        placement.tune(B.Pool(chunk, chunk_bytes=chunk), 1 << 20, W, 2, 3, measure)     # too small for the arrays


def test_fused_step_equals_local_step_plus_sync(B):
    import torch
    W, H, d = 8, 3, D_SMALL
    rng = np.random.default_rng(6)
    a = B.LocalAdaAlter(d, W, H, 0.5, 1.0); a.init_state()
    b = B.LocalAdaAlter(d, W, H, 0.5, 1.0); b.init_state()
    # the same with every thread-to-worker mapping: all W workers per thread in batches of 8, 4, 1, and one
    # worker per thread block (0)
    others = []
    for tile in (8, 0, 4, 1):
        c = B.LocalAdaAlter(d, W, H, 0.5, 1.0); c.init_state(); c.set_tile(tile)
        others.append(c)
    for t in range(1, 3 * H + 1):
        G = dev(rng.standard_normal((W, d)).astype(np.float32))
        a.step_dense(G)
        b.local_step_dense(G)
        for c in others:
            c.step_dense(G)
        if t % H == 0:
            b.sync()
        assert a.counters() == b.counters()
        torch.cuda.synchronize()
        for c in others[:2]:       # batch of 8 / one worker per block: the same arithmetic as the default
            assert torch.equal(a.x, c.x) and torch.equal(a.acc, c.acc), f"mapping differs at t={t}"
        for c in others[2:]:
            assert torch.allclose(a.x, c.x, rtol=1e-5, atol=1e-5) and torch.allclose(a.acc, c.acc, rtol=1e-5)
    assert torch.equal(a.x, b.x) and torch.equal(a.acc, b.acc) and torch.equal(a.snap, b.snap)


@pytest.mark.parametrize("W,H,d,gen", [(8, 4, D_SMALL, False), (8, 4, D_SMALL, True), (4, 1, 4 * 500, True),
                                         (3, 3, 1001, False), (2, 5, 4 * 64, True), (16, 2, 4 * 300, False)])
def test_lazy_replicas_bit_identical_to_default(B, W, H, d, gen):
    """With lazy replicas the post-sync state is kept once (row 0 of x, snap) until the next step; every
    result must be bit-identical to the default mode, and match the oracle."""
    import torch
    say(f"lazy replicas W={W} H={H} d={d} gen={gen}")
    rng = np.random.default_rng(23)
    x0 = rng.standard_normal(d).astype(np.float32)
    a = rng.uniform(0.1, 10, d).astype(np.float32); xs = rng.standard_normal(d).astype(np.float32)
    o = Oracle(d, W, H, 0.5, 1.0); o.init_state(x0)
    ref = B.LocalAdaAlter(d, W, H, 0.5, 1.0); ref.init_state(dev(x0))
    lz = B.LocalAdaAlter(d, W, H, 0.5, 1.0); lz.set_lazy_replicas(True); lz.init_state(dev(x0))
    if gen:
        o.set_generator(oracle.GEN_QUADRATIC, 3, a, xs, None, oracle.OFF_PHILOX, 0.1, 0.1)
        for inst in (ref, lz):
            inst.set_generator(B.GEN_QUADRATIC, 3, dev(a), dev(xs), None, B.OFF_PHILOX, 0.1, 0.1)
    sc = parity.Scale(o)
    for t in range(1, 3 * H + 2):
        fused = t % 2 == 0 or H == 1                 # alternate the whole-iteration call with local step (+ sync)
        if gen:
            if t == H + 1:                           # a gradient read straight from the collapsed state
                assert torch.equal(lz.generate_gradient(), ref.generate_gradient())
            o.local_step_gen()
            for inst in (ref, lz):
                inst.step_gen() if fused else inst.local_step_gen()
        else:
            G = rng.standard_normal((W, d)).astype(np.float32)
            o.local_step_dense(G)
            for inst in (ref, lz):
                inst.step_dense(dev(G)) if fused else inst.local_step_dense(dev(G))
        sc.update(o)
        if t % H == 0:
            o.sync()
            if not fused:
                ref.sync(); lz.sync()
            torch.cuda.synchronize()                 # collapsed: only row 0 of x and snap are current
            assert torch.equal(lz.x[0], ref.x[0]) and torch.equal(lz.snap, ref.snap), f"collapsed state t={t}"
        else:
            torch.cuda.synchronize()
            assert torch.equal(lz.x, ref.x) and torch.equal(lz.acc, ref.acc) and torch.equal(lz.snap, ref.snap), t
        assert lz.counters() == ref.counters() == (o.t, o.steps_since_sync)
    lz.materialize()
    torch.cuda.synchronize()
    assert torch.equal(lz.x, ref.x) and torch.equal(lz.acc, ref.acc) and torch.equal(lz.snap, ref.snap)
    bar, fl = (1e-5, 1.0) if gen else (parity.FULL_RUN, parity.FLOOR_X)
    parity.assert_state(host(lz.x), host(lz.acc), host(lz.snap), o, bar, floor_x=fl, what="lazy", scale=sc)


def test_lazy_replicas_materialize_paths(B):
    """Collapsed state followed by a sparse step, by switching the option off, and by an explicit materialize."""
    import torch
    W, H, rows, row_len = 4, 2, 50, 8
    d = rows * row_len
    rng = np.random.default_rng(29)
    o = Oracle(d, W, H, 0.5, 1.0); o.init_state()
    g = B.LocalAdaAlter(d, W, H, 0.5, 1.0); g.set_lazy_replicas(True); g.init_state()
    sc = parity.Scale(o)

    def dense():
        G = rng.standard_normal((W, d)).astype(np.float32)
        o.step_dense(G); g.step_dense(dev(G)); sc.update(o)

    dense(); dense()                                           # second one averages and leaves the state collapsed
    idx = np.stack([rng.permutation(rows)[:10] for _ in range(W)]).astype(np.int32)
    vals = rng.standard_normal((W, 10, row_len)).astype(np.float32)
    o.local_step_sparse(idx, vals, row_len); g.local_step_sparse(dev(idx), dev(vals), row_len); sc.update(o)
    parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, parity.FULL_RUN, what="sparse after collapse", scale=sc)
    o.sync(); g.sync()                                         # sparse sync: rows only, never collapses
    parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, parity.FULL_RUN, what="sparse sync", scale=sc)
    dense(); dense()
    g.set_lazy_replicas(False)                                 # expands the collapsed state
    parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, parity.FULL_RUN, what="option off", scale=sc)
    dense(); dense()
    parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, parity.FULL_RUN, what="default again", scale=sc)
    g.set_lazy_replicas(True)
    dense()
    G = rng.standard_normal((W, d)).astype(np.float32)
    o.local_step_dense(G); g.local_step_dense(dev(G)); sc.update(o)
    o.sync(); g.sync()                                         # stand-alone mean kernel, collapsing
    g.materialize(); g.materialize()                           # second call is a no-op
    parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, parity.FULL_RUN, what="materialize", scale=sc)


@pytest.mark.parametrize("off_mode,W,d", [("philox", 8, D_SMALL), ("array", 4, 4 * 2500), ("none", 3, 4 * 700 + 1),
                                          ("philox", 5, 999)])
def test_diagnostics_match_oracle(B, off_mode, W, d):
    say(f"diagnostics off={off_mode} W={W} d={d}")
    H = 3
    rng = np.random.default_rng(43)
    a = rng.uniform(0.1, 10, d).astype(np.float32); xs = rng.standard_normal(d).astype(np.float32)
    off = (0.1 * rng.standard_normal((W, d))).astype(np.float32)
    x0 = rng.standard_normal(d).astype(np.float32)
    om = {"none": oracle.OFF_NONE, "array": oracle.OFF_ARRAY, "philox": oracle.OFF_PHILOX}[off_mode]
    o = Oracle(d, W, H, 0.5, 1.0); o.init_state(x0)
    o.set_generator(oracle.GEN_QUADRATIC, 17, a, xs, off if off_mode == "array" else None, om, 0.1, 0.1)
    g = B.LocalAdaAlter(d, W, H, 0.5, 1.0); g.set_lazy_replicas(True); g.init_state(dev(x0))
    g.set_generator(B.GEN_QUADRATIC, 17, dev(a), dev(xs), dev(off) if off_mode == "array" else None, om, 0.1, 0.1)
    for t in range(1, 2 * H + 2):
        want, got = o.diagnostics(), g.diagnostics()           # at t = H + 1 the GPU state is collapsed
        for k in range(3):
            assert abs(got[k] - want[k]) <= 2e-5 * max(want[k], 1e-3 * want[0]), (t, k, got, want)
        o.step_gen(); g.step_gen()
    assert g.diagnostics()[2] > 0
    h = B.LocalAdaAlter(d, W, H, 0.5, 1.0); h.init_state()
    with pytest.raises(B.LaaError) as ei:
        h.diagnostics()
    assert ei.value.code == B.EMODE


def test_checkpoint_resume_continues_bit_identically(B):
    """Save x, acc, snap and the counters in the middle of a period, restore them into a fresh handle: the
    continuation (generator included) equals the uninterrupted run bit for bit."""
    import torch
    W, H, d = 4, 5, D_SMALL
    rng = np.random.default_rng(47)
    a = dev(rng.uniform(0.1, 10, d).astype(np.float32)); xs = dev(rng.standard_normal(d).astype(np.float32))
    ref = B.LocalAdaAlter(d, W, H, 0.5, 1.0); ref.set_lazy_replicas(True); ref.init_state()
    ref.set_generator(B.GEN_QUADRATIC, 8, a, xs, None, B.OFF_PHILOX, 0.1, 0.1)
    for _ in range(H + 2):
        ref.step_gen()
    ref.materialize()
    torch.cuda.synchronize()
    saved = (ref.x.clone(), ref.acc.clone(), ref.snap.clone(), ref.counters())
    assert saved[3] == (H + 2, 2)
    res = B.LocalAdaAlter(d, W, H, 0.5, 1.0); res.set_lazy_replicas(True)
    res.x.copy_(saved[0]); res.acc.copy_(saved[1]); res.snap.copy_(saved[2])
    res.set_counters(*saved[3])
    res.set_generator(B.GEN_QUADRATIC, 8, a, xs, None, B.OFF_PHILOX, 0.1, 0.1)
    for _ in range(2 * H):
        ref.step_gen(); res.step_gen()
    ref.materialize(); res.materialize()
    torch.cuda.synchronize()
    assert res.counters() == ref.counters()
    assert torch.equal(res.x, ref.x) and torch.equal(res.acc, ref.acc) and torch.equal(res.snap, ref.snap)


def test_runs_on_the_callers_stream(B):
    """All work is enqueued on the stream handed to laa_attach: a side stream here.  Inputs are produced on that stream
    right before each step (no host synchronisation in between) and results are read after synchronising it alone."""
    import torch
    W, H, d = 4, 3, 4 * 64 * 9
    rng = np.random.default_rng(67)
    Gs = [rng.standard_normal((W, d)).astype(np.float32) for _ in range(2 * H + 1)]
    o = Oracle(d, W, H, 0.5, 1.0); o.init_state()
    sc = parity.Scale(o)
    side = torch.cuda.Stream(device="cuda:0")
    with torch.cuda.stream(side):
        g = B.LocalAdaAlter(d, W, H, 0.5, 1.0)
        assert g.stream.cuda_stream == side.cuda_stream and side.cuda_stream != 0
        g.set_lazy_replicas(True); g.init_state()
        staged = [torch.from_numpy(G).pin_memory() for G in Gs]
        buf = torch.empty((W, d), device="cuda:0")
        for G, Gh in zip(Gs, staged):
            buf.copy_(Gh, non_blocking=True)        # same stream: ordered before the step that reads it
            g.step_dense(buf)
            o.step_dense(G); sc.update(o)
        g.materialize()
    side.synchronize()
    parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, parity.FULL_RUN, what="side stream", scale=sc)


@pytest.mark.parametrize("lazy,H,warmup,side,replays", [(True, 4, 0, True, 7), (False, 3, 0, True, 8),
                                                          (True, 1, 0, True, 7), (True, 2, 5, True, 5),
                                                          (True, 4, 0, False, 0)])
def test_replayed_periods_equal_step_by_step(B, lazy, H, warmup, side, replays):
    """laa_run_periods_gen (one HIP graph per period, replayed) against the same number of laa_step_gen calls: bit for
    bit after every call, with eager work, synchronisations and reads between the replays."""
    import torch
    say(f"graph periods lazy={lazy} H={H} warmup={warmup} side_stream={side}")
    W, d = 4, 4 * 64 * 5
    rng = np.random.default_rng(83)
    stream = torch.cuda.Stream(device="cuda:0") if side else torch.cuda.current_stream()
    with torch.cuda.stream(stream):
        a = dev(rng.uniform(0.1, 10, d).astype(np.float32)); xs = dev(rng.standard_normal(d).astype(np.float32))
        torch.cuda.synchronize()
        pair = []
        for _ in range(2):
            u = B.LocalAdaAlter(d, W, H, 0.5, 1.0); u.set_lazy_replicas(lazy); u.set_warmup(warmup); u.init_state()
            u.set_generator(B.GEN_QUADRATIC, 21, a, xs, None, B.OFF_PHILOX, 0.1, 0.1)
            pair.append(u)
        ref, g = pair
        for n in (1, 2, 1, 3, 2):
            for _ in range(n * H):
                ref.step_gen()
            g.run_periods_gen(n)
            assert g.counters() == ref.counters()
            dg, dr = g.diagnostics(), ref.diagnostics()          # synchronises; reads the (possibly collapsed) state
            assert dg == dr
            g.step_gen(); ref.step_gen()                          # eager work between the replays ...
            for _ in range(H - 1):
                g.step_gen(); ref.step_gen()                      # ... up to the next period boundary
            torch.cuda.synchronize()
            g.materialize(); ref.materialize()
            torch.cuda.synchronize()
            assert torch.equal(g.x, ref.x) and torch.equal(g.acc, ref.acc) and torch.equal(g.snap, ref.snap), n
            assert g.bytes_moved() == ref.bytes_moved()
    # 9 periods asked for (each call starts from full replicas because of the materialize above); the first of each
    # kind (from full replicas, from the collapsed state) outside the warm-up and those inside the
    # warm-up run as plain launches, and so does everything on the default stream
    assert g.replay_count() == replays and ref.replay_count() == 0
    if H > 1:
        g.local_step_gen()
        with pytest.raises(B.LaaError):
            g.run_periods_gen(1)                                  # not at a period boundary


def test_sync_due_early_sync_and_noop_sync(B):
    W, H, d = 2, 2, 64
    g = B.LocalAdaAlter(d, W, H, 0.5, 1.0); g.init_state()
    o = Oracle(d, W, H, 0.5, 1.0); o.init_state()
    G = np.ones((W, d), dtype=np.float32)
    g.sync()                                         # nothing to do
    assert g.counters() == (0, 0)
    g.local_step_dense(dev(G)); g.local_step_dense(dev(G))
    with pytest.raises(B.LaaError) as ei:
        g.local_step_dense(dev(G))
    assert ei.value.code == B.ESYNCDUE
    g.sync()
    g.local_step_dense(dev(G)); g.sync()             # early sync, t' restarts
    g.local_step_dense(dev(G))
    for _ in range(2):
        o.local_step_dense(G)
    o.sync(); o.local_step_dense(G); o.sync(); o.local_step_dense(G)
    parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, parity.ONE_STEP, what="early sync")
    with pytest.raises(B.LaaError) as ei:
        g.local_step_gen()
    assert ei.value.code == B.EMODE


def _gen_scale(a, x, xs, off_scale, noise_scale):
    """Magnitude of the terms that make up g = a (x - (xstar + off)) + noise_scale n."""
    return np.abs(a)[None, :] * (np.abs(x) + np.abs(xs)[None, :] + 4 * off_scale) + 5 * noise_scale


@pytest.mark.parametrize("mode,off_mode,W,d,tile", [("quad", "none", 4, D_SMALL, None), ("quad", "array", 4, D_SMALL, None),
                                                    ("quad", "philox", 8, D_SMALL, None),
                                                    ("quad", "philox", 3, 4 * 300 + 2, None),
                                                    ("noise", "none", 8, D_SMALL, None), ("noise", "none", 2, 999, None),
                                                    ("quad", "philox", 8, D_SMALL, 0), ("quad", "array", 5, 4 * 701, 0),
                                                    ("noise", "none", 3, 4 * 64 * 9, 0), ("quad", "philox", 16, 4 * 333, 4)])
def test_generator_gradient_and_fused_step(B, mode, off_mode, W, d, tile):
    import torch
    say(f"generator mode={mode} off={off_mode} W={W} d={d} tile={tile}")
    H, seed = 4, 1234567890123
    rng = np.random.default_rng(7)
    a = rng.uniform(0.1, 10, d).astype(np.float32)
    xs = rng.standard_normal(d).astype(np.float32)
    off = (0.1 * rng.standard_normal((W, d))).astype(np.float32)
    x0 = rng.standard_normal(d).astype(np.float32)
    gm = {"quad": oracle.GEN_QUADRATIC, "noise": oracle.GEN_NOISE}[mode]
    om = {"none": oracle.OFF_NONE, "array": oracle.OFF_ARRAY, "philox": oracle.OFF_PHILOX}[off_mode]
    o = Oracle(d, W, H, 0.5, 1.0); o.init_state(x0)
    o.set_generator(gm, seed, a, xs, off if off_mode == "array" else None, om, 0.1, 0.1)
    g = B.LocalAdaAlter(d, W, H, 0.5, 1.0); g.init_state(dev(x0))
    u = B.LocalAdaAlter(d, W, H, 0.5, 1.0); u.init_state(dev(x0))       # unfused twin: generate, then explicit step
    da, dxs, doff = dev(a), dev(xs), dev(off)
    if tile is not None:
        g.set_tile(tile)
        if tile:
            u.set_tile(tile)         # same batches, hence the same order of the worker-axis sum
    for inst in (g, u):
        inst.set_generator(gm, seed, da, dxs if mode == "quad" else None, doff if off_mode == "array" else None,
                           om, 0.1, 0.1)
    for t in range(1, 2 * H + 2):
        x_before = o.x
        G_ref = o.gradient(t)
        G_gpu = host(g.generate_gradient())
        scale = _gen_scale(a, x_before, xs, 0.1, 0.1) if mode == "quad" else np.abs(a)[None, :] * 5
        err = np.max(np.abs(G_gpu - G_ref) / scale)
        assert err <= 1e-6, f"gradient at t={t}: {err:.2e}"
        Gu = u.generate_gradient()
        den = np.sqrt(o.snap + (o.steps_since_sync + 1) * 1.0)[None, :]
        g.step_gen(); u.step_dense(Gu); o.step_gen()
        torch.cuda.synchronize()
        assert torch.equal(g.x, u.x) and torch.equal(g.acc, u.acc), f"fused != unfused at t={t}"
        if t == 1:                   # both sides start from the same state: the bound the arithmetic gives, no floor
            r = parity.assert_one_step_generated(host(g.x), host(g.acc), x_before, o, G_ref, scale, 0.5, den, "gen t=1")
            say(f"   one generated step: {r[0]:.2f} (x), {r[1]:.2f} (acc) of the 1e-6 bound")
        bar = 1e-5
        parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, bar, floor_x=1.0, what=f"gen t={t}")


@pytest.mark.parametrize("noise_scale,off_scale", [(0.0, 0.1), (0.1, 0.0), (0.0, 0.0), (2.5, 0.01), (1e-3, 3.0)])
def test_generator_scales(B, noise_scale, off_scale):
    """Standard deviations of the noise and of the per-worker offsets away from the workloads' 0.1, zero included
    (a zero scale must switch its term off exactly: the kernels fold the scale into the Box-Muller radius)."""
    import torch
    W, H, d = 4, 3, 4 * 64 * 5 + 8
    rng = np.random.default_rng(29)
    a = rng.uniform(0.1, 10, d).astype(np.float32); xs = rng.standard_normal(d).astype(np.float32)
    x0 = rng.standard_normal(d).astype(np.float32)
    o = Oracle(d, W, H, 0.05, 1.0); o.init_state(x0)
    o.set_generator(oracle.GEN_QUADRATIC, 11, a, xs, None, oracle.OFF_PHILOX, noise_scale, off_scale)
    g = B.LocalAdaAlter(d, W, H, 0.05, 1.0); g.init_state(dev(x0))
    g.set_generator(B.GEN_QUADRATIC, 11, dev(a), dev(xs), None, B.OFF_PHILOX, noise_scale, off_scale)
    for t in range(1, 2 * H + 1):
        G_ref, G_gpu = o.gradient(t), host(g.generate_gradient())
        S = _gen_scale(a, o.x, xs, off_scale, noise_scale)
        assert np.max(np.abs(G_gpu - G_ref) / np.maximum(S, 1e-30)) <= 1e-6, t
        if noise_scale == 0.0 and off_scale == 0.0:        # nothing random left: every worker sees a (x - xstar)
            assert np.array_equal(G_gpu, (a[None, :] * (host(g.x) - xs[None, :])).astype(np.float32))
        o.step_gen(); g.step_gen()
    parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, 1e-5, floor_x=1.0, what="generator scales")
    with pytest.raises(B.LaaError) as ei:
        g.set_generator(B.GEN_QUADRATIC, 11, dev(a), dev(xs), None, B.OFF_PHILOX, -0.1, 0.1)
    assert ei.value.code == B.EINVAL


@pytest.mark.parametrize("d,split", [(4 * 64 * 11, 4 * 64 * 4), (4 * 300 + 2, 4 * 77)])
def test_shard_by_columns_equals_the_unsplit_run(B, d, split):
    """Two handles that hold columns [0, split) and [split, d) with laa_set_shard reproduce the unsplit run bit for
    bit, syncs and Philox offsets included (nothing crosses the column axis)."""
    import torch
    W, H = 4, 3
    rng = np.random.default_rng(53)
    a = rng.uniform(0.1, 10, d).astype(np.float32); xs = rng.standard_normal(d).astype(np.float32)
    x0 = rng.standard_normal(d).astype(np.float32)
    full = B.LocalAdaAlter(d, W, H, 0.5, 1.0); full.init_state(dev(x0))
    full.set_generator(B.GEN_QUADRATIC, 77, dev(a), dev(xs), None, B.OFF_PHILOX, 0.1, 0.1)
    parts = []
    for lo, hi in ((0, split), (split, d)):
        p = B.LocalAdaAlter(hi - lo, W, H, 0.5, 1.0); p.init_state(dev(x0[lo:hi]))
        p.set_shard(lo, 0)
        p.set_generator(B.GEN_QUADRATIC, 77, dev(a[lo:hi]), dev(xs[lo:hi]), None, B.OFF_PHILOX, 0.1, 0.1)
        parts.append(p)
    for _ in range(2 * H + 1):
        full.step_gen()
        for p in parts:
            p.step_gen()
    torch.cuda.synchronize()
    for name in ("x", "acc", "snap"):
        whole = getattr(full, name)
        glued = torch.cat([getattr(p, name) for p in parts], dim=-1)
        assert torch.equal(whole, glued), name
    df = full.diagnostics()
    dp = [p.diagnostics() for p in parts]
    assert np.allclose(df, np.sum(dp, axis=0), rtol=1e-12, atol=0)      # the three diagnostics are sums over columns


def test_shard_by_workers_local_steps_equal_the_unsplit_run(B):
    """One or two workers per handle (the deployment of Algorithm 3): their local steps draw the global worker's random
    numbers; averaging the shards' rows by hand gives the unsplit run's Synchronize."""
    import torch
    W, H, d = 4, 3, D_SMALL
    rng = np.random.default_rng(59)
    a = dev(rng.uniform(0.1, 10, d).astype(np.float32)); xs = dev(rng.standard_normal(d).astype(np.float32))
    full = B.LocalAdaAlter(d, W, H, 0.5, 1.0); full.init_state()
    full.set_generator(B.GEN_QUADRATIC, 78, a, xs, None, B.OFF_PHILOX, 0.1, 0.1)
    parts = []
    for w0, wn in ((0, 1), (1, 2), (3, 1)):
        p = B.LocalAdaAlter(d, wn, H, 0.5, 1.0); p.init_state()
        p.set_shard(0, w0)
        p.set_generator(B.GEN_QUADRATIC, 78, a, xs, None, B.OFF_PHILOX, 0.1, 0.1)
        parts.append(p)
    for _ in range(H):
        full.local_step_gen()
        for p in parts:
            p.local_step_gen()
    torch.cuda.synchronize()
    px = torch.cat([p.x for p in parts]); pa = torch.cat([p.acc for p in parts])
    assert torch.equal(full.x, px) and torch.equal(full.acc, pa)
    full.sync()
    torch.cuda.synchronize()
    # the all-reduce a deployment would run: same balanced order as the kernel's register tree for W = 4
    mx = ((px[0] + px[1]) + (px[2] + px[3])) * 0.25
    ma = ((pa[0] + pa[1]) + (pa[2] + pa[3])) * 0.25
    assert torch.equal(full.x[0], mx) and torch.equal(full.snap, ma)


def test_generator_counters_beyond_32_bits(B):
    """A shard whose first column is past 2^34: the block index j/4 no longer fits the first counter word and its high
    half goes into the stream word; the oracle follows the same global columns."""
    import torch
    W, H, d = 3, 2, 4 * 64 * 3 + 4
    first = (1 << 34) - 4 * 100            # the shard straddles the point where j/4 reaches 2^32
    rng = np.random.default_rng(61)
    a = rng.uniform(0.1, 10, d).astype(np.float32); xs = rng.standard_normal(d).astype(np.float32)
    o = Oracle(d, W, H, 0.5, 1.0); o.set_columns(first + np.arange(d, dtype=np.int64)); o.init_state()
    o.set_generator(oracle.GEN_QUADRATIC, 5, a, xs, None, oracle.OFF_PHILOX, 0.1, 0.1)
    g = B.LocalAdaAlter(d, W, H, 0.5, 1.0); g.init_state(); g.set_shard(first, 0)
    g.set_generator(B.GEN_QUADRATIC, 5, dev(a), dev(xs), None, B.OFF_PHILOX, 0.1, 0.1)
    low = B.LocalAdaAlter(d, W, H, 0.5, 1.0); low.init_state()          # same shard without the base: must differ
    low.set_generator(B.GEN_QUADRATIC, 5, dev(a), dev(xs), None, B.OFF_PHILOX, 0.1, 0.1)
    for t in range(1, 2 * H + 2):
        G_ref = o.gradient(t)
        G_gpu = host(g.generate_gradient())
        assert np.max(np.abs(G_gpu - G_ref) / _gen_scale(a, o.x, xs, 0.1, 0.1)) <= 1e-6, t
        if t == 1:
            G_low = host(low.generate_gradient())
            assert np.mean(np.abs(G_low - G_ref) > 1e-3) > 0.9
        g.step_gen(); o.step_gen()
    torch.cuda.synchronize()
    parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, 1e-5, floor_x=1.0, what="high columns")


def test_generator_statistics_on_device(B):
    """The device normals themselves: moments over 4M draws (noise mode with a = 1 writes n directly)."""
    import torch
    d, W = 1 << 20, 4
    g = B.LocalAdaAlter(d, W, 4, 0.5, 1.0); g.init_state()
    ones = torch.ones(d, device="cuda:0")
    g.set_generator(B.GEN_NOISE, 99, ones)
    n = host(g.generate_gradient()).astype(np.float64).ravel()
    N = n.size
    assert abs(n.mean()) < 4 / np.sqrt(N) and abs(n.var() - 1) < 4 * np.sqrt(2 / N)
    assert abs(((n - n.mean()) ** 3).mean()) < 4 * np.sqrt(6 / N)
    assert abs((n ** 4).mean() - 3) < 4 * np.sqrt(96 / N)


@pytest.mark.parametrize("W,rows,row_len,k,H", [(3, 1000, 32, 100, 3), (8, 5000, 512, 300, 4), (4, 257, 4, 64, 2),
                                               (2, 100, 260, 100, 2)])
def test_sparse_steps_match_oracle_and_dirty_rows_exact(B, W, rows, row_len, k, H):
    say(f"sparse W={W} rows={rows} row_len={row_len} k={k}")
    d = rows * row_len
    rng = np.random.default_rng(11)
    zipf = wl.ZipfRows(rows, 1.1)
    x0 = rng.standard_normal(d).astype(np.float32)
    o = Oracle(d, W, H, 0.5, 1.0); o.init_state(x0)
    g = B.LocalAdaAlter(d, W, H, 0.5, 1.0); g.init_state(dev(x0))
    sc = parity.Scale(o)
    for t in range(1, 2 * H + 2):
        idx, vals = wl.sparse_step(zipf, W, k, row_len, 3, t)
        o.local_step_sparse(idx, vals, row_len)
        g.local_step_sparse(dev(idx), dev(vals), row_len)
        sc.update(o)
        assert np.array_equal(g.dirty_rows(), o.dirty_rows()), f"dirty rows differ at t={t}"
        if t == 1:
            parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, parity.ONE_STEP, what="sparse one step",
                                scale=sc)
        if t % H == 0:
            o.sync(); g.sync()
            assert g.dirty_rows().size == 0
    parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, parity.FULL_RUN, what="sparse run", scale=sc)
    assert g.counters(with_bad=True)[2] == 0


def test_sparse_edge_cases(B):
    import torch
    W, rows, row_len, H = 2, 64, 8, 2
    d = rows * row_len
    g = B.LocalAdaAlter(d, W, H, 0.5, 1.0); g.init_state()
    o = Oracle(d, W, H, 0.5, 1.0); o.init_state()
    # k = 0: a step that touches nothing still counts as a step
    g.local_step_sparse(None, None, row_len)
    o.local_step_sparse(np.zeros((W, 0), np.int32), np.zeros((W, 0, row_len)), row_len)
    assert g.counters() == (1, 1) and g.dirty_rows().size == 0
    # out-of-range rows are skipped and counted; valid ones applied
    idx = np.array([[3, 64, 7], [-1, 5, 63]], dtype=np.int32)
    vals = np.ones((W, 3, row_len), dtype=np.float32)
    g.local_step_sparse(dev(idx), dev(vals), row_len)
    idx_ok = np.array([[3, 7], [5, 63]], dtype=np.int32)
    o.local_step_sparse(idx_ok, np.ones((W, 2, row_len)), row_len)
    assert g.counters(with_bad=True) == (2, 0 + 2, 2)
    assert np.array_equal(g.dirty_rows(), np.array([3, 5, 7, 63], dtype=np.int32))
    g.sync(); o.sync()
    parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, parity.ONE_STEP, what="sparse edge")
    # the sparse sync must leave untouched rows alone and equal the dense sync on touched rows
    x = host(g.x).reshape(W, rows, row_len)
    assert np.all(x[:, [0, 1, 2, 4, 6, 62]] == 0.0)
    with pytest.raises(B.LaaError):
        g.local_step_sparse(dev(idx), dev(vals), 6)            # row_len not a multiple of 4
    # mixed dense + sparse in one period falls back to the dense mean
    G = np.random.default_rng(1).standard_normal((W, d)).astype(np.float32)
    sc = parity.Scale(o)
    g.local_step_dense(dev(G)); o.local_step_dense(G); sc.update(o)
    g.local_step_sparse(dev(idx_ok), dev(vals[:, :2]), row_len); o.local_step_sparse(idx_ok, vals[:, :2], row_len)
    sc.update(o)
    g.sync(); o.sync()
    parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, parity.FULL_RUN, what="mixed period", scale=sc)


def test_other_arrays_attached_mid_period_are_averaged_whole(B):
    """Arrays handed over in the middle of a period may differ between workers anywhere, not only in the rows the
    handle saw being stepped: the next averaging takes the whole table."""
    import torch
    W, rows, row_len, H = 4, 50, 8, 3
    d = rows * row_len
    g = B.LocalAdaAlter(d, W, H, 0.5, 1.0); g.init_state()
    idx = np.array([[1], [1], [7], [9]], dtype=np.int32)
    g.local_step_sparse(dev(idx), dev(np.ones((W, 1, row_len), dtype=np.float32)), row_len)
    x2, acc2, snap2 = g.x.clone(), g.acc.clone(), g.snap.clone()
    x2[2, 30 * row_len] = 4.0                        # a row that no sparse step listed
    g.attach(x2, acc2, snap2)
    assert g.counters() == (1, 1)
    g.sync()
    torch.cuda.synchronize()
    assert torch.all(g.x[:, 30 * row_len] == 1.0)    # (0 + 0 + 4 + 0) / 4 on every worker
    assert np.array_equal(g.dirty_rows(), np.zeros(0, dtype=np.int32))
    # at a period boundary the handle keeps relying on the listed rows
    g.local_step_sparse(dev(idx), dev(np.ones((W, 1, row_len), dtype=np.float32)), row_len)
    g.sync()
    torch.cuda.synchronize()
    assert all(torch.equal(g.x[0], g.x[w]) and torch.equal(g.acc[w], g.snap) for w in range(W))


@pytest.mark.parametrize("W,tile,row_len", [(8, 8, 16), (8, 4, 16), (8, 2, 16), (4, 1, 16), (2, 2, 16), (8, 8, 520),
                                             (64, 8, 8), (80, 8, 8), (16, 4, 260), (3, 1, 16), (6, 2, 520), (1, 1, 16)])
def test_sparse_sync_equals_dense_sync_bit_for_bit(B, W, tile, row_len):
    """After sparse-only steps the averaging touches the listed rows only, and of a listed row it reads the workers
    that stepped it plus one that did not (the others hold the same values).  On the listed rows this must equal the
    averaging of the whole table bit for bit, with the same batches of workers (laa_set_tile) in both; for W a power
    of two up to 8 the mean of equal values is exact, so the rows not listed agree as well."""
    import torch
    rows, k, H = 300, 40, 3
    d = rows * row_len
    zipf = wl.ZipfRows(rows, 1.1)
    x0 = dev(np.random.default_rng(91).standard_normal(d).astype(np.float32))
    sp = B.LocalAdaAlter(d, W, H, 0.5, 1.0); sp.set_tile(tile); sp.init_state(x0)
    de = B.LocalAdaAlter(d, W, H, 0.5, 1.0); de.set_tile(tile); de.init_state(x0)
    for period in range(2):
        for t in range(1, H + 1):
            idx, vals = wl.sparse_step(zipf, W, k, row_len, 17, period * H + t)
            sp.local_step_sparse(dev(idx), dev(vals), row_len)
            de.local_step_sparse(dev(idx), dev(vals), row_len)
        listed = sp.dirty_rows()
        de.set_counters(*de.counters())          # forgets which rows were touched: the next sync averages everything
        sp.sync(); de.sync()
        torch.cuda.synchronize()
        if W & (W - 1) == 0 and W <= 8:
            assert torch.equal(sp.x, de.x) and torch.equal(sp.acc, de.acc) and torch.equal(sp.snap, de.snap), period
        else:
            cols = torch.from_numpy((listed[:, None].astype(np.int64) * row_len + np.arange(row_len)[None, :]).ravel()).to("cuda:0")
            for got, ref in ((sp.x, de.x), (sp.acc, de.acc), (sp.snap, de.snap)):
                assert torch.equal(got.index_select(got.dim() - 1, cols), ref.index_select(ref.dim() - 1, cols)), period
            # carry on from one common state: the rows not listed differ in the last bit after a whole-table mean
            sp.x.copy_(de.x); sp.acc.copy_(de.acc); sp.snap.copy_(de.snap)
        assert listed.size > 0 and (W == 1 or W > 64 or listed.size < rows)       # 80 workers list every row
    if W > 64:        # no per-row record of the workers: every worker's rows are read, and counted as such
        moved, literal = sp.bytes_moved(literal=True)
        assert moved == literal


def _zipf_with_repeats(rows, W, k, rng, s=1.1):
    """[W][k] rows drawn independently from Zipf(s): popular rows repeat within a worker's list."""
    z = wl.ZipfRows(rows, s)
    return np.minimum(np.searchsorted(z.cdf, rng.random((W, k))), rows - 1).astype(np.int32)


def _abs_gradient(idx, vals, d, row_len):
    """sum of |entries| per (worker, coordinate): the magnitude of the terms that make up the summed gradient."""
    W, k = idx.shape
    gabs = np.zeros((W, d // row_len, row_len))
    for w in range(W):
        np.add.at(gabs[w], idx[w], np.abs(vals[w].astype(np.float64)))
    return gabs.reshape(W, d)


def test_sparse_coalesce_is_bit_identical_on_lists_without_repeats(B):
    import torch
    W, rows, row_len, k, H = 4, 3000, 64, 500, 3
    d = rows * row_len
    zipf = wl.ZipfRows(rows, 1.1)
    p = B.LocalAdaAlter(d, W, H, 0.5, 1.0); p.init_state()
    c = B.LocalAdaAlter(d, W, H, 0.5, 1.0); c.init_state(); c.set_sparse_coalesce(True)
    for t in range(1, 2 * H + 2):
        idx, vals = wl.sparse_step(zipf, W, k, row_len, 5, t)
        di, dv = dev(idx), dev(vals)
        p.step_sparse(di, dv, row_len); c.step_sparse(di, dv, row_len)
        assert np.array_equal(p.dirty_rows(), c.dirty_rows())
    torch.cuda.synchronize()
    assert torch.equal(p.x, c.x) and torch.equal(p.acc, c.acc) and torch.equal(p.snap, c.snap)


@pytest.mark.parametrize("W,rows,row_len,k,H,hot", [(3, 50, 32, 100, 3, False), (8, 5000, 512, 300, 4, False),
                                                   (2, 7, 4, 1, 2, False), (4, 100, 260, 777, 2, False),
                                                   (2, 64, 8, 1500, 2, True), (2, 20000, 4, 8192, 2, False)])
def test_sparse_coalesce_repeated_rows_match_oracle(B, W, rows, row_len, k, H, hot):
    """Rows that a worker lists several times: the oracle applies Algorithm 3 to the summed gradient; so must the GPU.
    Bars: the fp32 sum of L entries in list order is off by at most (L-1) 2^-24 of the sum of their magnitudes."""
    say(f"coalesce W={W} rows={rows} row_len={row_len} k={k} hot={hot}")
    d = rows * row_len
    rng = np.random.default_rng(71)
    x0 = rng.standard_normal(d).astype(np.float32)
    o = Oracle(d, W, H, 0.5, 1.0); o.init_state(x0)
    g = B.LocalAdaAlter(d, W, H, 0.5, 1.0); g.init_state(dev(x0)); g.set_sparse_coalesce(True)
    sx = np.abs(o.x); sb = np.ones((W, d))
    L_max = 1
    for t in range(1, 2 * H + 2):
        idx = _zipf_with_repeats(rows, W, k, rng)
        if hot:
            idx[0, :] = 5                      # one worker names a single row k times
        vals = (0.1 * rng.standard_normal((W, k, row_len))).astype(np.float32)
        L_max = max(L_max, max(np.bincount(idx[w]).max() for w in range(W)))
        gabs = _abs_gradient(idx, vals, d, row_len)
        o.local_step_sparse(idx, vals, row_len)
        g.local_step_sparse(dev(idx), dev(vals), row_len)
        assert np.array_equal(g.dirty_rows(), o.dirty_rows()), f"dirty rows differ at t={t}"
        if t % H == 0:
            o.sync(); g.sync()
        np.maximum(sx, np.abs(o.x), out=sx); np.maximum(sx, 0.5 * gabs, out=sx)        # eta = 0.5, denominators >= 1
        np.maximum(sb, gabs * gabs, out=sb)
        bar = 1e-5 + 2 * (L_max - 1) * 2.0 ** -24
        ex = np.max(np.abs(host(g.x) - o.x) / np.maximum(sx, 1e-3))
        eb = np.max(np.abs(host(g.acc) - o.acc) / np.maximum(np.abs(o.acc), sb))
        es = np.max(np.abs(host(g.snap) - o.snap) / np.maximum(np.abs(o.snap), sb.max(axis=0)))
        assert ex <= bar and eb <= bar and es <= bar, f"t={t} L_max={L_max}: x {ex:.2e} acc {eb:.2e} snap {es:.2e} > {bar:.1e}"
    assert L_max > 1 or k == 1


def test_sparse_coalesce_bad_rows_and_limit(B):
    W, rows, row_len, k, H = 2, 40, 8, 12, 2
    d = rows * row_len
    rng = np.random.default_rng(73)
    idx = _zipf_with_repeats(rows, W, k, rng)
    vals = rng.standard_normal((W, k, row_len)).astype(np.float32)
    bad = idx.copy(); bad[0, 3] = rows; bad[1, 0] = -7; bad[1, 11] = 2 ** 31 - 1
    # the oracle sees the same lists with each bad entry replaced by a repeat of another listed row with zero values
    ok = idx.copy(); ok[0, 3] = idx[0, 0]; ok[1, 0] = idx[1, 1]; ok[1, 11] = idx[1, 1]
    v_ok = vals.copy(); v_ok[0, 3] = 0; v_ok[1, 0] = 0; v_ok[1, 11] = 0
    o = Oracle(d, W, H, 0.5, 1.0); o.init_state()
    g = B.LocalAdaAlter(d, W, H, 0.5, 1.0); g.init_state(); g.set_sparse_coalesce(True)
    g.local_step_sparse(dev(bad), dev(vals), row_len)
    o.local_step_sparse(ok, v_ok, row_len)
    assert g.counters(with_bad=True) == (1, 1, 3)
    assert np.array_equal(g.dirty_rows(), o.dirty_rows())
    g.sync(); o.sync()
    gabs = _abs_gradient(ok, v_ok, d, row_len)
    ex = np.max(np.abs(host(g.x) - o.x) / np.maximum(np.maximum(np.abs(o.x), 0.5 * gabs.max(axis=0)), 1e-3))
    eb = np.max(np.abs(host(g.acc) - o.acc) / np.maximum(np.abs(o.acc), (gabs * gabs).max(axis=0)))
    assert ex <= 1e-5 and eb <= 1e-5, f"coalesce with bad rows: x {ex:.2e} acc {eb:.2e}"
    big = B.LocalAdaAlter(4 * 9000, 1, 2, 0.5, 1.0); big.init_state(); big.set_sparse_coalesce(True)
    import torch
    with pytest.raises(B.LaaError):
        big.local_step_sparse(torch.zeros((1, 8193), dtype=torch.int32, device="cuda:0"),
                              torch.zeros((1, 8193, 4), device="cuda:0"), 4)
    big.set_sparse_coalesce(False)             # the plain step has no such limit
    big.local_step_sparse(torch.arange(8193, dtype=torch.int32, device="cuda:0").reshape(1, -1),
                          torch.zeros((1, 8193, 4), device="cuda:0"), 4)


@pytest.mark.parametrize("seed", range(20))
def test_random_call_sequences_follow_the_oracle(B, seed):
    """Seeded random sequences over the whole boundary (explicit, generated and row-sparse steps, local and fused;
    early, due and empty syncs; lazy replicas and row coalescing switched on and off; materialize; resume; whole
    periods; diagnostics; dirty rows; tile changes)
    against the same calls on the oracle.  The test keeps its own model of when the state is held collapsed (row 0 of
    x and snap), so that it reads only what is defined and never disturbs the library's bookkeeping."""
    import torch
    rng = np.random.default_rng(1000 + seed)
    W, H = int(rng.choice([2, 4, 8])), int(rng.integers(1, 5))
    rows, row_len = 48, 8
    d = rows * row_len
    a = rng.uniform(0.1, 10, d).astype(np.float32); xs = rng.standard_normal(d).astype(np.float32)
    x0 = rng.standard_normal(d).astype(np.float32)
    o = Oracle(d, W, H, 0.3, 0.5); o.init_state(x0)
    o.set_generator(oracle.GEN_QUADRATIC, seed, a, xs, None, oracle.OFF_PHILOX, 0.1, 0.1)
    g = B.LocalAdaAlter(d, W, H, 0.3, 0.5); g.init_state(dev(x0))
    g.set_generator(B.GEN_QUADRATIC, seed, dev(a), dev(xs), None, B.OFF_PHILOX, 0.1, 0.1)
    m = {"lazy": False, "collapsed": False, "sparse_only": True, "sparse_ever": False, "coalesce": False,
         "dirty_known": True}
    log = []

    def averaged_by_sync():           # laa_sync with steps pending (also the tail of a fused sparse step)
        if not (m["sparse_only"] and m["sparse_ever"]):
            m["collapsed"] = m["lazy"]                 # whole-table mean; touched rows only leave it expanded
        m["sparse_only"] = True

    for n in range(60):
        s_before = o.steps_since_sync
        ops = ["sync", "lazy", "materialize", "diag", "dirty", "tile", "coalesce", "resume"]
        if s_before < H:
            ops += ["dense", "dense", "gen", "gen", "sparse", "sparse", "ldense", "lgen", "lsparse"]
        if s_before == 0:
            ops += ["periods"]
        op = str(rng.choice(ops))
        log.append(op)
        if op in ("dense", "ldense", "gen", "lgen"):
            if op.endswith("dense"):
                G = rng.standard_normal((W, d)).astype(np.float32)
                (g.step_dense if op == "dense" else g.local_step_dense)(dev(G))
                (o.step_dense if op == "dense" else o.local_step_dense)(G)
            else:
                (g.step_gen if op == "gen" else g.local_step_gen)()
                (o.step_gen if op == "gen" else o.local_step_gen)()
            m["collapsed"], m["sparse_only"] = False, False
            if o.steps_since_sync == 0:                # the fused step averaged in the same pass
                m["collapsed"], m["sparse_only"] = m["lazy"], True
        elif op in ("sparse", "lsparse"):
            k = int(rng.integers(0, 20))
            idx = np.stack([rng.permutation(rows)[:k] for _ in range(W)]).astype(np.int32).reshape(W, k)
            if m["coalesce"] and k:                    # lists may then name a row several times
                idx = rng.integers(0, max(k // 2, 1), size=(W, k)).astype(np.int32)
            vals = rng.integers(-3, 4, size=(W, k, row_len)).astype(np.float32)      # sums of repeats are exact
            (g.step_sparse if op == "sparse" else g.local_step_sparse)(dev(idx) if k else None,
                                                                       dev(vals) if k else None, row_len)
            (o.step_sparse if op == "sparse" else o.local_step_sparse)(idx, vals, row_len)
            m["collapsed"], m["sparse_ever"] = False, True        # a sparse step expands the state first
            if o.steps_since_sync == 0:
                averaged_by_sync()
        elif op == "sync":
            g.sync(); o.sync()
            if s_before > 0:
                averaged_by_sync()
        elif op == "lazy":
            m["lazy"] = not m["lazy"]
            g.set_lazy_replicas(m["lazy"])
            if not m["lazy"]:
                m["collapsed"] = False                 # switching it off expands the state
        elif op == "materialize":
            g.materialize(); m["collapsed"] = False
        elif op == "coalesce":
            m["coalesce"] = not m["coalesce"]
            g.set_sparse_coalesce(m["coalesce"])
        elif op == "resume":                           # as after restoring a checkpoint into the same arrays
            g.materialize()
            g.set_counters(*g.counters())
            m["collapsed"], m["sparse_only"] = False, False
            m["dirty_known"] = o.steps_since_sync == 0          # the rows touched before a resume are forgotten
        elif op == "periods":
            n_p = int(rng.integers(1, 3))
            g.run_periods_gen(n_p)
            for _ in range(n_p * H):
                o.step_gen()
            m["collapsed"], m["sparse_only"] = m["lazy"], True
        elif op == "diag":
            got, want = g.diagnostics(), o.diagnostics()
            for k in range(3):
                assert abs(got[k] - want[k]) <= 2e-5 * max(want[k], 1e-3 * want[0]), (log, k, got, want)
        elif op == "dirty":
            if m["dirty_known"]:
                assert np.array_equal(g.dirty_rows(), o.dirty_rows()), log
        elif op == "tile":
            g.set_tile(int(rng.choice([t for t in (1, 2, 4, 8) if W % t == 0])))
        assert g.counters() == (o.t, o.steps_since_sync), log
        if o.steps_since_sync == 0:
            m["dirty_known"] = True
        torch.cuda.synchronize()
        gx, ga, gs = host(g.x), host(g.acc), host(g.snap)
        if m["collapsed"]:                             # defined: row 0 of x and snap
            gx, ga = np.broadcast_to(gx[:1], gx.shape), np.broadcast_to(gs[None, :], ga.shape)
        ex = parity.rel_err(gx, o.x, 1.0); eb = parity.rel_err(ga, o.acc, 1e-3); es = parity.rel_err(gs, o.snap, 1e-3)
        assert ex <= 1e-5 and eb <= 1e-5 and es <= 1e-5, f"after {log}: x {ex:.2e} acc {eb:.2e} snap {es:.2e}"


def test_byte_counters(B):
    """laa_bytes_moved: what the launches move (collapsed state counted as such) and the literal traffic of the same
    iterations as separate step and Synchronize passes over full replicas."""
    W, H, d = 8, 4, 4 * 64 * 6
    rng = np.random.default_rng(3)
    a, xs = dev(rng.uniform(0.1, 10, d).astype(np.float32)), dev(rng.standard_normal(d).astype(np.float32))
    inputs = 8                                   # a, xstar once per column
    plain, lit_step, lit_sync = 16 * W + 4 + inputs, 16 * W + 4 + inputs, 16 * W + 4
    g = B.LocalAdaAlter(d, W, H, 0.5, 1.0); g.set_lazy_replicas(True); g.init_state()
    g.set_generator(B.GEN_QUADRATIC, 1, a, xs, None, B.OFF_PHILOX, 0.1, 0.1)
    for _ in range(2 * H):
        g.step_gen()
    averaging = (8 * W + 4) + inputs + 8         # reads every replica, writes row 0 of x and snap
    after = 8 + inputs + 8 * W                   # reads row 0 of x and snap, writes every replica
    moved = ((H - 1) * plain + averaging) + (after + (H - 2) * plain + averaging)
    literal = 2 * H * lit_step + 2 * lit_sync
    assert g.bytes_moved(literal=True) == (moved * d, literal * d)
    g.materialize()                              # reads row 0 of x and snap, writes the other 2W - 1 rows
    assert g.bytes_moved(literal=True) == ((moved + 8 + 8 * W - 4) * d, literal * d)
    # the same period without lazy replicas: fusing alone saves the second read of x and acc
    f = B.LocalAdaAlter(d, W, H, 0.5, 1.0); f.init_state()
    f.set_generator(B.GEN_QUADRATIC, 1, a, xs, None, B.OFF_PHILOX, 0.1, 0.1)
    for _ in range(H):
        f.step_gen()
    assert f.bytes_moved(literal=True) == (((H - 1) * plain + 16 * W + 8 + inputs) * d, (H * lit_step + lit_sync) * d)
    f.init_state()                               # counters restart
    for _ in range(H):
        f.local_step_gen()
    f.sync()                                     # unfused: both counters are the literal traffic
    assert f.bytes_moved(literal=True) == ((H * lit_step + lit_sync) * d,) * 2
    # H = 1 with lazy replicas: the state stays collapsed, 8 bytes in and 8 bytes out per column
    h1 = B.LocalAdaAlter(d, W, 1, 0.5, 1.0); h1.set_lazy_replicas(True); h1.init_state()
    h1.set_generator(B.GEN_QUADRATIC, 1, a, xs, None, B.OFF_PHILOX, 0.1, 0.1)
    for _ in range(3):
        h1.step_gen()
    assert h1.bytes_moved(literal=True) == ((averaging + 2 * (8 + inputs + 8)) * d, 3 * (lit_step + lit_sync) * d)
    # sparse period: the rows that the averaging touched are counted on the device
    rows, row_len, k = 100, 8, 10
    sp = B.LocalAdaAlter(rows * row_len, 4, 2, 0.5, 1.0); sp.init_state()
    zipf = wl.ZipfRows(rows, 1.1)
    workers_of = {}                              # row -> the workers that stepped it in this period
    for t in (1, 2):
        idx, vals = wl.sparse_step(zipf, 4, k, row_len, 9, t)
        sp.local_step_sparse(dev(idx), dev(vals), row_len)
        for w in range(4):
            for r in idx[w]:
                workers_of.setdefault(int(r), set()).add(w)
    n_dirty = sp.dirty_rows().size
    assert n_dirty == len(workers_of) and 0 < n_dirty <= 2 * 4 * k
    step_b = 2 * 4 * k * (24 * row_len + 4)
    assert sp.bytes_moved(literal=True) == (step_b, step_b)
    sp.sync()
    # per listed row the averaging reads x and acc of the workers that stepped it and of one that did not (the others
    # hold the same values), and writes every worker's rows and snap; literally it reads every worker's rows
    reads = sum(len(ws) + (1 if len(ws) < 4 else 0) for ws in workers_of.values())
    assert any(len(ws) < 4 for ws in workers_of.values())
    assert sp.bytes_moved(literal=True) == (step_b + (2 * reads + n_dirty * (2 * 4 + 1)) * 4 * row_len,
                                            step_b + n_dirty * (16 * 4 + 4) * row_len)
    sp.init_state()
    assert sp.bytes_moved(literal=True) == (0, 0)


def test_warmup_learning_rate(B):
    W, H, d, T = 4, 4, 4 * 300, 12
    rng = np.random.default_rng(12)
    o = Oracle(d, W, H, 0.5, 1.0); o.init_state(); o.set_warmup(5)
    g = B.LocalAdaAlter(d, W, H, 0.5, 1.0); g.init_state(); g.set_warmup(5)
    sc = parity.Scale(o)
    for t in range(1, T + 1):
        G = rng.standard_normal((W, d)).astype(np.float32)
        o.local_step_dense(G); sc.update(o)
        if t % H == 0:
            o.sync()
        g.step_dense(dev(G))
    parity.assert_state(host(g.x), host(g.acc), host(g.snap), o, parity.FULL_RUN, what="warm-up", scale=sc)


@pytest.mark.parametrize("W,d", [(4, D_SMALL), (3, 4 * 100 + 1), (8, 4 * 1000)])
def test_adagrad_and_local_sgd_variants(B, W, d):
    H, T = 3, 9
    rng = np.random.default_rng(13)
    Gs = [rng.standard_normal((W, d)).astype(np.float32) for _ in range(T)]
    import torch
    o = Oracle(d, W, 1, 0.3, 0.1, 0.0); o.init_state()
    g = B.LocalAdaAlter(d, W, 1, 0.3, 0.1, b0=0.0); g.set_algorithm(B.ALGO_DIST_ADAGRAD); g.init_state()
    z = B.LocalAdaAlter(d, W, 1, 0.3, 0.1, b0=0.0); z.set_algorithm(B.ALGO_DIST_ADAGRAD); z.set_lazy_replicas(True)
    z.init_state()                      # the single iterate of Algorithm 1 kept in row 0 of x and in snap
    sc = parity.Scale(o)
    for G in Gs:
        o.adagrad_step_dense(G); g.step_dense(dev(G)); z.step_dense(dev(G)); sc.update(o)
    assert parity.rel_err(host(g.x), o.x, 1e-3, sc.s) <= parity.FULL_RUN
    assert parity.rel_err(host(g.snap), o.snap, 1e-3) <= parity.FULL_RUN
    z.materialize()
    torch.cuda.synchronize()
    assert torch.equal(z.x, g.x) and torch.equal(z.acc, g.acc) and torch.equal(z.snap, g.snap)
    o = Oracle(d, W, H, 0.3, 0.1); o.init_state()
    g = B.LocalAdaAlter(d, W, H, 0.3, 0.1); g.set_algorithm(B.ALGO_LOCAL_SGD); g.init_state()
    sc = parity.Scale(o)
    for t, G in enumerate(Gs):
        o.localsgd_step_dense(G); g.step_dense(dev(G)); sc.update(o)
        assert parity.rel_err(host(g.x), o.x, 1e-3, sc.s) <= parity.FULL_RUN, f"local sgd t={t + 1}"
    with pytest.raises(B.LaaError):
        g.local_step_dense(dev(Gs[0]))


@pytest.mark.parametrize("algo,mode,off_mode,W,d,lazy", [
    ("adagrad", "quad", "philox", 8, D_SMALL, False), ("adagrad", "quad", "philox", 8, D_SMALL, True),
    ("adagrad", "quad", "array", 3, 4 * 300 + 3, False), ("adagrad", "quad", "none", 3, 4 * 300 + 3, True),
    ("adagrad", "noise", "none", 8, 4 * 64 * 5, True), ("adagrad", "noise", "none", 3, 1001, False),
    ("adagrad", "quad", "philox", 16, 4 * 333, True),
    ("sgd", "quad", "philox", 8, D_SMALL, False), ("sgd", "quad", "array", 3, 4 * 300 + 3, False),
    ("sgd", "noise", "none", 3, 1001, False), ("sgd", "noise", "none", 8, 4 * 64 * 5, True),
    ("sgd", "quad", "philox", 16, 4 * 333, True)])
def test_generator_fed_adagrad_and_local_sgd(B, algo, mode, off_mode, W, d, lazy):
    """Algorithms 1 and 2 with the gradient generated in the kernel, against the oracle's gradient followed by its
    Algorithm 1 / Algorithm 2 step: each worker's gradient is evaluated at its own iterate with its own random
    numbers (Algorithm 1: at the one shared iterate, also when that is kept in row 0 only)."""
    import torch
    say(f"generator-fed {algo} mode={mode} off={off_mode} W={W} d={d} lazy={lazy}")
    H, T, seed = (1, 7, 424242) if algo == "adagrad" else (3, 10, 434343)
    eta, eps, b0 = (0.3, 1.0, 0.0) if algo == "adagrad" else (0.05, 1.0, 1.0)       # eta a < 2 for plain SGD
    rng = np.random.default_rng(19)
    a = rng.uniform(0.1, 10, d).astype(np.float32)
    xs = rng.standard_normal(d).astype(np.float32)
    off = (0.1 * rng.standard_normal((W, d))).astype(np.float32)
    x0 = rng.standard_normal(d).astype(np.float32)
    gm = {"quad": oracle.GEN_QUADRATIC, "noise": oracle.GEN_NOISE}[mode]
    om = {"none": oracle.OFF_NONE, "array": oracle.OFF_ARRAY, "philox": oracle.OFF_PHILOX}[off_mode]
    o = Oracle(d, W, H, eta, eps, b0); o.init_state(x0)
    o.set_generator(gm, seed, a, xs, off if off_mode == "array" else None, om, 0.1, 0.1)
    g = B.LocalAdaAlter(d, W, H, eta, eps, b0=b0)
    g.set_algorithm(B.ALGO_DIST_ADAGRAD if algo == "adagrad" else B.ALGO_LOCAL_SGD)
    g.set_lazy_replicas(lazy)
    g.init_state(dev(x0))
    g.set_generator(gm, seed, dev(a), dev(xs) if mode == "quad" else None, dev(off) if off_mode == "array" else None,
                    om, 0.1, 0.1)
    single = algo == "adagrad" and lazy          # Algorithm 1's one iterate lives in row 0 of x and in snap
    sc = parity.Scale(o)
    S2 = np.zeros(d)                             # largest squared magnitude of the gradient's terms so far, per column
    for t in range(1, T + 1):
        x_before = o.x
        G_ref = o.gradient(t)
        G_gpu = host(g.generate_gradient())
        scale = _gen_scale(a, x_before, xs, 0.1, 0.1) if mode == "quad" else np.abs(a)[None, :] * 5
        err = np.max(np.abs(G_gpu - G_ref) / scale)
        assert err <= 1e-6, f"gradient at t={t}: {err:.2e}"
        np.maximum(S2, np.max(scale * np.ones((W, 1)), axis=0) ** 2, out=S2)
        (o.adagrad_step_dense if algo == "adagrad" else o.localsgd_step_dense)(G_ref)
        g.step_gen(); sc.update(o)
        assert g.counters()[0] == o.t
        gx = host(g.x)
        if single:
            gx = np.broadcast_to(gx[:1], gx.shape)
        ex = parity.rel_err(gx, o.x, 1.0, sc.s)
        assert ex <= 1e-5, f"{algo} t={t}: x {ex:.2e}"
        if algo == "adagrad":
            # B2 starts at 0 here (Algorithm 1), so its error is relative to the squared magnitude of the gradient's
            # terms: d(g^2) = 2 g dg with dg bounded by 1e-6 of that magnitude, whatever cancels inside g
            es = parity.rel_err(host(g.snap), o.snap, 1e-3, S2)
            assert es <= 1e-5, f"adagrad t={t}: B2 {es:.2e}"
    if single:
        g.materialize()
        torch.cuda.synchronize()
        assert all(torch.equal(g.x[0], g.x[w]) and torch.equal(g.acc[w], g.snap) for w in range(W))
    if algo == "adagrad":
        assert parity.rel_err(host(g.acc), o.acc, 1e-3, S2[None, :]) <= 1e-5


# ------------------------------------------------------------------------------------------ benchmark configurations
def _quadratic_setup(B, c, n_groups, off_mode="philox", bench_layout=False):
    """GPU instance at the full size of workload c and an oracle that follows a sample of its columns.
    bench_layout: the launch configuration bench.py times (spread row pitch, lazy replicas)."""
    cols = wl.column_sample(c.d, n_groups, seed=1)
    a = wl.curvature(c.d, c.seed, c.a_dist)
    xs = wl.optimum(c.d, c.seed)
    om = {"philox": oracle.OFF_PHILOX, "none": oracle.OFF_NONE}[off_mode]
    o = Oracle(len(cols), c.W, c.H, c.eta, c.eps)
    o.set_columns(cols); o.init_state()
    o.set_generator(oracle.GEN_QUADRATIC, c.seed, a[cols], xs[cols], None, om, c.noise_scale, c.off_scale)
    o.sample_a, o.sample_xs = a[cols], xs[cols]
    if bench_layout:
        # as bench.py sets the workload up: arrays at a measured placement inside a pool of most of the free memory
        # (fewer candidates here), the rest of the pool released, lazy replicas on
        import torch
        from paper_1911_09030_amd import placement
        pool = B.Pool(int(torch.cuda.mem_get_info()[0] * 0.9))
        measure = placement.quadratic_step_timer(c.d, c.W, c.eta, c.eps, c.seed, om, c.noise_scale, c.off_scale)
        best = placement.tune(pool, c.d, c.W, 2, 3, measure, n_random=8, seed=c.seed, refine=1)
        (bx, bacc), (bsnap, da, dxs) = placement.views(pool, c.d, c.W, best)
        pool.trim(best.ranges(c.d, c.W))
        say(f"   placement: {best.tried} timed, best {best.ms:.3f} ms, slowest {best.slowest_ms:.3f} ms")
        g = B.LocalAdaAlter(c.d, c.W, c.H, c.eta, c.eps, x=bx, acc=bacc, snap=bsnap, pitch=best.pitch)
        g._keep_backing = pool
        g.set_lazy_replicas(True)
        da.copy_(torch.from_numpy(a)); dxs.copy_(torch.from_numpy(xs))
    else:
        g = B.LocalAdaAlter(c.d, c.W, c.H, c.eta, c.eps)
        da, dxs = dev(a), dev(xs)
    g.init_state()
    g.set_generator(B.GEN_QUADRATIC, c.seed, da, dxs, None, om, c.noise_scale, c.off_scale)
    return cols, o, g


def _sampled(t, cols):
    import torch
    idx = torch.from_numpy(cols).to("cuda:0")
    return host(t.index_select(t.dim() - 1, idx))


def _first_step_with_bound(c, cols, o, g, what):
    """Iteration 1 of a quadratic workload on both sides (same initial state), checked against the one-step bound
    the arithmetic gives (parity.assert_one_step_generated) on the sampled columns."""
    x_before, G_ref = o.x, o.gradient(1)
    S = _gen_scale(o.sample_a, x_before, o.sample_xs, c.off_scale, c.noise_scale)
    den = np.sqrt(o.snap + c.eps * c.eps)[None, :]
    o.step_gen(); g.step_gen()
    r = parity.assert_one_step_generated(_sampled(g.x, cols), _sampled(g.acc, cols), x_before, o, G_ref, S, c.eta, den, what)
    say(f"   {what}: one generated step is {r[0]:.2f} (x), {r[1]:.2f} (acc) of the 1e-6 bound")


def test_config1_full_run_on_sampled_columns(B):
    """d=2^20, W=4, H=4, T=64 (the small configuration), full length, oracle on 4096 sampled columns."""
    c = wl.WORKLOADS["c1"]
    cols, o, g = _quadratic_setup(B, c, 1024)
    _first_step_with_bound(c, cols, o, g, "c1 t=1")
    for t in range(2, c.T + 1):
        o.step_gen(); g.step_gen()
        if t in (c.H, c.T):
            e = parity.assert_state(_sampled(g.x, cols), _sampled(g.acc, cols), _sampled(g.snap, cols), o, 1e-5,
                                    floor_x=1.0, what=f"c1 t={t}")
            say(f"   c1 t={t} rel err", e)
    # after the last sync all workers agree exactly, everywhere
    import torch
    assert all(torch.equal(g.x[0], g.x[w]) and torch.equal(g.acc[0], g.acc[w]) for w in range(1, c.W))
    assert torch.equal(g.acc[0], g.snap)


def test_config2_full_length_on_sampled_columns(B):
    """d=25M, W=8, H=8, curvature log-uniform on [1e-3, 1e2], all T = 256 iterations; the oracle follows 4096 columns."""
    c = wl.WORKLOADS["c2"]
    cols, o, g = _quadratic_setup(B, c, 1024)
    _first_step_with_bound(c, cols, o, g, "c2 t=1")
    for t in range(2, c.T + 1):
        o.step_gen(); g.step_gen()
        if t in (2 * c.H + 1, c.T):
            e = parity.assert_state(_sampled(g.x, cols), _sampled(g.acc, cols), _sampled(g.snap, cols), o, 1e-5,
                                    floor_x=1.0, what=f"c2 t={t}")
            say(f"   c2 t={t} rel err", e)


def test_config5_headline_size_two_periods_on_sampled_columns(B):
    """d=400M, W=8, H=16 in the launch configuration the benchmark times (fused step, Philox offsets)."""
    import torch
    c = wl.WORKLOADS["c5"]
    cols, o, g = _quadratic_setup(B, c, 512, bench_layout=True)
    _first_step_with_bound(c, cols, o, g, "c5 t=1")
    for t in range(2, 2 * c.H + 1):
        o.step_gen(); g.step_gen()
    g.materialize()                                   # the last iteration averaged: expand the collapsed state
    e = parity.assert_state(_sampled(g.x, cols), _sampled(g.acc, cols), _sampled(g.snap, cols), o, 1e-5,
                            floor_x=1.0, what="c5")
    say("   c5 rel err", e)
    # properties that hold at any size: consensus after the sync, snap == acc, accumulator >= b0^2
    assert torch.equal(g.x[0], g.x[c.W - 1]) and torch.equal(g.acc[3], g.snap)
    assert float(g.snap.min()) >= 1.0
    del g
    torch.cuda.empty_cache()


def test_config5_full_length_on_sampled_columns(B):
    """The headline configuration for all of its T = 1024 iterations (64 periods) in the benchmark's launch
    configuration; the oracle follows 2048 sampled columns.  Checked after the first period, a quarter of the run and
    at the end."""
    import torch
    c = wl.WORKLOADS["c5"]
    cols, o, g = _quadratic_setup(B, c, 512, bench_layout=True)
    for t in range(1, c.T + 1):
        o.step_gen(); g.step_gen()
        if t in (c.H, c.T // 4, c.T):
            torch.cuda.synchronize()
            gx = _sampled(g.x[:1], cols); gs = _sampled(g.snap, cols)        # just averaged: row 0 and snap hold it all
            ex = parity.rel_err(gx, o.x[:1], 1.0); es = parity.rel_err(gs, o.snap, 1e-3)
            say(f"   c5 t={t}: rel err x {ex:.2e} snap {es:.2e}")
            assert ex <= 1e-5 and es <= 1e-5, f"c5 at t={t}: x {ex:.2e} snap {es:.2e}"
    g.materialize()
    parity.assert_state(_sampled(g.x, cols), _sampled(g.acc, cols), _sampled(g.snap, cols), o, 1e-5, floor_x=1.0,
                        what="c5 full length")
    assert g.counters() == (c.T, 0)
    del g
    torch.cuda.empty_cache()


def test_config5_size_adagrad_and_local_sgd_on_sampled_columns(B):
    """Algorithms 1 and 2 on the headline workload's inputs at its full size (d = 4e8, W = 8): the kernels that
    `bench.py --algorithm` times, with 64-bit column offsets in reach.  The oracle follows 2048 sampled columns (the
    last column group among them): its gradient at every iteration, then its Algorithm 1 / Algorithm 2 step."""
    import torch
    c = wl.WORKLOADS["c5"]
    cols = wl.column_sample(c.d, 512, seed=2)
    a, xs = wl.curvature(c.d, c.seed, c.a_dist), wl.optimum(c.d, c.seed)
    da, dxs = dev(a), dev(xs)
    sa, sxs = a[cols], xs[cols]
    del a, xs
    x = torch.empty((c.W, c.d), dtype=torch.float32, device="cuda:0")
    acc = torch.empty_like(x)
    snap = torch.empty(c.d, dtype=torch.float32, device="cuda:0")
    for algo, lazy in (("adagrad", False), ("adagrad", True), ("sgd", False)):
        say(f"   {algo} lazy={lazy} at d={c.d}")
        H, T, b0 = (1, 5, 0.0) if algo == "adagrad" else (c.H, c.H + 2, 1.0)
        o = Oracle(len(cols), c.W, H, c.eta, c.eps, b0)
        o.set_columns(cols); o.init_state()
        o.set_generator(oracle.GEN_QUADRATIC, c.seed, sa, sxs, None, oracle.OFF_PHILOX, c.noise_scale, c.off_scale)
        g = B.LocalAdaAlter(c.d, c.W, H, c.eta, c.eps, b0=b0, x=x, acc=acc, snap=snap)
        g.set_algorithm(B.ALGO_DIST_ADAGRAD if algo == "adagrad" else B.ALGO_LOCAL_SGD)
        g.set_lazy_replicas(lazy)
        g.init_state()
        g.set_generator(B.GEN_QUADRATIC, c.seed, da, dxs, None, B.OFF_PHILOX, c.noise_scale, c.off_scale)
        sc = parity.Scale(o)
        S2 = np.zeros(len(cols))
        for t in range(1, T + 1):
            S = _gen_scale(sa, o.x, sxs, c.off_scale, c.noise_scale)
            np.maximum(S2, np.max(S * np.ones((c.W, 1)), axis=0) ** 2, out=S2)
            G_ref = o.gradient(t)
            (o.adagrad_step_dense if algo == "adagrad" else o.localsgd_step_dense)(G_ref)
            g.step_gen(); sc.update(o)
        if algo == "adagrad" and lazy:
            g.materialize()
        ex = parity.rel_err(_sampled(g.x, cols), o.x, 1.0, sc.s)
        say(f"   {algo} lazy={lazy}: rel err x {ex:.2e}")
        assert ex <= 1e-5, f"{algo} lazy={lazy}: x {ex:.2e}"
        if algo == "adagrad":
            es = parity.rel_err(_sampled(g.snap, cols), o.snap, 1e-3, S2)
            assert es <= 1e-5, f"adagrad lazy={lazy}: B2 {es:.2e}"
            assert torch.equal(g.x[0], g.x[c.W - 1]) and torch.equal(g.acc[c.W - 1], g.snap)
        else:       # T = H + 2: two local steps after the averaging, the workers have moved apart again
            assert not torch.equal(g.x[0], g.x[c.W - 1])
        assert g.counters()[0] == T
        g.close()
    del x, acc, snap, da, dxs
    torch.cuda.empty_cache()


@pytest.mark.parametrize("H,T", [(1, 64), (4, 128), (16, 512), (64, 128)])
def test_config3_explicit_gradient_pool(B, H, T):
    """d=100M, W=8: dense gradients N(0, sigma_j^2) precomputed into HBM, streamed by the explicit-gradient step; the
    configuration's four synchronisation periods, its full length T = 512 at the default H = 16."""
    import torch
    c = wl.WORKLOADS["c3"]
    say(f"c3 H={H} T={T}")
    sig = wl.sigma(c.d, c.seed)
    cols = wl.column_sample(c.d, 512, seed=2)
    g = B.LocalAdaAlter(c.d, c.W, H, c.eta, c.eps); g.init_state()
    g.set_generator(B.GEN_NOISE, c.seed, dev(sig))
    o = Oracle(len(cols), c.W, H, c.eta, c.eps); o.set_columns(cols); o.init_state()
    o.set_generator(oracle.GEN_NOISE, c.seed, sig[cols])
    pool = g.rows()
    sc = parity.Scale(o)
    for t in range(1, T + 1):
        g.generate_gradient(pool)                       # materialise this iteration's gradient, then stream it
        G_ref = o.gradient(t)
        G_gpu = _sampled(pool, cols)
        assert np.max(np.abs(G_gpu - G_ref) / (np.abs(sig[cols])[None, :] * 5)) <= 1e-6
        g.step_dense(pool)                              # identical gradient bits from here on
        o.local_step_dense(G_gpu); sc.update(o)
        if t % H == 0:
            o.sync()
        if t == 1:
            parity.assert_state(_sampled(g.x, cols), _sampled(g.acc, cols), _sampled(g.snap, cols), o,
                                parity.ONE_STEP, what="c3 one step", scale=sc)
    e = parity.assert_state(_sampled(g.x, cols), _sampled(g.acc, cols), _sampled(g.snap, cols), o, parity.FULL_RUN,
                            what="c3", scale=sc)
    say("   c3 rel err", e)
    del g, pool
    torch.cuda.empty_cache()


def test_config4_embedding_table_and_dense_blocks_full_length(B):
    """800,000 x 512 table, W=8, k=8192 Zipf(1.1) rows per worker and step, plus the 4 dense 2048 x 8192 blocks with
    the noise generator, for all T = 256 iterations of the configuration (16 periods of H = 16), as the benchmark
    runs it: row-sparse step + averaging of the touched rows on the table's handle, fused generator step with lazy
    replicas on the dense blocks' handle.  The oracle follows a sample of table rows (the 8 most frequent, 24 drawn
    from the first period's rows, 16 from the tail of the vocabulary) and a sample of the blocks' columns.  Row sets
    are drawn afresh for every iteration; the row values are drawn for the 16 iterations of the first period and
    used again in the later ones (drawing 33 M normals per iteration on the host would take minutes)."""
    import torch
    c = wl.WORKLOADS["c4"]
    H, T = c.H, c.T
    zipf = wl.ZipfRows(c.rows, c.zipf_s)
    g = B.LocalAdaAlter(c.d, c.W, H, c.eta, c.eps); g.init_state()
    first_period = [wl.sparse_step(zipf, c.W, c.k, c.row_len, c.seed, t, c.val_sigma) for t in range(1, H + 1)]
    vals_dev = [dev(v) for _, v in first_period]
    rng = np.random.default_rng(4)
    seen = np.unique(np.concatenate([i.ravel() for i, _ in first_period]))
    tail = np.arange(c.rows - 1, c.rows - 1 - 16 * 997, -997)                    # 16 rows from the rare end
    sample = np.unique(np.concatenate([np.arange(8), rng.choice(seen, 24, replace=False), tail]))
    remap = -np.ones(c.rows, dtype=np.int64); remap[sample] = np.arange(sample.size)
    o = Oracle(sample.size * c.row_len, c.W, H, c.eta, c.eps); o.init_state()
    # the dense blocks: one handle over their concatenation, as in the benchmark
    dd = sum(r * q for r, q in c.dense_blocks)
    sig = wl.sigma(dd, c.seed)
    dcols = wl.column_sample(dd, 256, seed=3)
    gd = B.LocalAdaAlter(dd, c.W, H, c.eta, c.eps); gd.set_lazy_replicas(True); gd.init_state()
    gd.set_generator(B.GEN_NOISE, c.seed, dev(sig))
    od = Oracle(len(dcols), c.W, H, c.eta, c.eps); od.set_columns(dcols); od.init_state()
    od.set_generator(oracle.GEN_NOISE, c.seed, sig[dcols])
    union, ever = set(), set()
    sc = parity.Scale(o)
    cols = (sample[:, None] * c.row_len + np.arange(c.row_len)[None, :]).reshape(-1)
    for t in range(1, T + 1):
        if t <= H:
            idx, vals = first_period[t - 1]
        else:
            idx = wl.sparse_step(zipf, c.W, c.k, c.row_len, c.seed, t, with_vals=False)[0]
            vals = first_period[(t - 1) % H][1]
        g.local_step_sparse(dev(idx), vals_dev[(t - 1) % H], c.row_len)
        # the oracle takes the dense step on the scattered gradient of the sampled rows: that is the definition
        G = np.zeros((c.W, sample.size, c.row_len))
        for w in range(c.W):
            m = remap[idx[w]]
            G[w, m[m >= 0]] = vals[w][m >= 0]
        o.local_step_dense(G.reshape(c.W, -1)); sc.update(o)
        rows_t = set(idx.ravel().tolist())
        union |= rows_t; ever |= rows_t
        gd.step_gen(); od.step_gen()
        if t == 1:
            assert np.array_equal(g.dirty_rows(), np.array(sorted(union), dtype=np.int32))
        if t % H == 0:
            if t in (H, T):
                assert np.array_equal(g.dirty_rows(), np.array(sorted(union), dtype=np.int32)), f"dirty rows at t={t}"
            g.sync(); o.sync(); union = set()
        if t in (1, H, T // 2, T):
            torch.cuda.synchronize()
            e = parity.assert_state(_sampled(g.x, cols), _sampled(g.acc, cols), _sampled(g.snap, cols), o,
                                    parity.FULL_RUN, what=f"c4 table t={t}", scale=sc)
            if t % H == 0:                # the blocks were just averaged: row 0 of x and snap hold the state
                ex = parity.rel_err(_sampled(gd.x[:1], dcols), od.x[:1], 1.0)
                es = parity.rel_err(_sampled(gd.snap, dcols), od.snap, 1e-3)
            else:
                ex = parity.rel_err(_sampled(gd.x, dcols), od.x, 1.0)
                es = parity.rel_err(_sampled(gd.acc, dcols), od.acc, 1e-3)
            say(f"   c4 t={t}: table rel err {e}, dense blocks x {ex:.2e} B2 {es:.2e}")
            assert ex <= 1e-5 and es <= 1e-5, f"c4 dense blocks at t={t}: x {ex:.2e} B2 {es:.2e}"
    assert g.counters(with_bad=True) == (T, 0, 0) and gd.counters() == (T, 0)
    gd.materialize()
    parity.assert_state(_sampled(gd.x, dcols), _sampled(gd.acc, dcols), _sampled(gd.snap, dcols), od, 1e-5,
                        floor_x=1.0, what="c4 dense blocks")
    # sampled rows nobody touched keep their initial state on every worker, bit for bit
    never = np.array([r for r in sample if r not in ever], dtype=np.int64)
    assert never.size > 0
    nv = (never[:, None] * c.row_len + np.arange(c.row_len)[None, :]).reshape(-1)
    assert np.all(_sampled(g.x, nv) == 0.0) and np.all(_sampled(g.acc, nv) == 1.0) and np.all(_sampled(g.snap, nv) == 1.0)
    del g, gd
    torch.cuda.empty_cache()
