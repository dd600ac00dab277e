"""Pins for the CPU oracle: each function checks the oracle (given as a loaded
oracle library) against something the paper or the mathematics fixes, and raises
AssertionError when it does not hold.  test_oracle_pins.py runs them on the real
oracle (must pass) and on builds with a planted mistake (at least one must fail).

Citations are to arXiv 1911.09030.
"""
from __future__ import annotations

import os
from decimal import Decimal, getcontext

import numpy as np

import oracle
from oracle import Oracle

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _tol(lib):
    # fp64 oracle: essentially exact; fp32 build: a few ulp per step
    return 1e-12 if lib.real_bytes == 8 else 2e-6


def _close(got, want, tol, what):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    err = np.max(np.abs(got - want) / np.maximum(np.abs(want), 1.0))
    assert err <= tol, f"{what}: max err {err:.3e} > {tol:.1e}"


def _rand_grads(T, W, d, seed, scale=1.0):
    return scale * np.random.default_rng(seed).standard_normal((T, W, d))


# --------------------------------------------------------------------------- Algorithm 3
def pin_literal_history(lib):
    """Algorithm 3 evaluated literally: every x_{i,t} and B^2_{i,t} kept for all t, the
    denominator read back as B^2_{i,t-t'} by its time index, 50-digit decimal arithmetic."""
    getcontext().prec = 50
    for (W, H, T, d, eta, eps, b0, seed) in [(3, 4, 11, 2, 0.5, 1.0, 1.0, 1), (2, 3, 9, 3, 0.3, 0.5, 1.5, 2),
                                             (4, 1, 5, 2, 0.7, 1.0, 1.0, 3), (1, 5, 10, 2, 0.2, 2.0, 1.0, 4)]:
        G = _rand_grads(T, W, d, seed, 2.0)
        o = Oracle(d, W, H, eta, eps, b0, lib=lib)
        x0 = np.random.default_rng(seed + 100).standard_normal(d)
        o.init_state(x0)
        # history arrays indexed [t][i][j], t = 0..T
        X = [[[Decimal(float(o.x[i, j])) for j in range(d)] for i in range(W)]]
        B = [[[Decimal(b0) * Decimal(b0) for j in range(d)] for i in range(W)]]
        De, Dp2 = Decimal(eta), Decimal(eps) * Decimal(eps)
        for t in range(1, T + 1):
            tp = (t - 1) % H + 1
            Gt = np.asarray(o._real(G[t - 1]), dtype=np.float64)       # the values the oracle receives
            y = [[None] * d for _ in range(W)]
            A = [[None] * d for _ in range(W)]
            for i in range(W):
                for j in range(d):
                    g = Decimal(float(Gt[i, j]))
                    y[i][j] = X[t - 1][i][j] - De * g / (B[t - tp][i][j] + tp * Dp2).sqrt()
                    A[i][j] = B[t - 1][i][j] + g * g
            if t % H != 0:
                X.append(y); B.append(A)
            else:
                mx = [sum(y[k][j] for k in range(W)) / W for j in range(d)]
                mb = [sum(A[k][j] for k in range(W)) / W for j in range(d)]
                X.append([[mx[j] for j in range(d)] for _ in range(W)])
                B.append([[mb[j] for j in range(d)] for _ in range(W)])
            o.step_dense(G[t - 1])
            want_x = np.array([[float(v) for v in row] for row in X[t]])
            want_b = np.array([[float(v) for v in row] for row in B[t]])
            _close(o.x, want_x, _tol(lib), f"literal Alg.3 x at t={t} (W={W},H={H})")
            _close(o.acc, want_b, _tol(lib), f"literal Alg.3 B^2 at t={t} (W={W},H={H})")


def pin_closed_form_constant_gradient(lib):
    """Constant gradient: closed-form trajectory; for c^2 = eps^2 it does not depend on H."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "constant_gradient_closed_form.txt")) if l[0] != "#"]
    for c, H, xT, accT in rows:
        c, H, xT, accT = float(c), int(H), float(xT), float(accT)
        for W in (1, 3):
            o = Oracle(5, W, H, 0.5, 1.0, 1.0, lib=lib)
            o.init_state()
            for _ in range(8):
                o.step_dense(np.full((W, 5), c))
            _close(o.x, np.full((W, 5), xT), max(_tol(lib), 2e-10), f"closed form x_8 c={c} H={H}")
            _close(o.acc, np.full((W, 5), accT), _tol(lib), f"closed form acc_8 c={c} H={H}")
    # general parameters, formula evaluated here
    eta, eps, b0, c, T, x0 = 0.3, 0.7, 1.2, -1.7, 13, 0.4
    for H in (1, 2, 5, 13):
        o = Oracle(2, 2, H, eta, eps, b0, lib=lib)
        o.init_state(np.full(2, x0))
        for _ in range(T):
            o.step_dense(np.full((2, 2), c))
        # at the end T may sit inside a period: then acc is still the local one, same formula
        want = x0 - eta * c * sum(1.0 / np.sqrt(b0 * b0 + H * ((t - 1) // H) * c * c + ((t - 1) % H + 1) * eps * eps)
                                  for t in range(1, T + 1))
        _close(o.x, np.full((2, 2), want), _tol(lib), f"closed form general H={H}")
        _close(o.acc, np.full((2, 2), b0 * b0 + T * c * c), _tol(lib), f"closed form acc general H={H}")


def pin_h1_is_sync_adaalter(lib):
    """H = 1 (Section 4.2, last sentence of the lazy-update paragraph): one shared iterate with
    x -= eta mean(g)/sqrt(B^2 + eps^2), B^2 += mean(g^2) -- the old B^2 under the root."""
    W, d, T, eta, eps = 4, 7, 12, 0.4, 0.8
    G = _rand_grads(T, W, d, 11, 1.5)
    o = Oracle(d, W, 1, eta, eps, 1.0, lib=lib)
    o.init_state()
    x = np.zeros(d); b2 = np.ones(d)
    for t in range(T):
        Gt = np.asarray(o._real(G[t]), dtype=np.float64)
        x = x - eta * Gt.mean(axis=0) / np.sqrt(b2 + eps * eps)
        b2 = b2 + (Gt * Gt).mean(axis=0)
        o.step_dense(G[t])
        _close(o.x, np.tile(x, (W, 1)), _tol(lib), f"H=1 x at t={t + 1}")
        _close(o.snap, b2, _tol(lib), f"H=1 B^2 at t={t + 1}")


def pin_w1_is_serial(lib):
    """n = 1: averaging is the identity; a serial loop whose root term is refreshed every H steps."""
    d, T, H, eta, eps = 6, 14, 4, 0.5, 1.0
    G = _rand_grads(T, 1, d, 12)
    o = Oracle(d, 1, H, eta, eps, 1.0, lib=lib)
    o.init_state()
    x = np.zeros(d); run = np.ones(d); root = np.ones(d)
    for t in range(1, T + 1):
        g = np.asarray(o._real(G[t - 1][0]), dtype=np.float64)
        tp = (t - 1) % H + 1
        x = x - eta * g / np.sqrt(root + tp * eps * eps)
        run = run + g * g
        if t % H == 0:
            root = run.copy()
        o.step_dense(G[t - 1])
        _close(o.x[0], x, _tol(lib), f"W=1 x at t={t}")
        _close(o.acc[0], run, _tol(lib), f"W=1 acc at t={t}")


def pin_global_accumulator_and_invariants(lib):
    """Notation table: B^2_t = b0^2 + (1/n) sum_i sum_{s<=t} G_{i,s} o G_{i,s} at sync points;
    accumulators never decrease; the root term is shared and >= b0^2; after a sync every
    worker holds identical x and B^2."""
    W, d, T, H, b0 = 4, 9, 24, 6, 1.3
    G = _rand_grads(T, W, d, 13, 3.0)
    o = Oracle(d, W, H, 0.2, 0.5, b0, lib=lib)
    o.init_state()
    prev_acc, prev_snap = o.acc, o.snap
    for t in range(1, T + 1):
        o.step_dense(G[t - 1])
        acc, snap, x = o.acc, o.snap, o.x
        if t % H:
            assert np.all(acc >= prev_acc), "accumulator decreased in a local step"
            assert np.array_equal(snap, prev_snap), "root term changed between syncs"
        else:
            Gs = np.asarray(o._real(G[:t].reshape(-1, d)).reshape(t, W, d), dtype=np.float64)
            want = b0 * b0 + (Gs * Gs).sum(axis=0).mean(axis=0)
            _close(snap, want, 10 * _tol(lib), f"B^2_t definition at t={t}")
            assert np.all(snap >= prev_snap), "synced accumulator decreased"
            for w in range(1, W):
                assert np.array_equal(x[w], x[0]) and np.array_equal(acc[w], acc[0]), "no consensus after sync"
            assert np.array_equal(acc[0], snap)
        assert np.all(snap >= b0 * b0 * (1 - 1e-6))
        prev_acc, prev_snap = acc, snap


def pin_mean_iterate(lib):
    """Section 5 auxiliary iterate: the synced x equals the mean of the workers' local y, so over one
    period from a common start x_sync = x_start - eta * mean_i sum_s G_{i,s}/sqrt(B^2 + s eps^2)
    (appendix, unrolled iterate, with the square root of Algorithm 3)."""
    W, d, H, eta, eps = 5, 4, 7, 0.35, 0.9
    G = _rand_grads(H, W, d, 14)
    o = Oracle(d, W, H, eta, eps, 1.0, lib=lib)
    x0 = np.random.default_rng(5).standard_normal(d)
    o.init_state(x0)
    x0r = np.asarray(o.x[0], dtype=np.float64)
    for s in range(H):
        o.step_dense(G[s])
    Gr = np.asarray(o._real(G.reshape(-1, d)).reshape(H, W, d), dtype=np.float64)
    want = x0r - eta * sum(Gr[s].mean(axis=0) / np.sqrt(1.0 + (s + 1) * eps * eps) for s in range(H))
    _close(o.x[0], want, _tol(lib), "mean iterate after one period")


def pin_worker_permutation(lib):
    W, d, T, H = 4, 5, 8, 4
    G = _rand_grads(T, W, d, 15)
    perm = np.array([2, 0, 3, 1])
    a = Oracle(d, W, H, 0.5, 1.0, lib=lib); a.init_state()
    b = Oracle(d, W, H, 0.5, 1.0, lib=lib); b.init_state()
    for t in range(T):
        a.local_step_dense(G[t]); b.local_step_dense(G[t][perm])
        _close(b.x, a.x[perm], _tol(lib), "permuted local x")
        if (t + 1) % H == 0:
            a.sync(); b.sync()
            _close(b.x, a.x, 4 * _tol(lib), "synced x under permutation")
            _close(b.acc, a.acc, 4 * _tol(lib), "synced acc under permutation")


def pin_sync_due_and_early_sync(lib):
    o = Oracle(3, 2, 2, 0.5, 1.0, lib=lib); o.init_state()
    g = np.ones((2, 3))
    o.local_step_dense(g); o.local_step_dense(g)
    assert o.local_step_dense(g, rc_only=True) == oracle.ESYNCDUE
    o.sync()
    assert o.steps_since_sync == 0 and o.t == 2
    o.local_step_dense(g); o.sync()            # early sync restarts t' at 1
    o.local_step_dense(g)
    # root term: snap = 1 + 3 (three unit gradients), t' = 1
    want_last = -0.5 / np.sqrt(1 + 3 + 1)
    x_before = -0.5 / np.sqrt(2) - 0.5 / np.sqrt(3) - 0.5 / np.sqrt(1 + 2 + 1)
    _close(o.x, np.full((2, 3), x_before + want_last), _tol(lib), "early sync restarts t'")


# --------------------------------------------------------------------------- sparse
def pin_sparse_equals_dense(lib):
    W, rows, row_len, k, H = 3, 12, 4, 5, 3
    d = rows * row_len
    rng = np.random.default_rng(21)
    s = Oracle(d, W, H, 0.5, 1.0, lib=lib); s.init_state()
    e = Oracle(d, W, H, 0.5, 1.0, lib=lib); e.init_state()
    touched = set()
    for t in range(1, 7):
        idx = np.stack([rng.permutation(rows)[:k] for _ in range(W)]).astype(np.int32)
        vals = rng.standard_normal((W, k, row_len))
        G = np.zeros((W, rows, row_len))
        for w in range(W):
            G[w, idx[w]] = vals[w]
        s.local_step_sparse(idx, vals, row_len)
        e.local_step_dense(G.reshape(W, d))
        touched |= set(idx.ravel().tolist())
        assert np.array_equal(s.dirty_rows(), np.array(sorted(touched), dtype=np.int32)), "dirty rows"
        if t % H == 0:
            s.sync(); e.sync(); touched = set()
            assert s.dirty_rows().size == 0
        assert np.array_equal(s.x, e.x) and np.array_equal(s.acc, e.acc) and np.array_equal(s.snap, e.snap)
    # a row listed several times by one worker: the gradient of that row is the sum of the entries (a batch with a
    # repeated word), so the step equals the dense step with the summed gradient: acc grows by (sum)^2, not by
    # the sum of squares, and the denominator is the same for the whole sum
    s = Oracle(d, W, H, 0.5, 1.0, lib=lib); s.init_state()
    e = Oracle(d, W, H, 0.5, 1.0, lib=lib); e.init_state()
    idx = np.array([[2, 9, 2, 2, 5], [0, 0, 1, 1, 11], [7, 3, 4, 6, 7]], dtype=np.int32)
    vals = rng.integers(-4, 5, size=(W, k, row_len)).astype(np.float64)     # small integers: sums are exact
    G = np.zeros((W, rows, row_len))
    for w in range(W):
        np.add.at(G[w], idx[w], vals[w])
    s.local_step_sparse(idx, vals, row_len)
    e.local_step_dense(G.reshape(W, d))
    assert np.array_equal(s.x, e.x) and np.array_equal(s.acc, e.acc), "repeated rows must add up before the step"
    assert np.array_equal(s.acc.reshape(W, rows, row_len)[0, 2], 1.0 + (vals[0, 0] + vals[0, 2] + vals[0, 3]) ** 2)
    # untouched rows are exact no-ops
    o = Oracle(d, W, 4, 0.5, 1.0, lib=lib)
    x0 = rng.standard_normal(d); o.init_state(x0)
    x_init = o.x
    idx = np.tile(np.array([[1, 7]], dtype=np.int32), (W, 1))
    o.local_step_sparse(idx, np.ones((W, 2, row_len)), row_len)
    keep = np.ones(rows, bool); keep[[1, 7]] = False
    assert np.array_equal(o.x.reshape(W, rows, row_len)[:, keep], x_init.reshape(W, rows, row_len)[:, keep])
    assert np.all(o.acc.reshape(W, rows, row_len)[:, keep] == 1.0)
    assert np.all(o.acc.reshape(W, rows, row_len)[:, [1, 7]] == 2.0)


# --------------------------------------------------------------------------- generator
def pin_philox_kat(lib):
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(s, 16) for s in line.split()]
        out = oracle.philox4x32_10(v[0:4], v[4:6], lib=lib)
        assert [int(o) for o in out] == v[6:10], f"Philox4x32-10 KAT mismatch for counter {v[0:4]}"


def pin_normal_statistics(lib):
    from scipy import stats
    n = np.concatenate([oracle.normals4(7, oracle.STREAM_NOISE, q, q % 5, 1 + q % 3, lib=lib) for q in range(50_000)])
    N = n.size
    assert abs(n.mean()) < 4 / np.sqrt(N)
    assert abs(n.var() - 1) < 4 * np.sqrt(2 / N)
    assert abs(stats.skew(n)) < 4 * np.sqrt(6 / N)
    assert abs(stats.kurtosis(n)) < 4 * np.sqrt(24 / N)
    assert stats.kstest(n, "norm").pvalue > 1e-3
    quad = n.reshape(-1, 4)
    c = np.corrcoef(quad.T)
    assert np.max(np.abs(c - np.eye(4))) < 4 / np.sqrt(quad.shape[0])
    # different worker / iteration / stream / seed give different draws; same arguments repeat
    base = oracle.normals4(7, 3, 10, 1, 1, lib=lib)
    assert np.array_equal(base, oracle.normals4(7, 3, 10, 1, 1, lib=lib))
    for other in [(8, 3, 10, 1, 1), (7, 2, 10, 1, 1), (7, 3, 11, 1, 1), (7, 3, 10, 2, 1), (7, 3, 10, 1, 2),
                  (7 + (1 << 32), 3, 10, 1, 1)]:
        assert not np.array_equal(base, oracle.normals4(*other, lib=lib))


def pin_box_muller_from_words(lib):
    """Normals recomputed here from the raw Philox words: u = ((r>>9)+0.5)/2^23,
    (n0,n1) = sqrt(-2 ln u0)(cos 2 pi u1, sin 2 pi u1), (n2,n3) from (u2,u3)."""
    for (seed, stream, q, w, t) in [(0, 3, 0, 0, 1), (5, 2, 123456, 3, 0), ((9 << 32) + 4, 3, (1 << 32) + 17, 7, 1 << 20)]:
        r = oracle.philox4x32_10([q & 0xFFFFFFFF, w, t & 0xFFFFFFFF, stream + (q >> 32) * 16],
                                 [seed & 0xFFFFFFFF, seed >> 32], lib=lib).astype(np.float64)
        u = (np.floor(r / 512.0) + 0.5) / 8388608.0
        assert np.all((u > 0) & (u < 1)) and np.array_equal(u, u.astype(np.float32).astype(np.float64))
        want = [np.sqrt(-2 * np.log(u[0])) * np.cos(2 * np.pi * u[1]), np.sqrt(-2 * np.log(u[0])) * np.sin(2 * np.pi * u[1]),
                np.sqrt(-2 * np.log(u[2])) * np.cos(2 * np.pi * u[3]), np.sqrt(-2 * np.log(u[2])) * np.sin(2 * np.pi * u[3])]
        got = oracle.normals4(seed, stream, q, w, t, lib=lib)
        _close(got, want, 1e-12 if lib.real_bytes == 8 else 1e-5, "Box-Muller from words")


def pin_gradient_formula(lib):
    """g = a (x - (xstar + off)) + noise_scale n, and g = a n, rebuilt from normals4; column
    remapping equals slicing the full problem."""
    W, d, seed = 3, 16, 42
    rng = np.random.default_rng(3)
    a = rng.uniform(0.1, 10, d); xs = rng.standard_normal(d); off = 0.1 * rng.standard_normal((W, d))
    x0 = rng.standard_normal(d)
    for off_mode in (oracle.OFF_NONE, oracle.OFF_ARRAY, oracle.OFF_PHILOX):
        o = Oracle(d, W, 4, 0.5, 1.0, lib=lib); o.init_state(x0)
        o.set_generator(oracle.GEN_QUADRATIC, seed, a, xs, off if off_mode == oracle.OFF_ARRAY else None,
                        off_mode, noise_scale=0.2, off_scale=0.3)
        ar, xr, x0r = (np.asarray(o._real(v), dtype=np.float64) for v in (a, xs, x0))
        offr = np.asarray(o._real(off), dtype=np.float64)
        for t in (1, 2):
            want = np.empty((W, d))
            for w in range(W):
                for j in range(d):
                    n = oracle.normals4(seed, 3, j // 4, w, t, lib=lib)[j % 4]
                    sh = {oracle.OFF_NONE: 0.0, oracle.OFF_ARRAY: offr[w, j],
                          oracle.OFF_PHILOX: 0.3 * float(oracle.normals4(seed, 2, j // 4, w, 0, lib=lib)[j % 4])}[off_mode]
                    want[w, j] = ar[j] * (x0r[j] - (xr[j] + sh)) + 0.2 * float(n)
            _close(o.gradient(t), want, _tol(lib) * 10, f"quadratic gradient off_mode={off_mode}")
    o = Oracle(d, W, 4, 0.5, 1.0, lib=lib); o.init_state(x0)
    o.set_generator(oracle.GEN_NOISE, seed, a)
    want = np.array([[np.asarray(o._real(a), dtype=np.float64)[j] * float(oracle.normals4(seed, 3, j // 4, w, 5, lib=lib)[j % 4])
                      for j in range(d)] for w in range(W)])
    _close(o.gradient(5), want, _tol(lib) * 10, "noise gradient")
    # a generator step is the dense step on that gradient
    p = Oracle(d, W, 4, 0.5, 1.0, lib=lib); p.init_state(x0)
    p.set_generator(oracle.GEN_QUADRATIC, seed, a, xs, None, oracle.OFF_PHILOX)
    q = Oracle(d, W, 4, 0.5, 1.0, lib=lib); q.init_state(x0)
    for t in range(1, 6):
        g = p.gradient(t)
        p.step_gen(); q.step_dense(g)
        assert np.array_equal(p.x, q.x) and np.array_equal(p.acc, q.acc)
    # columns: a run on a subset of columns with absolute coordinates equals the slice of the full run
    cols = np.array([4, 5, 6, 7, 12, 13, 14, 15, 2])
    full = Oracle(d, W, 2, 0.5, 1.0, lib=lib); full.init_state(x0)
    full.set_generator(oracle.GEN_QUADRATIC, seed, a, xs, None, oracle.OFF_PHILOX)
    part = Oracle(len(cols), W, 2, 0.5, 1.0, lib=lib); part.set_columns(cols); part.init_state(x0[cols])
    part.set_generator(oracle.GEN_QUADRATIC, seed, a[cols], xs[cols], None, oracle.OFF_PHILOX)
    for _ in range(5):
        full.step_gen(); part.step_gen()
    assert np.array_equal(full.x[:, cols], part.x) and np.array_equal(full.acc[:, cols], part.acc)


# --------------------------------------------------------------------------- Section 6.2, Algorithms 1 and 2
def pin_warmup(lib):
    """eta_t = eta min(1, t/warmup): with g = eps the H-independent closed form becomes a weighted sum."""
    eta, eps, T, wu = 0.5, 1.0, 12, 5
    for H in (1, 3, 12):
        o = Oracle(2, 2, H, eta, eps, 1.0, lib=lib); o.init_state(); o.set_warmup(wu)
        for _ in range(T):
            o.step_dense(np.full((2, 2), eps))
        want = -sum(eta * min(1.0, t / wu) * eps / np.sqrt(1 + t * eps * eps) for t in range(1, T + 1))
        _close(o.x, np.full((2, 2), want), _tol(lib), f"warm-up closed form H={H}")


def pin_adagrad_and_local_sgd(lib):
    """Algorithm 1 with explicit gradients: x_T = x0 - eta sum_t gbar_t / sqrt(sum_{s<=t} gbar_s^2 + eps^2), gbar the
    worker mean, B^2_0 = 0.  Algorithm 2 with gradients that do not depend on x: at every sync point
    x = x0 - eta sum_t gbar_t, and in between each worker has moved by its own gradients."""
    W, d, T, eta, eps = 3, 5, 9, 0.3, 0.1
    G = _rand_grads(T, W, d, 31)
    o = Oracle(d, W, 1, eta, eps, 0.0, lib=lib); o.init_state()
    for t in range(T):
        o.adagrad_step_dense(G[t])
    Gr = np.asarray(o._real(G.reshape(-1, d)).reshape(T, W, d), dtype=np.float64)
    gb = Gr.mean(axis=1)
    want = -eta * (gb / np.sqrt(np.cumsum(gb * gb, axis=0) + eps * eps)).sum(axis=0)
    _close(o.x, np.tile(want, (W, 1)), _tol(lib) * 4, "Distributed AdaGrad closed form")
    H = 3
    s = Oracle(d, W, H, eta, eps, 1.0, lib=lib); s.init_state()
    for t in range(1, T + 1):
        s.localsgd_step_dense(G[t - 1])
        last_sync = (t // H) * H
        base = -eta * gb[:last_sync].sum(axis=0)
        want = base[None, :] - eta * Gr[last_sync:t].sum(axis=0)
        _close(s.x, want, _tol(lib) * 4, f"Local SGD at t={t}")


def pin_diagnostics(lib):
    """Section 5's mean iterate: ||xbar - xstar||^2, ||grad F(xbar)||^2 with grad F(xbar) = a (xbar - xstar - mean off)
    for the quadratic objective, and the mean squared distance of the workers from xbar -- recomputed with numpy;
    at xbar = xstar + mean off the gradient vanishes."""
    W, d = 4, 12
    rng = np.random.default_rng(41)
    a = rng.uniform(0.1, 10, d); xs = rng.standard_normal(d); off = 0.3 * rng.standard_normal((W, d))
    o = Oracle(d, W, 5, 0.5, 1.0, lib=lib); o.init_state(rng.standard_normal(d))
    o.set_generator(oracle.GEN_QUADRATIC, 9, a, xs, off, oracle.OFF_ARRAY, 0.1, 0.1)
    for _ in range(3):
        o.local_step_gen()
    x = o.x.astype(np.float64)
    ar, xr, offr = (np.asarray(o._real(v), dtype=np.float64) for v in (a, xs, off))
    xbar = x.mean(axis=0)
    want = (np.sum((xbar - xr) ** 2), np.sum((ar * (xbar - xr - offr.mean(axis=0))) ** 2), np.mean(np.sum((x - xbar) ** 2, axis=1)))
    _close(o.diagnostics(), want, 1e-12 if lib.real_bytes == 8 else 1e-5, "diagnostics")
    p = Oracle(d, W, 5, 0.5, 1.0, lib=lib)
    p.init_state(xr + offr.mean(axis=0))
    p.set_generator(oracle.GEN_QUADRATIC, 9, a, xs, off, oracle.OFF_ARRAY, 0.1, 0.1)
    g = p.diagnostics()
    assert g[1] <= 1e-10 and g[2] == 0.0 and abs(g[0] - np.sum(offr.mean(axis=0) ** 2)) <= 1e-6


ALL_PINS = [pin_diagnostics, pin_literal_history, pin_closed_form_constant_gradient, pin_h1_is_sync_adaalter, pin_w1_is_serial,
            pin_global_accumulator_and_invariants, pin_mean_iterate, pin_worker_permutation,
            pin_sync_due_and_early_sync, pin_sparse_equals_dense, pin_philox_kat, pin_normal_statistics,
            pin_box_muller_from_words, pin_gradient_formula, pin_warmup, pin_adagrad_and_local_sgd]
