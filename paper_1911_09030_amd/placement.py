"""Choosing where the state arrays live in device memory by measurement.

On MI355X the rate of a kernel that streams the 2W rows of x and acc and a few [d] vectors at once depends on
where these arrays sit in physical memory relative to one another: inside one 260 GB range the plain step of the
d = 4e8, W = 8 workload took between 8.70 and 10.2 ms over 235 placements (0.80 to 0.69 of the HBM peak), most
likely because the streams share DRAM banks in some placements and not in others, and the address-to-bank mapping is
not documented.  So the placement is measured: take a pool of most of the free memory (binding.Pool), time the
caller's step on candidate placements inside it, keep the best and release the rest of the pool.

Nothing here is part of the optimizer's arithmetic; it only decides at which addresses the caller's arrays start.
"""
from __future__ import annotations

import random
from dataclasses import dataclass

ALIGN = 1024            # elements: arrays start at multiples of 4 KiB


@dataclass
class Layout:
    pitch: int                   # elements between consecutive worker rows of every [W][d] matrix
    matrices: list               # element offset of each matrix in the pool
    vectors: list                # element offset of each [d] vector
    ms: float = float("inf")     # measured time of the caller's step

    def ranges(self, d, W):
        """(offset, length) in elements of every array, for Pool.trim."""
        out = [(m + w * self.pitch, d) for m in self.matrices for w in range(W)]
        return out + [(v, d) for v in self.vectors]


def _round_up(n, a=ALIGN):
    return (n + a - 1) // a * a


def _disjoint(spans):
    spans = sorted(spans)
    return all(spans[i][1] <= spans[i + 1][0] for i in range(len(spans) - 1))


def candidates(pool_elems, d, W, n_matrices, n_vectors, n_random, seed):
    """Everything packed back to back from a grid of start offsets, then seeded random placements of every matrix
    (rows packed or a little apart) and of the block of vectors."""
    dp = _round_up(d)
    out = []
    packed_len = (n_matrices * W + n_vectors) * dp
    n_grid = 16
    for k in range(n_grid):
        b = _round_up((pool_elems - packed_len) * k // max(n_grid - 1, 1)) if pool_elems > packed_len else 0
        if b + packed_len > pool_elems:
            continue
        out.append(Layout(dp, [b + m * W * dp for m in range(n_matrices)],
                          [b + n_matrices * W * dp + v * dp for v in range(n_vectors)]))
    rng = random.Random(seed)
    tries = 0
    while len(out) < n_grid + n_random and tries < 50 * n_random:
        tries += 1
        pitch = _round_up(int(dp * rng.choice((1.0, 1.0, 1.25, 1.5, 2.0))))
        mats = [_round_up(rng.randrange(0, max(pool_elems - W * pitch, 1))) for _ in range(n_matrices)]
        vb = _round_up(rng.randrange(0, max(pool_elems - n_vectors * dp, 1)))
        spans = [(m, m + (W - 1) * pitch + d) for m in mats] + [(vb, vb + (n_vectors - 1) * dp + d)]
        if max(e for _, e in spans) > pool_elems or not _disjoint(spans):
            continue
        out.append(Layout(pitch, mats, [vb + v * dp for v in range(n_vectors)]))
    return out


def tune(pool, d, W, n_matrices, n_vectors, measure, n_random=48, seed=0, confirm=3, refine=6, log=None):
    """Time measure(matrices, vectors, pitch) -> milliseconds on candidate placements inside `pool` and return the
    fastest Layout: first the candidates, then `refine` variations of each of the best four (one array group moved
    elsewhere); the three best are timed a second time and the best of those wins.  `matrices` are [W][d]
    float32 views with row pitch `pitch`, `vectors` are [d] views; measure must leave nothing running."""
    pool_elems = pool.nbytes // 4
    tried = []
    for lay in candidates(pool_elems, d, W, n_matrices, n_vectors, n_random, seed):
        lay.ms = _run(pool, d, W, lay, measure)
        tried.append(lay)
        if log:
            log(f"placement pitch {lay.pitch} matrices {lay.matrices} vectors {lay.vectors[0]}: {lay.ms:.4f} ms")
    if not tried:
        raise ValueError("the pool is too small for the arrays")
    tried.sort(key=lambda l: l.ms)
    # second stage: around the best few, move one part of the placement (a matrix or the block of vectors) elsewhere
    rng = random.Random(seed + 1)
    dp = _round_up(d)
    for parent in list(tried[:4]):
        for _ in range(refine):
            mats, vb = list(parent.matrices), parent.vectors[0]
            k = rng.randrange(len(mats) + 1)
            if k < len(mats):
                mats[k] = _round_up(rng.randrange(0, max(pool_elems - W * parent.pitch, 1)))
            else:
                vb = _round_up(rng.randrange(0, max(pool_elems - n_vectors * dp, 1)))
            spans = [(m, m + (W - 1) * parent.pitch + d) for m in mats] + [(vb, vb + (n_vectors - 1) * dp + d)]
            if max(e for _, e in spans) > pool_elems or not _disjoint(spans):
                continue
            lay = Layout(parent.pitch, mats, [vb + v * dp for v in range(n_vectors)])
            lay.ms = _run(pool, d, W, lay, measure)
            tried.append(lay)
            if log:
                log(f"placement (refined) pitch {lay.pitch} matrices {lay.matrices} vectors {lay.vectors[0]}: {lay.ms:.4f} ms")
    tried.sort(key=lambda l: l.ms)
    best = tried[0]
    for lay in tried[:confirm]:
        lay.ms = max(lay.ms, _run(pool, d, W, lay, measure))       # the slower of its two timings
    best = min(tried[:confirm], key=lambda l: l.ms)
    best.tried = len(tried)
    best.slowest_ms = tried[-1].ms
    best.median_ms = tried[len(tried) // 2].ms
    return best


def views(pool, d, W, lay):
    mats = [pool.tensor(m, (W, d), (lay.pitch, 1)) for m in lay.matrices]
    vecs = [pool.tensor(v, (d,)) for v in lay.vectors]
    return mats, vecs


def _run(pool, d, W, lay, measure):
    mats, vecs = views(pool, d, W, lay)
    return float(measure(mats, vecs, lay.pitch))


def event_median_ms(step, n=5):
    """Median duration of n calls of step(), each between two events on the current stream."""
    import torch
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
    ev[0].record()
    for i in range(n):
        step()
        ev[i + 1].record()
    torch.cuda.synchronize()
    return sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(n))[n // 2]


def generator_step_timer(d, W, eta, eps, seed, mode, off_mode, noise_scale, off_scale, tile=None, algorithm=None,
                         lazy=False):
    """measure() for tune(): the plain generator step (no averaging in reach) on arrays at a candidate placement.
    Quadratic mode: matrices (x, acc[, stored offsets]), vectors (snap, a, xstar); noise mode: matrices (x, acc),
    vectors (snap, a).  The inputs are constants: the step's duration does not depend on their values.
    `algorithm` (a binding.ALGO_* value) times the step of that algorithm instead of Local AdaAlter's; `lazy` switches
    lazy replicas on (it changes the kernel of Distributed AdaGrad, whose every step averages)."""
    from . import binding as B

    def measure(mats, vecs, pitch):
        vecs[1].fill_(1.0)
        xstar = None
        if mode == B.GEN_QUADRATIC:
            xstar = vecs[2]
            xstar.fill_(0.5)
        off = None
        if off_mode == B.OFF_ARRAY:
            off = mats[2]
            off.zero_()
        h = B.LocalAdaAlter(d, W, 1 << 30, eta, eps, x=mats[0], acc=mats[1], snap=vecs[0], pitch=pitch)
        if algorithm is not None:
            h.set_algorithm(algorithm)
        if lazy:
            h.set_lazy_replicas(True)
        h.init_state()
        h.set_generator(mode, seed, vecs[1], xstar, off, off_mode, noise_scale, off_scale)
        if tile is not None:
            h.set_tile(tile)
        h.step_gen()
        ms = event_median_ms(h.step_gen)
        h.close()
        return ms

    return measure


def quadratic_step_timer(d, W, eta, eps, seed, off_mode, noise_scale, off_scale, tile=None, algorithm=None, lazy=False):
    from . import binding as B
    return generator_step_timer(d, W, eta, eps, seed, B.GEN_QUADRATIC, off_mode, noise_scale, off_scale, tile, algorithm, lazy)


def averaging_timer(d, W, eta, eps):
    """measure() for tune(): the Synchronize pass over the whole of x, acc, snap (matrices (x, acc), vectors
    (snap,)): 2W read and 2W + 1 write streams, the pattern of the averaging of touched rows on a row-sparse table."""
    from . import binding as B

    def measure(mats, vecs, pitch):
        h = B.LocalAdaAlter(d, W, 1 << 30, eta, eps, x=mats[0], acc=mats[1], snap=vecs[0], pitch=pitch)
        h.init_state()

        def one():
            h.set_counters(1, 1)          # one local step pending, touched rows unknown: the next sync takes the whole table
            h.sync()
        one()
        ms = event_median_ms(one)
        h.close()
        return ms

    return measure
