"""Host logic of the placement tuner (no GPU): candidates lie inside the pool and do not overlap, the fastest one wins,
the second stage only keeps valid variations."""
import random

import pytest

from paper_1911_09030_amd import placement as P


class FakePool:
    """Stands in for binding.Pool: views are just (offset, shape, strides) records."""

    def __init__(self, nbytes):
        self.nbytes = nbytes

    def tensor(self, offset, shape, strides=None):
        return ("view", offset, tuple(shape), strides)


def _check(lay, pool_elems, d, W, n_mat, n_vec):
    assert lay.pitch >= d and lay.pitch % P.ALIGN == 0
    assert len(lay.matrices) == n_mat and len(lay.vectors) == n_vec
    spans = sorted(lay.ranges(d, W))
    assert len(spans) == n_mat * W + n_vec
    assert all(o % P.ALIGN == 0 for o, _ in spans)
    assert spans[0][0] >= 0 and spans[-1][0] + spans[-1][1] <= pool_elems
    assert all(a + n <= b for (a, n), (b, _) in zip(spans, spans[1:])), "arrays overlap"


@pytest.mark.parametrize("d,W,n_mat,n_vec,pool_elems", [(400_000_000, 8, 2, 3, 65_000_000_000), (100_000_000, 8, 6, 2, 65_000_000_000),
                                                        (8448, 4, 2, 3, 20_971_520), (1001, 3, 2, 1, 200_000)])
def test_candidates_are_valid(d, W, n_mat, n_vec, pool_elems):
    c = P.candidates(pool_elems, d, W, n_mat, n_vec, 48, seed=0)
    assert len(c) > 16
    for lay in c:
        _check(lay, pool_elems, d, W, n_mat, n_vec)
    again = P.candidates(pool_elems, d, W, n_mat, n_vec, 48, seed=0)
    assert [(l.pitch, l.matrices, l.vectors) for l in c] == [(l.pitch, l.matrices, l.vectors) for l in again]     # seeded
    assert P.candidates(1000, d, W, n_mat, n_vec, 8, seed=0) == []                                              # pool too small


def test_tune_picks_the_fastest_and_confirms_it():
    d, W, pool = 8448, 4, FakePool(4 * 20_971_520)
    rng = random.Random(5)
    calls = []

    def measure(mats, vecs, pitch):
        assert len(mats) == 2 and len(vecs) == 3 and mats[0][2] == (W, d) and mats[0][3] == (pitch, 1)
        # a deterministic "duration" per placement: the same placement measures the same both times
        ms = 8.0 + (hash((mats[0][1], mats[1][1], vecs[0][1])) % 1000) / 500.0
        calls.append(ms)
        return ms

    best = P.tune(pool, d, W, 2, 3, measure, n_random=20, seed=2, refine=3)
    assert best.ms == min(calls) and best.tried == len(calls) - 3
    assert best.tried > 16 + 20                       # the second stage added variations
    assert best.median_ms >= best.ms and best.slowest_ms == max(calls)
    _check(best, pool.nbytes // 4, d, W, 2, 3)
    with pytest.raises(ValueError):
        P.tune(FakePool(4096), d, W, 2, 3, measure)
