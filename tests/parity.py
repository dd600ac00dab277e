"""Error metrics shared by the parity tests.

Per-element relative error  |got_j - ref_j| / max(|ref_j|, s_j, floor).

s_j is the largest magnitude the oracle's x_j has had so far on the run (tracked by Scale): an fp32 iterate
x - eta g / den cannot be more accurate than an ulp of its largest operand, so when an update cancels most of x
the error is relative to what was cancelled, not to the small remainder.  `floor` guards exact zeros.

Bars: explicit-gradient runs (both sides receive the same gradient bits) use floor 1e-3 for x and
1e-3 for the accumulators, 1e-6 after one step and 1e-5 after a full run.  Generator-fed runs compare the
generated gradient separately against the magnitude of its terms, and use floor 1 for x (the scale of the
quadratic's optimum): the gradient is itself an fp32 quantity with cancellation between a (x - xstar - off)
and the noise term, which no fp32 implementation can avoid.
"""
import numpy as np

ONE_STEP = 1e-6
FULL_RUN = 1e-5
FLOOR_X = 1e-3
FLOOR_B = 1e-3


class Scale:
    """Running elementwise maximum of |x| over the oracle's trajectory."""

    def __init__(self, ora):
        self.s = np.abs(ora.x)

    def update(self, ora):
        np.maximum(self.s, np.abs(ora.x), out=self.s)
        return self


def rel_err(got, ref, floor, scale=None):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if not ref.size:
        return 0.0
    den = np.maximum(np.abs(ref), floor)
    if scale is not None:
        den = np.maximum(den, scale)
    return float(np.max(np.abs(got - ref) / den))


def assert_state(got_x, got_acc, got_snap, ora, bar, floor_x=FLOOR_X, floor_b=FLOOR_B, what="", scale=None):
    ex = rel_err(got_x, ora.x, floor_x, None if scale is None else scale.s)
    eb = rel_err(got_acc, ora.acc, floor_b)
    es = rel_err(got_snap, ora.snap, floor_b)
    assert ex <= bar and eb <= bar and es <= bar, f"{what}: rel err x {ex:.2e} acc {eb:.2e} snap {es:.2e} > {bar:.0e}"
    return ex, eb, es


def assert_one_step_generated(got_x, got_acc, x_before, ora, g_ref, S, eta, den, what=""):
    """One generator-fed step against the oracle, with the bound the arithmetic gives instead of a floor.

    The generated gradient is within 1e-6 S of the oracle's (S = magnitude of its terms, asserted separately), so
    x' = x - eta g / den is within eta (1e-6 S) / den plus a few roundings of the larger of |x|, |x'|:
        |dx|   <= 1e-6 (max(|x|, |x'|) + eta S / den)
    and acc' = acc + g^2 within 2 |g| (1e-6 S) plus one rounding of acc':
        |dacc| <= 1e-6 (acc' + 2 |g| S)
    """
    got_x = np.asarray(got_x, dtype=np.float64)
    got_acc = np.asarray(got_acc, dtype=np.float64)
    bx = ONE_STEP * (np.maximum(np.abs(x_before), np.abs(ora.x)) + abs(eta) * S / den)
    bb = ONE_STEP * (np.abs(ora.acc) + 2 * np.abs(g_ref) * S)
    rx = float(np.max(np.abs(got_x - ora.x) / bx))
    rb = float(np.max(np.abs(got_acc - ora.acc) / bb))
    assert rx <= 1.0 and rb <= 1.0, f"{what}: one generated step is {rx:.2f} (x) and {rb:.2f} (acc) of the 1e-6 bound"
    return rx, rb
