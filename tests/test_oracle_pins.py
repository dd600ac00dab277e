"""CPU tests: the oracle against what the paper and the mathematics fix (no GPU)."""
import numpy as np
import pytest

import oracle
import pins

PLANTS = ["ORA_PLANT_RUNNING_DENOM", "ORA_PLANT_NO_SQRT", "ORA_PLANT_PAD_ONE", "ORA_PLANT_PAD_OFF_BY_ONE",
          "ORA_PLANT_PLUS", "ORA_PLANT_ACC_ABS", "ORA_PLANT_SYNC_NO_ACC", "ORA_PLANT_GRAD_OFFSET_SIGN",
          "ORA_PLANT_SINCOS_SWAPPED", "ORA_PLANT_ADAGRAD_OLD_B2", "ORA_PLANT_SPARSE_LAST_WINS"]


@pytest.mark.parametrize("pin", pins.ALL_PINS, ids=lambda f: f.__name__)
def test_pin_fp64(pin, ora64):
    pin(ora64)


@pytest.mark.parametrize("pin", pins.ALL_PINS, ids=lambda f: f.__name__)
def test_pin_fp32_build(pin, ora32):
    pin(ora32)


@pytest.mark.parametrize("plant", PLANTS)
def test_planted_mistake_is_caught(plant, tmp_path):
    """A build of the oracle with one deliberate mistake must fail at least one pin."""
    path = oracle.build("f64", out=str(tmp_path / f"bad_{plant}.so"), defines=(plant,), force=True)
    lib = oracle.load(path=path)
    failed = []
    for pin in pins.ALL_PINS:
        if pin is pins.pin_normal_statistics:      # slow and not meant to see these
            continue
        try:
            pin(lib)
        except AssertionError:
            failed.append(pin.__name__)
    assert failed, f"{plant} slipped through every pin"


def test_worked_example_two_workers():
    """W=2, H=2, eta=0.5, eps=b0=1, d=1, gradients (1,2,-1,0.5) and (3,-2,1,1.5), unrolled by hand from
    Algorithm 3: t=1 roots are sqrt(1+1); t=2 sqrt(1+2) then the mean; t=3 sqrt(10+1); t=4 sqrt(10+2)."""
    o = oracle.Oracle(1, 2, 2, 0.5, 1.0)
    o.init_state()
    r2, r3, r11, r12 = np.sqrt(2.0), np.sqrt(3.0), np.sqrt(11.0), np.sqrt(12.0)
    o.step_dense([[1.0], [3.0]])
    assert np.allclose(o.x.ravel(), [-0.5 / r2, -1.5 / r2], rtol=1e-14) and np.array_equal(o.acc.ravel(), [2, 10])
    assert o.snap[0] == 1.0
    o.step_dense([[2.0], [-2.0]])
    m = ((-0.5 / r2 - 1.0 / r3) + (-1.5 / r2 + 1.0 / r3)) / 2
    assert np.allclose(o.x.ravel(), [m, m], rtol=1e-14) and np.array_equal(o.acc.ravel(), [10, 10])
    assert abs(m + 0.7071067811865476) < 1e-15 and o.snap[0] == 10.0
    o.step_dense([[-1.0], [1.0]])
    assert np.allclose(o.x.ravel(), [m + 0.5 / r11, m - 0.5 / r11], rtol=1e-14) and np.array_equal(o.acc.ravel(), [11, 11])
    o.step_dense([[0.5], [1.5]])
    m2 = m - (0.25 + 0.75) / r12 / 2
    assert np.allclose(o.x.ravel(), [m2, m2], rtol=1e-14) and np.array_equal(o.acc.ravel(), [12.25, 12.25])


def test_h1_differs_from_adagrad():
    """Section 4.2: even with H=1 the method is not AdaGrad (the root sees the accumulator one step late,
    and the mean of squares rather than the square of the mean)."""
    G = np.random.default_rng(0).standard_normal((6, 3, 4))
    a = oracle.Oracle(4, 3, 1, 0.5, 1.0, 1.0); a.init_state()
    b = oracle.Oracle(4, 3, 1, 0.5, 1.0, 1.0); b.init_state()
    for t in range(6):
        a.step_dense(G[t]); b.adagrad_step_dense(G[t])
    assert np.max(np.abs(a.x - b.x)) > 1e-3


def test_create_rejects_bad_arguments():
    for args in [(0, 1, 1, 0.5, 1.0), (4, 0, 1, 0.5, 1.0), (4, 1, 0, 0.5, 1.0), (4, 1, 1, float("nan"), 1.0),
                 (4, 1, 1, 0.5, -1.0)]:
        with pytest.raises(ValueError):
            oracle.Oracle(*args)


def test_tolerance_calibration_fp32_statements_meet_the_gpu_bars():
    """The same statements evaluated in fp32 (the oracle's fp32 build) stay within the bars the GPU tests use,
    i.e. the bars are what fp32 arithmetic can deliver and no looser."""
    import parity
    from paper_1911_09030_amd import workloads as wl
    # explicit gradients: identical inputs on both sides
    W, H, d, T = 4, 4, 4096, 32
    rng = np.random.default_rng(3)
    x0 = rng.standard_normal(d).astype(np.float32)
    sig = np.power(10.0, rng.uniform(-3, 1, d)).astype(np.float32)
    o64 = oracle.Oracle(d, W, H, 0.5, 1.0); o64.init_state(x0)
    o32 = oracle.Oracle(d, W, H, 0.5, 1.0, precision="f32"); o32.init_state(x0)
    sc = parity.Scale(o64)
    for t in range(1, T + 1):
        G = rng.standard_normal((W, d)).astype(np.float32) * sig[None, :]
        o64.local_step_dense(G); o32.local_step_dense(G); sc.update(o64)
        if t == 1:
            parity.assert_state(o32.x, o32.acc, o32.snap, o64, parity.ONE_STEP, what="fp32 one step", scale=sc)
        if t % H == 0:
            o64.sync(); o32.sync()
    parity.assert_state(o32.x, o32.acc, o32.snap, o64, parity.FULL_RUN, what="fp32 full run", scale=sc)
    # generator-fed, the small configuration on a column sample, full length
    c = wl.WORKLOADS["c1"]
    cols = wl.column_sample(c.d, 512, seed=1)
    a = wl.curvature(c.d, c.seed, c.a_dist)[cols]; xs = wl.optimum(c.d, c.seed)[cols]
    runs = []
    for prec in ("f64", "f32"):
        o = oracle.Oracle(len(cols), c.W, c.H, c.eta, c.eps, precision=prec)
        o.set_columns(cols); o.init_state()
        o.set_generator(oracle.GEN_QUADRATIC, c.seed, a, xs, None, oracle.OFF_PHILOX, c.noise_scale, c.off_scale)
        for _ in range(c.T):
            o.step_gen()
        runs.append(o)
    parity.assert_state(runs[1].x, runs[1].acc, runs[1].snap, runs[0], 1e-5, floor_x=1.0, what="fp32 generator run")


def test_noise_grows_with_the_sync_period():
    """Section 5, remark after the theorem: compared with H = 1, local steps add noise that grows with H.  On the
    small quadratic configuration the workers' drift (1/n) sum_i ||x_i - xbar||^2 just before a synchronisation
    (the quantity the proof bounds by the H^2 term) grows with H."""
    from paper_1911_09030_amd import workloads as wl
    c = wl.WORKLOADS["c1"]
    cols = wl.column_sample(c.d, 256, seed=3)
    a = wl.curvature(c.d, c.seed, c.a_dist)[cols]; xs = wl.optimum(c.d, c.seed)[cols]
    drift = {}
    for H in (1, 4, 16):
        o = oracle.Oracle(len(cols), c.W, H, c.eta, c.eps)
        o.set_columns(cols); o.init_state()
        o.set_generator(oracle.GEN_QUADRATIC, c.seed, a, xs, None, oracle.OFF_PHILOX, c.noise_scale, c.off_scale)
        for t in range(1, c.T + 1):
            o.local_step_gen()
            if t == c.T:
                drift[H] = o.diagnostics()[2]
            if t % H == 0:
                o.sync()
    assert drift[1] < drift[4] < drift[16]
