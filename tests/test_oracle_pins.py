"""CPU tests: the oracle against what the paper and the mathematics fix (no GPU)."""
import numpy as np
import pytest

import oracle
import pins

PLANTS = ["ORA_PLANT_RUNNING_DENOM", "ORA_PLANT_NO_SQRT", "ORA_PLANT_PAD_ONE", "ORA_PLANT_PAD_OFF_BY_ONE",
          "ORA_PLANT_PLUS", "ORA_PLANT_ACC_ABS", "ORA_PLANT_SYNC_NO_ACC", "ORA_PLANT_GRAD_OFFSET_SIGN",
          "ORA_PLANT_SINCOS_SWAPPED", "ORA_PLANT_ADAGRAD_OLD_B2"]


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
