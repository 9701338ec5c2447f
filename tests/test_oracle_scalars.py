"""Pins for the per-step scalars: exact rational arithmetic, not libm."""
from fractions import Fraction

import numpy as np
import pytest

import oracle


def _exact_bias_corrections(beta1, beta2, step):
    b1 = Fraction(float(np.float32(beta1)))
    b2 = Fraction(float(np.float32(beta2)))
    return 1 - b1 ** step, 1 - b2 ** step


@pytest.mark.parametrize("step", [1, 2, 10, 100, 1000, 100000])
def test_bias_corrections_match_exact_rationals(step):
    cfg = oracle.config(step=step)
    s = oracle.scalars(cfg)
    bc1, bc2 = _exact_bias_corrections(0.9, 0.999, step)
    assert abs(Fraction(s.bc1) - bc1) <= abs(bc1) * Fraction(1, 2 ** 48)
    assert abs(Fraction(s.bc2) - bc2) <= abs(bc2) * Fraction(1, 2 ** 44)  # 1 - x loses a few bits at small steps
    # step size lr / bc1 and 1/sqrt(bc2), each rounded once to fp32
    lr = Fraction(float(np.float32(1e-3)))
    assert s.step_size == np.float32(float(lr / bc1))
    want = np.float32(1.0 / np.sqrt(float(bc2)))
    assert abs(int(np.float32(s.inv_sqrt_bc2).view(np.uint32)) - int(want.view(np.uint32))) <= 1
    assert s.decay == np.float32(float(lr * Fraction(float(np.float32(0.01)))))
    assert s.omb1 == np.float32(float(1 - Fraction(float(np.float32(0.9)))))
    assert s.omb2 == np.float32(float(1 - Fraction(float(np.float32(0.999)))))


def test_printed_decimal_values_of_the_bias_corrections():
    """1 - 0.9^10, 1 - 0.999^10, 1 - 0.9^100, 1 - 0.999^100 to the digits a float32 beta allows."""
    s10 = oracle.scalars(oracle.config(step=10))
    s100 = oracle.scalars(oracle.config(step=100))
    assert s10.bc1 == pytest.approx(0.6513215599, rel=2e-7)
    assert s10.bc2 == pytest.approx(0.0099551198, rel=2e-5)   # float32(0.999) differs from 0.999 by 1.7e-8
    assert s100.bc1 == pytest.approx(0.9999734386, rel=1e-9)
    assert s100.bc2 == pytest.approx(0.0952078529, rel=2e-5)
    s1 = oracle.scalars(oracle.config(step=1))
    assert s1.bc1 == 1.0 - float(np.float32(0.9))
    assert s1.bc2 == 1.0 - float(np.float32(0.999))


def test_first_step_scalars_make_mhat_equal_g():
    # step 1: step_size * (1-b1) == lr and inv_sqrt_bc2^2 * (1-b2) == 1 up to fp32 rounding
    s = oracle.scalars(oracle.config(step=1))
    assert float(s.step_size) * float(s.omb1) == pytest.approx(1e-3, rel=3e-7)
    assert float(s.inv_sqrt_bc2) ** 2 * float(s.omb2) == pytest.approx(1.0, rel=3e-7)


def test_clip_and_gscale():
    cfg = oracle.config(step=10, loss_scale=65536.0, max_grad_norm=1.0)
    # sumsq chosen so that sqrt(sumsq)/65536 = 4 exactly
    s = oracle.scalars(cfg, sumsq=(4.0 * 65536.0) ** 2)
    assert s.norm == 4.0
    assert s.clip == 1.0 / (4.0 + 1e-6)
    assert s.gscale == np.float32(s.clip / 65536.0)
    # below the threshold nothing is clipped and gscale is exactly 1/loss_scale
    s = oracle.scalars(cfg, sumsq=(0.5 * 65536.0) ** 2)
    assert s.clip == 1.0 and s.gscale == np.float32(2.0 ** -16)
    # no norm given: clip is 1 whatever max_grad_norm says
    s = oracle.scalars(cfg)
    assert s.clip == 1.0
    # clipping off
    s = oracle.scalars(oracle.config(step=10, max_grad_norm=0.0), sumsq=1e12)
    assert s.clip == 1.0 and s.gscale == 1.0
    # Adam-with-L2 mode has no decoupled decay
    assert oracle.scalars(oracle.config(mode=oracle.MODE_ADAM_L2)).decay == 0.0


@pytest.mark.parametrize("bad", [dict(step=0), dict(loss_scale=0.0), dict(loss_scale=float("inf")),
                                 dict(beta1=1.0), dict(beta2=-0.1), dict(eps=-1.0), dict(mode=7),
                                 dict(loss_scale=float("nan"))])
def test_bad_configurations_are_rejected(bad):
    with pytest.raises(ValueError):
        oracle.scalars(oracle.config(**bad))
