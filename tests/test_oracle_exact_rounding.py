"""Pin of the oracle's rounding behaviour: every element operation is one correctly rounded binary32
operation, fused only where a fused multiply-add is written.

The other pins bound the oracle against the textbook definition in extended precision; they cannot see
whether the C compiler contracted a multiply and an add that were written apart, split one that was
written fused, or kept excess precision.  Here each operation of the sequence is evaluated exactly in
rational arithmetic (`fractions.Fraction`, integer square root) and rounded once to binary32 by a
rounding routine written for this test (nearest, ties to even, gradual underflow); the oracle must agree
bit for bit.  The per-step scalars are taken from the oracle's own scalar routine, which the scalar
pins cover, so this test isolates the element loop.
"""
from fractions import Fraction
from math import isqrt

import numpy as np
import pytest

import oracle


def round_f32(q: Fraction) -> Fraction:
    """The binary32 value nearest to q (ties to even, subnormals kept); q stays below the overflow range."""
    if q == 0:
        return Fraction(0)
    sign = -1 if q < 0 else 1
    a = abs(q)
    e = a.numerator.bit_length() - a.denominator.bit_length()      # floor(log2 a) or one more
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    ulp = Fraction(2) ** (max(e, -126) - 23)
    scaled = a / ulp
    n = scaled.numerator // scaled.denominator
    rem = scaled - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and n % 2 == 1):
        n += 1
    r = n * ulp
    assert r < Fraction(2) ** 128
    return sign * r


def sqrt_f32(v: Fraction) -> Fraction:
    """Correctly rounded binary32 square root of a non-negative binary32 value.  The root is taken to
    200 fractional bits first; the root of a 24-bit number cannot lie that close to a rounding boundary."""
    assert v >= 0
    k = 200
    t = isqrt((v.numerator << (2 * k)) // v.denominator)
    if t * t * v.denominator == v.numerator << (2 * k):
        return round_f32(Fraction(t, 1 << k))                      # exact root
    return round_f32(Fraction(2 * t + 1, 1 << (k + 1)))            # strictly between t and t+1: same rounding


def F(x) -> Fraction:
    return Fraction(float(np.float32(x)))


def exact_step(p, m, v, g, s, cfg):
    """The element sequence with every operation rounded once.  s: the oracle's scalars."""
    beta1, beta2, eps, wd = F(cfg.beta1), F(cfg.beta2), F(cfg.eps), F(cfg.weight_decay)
    omb1, omb2, step_size, isb, decay, gscale = (F(s.omb1), F(s.omb2), F(s.step_size), F(s.inv_sqrt_bc2),
                                                 F(s.decay), F(s.gscale))
    gi = round_f32(g * gscale)
    if cfg.mode == oracle.MODE_ADAM_L2:
        gi = round_f32(wd * p + gi)                                 # fused
    m1 = round_f32(beta1 * m + round_f32(omb1 * gi))                # fma(beta1, m, omb1*g)
    v1 = round_f32(beta2 * v + round_f32(omb2 * round_f32(gi * gi)))
    d = round_f32(sqrt_f32(v1) * isb + eps)
    q = round_f32(m1 / d)
    pd = round_f32(-decay * p + p)
    p1 = round_f32(-step_size * q + pd)
    return p1, m1, v1


def _bits(x: Fraction) -> int:
    return int(np.float32(float(x)).view(np.uint32))


def _cases(dtype, n, seed):
    rng = np.random.default_rng(seed)
    p = rng.normal(0, 0.02, n).astype(np.float32)
    m = rng.normal(0, 1e-4, n).astype(np.float32)
    v = np.abs(rng.normal(0, 1e-6, n)).astype(np.float32)
    gf = rng.normal(0, 1e-3, n).astype(np.float32)
    # values that exercise gradual underflow, exact zeros and cancellation
    m[:8] = np.float32([1e-40, -3e-42, 0, 1e-38, -1e-39, 2e-45, 0, 1e-30])
    v[8:16] = np.float32([0, 1e-44, 1e-40, 3e-39, 0, 1e-38, 1e-20, 1e-45])
    gf[16:24] = np.float32([0, 1e-30, -1e-30, 1e-20, 0, 6e-8, -6e-8, 1.0])
    p[24:28] = np.float32([0, 1e-40, -1e-38, 1e3])
    g = oracle.cast(gf, dtype)
    return p, m, v, g


@pytest.mark.parametrize("dtype", [oracle.BF16, oracle.FP16])
@pytest.mark.parametrize("mode", [oracle.MODE_ADAMW, oracle.MODE_ADAM_L2])
@pytest.mark.parametrize("step,loss_scale,max_norm", [(1, 1.0, 0.0), (10, 1.0, 0.0), (1000, 3.7, 0.01)])
def test_element_loop_is_correctly_rounded_operation_by_operation(dtype, mode, step, loss_scale, max_norm):
    n = 400
    p, m, v, g = _cases(dtype, n, seed=step * 7 + dtype + 3 * mode)
    cfg = oracle.config(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, step=step,
                        loss_scale=loss_scale, max_grad_norm=max_norm, mode=mode)
    sumsq = None
    if max_norm > 0:
        sumsq, flag = oracle.grad_sumsq([g], dtype)
        assert flag == 0
    s = oracle.scalars(cfg, sumsq)
    if max_norm > 0:
        assert s.clip < 1.0
    gw = oracle.widen(g, dtype)
    po, mo, vo = p.copy(), m.copy(), v.copy()
    assert oracle.adamw(po, mo, vo, g, None, dtype, cfg, sumsq, 0) == 0
    for i in range(n):
        p1, m1, v1 = exact_step(F(p[i]), F(m[i]), F(v[i]), F(gw[i]), s, cfg)
        got = (int(po[i].view(np.uint32)), int(mo[i].view(np.uint32)), int(vo[i].view(np.uint32)))
        want = (_bits(p1), _bits(m1), _bits(v1))
        # +0 and -0 are one value to the rational model: compare them as equal
        got = tuple(b & 0x7FFFFFFF if (b & 0x7FFFFFFF) == 0 else b for b in got)
        assert got == want, f"element {i}: p,m,v bits {got} != {want} (inputs {p[i]!r} {m[i]!r} {v[i]!r} {gw[i]!r})"


def test_the_rounding_routine_itself():
    """round_f32 against numpy's conversion on values whose rounding is known, so that the routine above is
    not trusted blindly: exact values, ties to even, subnormals, the smallest subnormal's half."""
    one = Fraction(1)
    eps = Fraction(2) ** -23
    assert round_f32(one + eps / 2) == one                           # tie -> even (1.0)
    assert round_f32(one + eps + eps / 2) == one + 2 * eps           # tie -> even (odd neighbour skipped)
    assert round_f32(one + eps / 2 + Fraction(2) ** -60) == one + eps
    assert round_f32(Fraction(2) ** -150) == 0                       # half of the smallest subnormal: tie -> 0
    assert round_f32(Fraction(2) ** -150 + Fraction(2) ** -200) == Fraction(2) ** -149
    assert round_f32(Fraction(3, 2) * Fraction(2) ** -149) == Fraction(2) ** -148
    rng = np.random.default_rng(5)
    for x in rng.normal(0, 1, 200).astype(np.float64) * 10.0 ** rng.integers(-44, 30, 200):
        assert float(round_f32(Fraction(float(x)))) == float(np.float32(x))
    for x in (0.0, 2.0, 4.0, 0.25, 1e-40, 2.25, 3.0, 1e-10):
        v = Fraction(float(np.float32(x)))
        assert float(sqrt_f32(v)) == float(np.sqrt(np.float32(x), dtype=np.float32))
