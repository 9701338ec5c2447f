"""Pins for the oracle's sum of squares and overflow flag."""
import math

import numpy as np
import pytest

import oracle


def _bf16_trunc(x):
    return (np.asarray(x, np.float32).view(np.uint32) >> 16).astype(np.uint16)


def test_constant_input_closed_form():
    for dt, bits, val in ((oracle.BF16, 0x3E80, 0.25), (oracle.FP16, 0x3400, 0.25)):
        g = np.full(1 << 16, bits, np.uint16)
        ss, flag = oracle.grad_sumsq([g], dt)
        assert ss == val * val * (1 << 16) and flag == 0
        norm, _ = oracle.grad_norm([g], dt, loss_scale=4.0)
        assert norm == 0.25 * 256 / 4.0


@pytest.mark.parametrize("dt", [oracle.BF16, oracle.FP16])
def test_random_input_against_exactly_rounded_sum(dt):
    rng = np.random.default_rng(21)
    x = rng.normal(0, 1e-3, 300_000).astype(np.float32) * (65536 if dt == oracle.FP16 else 1)
    g = x.astype(np.float16).view(np.uint16) if dt == oracle.FP16 else _bf16_trunc(x)
    wide = oracle.widen(g, dt).astype(np.float64)
    want = math.fsum((wide * wide).tolist())       # squares exact in double; fsum rounds once
    ss, flag = oracle.grad_sumsq([g[:100_000], g[100_000:100_007], g[100_007:]], dt)
    assert flag == 0
    assert abs(ss - want) <= 2 * np.spacing(want)


def test_statistical_norm_of_unit_variance_gradients():
    # gradients N(0, 1e-3) over N elements: norm ~ 1e-3 sqrt(N)
    import zi_synth
    n = 1 << 20
    g = np.empty(n, np.uint16)
    zi_synth.fill_normal_lp(g, n, 99, zi_synth.STREAM_G, zi_synth.BF16, std=1e-3)
    norm, flag = oracle.grad_norm([g], oracle.BF16)
    assert flag == 0
    assert norm == pytest.approx(1e-3 * math.sqrt(n), rel=5e-3)


@pytest.mark.parametrize("dt,specials,maxfinite", [
    (oracle.BF16, [0x7F80, 0xFF80, 0x7FC0, 0x7F81, 0xFFFF], [0x7F7F, 0xFF7F]),
    (oracle.FP16, [0x7C00, 0xFC00, 0x7E00, 0x7C01, 0xFFFF], [0x7BFF, 0xFBFF])])
def test_flag(dt, specials, maxfinite):
    n = 1003
    base = _bf16_trunc(np.random.default_rng(1).normal(0, 1e-3, n)) if dt == oracle.BF16 else \
        np.random.default_rng(1).normal(0, 1e-3, n).astype(np.float16).view(np.uint16)
    assert oracle.grad_sumsq([base], dt)[1] == 0
    for s in specials:
        for pos in (0, n - 1, 501):
            g = base.copy()
            g[pos] = s
            assert oracle.grad_sumsq([g], dt)[1] == 1
            assert oracle.grad_sumsq([base, g], dt)[1] == 1
    for s in maxfinite:
        g = base.copy()
        g[17] = s
        ss, flag = oracle.grad_sumsq([g], dt)
        assert flag == 0 and math.isfinite(ss)     # a huge finite gradient is not an overflow


def test_empty():
    assert oracle.grad_sumsq([], oracle.BF16) == (0.0, 0)
    assert oracle.grad_sumsq([np.empty(0, np.uint16)], oracle.FP16) == (0.0, 0)
