"""The explicit host-CPU step (the paper's own placement of the offloaded step) against the oracle.  No GPU."""
import numpy as np
import pytest

import oracle
import paper_2104_07857_amd as zi
import zi_synth
from ulp import is_nan_lp


def _state(n, dt, seed):
    spec = zi_synth.StateSpec(seed, dt, g_std=1e-3 if dt == zi.ZI_BF16 else 65.536)
    p = np.empty(n, np.float32); m = np.empty(n, np.float32); v = np.empty(n, np.float32)
    g = np.empty(n, np.uint16)
    spec.fill_p(p, n); spec.fill_m(m, n); spec.fill_v(v, n); spec.fill_g(g, n)
    return p, m, v, g


def _same_bits(a, b):
    na, nb = np.isnan(a), np.isnan(b)
    return np.array_equal(na, nb) and np.array_equal(a.view(np.uint32)[~na], b.view(np.uint32)[~nb])


@pytest.mark.parametrize("dt", [zi.ZI_BF16, zi.ZI_FP16])
@pytest.mark.parametrize("mode", [zi.ZI_MODE_ADAMW, zi.ZI_MODE_ADAM_L2])
@pytest.mark.parametrize("n,threads", [(0, 1), (1, 1), (7, 2), (8, 1), (1001, 3), ((1 << 18) + 5, 2), (700_001, 5)])
def test_bit_identical_to_the_oracle(n, threads, mode, dt):
    p, m, v, g = _state(n, dt, 100 + n)
    if n > 20:   # awkward parameters: NaN, inf, fp16-subnormal, fp16-overflow, -0, fp32 subnormal
        p[5:11] = [np.nan, np.inf, 3e-5, 1e5, -0.0, 1e-41]
        v[11] = 1e-42
        g[12] = 0
    kw = dict(step=10, loss_scale=1.0 if dt == zi.ZI_BF16 else 65536.0, max_grad_norm=0.05, mode=mode)
    pe, me, ve = p.copy(), m.copy(), v.copy()
    lpe = np.zeros(n, np.uint16)
    ss, fl = oracle.grad_sumsq([g], dt)
    oracle.adamw(pe, me, ve, g, lpe, dt, oracle.config(**kw), ss, fl)
    lp = np.zeros(n, np.uint16)
    tl = [(p, m, v, g, lp, n)]
    r = zi.zi_host_grad_norm(tl, dt, kw["loss_scale"], threads)
    assert r.found_inf == fl == 0 and abs(r.sumsq - ss) <= 1e-12 * max(ss, 1e-300)
    assert zi.zi_host_adamw_step(tl, dt, zi.make_config(**kw), r, threads) == zi.ZI_OK
    assert _same_bits(pe, p) and _same_bits(me, m) and _same_bits(ve, v)
    nan = is_nan_lp(lpe, dt)
    assert np.array_equal(nan, is_nan_lp(lp, dt)) and np.array_equal(lpe[~nan], lp[~nan])


def test_norm_does_not_depend_on_the_thread_count_and_flags_are_exact():
    dt = zi.ZI_FP16
    gs = [_state(n, dt, 7 + i)[3] for i, n in enumerate([(1 << 19) + 3, 0, 77, 300_000])]
    tl = [(None, None, None, g, None, g.size) for g in gs]
    ref = zi.zi_host_grad_norm(tl, dt, 4.0, 1)
    want, _ = oracle.grad_sumsq(gs, dt)
    assert abs(ref.sumsq - want) <= 1e-12 * want and ref.norm == np.sqrt(ref.sumsq) / 4.0
    for th in (2, 3, 8):
        r = zi.zi_host_grad_norm(tl, dt, 4.0, th)
        assert r.sumsq == ref.sumsq and r.found_inf == 0
    for special in (0x7C00, 0xFC00, 0x7E00, 0xFFFF):
        for idx, pos in ((0, 0), (0, (1 << 19) + 2), (2, 76), (3, 12345)):
            saved = gs[idx][pos]
            gs[idx][pos] = special
            assert zi.zi_host_grad_norm(tl, dt, 4.0, 3).found_inf == 1
            gs[idx][pos] = saved
    gs[0][5] = 0x7BFF                 # largest finite fp16 is not an overflow
    assert zi.zi_host_grad_norm(tl, dt, 4.0, 3).found_inf == 0


def test_overflow_skips_and_arguments_are_checked():
    n = 1000
    p, m, v, g = _state(n, zi.ZI_BF16, 3)
    lp = np.zeros(n, np.uint16)
    g[17] = 0x7F80
    tl = [(p, m, v, g, lp, n)]
    r = zi.zi_host_grad_norm(tl, zi.ZI_BF16, 1.0, 2)
    assert r.found_inf == 1
    before = [a.copy() for a in (p, m, v)]
    assert zi.zi_host_adamw_step(tl, zi.ZI_BF16, zi.make_config(step=3), r, 2) == zi.ZI_SKIPPED_OVERFLOW
    assert all(np.array_equal(a.view(np.uint32), b.view(np.uint32)) for a, b in zip(before, (p, m, v)))
    assert not lp.any()
    for bad in (dict(step=0), dict(beta1=1.0), dict(eps=-1.0), dict(loss_scale=0.0), dict(mode=9)):
        with pytest.raises(zi.ZiError) as e:
            zi.zi_host_adamw_step(tl, zi.ZI_BF16, zi.make_config(**bad), None, 1)
        assert e.value.status == zi.ZI_ERR_INVALID_ARG
    with pytest.raises(zi.ZiError):
        zi.zi_host_adamw_step(tl, zi.ZI_BF16, zi.make_config(), None, 0)
    with pytest.raises(zi.ZiError):
        zi.zi_host_adamw_step([(p, None, v, g, lp, n)], zi.ZI_BF16, zi.make_config(), None, 1)
    with pytest.raises(zi.ZiError) as e:
        zi.zi_host_adamw_step([(p.ctypes.data + 1, m, v, g, lp, 8)], zi.ZI_BF16, zi.make_config(), None, 1)
    assert e.value.status == zi.ZI_ERR_ALIGNMENT
    with pytest.raises(zi.ZiError):
        zi.zi_host_grad_norm(tl, 5, 1.0, 1)
    with pytest.raises(zi.ZiError):
        zi.zi_host_grad_norm(tl, zi.ZI_BF16, -1.0, 1)


@pytest.mark.parametrize("dt", [zi.ZI_BF16, zi.ZI_FP16])
@pytest.mark.parametrize("mode", [zi.ZI_MODE_ADAMW, zi.ZI_MODE_ADAM_L2])
def test_every_short_length_and_every_tail(dt, mode):
    """n = 0..17 and 8k + r: the padded last group runs the same eight-lane routine as the body, writes
    exactly n elements (the bytes behind every array stay as they were) and agrees with the oracle."""
    kw = dict(step=7, loss_scale=1.0 if dt == zi.ZI_BF16 else 1024.0, max_grad_norm=0.0, mode=mode, eps=0.0)
    for n in list(range(0, 18)) + [64 + r for r in range(8)]:
        p, m, v, g = _state(n + 8, dt, 900 + n)
        v[:] = np.abs(v) + np.float32(1e-12)                   # eps = 0: keep the denominator away from zero
        lp = np.full(n + 8, 0xABCD, np.uint16)
        guard = [a[n:].copy() for a in (p, m, v, lp)]
        pe, me, ve, lpe = p[:n].copy(), m[:n].copy(), v[:n].copy(), np.zeros(n, np.uint16)
        oracle.adamw(pe, me, ve, g[:n].copy(), lpe, dt, oracle.config(**kw), None, 0)
        assert zi.zi_host_adamw_step([(p, m, v, g, lp, n)], dt, zi.make_config(**kw), None, 2) == zi.ZI_OK
        assert _same_bits(pe, p[:n]) and _same_bits(me, m[:n]) and _same_bits(ve, v[:n]), n
        assert np.array_equal(lpe, lp[:n]), n
        for a, b in zip(guard, (p, m, v, lp)):
            assert np.array_equal(a.view(np.uint8), b[n:].view(np.uint8)), f"n={n}: wrote past the end"
        r = zi.zi_host_grad_norm([(None, None, None, g, None, n)], dt, 1.0, 1)
        want, _ = oracle.grad_sumsq([g[:n].copy()], dt)
        assert abs(r.sumsq - want) <= 1e-12 * max(want, 1e-300)


@pytest.mark.parametrize("dt", [zi.ZI_BF16, zi.ZI_FP16])
@pytest.mark.parametrize("mode", [zi.ZI_MODE_ADAMW, zi.ZI_MODE_ADAM_L2])
def test_pinned_to_exact_rational_arithmetic_not_only_to_the_oracle(dt, mode):
    """Every operation of the sequence evaluated exactly and rounded once (the model of
    test_oracle_exact_rounding.py): the vector code neither contracts, splits nor reorders anything."""
    from test_oracle_exact_rounding import F, _bits, _cases, exact_step
    n = 203                                                    # 25 full groups and a tail of 3
    p, m, v, g = _cases(dt, n, seed=77 + dt + 5 * mode)
    kw = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, step=10, loss_scale=3.7,
              max_grad_norm=0.01, mode=mode)
    ocfg = oracle.config(**kw)
    sumsq, flag = oracle.grad_sumsq([g], dt)
    s = oracle.scalars(ocfg, sumsq)
    gw = oracle.widen(g, dt)
    p0, m0, v0 = p.copy(), m.copy(), v.copy()
    r = zi.zi_host_grad_norm([(None, None, None, g, None, n)], dt, kw["loss_scale"], 1)
    assert zi.zi_host_adamw_step([(p, m, v, g, None, n)], dt, zi.make_config(**kw), r, 1) == zi.ZI_OK
    for i in range(n):
        p1, m1, v1 = exact_step(F(p0[i]), F(m0[i]), F(v0[i]), F(gw[i]), s, ocfg)
        got = tuple(int(a[i].view(np.uint32)) for a in (p, m, v))
        got = tuple(b & 0x7FFFFFFF if (b & 0x7FFFFFFF) == 0 else b for b in got)
        assert got == (_bits(p1), _bits(m1), _bits(v1)), f"element {i}"


def test_low_precision_copy_against_library_converters():
    """The copy the host step writes, against numpy's (fp16) and torch's (bf16) own conversions of the
    stored p': ties to even, subnormals, overflow to inf, NaN stays NaN."""
    import torch
    rng = np.random.default_rng(11)
    n = 4099
    base = np.concatenate([rng.normal(0, 1, n - 40).astype(np.float32) * np.float32(10.0) ** rng.integers(-8, 5, n - 40).astype(np.float32),
                           np.float32([1.00390625, 1.01171875, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 65504, 65520, 65519.99,
                                       6e-8, 2.98e-8, 2.9802322e-8, 3e-8, 1e-45, 3.3895314e38, 3.4e38, 1e30, -1e30,
                                       np.nan, -1.5, 0.0, 5.9604645e-8] * 2)])
    for dt in (zi.ZI_BF16, zi.ZI_FP16):
        p = base.copy()
        m = np.zeros(n, np.float32); v = np.zeros(n, np.float32); g = np.zeros(n, np.uint16)
        lp = np.zeros(n, np.uint16)
        # zero gradient, zero moments, no decay: p' = p exactly, so lp = cast(p)
        cfg = zi.make_config(lr=1e-3, weight_decay=0.0, step=1, eps=1e-8)
        assert zi.zi_host_adamw_step([(p, m, v, g, lp, n)], dt, cfg, None, 1) == zi.ZI_OK
        assert _same_bits(p, base)
        if dt == zi.ZI_FP16:
            with np.errstate(over="ignore"):
                want = base.astype(np.float16).view(np.uint16)
        else:
            want = torch.from_numpy(base).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        nan = np.isnan(base)
        assert np.array_equal(lp[~nan], want[~nan])
        assert is_nan_lp(lp, dt)[nan].all()


def test_overlapping_arrays_are_refused():
    n = 64
    buf = np.zeros(4 * n, np.float32)
    g = np.zeros(n, np.uint16); lp = np.zeros(n, np.uint16)
    cfg = zi.make_config()
    for step in (zi.zi_host_adamw_step, ):
        with pytest.raises(zi.ZiError) as e:            # m starts inside p
            step([(buf[0:n], buf[n // 2:n // 2 + n], buf[2 * n:3 * n], g, lp, n)], zi.ZI_BF16, cfg, None, 1)
        assert e.value.status == zi.ZI_ERR_INVALID_ARG and "overlap" in e.value.message
        with pytest.raises(zi.ZiError):                 # the copy lands inside v
            step([(buf[0:n], buf[n:2 * n], buf[2 * n:3 * n], g, buf[2 * n:].view(np.uint16)[7:], n)], zi.ZI_BF16, cfg, None, 1)
        with pytest.raises(zi.ZiError):                 # g and the copy share a byte
            both = np.zeros(2 * n, np.uint16)
            step([(buf[0:n], buf[n:2 * n], buf[2 * n:3 * n], both[:n], both[n - 1:], n)], zi.ZI_BF16, cfg, None, 1)
    assert not buf.any()
    # adjacent is fine
    assert zi.zi_host_adamw_step([(buf[0:n], buf[n:2 * n], buf[2 * n:3 * n], g, lp, n)], zi.ZI_BF16, cfg, None, 1) == 0
