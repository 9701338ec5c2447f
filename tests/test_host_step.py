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
