"""Pins for the oracle's update: closed forms, invariants, textbook evaluation in extended precision."""
import numpy as np
import pytest

import oracle
from ulp import ulp_dist_f32

LD = np.longdouble


def _bf16_trunc(x):
    return (np.asarray(x, np.float32).view(np.uint32) >> 16).astype(np.uint16)


def _state(n, seed=0, step1=False):
    rng = np.random.default_rng(seed)
    p = rng.normal(0, 0.02, n).astype(np.float32)
    g = _bf16_trunc(rng.normal(0, 1e-3, n))
    if step1:
        m = np.zeros(n, np.float32)
        v = np.zeros(n, np.float32)
    else:
        m = rng.normal(0, 1e-4, n).astype(np.float32)
        v = np.abs(rng.normal(0, 1e-6, n)).astype(np.float32)
    return p, m, v, g


def textbook(p, m, v, g_lp, dtype, cfg, sumsq=None, mutate=None):
    """Adam / AdamW as the standard definition writes it, in extended precision.

    m' = b1 m + (1-b1) g;  v' = b2 v + (1-b2) g^2;  mhat = m'/(1-b1^t);  vhat = v'/(1-b2^t);
    p' = p - lr wd p - lr mhat / (sqrt(vhat) + eps), g being the unscaled, clipped gradient.
    mutate plants one mistake, to show that the comparison below has the power to see it.
    """
    f = lambda x: LD(float(np.float32(x)))
    lr, b1, b2, eps, wd = f(cfg.lr), f(cfg.beta1), f(cfg.beta2), f(cfg.eps), f(cfg.weight_decay)
    t = int(cfg.step)
    ls = f(cfg.loss_scale)
    clip = LD(1)
    if sumsq is not None:
        norm = np.sqrt(LD(sumsq)) / ls
        if cfg.max_grad_norm > 0 and norm + LD(1e-6) > f(cfg.max_grad_norm):
            clip = f(cfg.max_grad_norm) / (norm + LD(1e-6))
    g = oracle.widen(g_lp, dtype).astype(LD) * (clip / ls)
    p, m, v = p.astype(LD), m.astype(LD), v.astype(LD)
    if cfg.mode == oracle.MODE_ADAM_L2:
        g = g + wd * p
    m1 = b1 * m + (1 - b1) * g
    v1 = b2 * v + (1 - b2) * g * g
    bc1 = 1 - b1 ** t
    bc2 = 1 - b2 ** t
    if mutate == "no_bias_correction":
        bc1 = bc2 = LD(1)
    mhat, vhat = m1 / bc1, v1 / bc2
    denom = np.sqrt(vhat) + eps
    if mutate == "eps_inside_sqrt":
        denom = np.sqrt(vhat + eps)
    decay = lr * wd * p if cfg.mode == oracle.MODE_ADAMW else 0
    if mutate == "decay_dropped":
        decay = 0
    upd = lr * mhat / denom
    if mutate == "wrong_sign":
        upd = -upd
    if mutate == "m_v_swapped_betas":
        m1 = b2 * m + (1 - b2) * g
    p1 = p - decay - upd
    return p1, m1, v1


def error_bounds(p, m, v, g_lp, dtype, cfg, sumsq=None):
    """A-priori rounding-error bounds of a binary32 evaluation with about ten roundings.

    Condition-aware: where b1 m and (1-b1) g cancel, the bound stays relative to the operands.
    """
    u = LD(2.0) ** -24
    p1, m1, v1 = textbook(p, m, v, g_lp, dtype, cfg, sumsq)
    f = lambda x: LD(float(np.float32(x)))
    b1, b2, eps, lr, wd = f(cfg.beta1), f(cfg.beta2), f(cfg.eps), f(cfg.lr), f(cfg.weight_decay)
    ls = f(cfg.loss_scale)
    clip = LD(1)
    if sumsq is not None:
        norm = np.sqrt(LD(sumsq)) / ls
        if cfg.max_grad_norm > 0 and norm + LD(1e-6) > f(cfg.max_grad_norm):
            clip = f(cfg.max_grad_norm) / (norm + LD(1e-6))
    g = oracle.widen(g_lp, dtype).astype(LD) * (clip / ls)
    pl, ml, vl = p.astype(LD), m.astype(LD), v.astype(LD)
    if cfg.mode == oracle.MODE_ADAM_L2:
        g_abs = np.abs(g) + np.abs(wd * pl)
        dg = 3 * u * g_abs
    else:
        g_abs = np.abs(g)
        dg = 2 * u * g_abs
    tiny = LD(2.0) ** -149
    dm = 3 * u * (np.abs(b1 * ml) + (1 - b1) * g_abs) + (1 - b1) * dg + tiny
    dv = 4 * u * (np.abs(b2 * vl) + (1 - b2) * g_abs ** 2) + (1 - b2) * 2 * g_abs * dg + tiny
    bc1 = 1 - b1 ** int(cfg.step)
    bc2 = 1 - b2 ** int(cfg.step)
    isb = 1 / np.sqrt(bc2)
    sq = np.sqrt(np.abs(v1))
    dsq = np.sqrt(np.abs(v1) + dv) - np.sqrt(np.maximum(np.abs(v1) - dv, 0)) + u * sq
    d = sq * isb + eps
    dd = dsq * isb + 2 * u * d
    q = m1 / d
    dq = dm / d + np.abs(q) * dd / d + u * np.abs(q)
    step = lr / bc1
    dp = 2 * u * (np.abs(pl) + np.abs(lr * wd * pl)) + step * dq + 3 * u * np.abs(step * q)
    return (p1, m1, v1), (dp, dm, dv)


def _run_oracle(p, m, v, g, dtype, cfg, sumsq=None, found_inf=0):
    p, m, v = p.copy(), m.copy(), v.copy()
    lp = np.zeros(p.size, np.uint16)
    rc = oracle.adamw(p, m, v, g, lp, dtype, cfg, sumsq, found_inf)
    return p, m, v, lp, rc


def _adversarial(n=4096, seed=11):
    rng = np.random.default_rng(seed)
    p, m, v, g = _state(n, seed)
    gf = oracle.widen(g, oracle.BF16)
    # cancellation in the first moment: b1 m ~ -(1-b1) g
    m[:512] = (-(1 - 0.9) / 0.9 * gf[:512] * (1 + rng.normal(0, 1e-4, 512))).astype(np.float32)
    g[512:600] = 0                      # zero gradients
    m[600:700] = 0
    v[700:800] = 0
    g[800:830] = _bf16_trunc(rng.normal(0, 1e-18, 30))   # squares underflow towards fp32 subnormals
    v[800:830] = 0
    g[830:860] = _bf16_trunc(rng.normal(0, 1e3, 30))     # huge gradients
    p[860:880] = 0
    p[880:890] = -0.0
    p[890:900] = rng.normal(0, 1e-30, 10).astype(np.float32)
    return p, m, v, g


@pytest.mark.parametrize("mode", [oracle.MODE_ADAMW, oracle.MODE_ADAM_L2])
@pytest.mark.parametrize("step", [1, 10, 100, 12345])
def test_against_textbook_in_extended_precision(step, mode):
    for make in (lambda: _state(50_000, seed=step), _adversarial):
        p, m, v, g = make()
        cfg = oracle.config(step=step, mode=mode)
        (p1, m1, v1), (dp, dm, dv) = error_bounds(p, m, v, g, oracle.BF16, cfg)
        po, mo, vo, _, rc = _run_oracle(p, m, v, g, oracle.BF16, cfg)
        assert rc == 0
        assert (np.abs(mo.astype(LD) - m1) <= dm).all()
        assert (np.abs(vo.astype(LD) - v1) <= dv).all()
        assert (np.abs(po.astype(LD) - p1) <= dp).all()


def test_against_textbook_with_loss_scale_and_clip_fp16():
    n = 30_000
    rng = np.random.default_rng(5)
    p, m, v, _ = _state(n, 5)
    g = (rng.normal(0, 1e-3, n) * 65536).astype(np.float16).view(np.uint16)
    cfg = oracle.config(step=10, loss_scale=65536.0, max_grad_norm=0.05)
    sumsq, flag = oracle.grad_sumsq([g], oracle.FP16)
    assert flag == 0
    s = oracle.scalars(cfg, sumsq)
    assert s.clip < 1.0                                  # the clip branch is taken
    (p1, m1, v1), (dp, dm, dv) = error_bounds(p, m, v, g, oracle.FP16, cfg, sumsq)
    po, mo, vo, lp, _ = _run_oracle(p, m, v, g, oracle.FP16, cfg, sumsq)
    assert (np.abs(mo.astype(LD) - m1) <= dm).all()
    assert (np.abs(vo.astype(LD) - v1) <= dv).all()
    assert (np.abs(po.astype(LD) - p1) <= dp).all()
    assert np.array_equal(lp, po.astype(np.float16).view(np.uint16))   # copy = RNE cast of the stored fp32 p'


@pytest.mark.parametrize("mutation", ["no_bias_correction", "eps_inside_sqrt", "decay_dropped", "wrong_sign",
                                      "m_v_swapped_betas"])
def test_the_textbook_comparison_sees_planted_mistakes(mutation):
    """Each plausible mistake, planted in the reference formula, lands far outside the bounds."""
    p, m, v, g = _state(20_000, seed=2)
    # eps = 1e-4 is comparable to sqrt(vhat) ~ 1e-2, so that its placement matters above rounding level
    cfg = oracle.config(step=10, eps=1e-4)
    (_, _, _), (dp, dm, dv) = error_bounds(p, m, v, g, oracle.BF16, cfg)
    pm, mm, vm = textbook(p, m, v, g, oracle.BF16, cfg, mutate=mutation)
    po, mo, vo, _, _ = _run_oracle(p, m, v, g, oracle.BF16, cfg)
    bad_p = (np.abs(po.astype(LD) - pm) > dp).mean()
    bad_m = (np.abs(mo.astype(LD) - mm) > dm).mean()
    assert max(bad_p, bad_m) > 0.9


def test_first_step_closed_form():
    """m = v = 0, step 1, no decay: p' - p = -lr g / (|g| + eps), about -lr sign(g)."""
    n = 1 << 16
    p, m, v, g = _state(n, seed=1, step1=True)
    cfg = oracle.config(step=1, weight_decay=0.0)
    po, mo, vo, _, _ = _run_oracle(p, m, v, g, oracle.BF16, cfg)
    gf = oracle.widen(g, oracle.BF16).astype(np.float64)
    lr, eps = float(np.float32(1e-3)), float(np.float32(1e-8))
    want = p.astype(np.float64) - lr * gf / (np.abs(gf) + eps)
    # rounding of p' itself (half an ulp of p) plus a few ulp of lr
    tol = np.spacing(np.abs(want).astype(np.float32)).astype(np.float64) * 0.5 + 4 * np.spacing(np.float32(lr))
    assert (np.abs(po.astype(np.float64) - want) <= tol).all()
    nz = gf != 0
    assert (np.sign(po.astype(np.float64) - p)[nz] == -np.sign(gf)[nz]).all()
    # |g| ~ 1e-3 >> eps: the move is lr to within 1e-4 relative for typical elements
    typical = np.abs(gf) > 1e-4
    moved = np.abs(po.astype(np.float64) - p.astype(np.float64))[typical]
    assert np.allclose(moved, lr, rtol=2e-4, atol=2 * np.spacing(np.float32(0.1)))
    # first moments are (1-b1) g and (1-b2) g^2
    assert np.allclose(mo, (1 - float(np.float32(0.9))) * gf, rtol=3e-7, atol=1e-45)
    assert np.allclose(vo, (1 - float(np.float32(0.999))) * gf * gf, rtol=3e-7, atol=1e-45)


def test_first_step_closed_form_with_decay():
    n = 4096
    p, m, v, g = _state(n, seed=4, step1=True)
    cfg = oracle.config(step=1, weight_decay=0.01)
    po, *_ = _run_oracle(p, m, v, g, oracle.BF16, cfg)
    gf = oracle.widen(g, oracle.BF16).astype(np.float64)
    lr, eps, wd = float(np.float32(1e-3)), float(np.float32(1e-8)), float(np.float32(0.01))
    want = p.astype(np.float64) * (1 - lr * wd) - lr * gf / (np.abs(gf) + eps)
    # two roundings at the magnitude of p (the decayed parameter, then the result) plus a few ulp of lr
    mag = np.maximum(np.abs(want), np.abs(p.astype(np.float64))).astype(np.float32)
    tol = 1.5 * np.spacing(mag).astype(np.float64) + 4 * np.spacing(np.float32(lr))
    assert (np.abs(po.astype(np.float64) - want) <= tol).all()


def test_invariants():
    n = 10_000
    p, m, v, g = _state(n, seed=8)
    cfg = oracle.config(step=10)
    po, mo, vo, lp, _ = _run_oracle(p, m, v, g, oracle.BF16, cfg)
    assert (vo >= 0).all()
    assert not np.isnan(po).any()

    # zero gradient, zero momentum, no decay: p is untouched, bit for bit; a -0 parameter stays a zero
    # (its sign is not kept: p - 0*p evaluates (+0) + (-0) = +0 under round to nearest)
    z = np.zeros(n, np.uint16)
    p2 = p.copy(); p2[:10] = -0.0
    cfg0 = oracle.config(step=10, weight_decay=0.0)
    po, mo, vo, lp, _ = _run_oracle(p2, np.zeros(n, np.float32), v, z, oracle.BF16, cfg0)
    assert np.array_equal(po.view(np.uint32)[10:], p2.view(np.uint32)[10:])
    assert (po[:10] == 0).all()
    assert not mo.any()
    assert np.array_equal(lp, oracle.cast(po, oracle.BF16))

    # zero gradient, no decay, nonzero momentum: m' = fl(b1 m), p moves against sign(m)
    po, mo, vo, _, _ = _run_oracle(p, m, v, z, oracle.BF16, cfg0)
    assert np.array_equal(mo, (np.float32(0.9) * m).astype(np.float32))
    assert np.array_equal(vo, (np.float32(0.999) * v).astype(np.float32))
    big = np.abs(m) > 1e-6
    assert (np.sign(po.astype(np.float64) - p)[big] == -np.sign(m)[big]).all()

    # decay only: p' = p - lr wd p with a single rounding
    po, *_ = _run_oracle(p, np.zeros(n, np.float32), v, z, oracle.BF16, oracle.config(step=10))
    decay = float(np.float32(float(np.float32(1e-3)) * float(np.float32(0.01))))
    want = (p.astype(np.float64) * (1 - decay)).astype(np.float32)
    assert np.array_equal(po, want)


def test_overflowed_step_changes_nothing():
    p, m, v, g = _state(5000, seed=9)
    g[1234] = 0x7F80  # +inf in bf16
    sumsq, flag = oracle.grad_sumsq([g], oracle.BF16)
    assert flag == 1
    po, mo, vo, lp, rc = _run_oracle(p, m, v, g, oracle.BF16, oracle.config(step=10), sumsq, flag)
    assert rc == 1
    assert np.array_equal(po.view(np.uint32), p.view(np.uint32))
    assert np.array_equal(mo.view(np.uint32), m.view(np.uint32))
    assert np.array_equal(vo.view(np.uint32), v.view(np.uint32))
    assert not lp.any()


@pytest.mark.parametrize("k", [0, 1, 7, 8, 1000, 4999, 5000])
def test_split_invariance(k):
    """The update is independent per element: stepping [0,k) and [k,n) apart equals stepping [0,n)."""
    n = 5000
    p, m, v, g = _state(n, seed=10)
    cfg = oracle.config(step=10)
    po, mo, vo, lp, _ = _run_oracle(p, m, v, g, oracle.BF16, cfg)
    pa, ma, va, la, _ = _run_oracle(p[:k], m[:k], v[:k], g[:k], oracle.BF16, cfg)
    pb, mb, vb, lb, _ = _run_oracle(p[k:], m[k:], v[k:], g[k:], oracle.BF16, cfg)
    assert np.array_equal(np.concatenate([pa, pb]).view(np.uint32), po.view(np.uint32))
    assert np.array_equal(np.concatenate([ma, mb]).view(np.uint32), mo.view(np.uint32))
    assert np.array_equal(np.concatenate([va, vb]).view(np.uint32), vo.view(np.uint32))
    assert np.array_equal(np.concatenate([la, lb]), lp)


@pytest.mark.parametrize("k", [1, 4, 16])
def test_power_of_two_loss_scale_is_invisible(k):
    """Gradients pre-multiplied by 2^k with loss_scale 2^k give the unscaled run, bit for bit."""
    n = 20_000
    rng = np.random.default_rng(12)
    p, m, v, _ = _state(n, 12)
    g32 = rng.normal(0, 1e-3, n).astype(np.float32)
    g = g32.astype(np.float16)
    # keep to values that stay normal fp16 numbers after scaling in both directions
    g = np.where(np.abs(g) < 2.0 ** -10, np.float16(2.0 ** -10), g).astype(np.float16)
    gs = (g.astype(np.float32) * np.float32(2.0 ** k)).astype(np.float16)
    assert np.array_equal(gs.astype(np.float32), g.astype(np.float32) * 2.0 ** k)
    a = _run_oracle(p, m, v, g.view(np.uint16), oracle.FP16, oracle.config(step=10))
    b = _run_oracle(p, m, v, gs.view(np.uint16), oracle.FP16, oracle.config(step=10, loss_scale=2.0 ** k))
    for x, y in zip(a[:4], b[:4]):
        assert np.array_equal(x, y)


def test_clip_closed_form_and_no_clip_below_threshold():
    """All-equal gradients c over N elements: norm = |c| sqrt(N), exactly, for powers of two / four."""
    n = 4096                      # sqrt = 64
    c = np.float32(0.5)
    g = np.full(n, _bf16_trunc(c), np.uint16)
    sumsq, flag = oracle.grad_sumsq([g], oracle.BF16)
    assert sumsq == 0.25 * n and flag == 0
    p, m, v, _ = _state(n, 13)
    cfg = oracle.config(step=10, max_grad_norm=1.0)
    s = oracle.scalars(cfg, sumsq)
    assert s.norm == 32.0 and s.clip == 1.0 / (32.0 + 1e-6)
    po, mo, vo, _, _ = _run_oracle(p, m, v, g, oracle.BF16, cfg, sumsq)
    # the clipped run equals an unclipped run on gradients scaled by the same fp32 factor
    gc = np.float32(s.gscale) * np.float32(0.5)
    want_m = (np.float32(0.9) * m.astype(np.float64) + float(np.float32(float(s.omb1) * float(gc)))).astype(np.float32)
    assert (ulp_dist_f32(mo, want_m) <= 1).all()
    # norm under the threshold: identical to the run without a norm
    cfg_hi = oracle.config(step=10, max_grad_norm=64.0)
    a = _run_oracle(p, m, v, g, oracle.BF16, cfg_hi, sumsq)
    b = _run_oracle(p, m, v, g, oracle.BF16, oracle.config(step=10))
    for x, y in zip(a[:4], b[:4]):
        assert np.array_equal(x, y)
