"""Parity of the HBM-resident fused AdamW step with the CPU oracle, element by element, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2104_07857_amd as zi
import zi_synth
from ulp import is_nan_lp
from gpu_util import (NormBuffers, compare_state, gen_numpy, oracle_cfg, progress, to_dev, to_np, zi_cfg)

pytestmark = pytest.mark.gpu

TILE = 512    # elements one workgroup covers


def _run_both(p, m, v, g, dt, ocfg, zcfg, with_lp=True, use_norm=False, offsets=None, norm_scale=None):
    """Steps numpy state through the oracle and through zi_adamw_step; returns (expected, got, info).
    norm_scale: loss scale handed to zi_grad_norm when it is to differ from the step's own."""
    n = p.size
    pe, me, ve = p.copy(), m.copy(), v.copy()
    lpe = np.zeros(n, np.uint16) if with_lp else None
    sumsq, flag = (None, 0)
    if use_norm:
        sumsq, flag = oracle.grad_sumsq([g], dt)
    rc = oracle.adamw(pe, me, ve, g, lpe, dt, ocfg, sumsq, flag)

    pad = 80
    off = offsets or (0, 0, 0, 0, 0)
    bufs = []
    for a, o in zip((p, m, v, g, np.zeros(n, np.uint16)), off):
        t = torch.zeros(n + pad, dtype=torch.float32 if a.dtype == np.float32 else torch.int16, device="cuda:0")
        t[o:o + n].copy_(to_dev(a))
        bufs.append(t)
    views = [b[o:o + n] for b, o in zip(bufs, off)]
    dp, dm, dv, dg, dlp = views
    nb = None
    if use_norm:
        nb = NormBuffers()
        zi.zi_grad_norm([(None, None, None, dg, None, n)], dt, norm_scale or ocfg.loss_scale, nb.out, nb.ws)
    st = zi.zi_adamw_step([(dp, dm, dv, dg, dlp if with_lp else None, n)], dt, zcfg,
                          None if nb is None else nb.out)
    assert st == zi.ZI_OK
    torch.cuda.synchronize()
    got = (to_np(dp), to_np(dm), to_np(dv), to_np(dlp) if with_lp else None)
    # nothing outside the views may have been touched
    for b, o, a in zip(bufs[:3], off[:3], (p, m, v)):
        assert not b[:o].any() and not b[o + n:].any()
    assert not bufs[4][:off[4]].any() and not bufs[4][off[4] + n:].any()
    return (pe, me, ve, lpe), got, dict(rc=rc, norm=nb.read() if nb else None, sumsq=sumsq, flag=flag)


def test_config0_first_step_one_mebi_elements():
    """Workload 0: 2^20 flat elements, bf16 gradients, m = v = 0, step 1, no loss scale."""
    w = zi_synth.workload("c0")
    n = w["numel"][0]
    p, m, v, g = gen_numpy(w["spec"], n)
    exp, got, _ = _run_both(p, m, v, g, zi.ZI_BF16, oracle_cfg(w), zi_cfg(w))
    rep = compare_state(exp, got, zi.ZI_BF16, "c0 ")
    progress("c0 parity: " + rep)
    assert not np.array_equal(got[0], p)       # the step did something


@pytest.mark.parametrize("dt", [zi.ZI_BF16, zi.ZI_FP16])
@pytest.mark.parametrize("n", [0, 1, 7, 8, 9, 15, 16, 17, TILE - 1, TILE, TILE + 1, 3 * TILE + 5, 100_003,
                               (1 << 20) + 13])
def test_sizes_spanning_tiles_and_ragged_tails(n, dt):
    w = zi_synth.workload("c1" if dt == zi.ZI_BF16 else "c3")
    spec = zi_synth.StateSpec(1234 + n, dt, g_std=w["spec"].g_std)
    p, m, v, g = gen_numpy(spec, n)
    ocfg, zcfg = oracle_cfg(w, loss_scale=1.0, max_grad_norm=0.0), zi_cfg(w, loss_scale=1.0, max_grad_norm=0.0)
    exp, got, _ = _run_both(p, m, v, g, dt, ocfg, zcfg)
    compare_state(exp, got, dt, f"n={n} ")


@pytest.mark.parametrize("mode", [zi.ZI_MODE_ADAMW, zi.ZI_MODE_ADAM_L2])
@pytest.mark.parametrize("step", [1, 10, 100, 100000])
def test_modes_and_steps(step, mode):
    n = 50_001
    w = zi_synth.workload("c1")
    p, m, v, g = gen_numpy(zi_synth.StateSpec(77 + step, zi.ZI_BF16), n)
    exp, got, _ = _run_both(p, m, v, g, zi.ZI_BF16, oracle_cfg(w, step=step, mode=mode),
                            zi_cfg(w, step=step, mode=mode))
    compare_state(exp, got, zi.ZI_BF16, f"step={step} mode={mode} ")


def test_without_low_precision_copy():
    n = 20_011
    w = zi_synth.workload("c1")
    p, m, v, g = gen_numpy(w["spec"], n)
    exp, got, _ = _run_both(p, m, v, g, zi.ZI_BF16, oracle_cfg(w), zi_cfg(w), with_lp=False)
    compare_state(exp, got, zi.ZI_BF16)


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5, 6, 7])
def test_common_misalignment(k):
    """All five arrays start k elements past an aligned address (a slice of a flat partition): the
    vector body then starts 64 - k elements in, on a 128-byte line of every array."""
    n = 3 * TILE + 11
    w = zi_synth.workload("c1")
    p, m, v, g = gen_numpy(zi_synth.StateSpec(500 + k, zi.ZI_BF16), n)
    exp, got, _ = _run_both(p, m, v, g, zi.ZI_BF16, oracle_cfg(w), zi_cfg(w), offsets=(k, k, k, k, k))
    compare_state(exp, got, zi.ZI_BF16, f"offset {k} ")


@pytest.mark.parametrize("offsets", [(1, 0, 0, 0, 0), (0, 0, 0, 1, 0), (0, 0, 0, 0, 3), (1, 2, 3, 5, 7),
                                     (4, 4, 4, 0, 0), (0, 0, 0, 4, 4), (0, 0, 0, 32, 32), (3, 3, 3, 35, 35),
                                     (31, 30, 29, 63, 1)])
def test_unrelated_misalignments(offsets):
    """Arrays with no common alignment: the lane vectors of some arrays are then only element-aligned."""
    n = 2 * TILE + 77
    w = zi_synth.workload("c1")
    p, m, v, g = gen_numpy(zi_synth.StateSpec(900 + sum(offsets), zi.ZI_BF16), n)
    exp, got, _ = _run_both(p, m, v, g, zi.ZI_BF16, oracle_cfg(w), zi_cfg(w), offsets=offsets)
    compare_state(exp, got, zi.ZI_BF16, f"offsets {offsets} ")


def test_adversarial_values():
    """Cancellation in the first moment, zero and huge gradients, zero / tiny / negative-zero parameters,
    variance in the fp32 subnormal range, fp16 copies that are subnormal or overflow."""
    n = 8192
    rng = np.random.default_rng(3)
    w = zi_synth.workload("c1")
    for dt in (zi.ZI_BF16, zi.ZI_FP16):
        p, m, v, g = gen_numpy(zi_synth.StateSpec(31, dt), n)
        gf = oracle.widen(g, dt)
        m[:512] = (-(0.1 / 0.9) * gf[:512] * (1 + rng.normal(0, 1e-4, 512))).astype(np.float32)
        g[512:600] = 0
        m[600:700] = 0
        v[700:800] = 0
        v[800:830] = 0
        g[800:830] = oracle.cast(rng.normal(0, 1e-18 if dt == zi.ZI_BF16 else 1e-7, 30).astype(np.float32), dt)
        g[830:860] = oracle.cast(rng.normal(0, 1e3, 30).astype(np.float32), dt)
        p[860:880] = 0
        p[880:890] = -0.0
        p[890:900] = rng.normal(0, 1e-30, 10).astype(np.float32)
        p[900:940] = rng.normal(0, 3e-5, 40).astype(np.float32)     # fp16 copy is subnormal
        p[940:960] = rng.normal(0, 1e5, 20).astype(np.float32)      # fp16 copy overflows to inf
        p[960:970] = rng.normal(0, 1e-41, 10).astype(np.float32)    # fp32 subnormal parameters
        v[970:980] = rng.uniform(0, 1e-42, 10).astype(np.float32)   # fp32 subnormal variance
        exp, got, _ = _run_both(p, m, v, g, dt, oracle_cfg(w), zi_cfg(w))
        compare_state(exp, got, dt, f"dt={dt} ")


def test_loss_scale_clip_and_overflow_skip_small():
    """Workload 3 in miniature: fp16 gradients scaled by 65536; run A plants +inf, run B clips to norm 1."""
    w = zi_synth.workload("c3")
    n = 300_007
    dt = zi.ZI_FP16
    p, m, v, g = gen_numpy(w["spec"], n)
    # run B (norm ~ 1e-3 sqrt(n) = 0.55 at this size, so the threshold is lowered to keep the clip active)
    over = dict(max_grad_norm=0.1)
    exp, got, info = _run_both(p, m, v, g, dt, oracle_cfg(w, **over), zi_cfg(w, **over), use_norm=True)
    sumsq, norm, flag = info["norm"]
    assert flag == 0 and info["flag"] == 0
    onorm = float(np.sqrt(info["sumsq"]) / 65536.0)
    assert abs(norm - onorm) <= 1e-6 * onorm
    assert abs(sumsq - info["sumsq"]) <= 1e-9 * info["sumsq"]
    assert onorm > 0.5 * 1e-3 * np.sqrt(n)
    progress("c3-small run B: " + compare_state(exp, got, dt, "run B ") + f"; norm {norm:.6f} vs {onorm:.6f}")
    assert oracle.scalars(oracle_cfg(w, **over), info["sumsq"]).clip < 0.2
    # run A: +inf at a seeded index -> nothing may change, not one bit
    j = zi_synth.pick_index(w["spec"].seed, 0x696E66, n)
    g2 = g.copy()
    g2[j] = 0x7C00
    exp, got, info = _run_both(p, m, v, g2, dt, oracle_cfg(w), zi_cfg(w), use_norm=True)
    assert info["rc"] == 1 and info["flag"] == 1 and info["norm"][2] == 1
    for a, b in zip((p, m, v), got[:3]):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    assert not got[3].any()


@pytest.mark.parametrize("max_norm", [0.05, 0.125])
@pytest.mark.parametrize("step_scale,norm_scale", [(65536.0, 65536.0), (65536.0, 1.0), (65536.0, 1024.0),
                                                   (1000.0, 1000.0), (1000.0, 65536.0), (3.0, 0.75)])
def test_clip_follows_the_steps_own_loss_scale_whatever_scale_the_reduction_was_given(step_scale, norm_scale,
                                                                                      max_norm):
    """The step takes the reduction's norm (and its 1 / (norm + 1e-6)) only when they were computed with the
    step's own loss scale and derives the norm from the sum of squares otherwise; a power-of-two loss scale or
    maximum norm is applied by an exact multiplication, any other by a division.  Every combination of these
    paths has to give the oracle's bits."""
    w = zi_synth.workload("c3")
    n = 70_001
    dt = zi.ZI_FP16
    spec = zi_synth.StateSpec(777, dt, g_std=w["spec"].g_std * step_scale / 65536.0)
    p, m, v, g = gen_numpy(spec, n)
    over = dict(loss_scale=step_scale, max_grad_norm=max_norm)
    exp, got, info = _run_both(p, m, v, g, dt, oracle_cfg(w, **over), zi_cfg(w, **over), use_norm=True,
                               norm_scale=norm_scale)
    assert info["flag"] == 0 and info["norm"][2] == 0
    assert oracle.scalars(oracle_cfg(w, **over), info["sumsq"]).clip < 0.6      # the clip is active
    want_norm = float(np.sqrt(info["sumsq"]) / norm_scale)
    assert abs(info["norm"][1] - want_norm) <= 1e-6 * want_norm                 # the reduction used its own scale
    progress(f"clip to {max_norm} with step scale {step_scale}, reduction scale {norm_scale}: "
             + compare_state(exp, got, dt, ""))


def test_power_of_two_loss_scale_is_invisible_on_the_device():
    n = 40_000
    rng = np.random.default_rng(12)
    w = zi_synth.workload("c1")
    p, m, v, _ = gen_numpy(zi_synth.StateSpec(12, zi.ZI_FP16), n)
    g = rng.normal(0, 1e-3, n).astype(np.float16)
    g = np.where(np.abs(g) < 2.0 ** -10, np.float16(2.0 ** -10), g).astype(np.float16)
    gs = (g.astype(np.float32) * np.float32(256.0)).astype(np.float16)
    _, a, _ = _run_both(p, m, v, g.view(np.uint16), zi.ZI_FP16, oracle_cfg(w), zi_cfg(w))
    _, b, _ = _run_both(p, m, v, gs.view(np.uint16), zi.ZI_FP16, oracle_cfg(w, loss_scale=256.0),
                        zi_cfg(w, loss_scale=256.0))
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_split_invariance_on_the_device():
    """Stepping [0,k) and [k,n) in two calls equals one call, bit for bit, for unaligned k too."""
    n = 5 * TILE + 123
    w = zi_synth.workload("c1")
    p, m, v, g = gen_numpy(zi_synth.StateSpec(41, zi.ZI_BF16), n)
    cfg = zi_cfg(w)
    whole = [to_dev(a) for a in (p, m, v, g)] + [torch.zeros(n, dtype=torch.int16, device="cuda:0")]
    zi.zi_adamw_step([tuple(whole) + (n,)], zi.ZI_BF16, cfg)
    for k in (1, 8, 1001, TILE, TILE + 3, n - 1):
        parts = [to_dev(a) for a in (p, m, v, g)] + [torch.zeros(n, dtype=torch.int16, device="cuda:0")]
        zi.zi_adamw_step([tuple(x[:k] for x in parts) + (k,), tuple(x[k:] for x in parts) + (n - k,)],
                         zi.ZI_BF16, cfg)
        torch.cuda.synchronize()
        for a, b in zip(whole, parts):
            assert torch.equal(a, b), f"k={k}"


def test_many_tensors_in_one_call_with_global_clip():
    """Workload 4 in miniature: 4 layers x 12 tensors at hidden size 96, one global norm, clip to 1."""
    h = 96
    w = zi_synth.workload("c4")
    numel = [n for _ in range(4) for (_, n) in zi_synth.transformer_layer_shapes(h)]
    dt = zi.ZI_BF16
    spec = zi_synth.StateSpec(w["spec"].seed, dt, g_std=2e-3)
    host = [gen_numpy(spec, n, tensor=i) for i, n in enumerate(numel)]
    ocfg, zcfg = oracle_cfg(w), zi_cfg(w)
    exp = [(p.copy(), m.copy(), v.copy(), g, np.zeros(p.size, np.uint16)) for (p, m, v, g) in host]
    info = oracle.step(exp, dt, ocfg, use_norm=True)
    assert info["found_inf"] == 0 and oracle.scalars(ocfg, info["sumsq"]).clip < 1.0
    devt = [tuple(to_dev(a) for a in t) + (torch.zeros(t[0].size, dtype=torch.int16, device="cuda:0"),)
            for t in host]
    nb = NormBuffers()
    zi.zi_grad_norm([(None, None, None, t[3], None) for t in devt], dt, ocfg.loss_scale, nb.out, nb.ws)
    zi.zi_adamw_step([t + (t[0].numel(),) for t in devt], dt, zcfg, nb.out)
    torch.cuda.synchronize()
    sumsq, norm, flag = nb.read()
    assert flag == 0 and abs(norm - info["norm"]) <= 1e-6 * info["norm"]
    worst = ""
    for i, (e, d) in enumerate(zip(exp, devt)):
        worst = compare_state((e[0], e[1], e[2], e[4]), (to_np(d[0]), to_np(d[1]), to_np(d[2]), to_np(d[4])),
                              dt, f"tensor {i} ")
    progress(f"c4-small: 48 tensors, norm {norm:.6f}; last tensor {worst}")


@pytest.mark.parametrize("dt", [zi.ZI_BF16, zi.ZI_FP16])
def test_every_fp32_pattern_through_the_copy(dt):
    """All 2^32 parameter patterns: with lr = 0 and zero g, m, v the step leaves p alone, so the
    low-precision output is the cast of every finite fp32 value; compared with the oracle's cast."""
    chunk = 1 << 27
    cfg = zi.make_config(lr=0.0, weight_decay=0.0, step=1)
    z32 = torch.zeros(chunk, dtype=torch.float32, device="cuda:0")
    zg = torch.zeros(chunk, dtype=torch.int16, device="cuda:0")
    bad = 0
    for c in range(0, 1 << 32, chunk):
        bits = np.arange(c, c + chunk, dtype=np.uint64).astype(np.uint32)
        p = torch.from_numpy(bits.view(np.int32)).to("cuda:0").view(torch.float32)
        m, v = z32.clone(), z32.clone()
        lp = torch.zeros(chunk, dtype=torch.int16, device="cuda:0")
        zi.zi_adamw_step([(p, m, v, zg, lp, chunk)], dt, cfg)
        want = oracle.cast(bits.view(np.float32), dt)
        got = to_np(lp)
        # +-inf turns into NaN on both sides (0 * inf in the decay and update terms), like NaN itself
        isnan = ~np.isfinite(bits.view(np.float32))
        if c == 0x80000000:
            want[0] = 0          # the parameter -0 comes back as +0 (see below), and so does its copy
        wrong = np.flatnonzero((want != got) & ~isnan)
        if wrong.size:
            progress("cast mismatches: " + ", ".join(
                f"p={bits[i]:#010x} want={want[i]:#06x} got={got[i]:#06x}" for i in wrong[:8]))
        bad += int(wrong.size)
        bad += int((~is_nan_lp(got[isnan], dt)).sum())
        # p itself: unchanged for every finite pattern (a -0 comes back as +0)
        pb = p.view(torch.int32).cpu().numpy().view(np.uint32)
        same = (pb == bits) | ((bits == 0x80000000) & (pb == 0)) | isnan
        if not same.all():
            progress("parameter changed: " + ", ".join(
                f"p={bits[i]:#010x} -> {pb[i]:#010x}" for i in np.flatnonzero(~same)[:8]))
        bad += int((~same).sum())
        if c % (1 << 30) == 0:
            progress(f"cast sweep dt={dt}: {c >> 27}/32 chunks, mismatches so far {bad}")
    assert bad == 0


def test_device_reproduces_the_oracle_golden_file():
    """The frozen oracle outputs under tests/golden/ (written by a script that calls only the oracle)."""
    from golden_util import load_cases
    for c in load_cases():
        n = c["in_p"].size
        p, m, v, g = (to_dev(c[k].copy()) for k in ("in_p", "in_m", "in_v", "in_g"))
        lp = torch.zeros(n, dtype=torch.int16, device="cuda:0")
        nb = None
        if c["use_norm"]:
            nb = NormBuffers()
            zi.zi_grad_norm([(None, None, None, g, None, n)], c["dtype"], c["kw"].get("loss_scale", 1.0), nb.out, nb.ws)
        zi.zi_adamw_step([(p, m, v, g, lp, n)], c["dtype"], zi.make_config(**c["kw"]), None if nb is None else nb.out)
        torch.cuda.synchronize()
        compare_state((c["out_p"], c["out_m"], c["out_v"], c["out_lp"]), (to_np(p), to_np(m), to_np(v), to_np(lp)),
                      c["dtype"], c["name"] + " ")


def test_ordinary_host_pointers_are_refused_not_dereferenced():
    """A pointer the GPU cannot reach is an argument error before any launch (page-locked host memory is fine)."""
    n = 1000
    w = zi_synth.workload("c1")
    p, m, v, g = gen_numpy(w["spec"], n)
    dp, dm, dv, dg = (to_dev(a) for a in (p, m, v, g))
    dlp = torch.zeros(n, dtype=torch.int16, device="cuda:0")
    good = [dp, dm, dv, dg, dlp]
    host = [p, m, v, g, np.zeros(n, np.uint16)]
    for k in range(5):
        args = list(good)
        args[k] = host[k]
        with pytest.raises(zi.ZiError) as ei:
            zi.zi_adamw_step([tuple(args) + (n,)], zi.ZI_BF16, zi_cfg(w))
        assert ei.value.status == zi.ZI_ERR_INVALID_ARG
    nb = NormBuffers()
    with pytest.raises(zi.ZiError):
        zi.zi_grad_norm([(None, None, None, g, None, n)], zi.ZI_BF16, 1.0, nb.out, nb.ws)
    with pytest.raises(zi.ZiError):
        zi.zi_adamw_step([(dp, dm, dv, dg, dlp, n)], zi.ZI_BF16, zi_cfg(w), np.zeros(4, np.float64))
    torch.cuda.synchronize()
    assert np.array_equal(to_np(dp), p)                       # nothing ran
    # a tensor whose end lies beyond its allocation's registered range is caught at its last byte
    pinned = torch.empty(n, dtype=torch.float32, pin_memory=True)
    pinned.numpy()[:] = p
    exp, _, _ = _run_both(p, m, v, g, zi.ZI_BF16, oracle_cfg(w), zi_cfg(w))
    zi.zi_adamw_step([(pinned, dm, dv, dg, dlp, n)], zi.ZI_BF16, zi_cfg(w))      # page-locked host memory works
    torch.cuda.synchronize()
    assert np.array_equal(pinned.numpy().view(np.uint32), exp[0].view(np.uint32))


@pytest.mark.parametrize("dt", [zi.ZI_BF16, zi.ZI_FP16])
def test_every_gradient_pattern(dt):
    """All 65,536 bit patterns of a low-precision gradient (subnormals, both zeros, the largest finite
    values; infinities and NaNs too: with no norm result nothing skips the step, NaN just propagates on
    both sides), each met with three different states."""
    w = zi_synth.workload("c1")
    g = np.tile(np.arange(65536, dtype=np.uint32).astype(np.uint16), 3)
    n = g.size
    p, m, v, _ = gen_numpy(zi_synth.StateSpec(4242 + dt, dt), n)
    m[65536:2 * 65536] = 0
    v[65536:2 * 65536] = 0                                     # first-step state for the middle copy
    ls = 1.0 if dt == zi.ZI_BF16 else 1024.0
    exp, got, _ = _run_both(p, m, v, g, dt, oracle_cfg(w, loss_scale=ls), zi_cfg(w, loss_scale=ls))
    special = np.isnan(exp[0])
    assert special.sum() >= 3 * 2 * 3                          # the NaN / inf patterns did reach the arithmetic
    for e, d in zip(exp[:3], got[:3]):
        assert np.array_equal(np.isnan(e), np.isnan(d))
    ok = ~special
    rep = compare_state(tuple(a[ok] for a in exp[:3]) + (exp[3][ok],), tuple(a[ok] for a in got[:3]) + (got[3][ok],),
                        dt, f"gradient patterns dt={dt} ")
    progress(f"all gradient patterns dt={dt}: {rep}")


@pytest.mark.parametrize("dt", [zi.ZI_BF16, zi.ZI_FP16])
def test_host_cpu_step_and_gpu_step_agree_bit_for_bit(dt):
    """The explicit host-CPU entry points against the HIP kernels on the same values (both follow the one
    written operation order): same norm to rounding, same p, m, v and copy, same skip decision."""
    n = 300_007
    spec = zi_synth.StateSpec(4242 + dt, dt, g_std=1e-3 if dt == zi.ZI_BF16 else 65.536)
    hp, hm, hv, hg = gen_numpy(spec, n)
    kw = dict(step=10, loss_scale=1.0 if dt == zi.ZI_BF16 else 65536.0, max_grad_norm=0.05)
    cfg = zi.make_config(**kw)
    p, m, v, g = to_dev(hp), to_dev(hm), to_dev(hv), to_dev(hg)
    lp = torch.zeros(n, dtype=torch.int16, device="cuda:0")
    nb = NormBuffers()
    tl = [(p, m, v, g, lp, n)]
    zi.zi_grad_norm(tl, dt, kw["loss_scale"], nb.out, nb.ws)
    zi.zi_adamw_step(tl, dt, cfg, nb.out)
    torch.cuda.synchronize()
    sumsq, norm, flag = nb.read()
    hlp = np.zeros(n, np.uint16)
    htl = [(hp, hm, hv, hg, hlp, n)]
    r = zi.zi_host_grad_norm(htl, dt, kw["loss_scale"], 4)
    assert r.found_inf == flag == 0 and abs(r.sumsq - sumsq) <= 1e-12 * sumsq
    # the step gets the very sum the GPU step read (the two reductions group their double sums differently)
    shared = zi.zi_norm_result(sumsq, norm, flag, 0)
    assert zi.zi_host_adamw_step(htl, dt, cfg, shared, 4) == zi.ZI_OK
    for name, h, d in (("p", hp, p), ("m", hm, m), ("v", hv, v)):
        assert np.array_equal(h.view(np.uint32), to_np(d).view(np.uint32)), name
    assert np.array_equal(hlp, to_np(lp))
    progress(f"host-CPU step == GPU step on {n} elements, dt={dt}")
