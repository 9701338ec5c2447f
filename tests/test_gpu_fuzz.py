"""Seeded random configurations and multi-step trajectories: the HIP path against the CPU oracle.

The fixed cases elsewhere pick their sizes, offsets and hyper-parameters by hand; here a seeded
generator draws them (tensor lists, ragged sizes, alignment offsets, both formats and modes, loss
scales that are and are not powers of two, clipping on and off), and a state is carried through many
consecutive steps (with one overflowing step in the middle) so that m and v take the values a real
run produces rather than the initial recipe's.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2104_07857_amd as zi
import zi_synth
from gpu_util import NormBuffers, TOL_NORM_REL, compare_state, gen_numpy, progress, to_dev, to_np

pytestmark = pytest.mark.gpu


def _draw_case(rng):
    dt = int(rng.choice([zi.ZI_BF16, zi.ZI_FP16]))
    loss_scale = float(rng.choice([1.0, 128.0, 65536.0, 3.7, 1000.0]))
    hp = dict(lr=float(10.0 ** rng.uniform(-6, -1)),
              beta1=float(rng.choice([0.0, 0.5, 0.9, 0.99])),
              beta2=float(rng.choice([0.0, 0.9, 0.999, 0.9999])),
              eps=float(rng.choice([1e-10, 1e-8, 1e-6, 1e-3])),
              weight_decay=float(rng.choice([0.0, 0.01, 0.3])),
              step=int(rng.choice([1, 2, 3, 10, 1000, 1_000_000])),
              loss_scale=loss_scale,
              max_grad_norm=float(rng.choice([0.0, 1.0, 0.05])),
              mode=int(rng.choice([zi.ZI_MODE_ADAMW, zi.ZI_MODE_ADAM_L2])))
    n_tensors = int(rng.integers(1, 6))
    sizes = [int(rng.choice([0, 1, int(rng.integers(2, 600)), int(rng.integers(600, 70_000))]))
             for _ in range(n_tensors)]
    # alignment: one common offset (every array line-aligned after the leading elements) or unrelated ones
    if rng.random() < 0.6:
        k = int(rng.integers(0, 70))
        offsets = [(k,) * 5 for _ in sizes]
    else:
        offsets = [tuple(int(x) for x in rng.integers(0, 70, 5)) for _ in sizes]
    g_std = 1e-3 * loss_scale * float(rng.choice([0.1, 1.0, 10.0]))
    if dt == zi.ZI_FP16:
        g_std = min(g_std, 2000.0)         # keep 6 sigma below the largest fp16 value
    with_lp = bool(rng.random() < 0.85)
    use_norm = bool(hp["max_grad_norm"] > 0 or rng.random() < 0.5)
    return dt, hp, sizes, offsets, g_std, with_lp, use_norm


def _place(a, off, pad=80):
    t = torch.zeros(a.size + pad, dtype=torch.float32 if a.dtype == np.float32 else torch.int16, device="cuda:0")
    t[off:off + a.size].copy_(to_dev(a))
    return t, t[off:off + a.size]


@pytest.mark.parametrize("seed", range(48))
def test_seeded_random_configuration(seed):
    rng = np.random.default_rng(0xF022 + seed)
    dt, hp, sizes, offsets, g_std, with_lp, use_norm = _draw_case(rng)
    spec = zi_synth.StateSpec(0xABC000 + seed, dt, g_std=g_std)
    host = [gen_numpy(spec, n, tensor=i) for i, n in enumerate(sizes)]
    ocfg = oracle.config(**hp)
    zcfg = zi.make_config(**hp)

    exp = [(p.copy(), m.copy(), v.copy(), g, np.zeros(p.size, np.uint16) if with_lp else None)
           for (p, m, v, g) in host]
    info = oracle.step(exp, dt, ocfg, use_norm=use_norm)

    bufs, views = [], []
    for (p, m, v, g), off in zip(host, offsets):
        placed = [_place(a, o) for a, o in zip((p, m, v, g, np.zeros(p.size, np.uint16)), off)]
        bufs.append([b for b, _ in placed])
        views.append([w for _, w in placed])
    nb = None
    if use_norm:
        nb = NormBuffers()
        zi.zi_grad_norm([(None, None, None, w[3], None, n) for w, n in zip(views, sizes)], dt, hp["loss_scale"],
                        nb.out, nb.ws)
    st = zi.zi_adamw_step([(w[0], w[1], w[2], w[3], w[4] if with_lp else None, n) for w, n in zip(views, sizes)],
                          dt, zcfg, None if nb is None else nb.out)
    torch.cuda.synchronize()
    assert st == zi.ZI_OK
    if use_norm:
        _, norm, flag = nb.read()
        assert flag == info["found_inf"] == 0
        assert abs(norm - info["norm"]) <= TOL_NORM_REL * max(info["norm"], 1e-300)
    rep = ""
    for i, (e, w, b, off, n) in enumerate(zip(exp, views, bufs, offsets, sizes)):
        got = (to_np(w[0]), to_np(w[1]), to_np(w[2]), to_np(w[4]) if with_lp else None)
        rep = compare_state((e[0], e[1], e[2], e[4]), got, dt, f"seed {seed} tensor {i} (n={n}) ")
        for a, o in zip(b, off):                     # nothing outside the views was touched
            assert not a[:o].any() and not a[o + n:].any()
        if not with_lp:
            assert not b[4].any()
    progress(f"fuzz seed {seed}: dt={dt} mode={hp['mode']} step={hp['step']} sizes={sizes} norm={use_norm} "
             f"lp={with_lp}; last tensor {rep}")


@pytest.mark.parametrize("dt,loss_scale,g_std", [(zi.ZI_BF16, 1.0, 1e-3), (zi.ZI_FP16, 4096.0, 4.0)])
def test_forty_consecutive_steps_follow_the_oracle(dt, loss_scale, g_std):
    """A state carried through 40 steps (fresh gradients each step, clip active, step 17 overflows and is
    skipped on both sides) stays within the bar of the oracle's trajectory at every fifth step and at
    the end.  The device's low-precision copy of step k is compared too."""
    n = 3 * 16384 + 77
    spec = zi_synth.StateSpec(0x7EA7 + dt, dt, g_std=g_std)
    p, m, v, _ = gen_numpy(spec, n)
    m[:] = 0
    v[:] = 0
    lp = np.zeros(n, np.uint16)
    dp, dm, dv = to_dev(p), to_dev(m), to_dev(v)
    dlp = torch.zeros(n, dtype=torch.int16, device="cuda:0")
    nb = NormBuffers()
    hp = dict(lr=3e-3, beta1=0.9, beta2=0.98, eps=1e-8, weight_decay=0.05, loss_scale=loss_scale, max_grad_norm=0.2)
    step = 0                              # the caller's count of steps actually taken
    for it in range(40):
        g = np.empty(n, np.uint16)
        spec.fill_g(g, n, 1 + it, 0)      # a new gradient stream per iteration
        if it == 17:
            g[n // 3] = 0x7F80 if dt == zi.ZI_BF16 else 0x7C00
        cfg_kw = dict(hp, step=step + 1)
        info = oracle.step([(p, m, v, g, lp)], dt, oracle.config(**cfg_kw), use_norm=True)
        dg = to_dev(g)
        zi.zi_grad_norm([(None, None, None, dg, None, n)], dt, loss_scale, nb.out, nb.ws)
        st = zi.zi_adamw_step([(dp, dm, dv, dg, dlp, n)], dt, zi.make_config(**cfg_kw), nb.out)
        torch.cuda.synchronize()
        _, norm, flag = nb.read()
        assert flag == info["found_inf"] == (1 if it == 17 else 0)
        if flag:
            assert info["skipped"]
        else:
            assert abs(norm - info["norm"]) <= TOL_NORM_REL * info["norm"]
            step += 1
        if it % 5 == 4 or it in (17, 39):
            rep = compare_state((p, m, v, lp), (to_np(dp), to_np(dm), to_np(dv), to_np(dlp)), dt, f"iteration {it} ")
            progress(f"trajectory dt={dt} iteration {it} (step {step}): {rep}")
    assert step == 39


def _host_array(a, where):
    """A copy of `a` in pinned ("pin"), ordinary ("page") or device ("dev") memory; (holder, numpy view or None)."""
    if where == "dev":
        return to_dev(a), None
    if where == "pin":
        t = torch.empty(max(a.size, 1), dtype=torch.float32 if a.dtype == np.float32 else torch.int16, pin_memory=True)
        view = t.numpy()[:a.size]
        view[:] = a if a.dtype == np.float32 else a.view(np.int16)
        return t, view
    c = a.copy()
    return c, c


@pytest.mark.parametrize("seed", range(24))
def test_seeded_random_streamed_lists(seed):
    """The streamed step on drawn lists: 1-120 tensors from empty to several chunks long, chunk size and
    slot count drawn too, state pinned or ordinary (ring), gradients / copy on the device or in host
    memory, with or without a norm result.  Compared with the oracle element by element."""
    rng = np.random.default_rng(0x5EA0 + seed)
    dt = int(rng.choice([zi.ZI_BF16, zi.ZI_FP16]))
    chunk_elems = int(rng.choice([1024, 4096, 16384]))
    n_slots = int(rng.integers(2, 6))
    n_tensors = int(rng.choice([1, 2, 5, 40, 120]))
    kinds = [0, 1, int(rng.integers(2, 200)), int(rng.integers(200, chunk_elems)), chunk_elems,
             int(rng.integers(chunk_elems + 1, 4 * chunk_elems))]
    weights = [0.05, 0.1, 0.35, 0.3, 0.05, 0.15]
    sizes = [int(kinds[k]) for k in rng.choice(len(kinds), n_tensors, p=weights)]
    state_where = str(rng.choice(["pin", "page"]))
    g_where = str(rng.choice(["dev", "pin", "page"]))
    lp_where = str(rng.choice(["dev", "pin", "page", "none"]))
    use_norm = bool(rng.random() < 0.7)
    loss_scale = float(rng.choice([1.0, 1024.0]))
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, step=int(rng.choice([1, 10, 500])),
              loss_scale=loss_scale, max_grad_norm=float(rng.choice([0.0, 0.5])),
              mode=int(rng.choice([zi.ZI_MODE_ADAMW, zi.ZI_MODE_ADAM_L2])))
    spec = zi_synth.StateSpec(0xBEE000 + seed, dt, g_std=1e-3 * loss_scale)
    host = [gen_numpy(spec, n, tensor=i) for i, n in enumerate(sizes)]
    exp = [(p.copy(), m.copy(), v.copy(), g, None if lp_where == "none" else np.zeros(p.size, np.uint16))
           for (p, m, v, g) in host]
    info = oracle.step(exp, dt, oracle.config(**hp), use_norm=use_norm)

    needs_ring = "page" in (state_where, g_where, lp_where)
    eng = zi.zi_engine_create(0, 4 * chunk_elems, n_slots)
    try:
        if needs_ring:
            zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_COPY_THREADS, int(rng.integers(1, 5)))
            zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_RING_SLOTS, int(rng.integers(2, 6)))
        holders, tl = [], []
        for (p, m, v, g) in host:
            hs = [_host_array(a, state_where) for a in (p, m, v)]
            hg = _host_array(g, g_where)
            hl = (None, None) if lp_where == "none" else _host_array(np.zeros(p.size, np.uint16), lp_where)
            holders.append((hs, hg, hl))
            tl.append((hs[0][0], hs[1][0], hs[2][0], hg[0], hl[0], p.size))
        nb = None
        if use_norm:
            nb = NormBuffers()
            zi.zi_grad_norm_streamed(eng, tl, dt, loss_scale, nb.out, nb.ws)
        st = zi.zi_adamw_step_streamed(eng, tl, dt, zi.make_config(**hp), None if nb is None else nb.out,
                                       torch.cuda.current_stream())
        assert st == zi.ZI_OK
        if use_norm:
            _, norm, flag = nb.read()
            assert flag == info["found_inf"] == 0
            assert abs(norm - info["norm"]) <= TOL_NORM_REL * max(info["norm"], 1e-300)
        _, uses = zi.zi_plan_chunks(sizes, chunk_elems)
        stats = zi.zi_engine_last_stats(eng)
        per_elem = 12 + (2 if g_where != "dev" else 0)
        assert stats.n_slot_uses == uses and stats.bytes_h2d == per_elem * sum(sizes)
        rep = ""
        for i, (e, (hs, hg, hl)) in enumerate(zip(exp, holders)):
            got_lp = None
            if lp_where != "none":
                got_lp = to_np(hl[0]) if lp_where == "dev" else np.asarray(hl[1]).view(np.uint16).copy()
            got = tuple(np.asarray(x[1]).copy() for x in hs) + (got_lp,)
            rep = compare_state((e[0], e[1], e[2], e[4]), got, dt, f"seed {seed} tensor {i} (n={sizes[i]}) ")
        progress(f"streamed fuzz seed {seed}: dt={dt} chunk={chunk_elems} slots={n_slots} tensors={n_tensors} "
                 f"state={state_where} g={g_where} lp={lp_where} norm={use_norm}: {uses} slot uses; last {rep}")
    finally:
        zi.zi_engine_destroy(eng)
