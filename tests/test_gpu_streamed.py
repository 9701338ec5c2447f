"""The streamed step (state in pinned host memory, chunked through HBM) against the oracle and the resident step."""
import os
import tempfile

import numpy as np
import pytest
import torch

import oracle
import paper_2104_07857_amd as zi
import zi_synth
from gpu_util import NormBuffers, compare_state, gen_numpy, oracle_cfg, progress, to_dev, to_np, zi_cfg

pytestmark = pytest.mark.gpu


def _pinned(a: np.ndarray) -> torch.Tensor:
    t = torch.empty(a.size, dtype=torch.float32, pin_memory=True)
    t.numpy()[:] = a
    return t


def _stream_list(engine, host, dt, ocfg, zcfg, use_norm, g_offset=0):
    """host: list of (p, m, v, g) numpy.  Returns expected (oracle) and got (streamed) lists + info."""
    exp = [(p.copy(), m.copy(), v.copy(), g, np.zeros(p.size, np.uint16)) for (p, m, v, g) in host]
    info = oracle.step(exp, dt, ocfg, use_norm)
    pinned = [tuple(_pinned(a) for a in t[:3]) for t in host]
    dg, dlp = [], []
    for t in host:
        n = t[3].size
        gbuf = torch.zeros(n + 8, dtype=torch.int16, device="cuda:0")
        lbuf = torch.zeros(n + 8, dtype=torch.int16, device="cuda:0")
        gbuf[g_offset:g_offset + n].copy_(to_dev(t[3]))
        dg.append(gbuf[g_offset:g_offset + n])
        dlp.append(lbuf[g_offset:g_offset + n])
    nb = None
    if use_norm:
        nb = NormBuffers()
        zi.zi_grad_norm([(None, None, None, g, None, g.numel()) for g in dg], dt, ocfg.loss_scale, nb.out, nb.ws)
    tl = [(pp, pm, pv, g, lp, g.numel()) for (pp, pm, pv), g, lp in zip(pinned, dg, dlp)]
    st = zi.zi_adamw_step_streamed(engine, tl, dt, zcfg, None if nb is None else nb.out,
                                   torch.cuda.current_stream())
    got = [(pp.numpy().copy(), pm.numpy().copy(), pv.numpy().copy(), to_np(lp))
           for (pp, pm, pv), lp in zip(pinned, dlp)]
    return exp, got, dict(status=st, oracle=info, norm=nb.read() if nb else None)


@pytest.fixture(scope="module")
def engine():
    e = zi.zi_engine_create(0, 64 * 1024, 3)          # 16384-element chunks: many slot uses at small sizes
    yield e
    zi.zi_engine_destroy(e)


@pytest.mark.parametrize("n", [1, 100, 16384 - 8, 16384, 16384 + 1, 5 * 16384 + 777, 40 * 16384])
def test_flat_state_with_tail_chunk(engine, n):
    w = zi_synth.workload("c2")
    host = [gen_numpy(zi_synth.StateSpec(2000 + n, zi.ZI_BF16), n)]
    exp, got, info = _stream_list(engine, host, zi.ZI_BF16, oracle_cfg(w), zi_cfg(w), use_norm=False)
    assert info["status"] == zi.ZI_OK
    rep = compare_state((exp[0][0], exp[0][1], exp[0][2], exp[0][4]), got[0], zi.ZI_BF16, f"n={n} ")
    st = zi.zi_engine_last_stats(engine)
    assert st.bytes_h2d == st.bytes_d2h == 12 * n
    assert st.n_slot_uses == (n + 16383) // 16384
    if n == 5 * 16384 + 777:
        progress("streamed flat: " + rep)


def test_streamed_equals_resident_bit_for_bit(engine):
    """Chunking must not change a single bit (the update is independent per element)."""
    n = 7 * 16384 + 4321
    w = zi_synth.workload("c2")
    host = [gen_numpy(zi_synth.StateSpec(77, zi.ZI_BF16), n)]
    _, got, _ = _stream_list(engine, host, zi.ZI_BF16, oracle_cfg(w), zi_cfg(w), use_norm=False)
    p, m, v, g = (to_dev(a) for a in host[0])
    lp = torch.zeros(n, dtype=torch.int16, device="cuda:0")
    zi.zi_adamw_step([(p, m, v, g, lp, n)], zi.ZI_BF16, zi_cfg(w))
    torch.cuda.synchronize()
    for a, b in zip(got[0], (to_np(p), to_np(m), to_np(v), to_np(lp))):
        assert np.array_equal(a.view(np.uint32) if a.dtype == np.float32 else a,
                              b.view(np.uint32) if b.dtype == np.float32 else b)


@pytest.mark.parametrize("g_offset", [0, 3])
def test_ragged_list_with_packing_and_global_clip(engine, g_offset):
    """Workload 4 in miniature: 4 layers x 12 tensors (hidden 128: weights span several chunks, biases
    and LayerNorm vectors are packed into shared slots), separate pinned arrays, one global clip."""
    h = 128
    w = zi_synth.workload("c4")
    numel = [n for _ in range(4) for (_, n) in zi_synth.transformer_layer_shapes(h)]
    spec = zi_synth.StateSpec(w["spec"].seed, zi.ZI_BF16, g_std=2e-3)
    host = [gen_numpy(spec, n, tensor=i) for i, n in enumerate(numel)]
    exp, got, info = _stream_list(engine, host, zi.ZI_BF16, oracle_cfg(w), zi_cfg(w), use_norm=True,
                                  g_offset=g_offset)
    assert info["status"] == zi.ZI_OK and info["oracle"]["found_inf"] == 0
    assert abs(info["norm"][1] - info["oracle"]["norm"]) <= 1e-6 * info["oracle"]["norm"]
    assert oracle.scalars(oracle_cfg(w), info["oracle"]["sumsq"]).clip < 1.0
    for i, (e, g) in enumerate(zip(exp, got)):
        rep = compare_state((e[0], e[1], e[2], e[4]), g, zi.ZI_BF16, f"tensor {i} ")
    segs, uses = zi.zi_plan_chunks(numel, 16384)
    st = zi.zi_engine_last_stats(engine)
    assert st.n_slot_uses == uses and st.bytes_h2d == 12 * sum(numel) == st.bytes_d2h
    progress(f"streamed ragged (g offset {g_offset}): {uses} slot uses, {st.n_kernels} launches; last {rep}")


@pytest.mark.parametrize("chunk_bytes,slots", [(4096, 2), (4096, 8), (1 << 20, 3), (1 << 22, 4)])
def test_chunk_size_and_slot_count_do_not_change_a_bit(chunk_bytes, slots):
    """Chunked processing equals unchunked processing for any chunk size, including chunks larger than
    the whole state, and any number of slots."""
    n = 300_007
    w = zi_synth.workload("c2")
    p, m, v, g = gen_numpy(zi_synth.StateSpec(55, zi.ZI_BF16), n)
    dp, dm, dv, dg = (to_dev(a) for a in (p, m, v, g))
    rlp = torch.zeros(n, dtype=torch.int16, device="cuda:0")
    zi.zi_adamw_step([(dp, dm, dv, dg, rlp, n)], zi.ZI_BF16, zi_cfg(w))
    pp, pm, pv = _pinned(p), _pinned(m), _pinned(v)
    lp = torch.zeros(n, dtype=torch.int16, device="cuda:0")
    eng = zi.zi_engine_create(0, chunk_bytes, slots)
    try:
        assert zi.zi_adamw_step_streamed(eng, [(pp, pm, pv, dg, lp, n)], zi.ZI_BF16, zi_cfg(w)) == zi.ZI_OK
        assert zi.zi_engine_last_stats(eng).n_slot_uses == -(-n // (chunk_bytes // 4))
    finally:
        zi.zi_engine_destroy(eng)
    torch.cuda.synchronize()
    for a, b in ((pp, dp), (pm, dm), (pv, dv)):
        assert np.array_equal(a.numpy().view(np.uint32), to_np(b).view(np.uint32))
    assert torch.equal(lp, rlp)


def test_streamed_without_low_precision_copy(engine):
    n = 3 * 16384 + 99
    w = zi_synth.workload("c2")
    p, m, v, g = gen_numpy(zi_synth.StateSpec(8, zi.ZI_BF16), n)
    pe, me, ve = p.copy(), m.copy(), v.copy()
    oracle.adamw(pe, me, ve, g, None, zi.ZI_BF16, oracle_cfg(w))
    pp, pm, pv = _pinned(p), _pinned(m), _pinned(v)
    assert zi.zi_adamw_step_streamed(engine, [(pp, pm, pv, to_dev(g), None, n)], zi.ZI_BF16, zi_cfg(w)) == zi.ZI_OK
    compare_state((pe, me, ve, None), (pp.numpy(), pm.numpy(), pv.numpy(), None), zi.ZI_BF16)


def test_overflow_skips_without_moving_state(engine):
    w = zi_synth.workload("c3")
    n = 3 * 16384 + 5
    p, m, v, g = gen_numpy(w["spec"], n)
    g[zi_synth.pick_index(1, 2, n)] = 0xFC00          # -inf
    exp, got, info = _stream_list(engine, [(p, m, v, g)], zi.ZI_FP16, oracle_cfg(w), zi_cfg(w), use_norm=True)
    assert info["status"] == zi.ZI_SKIPPED_OVERFLOW and info["oracle"]["skipped"]
    for a, b in zip((p, m, v), got[0][:3]):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    assert not got[0][3].any()
    st = zi.zi_engine_last_stats(engine)
    assert st.bytes_h2d == 0 and st.bytes_d2h == 0 and st.n_kernels == 0


def test_step_allocates_nothing_and_rejects_pageable_state(engine):
    n = 4 * 16384
    w = zi_synth.workload("c2")
    host = gen_numpy(w["spec"], n)
    pp, pm, pv = (_pinned(a) for a in host[:3])
    g = to_dev(host[3])
    lp = torch.zeros(n, dtype=torch.int16, device="cuda:0")
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(3):
        zi.zi_adamw_step_streamed(engine, [(pp, pm, pv, g, lp, n)], zi.ZI_BF16, zi_cfg(w))
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0, "the engine's step must not allocate device memory"
    pageable = np.zeros(n, np.float32)
    with pytest.raises(zi.ZiError) as e:
        zi.zi_adamw_step_streamed(engine, [(pageable, pm, pv, g, lp, n)], zi.ZI_BF16, zi_cfg(w))
    assert e.value.status == zi.ZI_ERR_INVALID_ARG and "pinned" in e.value.message


@pytest.mark.parametrize("hslots,threads", [(2, 1), (4, 3), (7, 6)])
def test_pageable_state_through_the_pinned_ring(hslots, threads):
    """State in ordinary host memory, staged through a small pinned ring by CPU threads: same bits as the
    resident step, for a flat tensor with a tail chunk and for a ragged list with packing."""
    w = zi_synth.workload("c4")
    eng = zi.zi_engine_create(0, 64 * 1024, 3)
    try:
        zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_COPY_THREADS, threads)
        zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_RING_SLOTS, hslots)
        h = 128
        lists = [[9 * 16384 + 1234], [n for _ in range(2) for (_, n) in zi_synth.transformer_layer_shapes(h)]]
        for numel in lists:
            spec = zi_synth.StateSpec(4321 + len(numel), zi.ZI_BF16, g_std=2e-3)
            host = [gen_numpy(spec, n, tensor=i) for i, n in enumerate(numel)]
            plain = [tuple(a.copy() for a in t[:3]) for t in host]           # ordinary numpy memory
            dg = [to_dev(t[3]) for t in host]
            dlp = [torch.zeros(t[3].size, dtype=torch.int16, device="cuda:0") for t in host]
            nb = NormBuffers()
            zi.zi_grad_norm([(None, None, None, g, None, g.numel()) for g in dg], zi.ZI_BF16, 1.0, nb.out, nb.ws)
            tl = [(pp, pm, pv, g, lp, g.numel()) for (pp, pm, pv), g, lp in zip(plain, dg, dlp)]
            st = zi.zi_adamw_step_streamed(eng, tl, zi.ZI_BF16, zi_cfg(w), nb.out, torch.cuda.current_stream())
            assert st == zi.ZI_OK
            stats = zi.zi_engine_last_stats(eng)
            assert stats.bytes_staged_host == 24 * sum(numel) and stats.bytes_h2d == 12 * sum(numel)
            # reference: the resident step on the same values
            for (p, m, v, g), (pp, pm, pv), lp in zip(host, plain, dlp):
                dp, dm, dv, dgg = (to_dev(a) for a in (p, m, v, g))
                rlp = torch.zeros(p.size, dtype=torch.int16, device="cuda:0")
                zi.zi_adamw_step([(dp, dm, dv, dgg, rlp, p.size)], zi.ZI_BF16, zi_cfg(w), nb.out)
                torch.cuda.synchronize()
                assert np.array_equal(pp.view(np.uint32), to_np(dp).view(np.uint32))
                assert np.array_equal(pm.view(np.uint32), to_np(dm).view(np.uint32))
                assert np.array_equal(pv.view(np.uint32), to_np(dv).view(np.uint32))
                assert torch.equal(lp, rlp)
        # turning the ring off again makes pageable state an error
        zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_RING_SLOTS, 0)
        with pytest.raises(zi.ZiError):
            zi.zi_adamw_step_streamed(eng, tl, zi.ZI_BF16, zi_cfg(w), nb.out)
        for bad in (1, 17, -1):
            with pytest.raises(zi.ZiError):
                zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_RING_SLOTS, bad)
        with pytest.raises(zi.ZiError):
            zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_COPY_THREADS, 0)
    finally:
        zi.zi_engine_destroy(eng)


def _pinned16(a: np.ndarray) -> torch.Tensor:
    t = torch.empty(a.size, dtype=torch.int16, pin_memory=True)
    t.numpy()[:] = a.view(np.int16)
    return t


@pytest.mark.parametrize("placement", ["g_pinned", "lp_pinned", "both_pinned", "all_pageable", "g_pageable_state_pinned"])
def test_gradients_and_copy_in_host_memory(placement):
    """Gradient-side offload: gradients and / or the low-precision copy live in host memory and travel with
    their chunk of state; the norm is reduced from host-resident gradients too.  Same bits as resident."""
    w = zi_synth.workload("c4")
    dt = zi.ZI_BF16
    eng = zi.zi_engine_create(0, 64 * 1024, 3)
    try:
        zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_RING_SLOTS, 4)
        h = 128
        for numel in ([7 * 16384 + 4322], [n for _ in range(2) for (_, n) in zi_synth.transformer_layer_shapes(h)]):
            spec = zi_synth.StateSpec(99 + len(numel), dt, g_std=2e-3)
            host = [gen_numpy(spec, n, tensor=i) for i, n in enumerate(numel)]
            ocfg, zcfg = oracle_cfg(w), zi_cfg(w)
            exp = [(p.copy(), m.copy(), v.copy(), g, np.zeros(p.size, np.uint16)) for (p, m, v, g) in host]
            info = oracle.step(exp, dt, ocfg, use_norm=True)
            tl, keep = [], []
            for (p, m, v, g) in host:
                if placement == "all_pageable":
                    sp, sm, sv = p.copy(), m.copy(), v.copy()
                    sg, slp = g.copy(), np.zeros(g.size, np.uint16)
                else:
                    sp, sm, sv = _pinned(p), _pinned(m), _pinned(v)
                    sg = to_dev(g)
                    slp = torch.zeros(g.size, dtype=torch.int16, device="cuda:0")
                    if placement in ("g_pinned", "both_pinned"):
                        sg = _pinned16(g)
                    if placement == "g_pageable_state_pinned":
                        sg = g.copy()
                    if placement in ("lp_pinned", "both_pinned"):
                        slp = torch.zeros(g.size, dtype=torch.int16, pin_memory=True)
                keep.append((sp, sm, sv, sg, slp))
                tl.append((sp, sm, sv, sg, slp, g.size))
            nb = NormBuffers()
            zi.zi_grad_norm_streamed(eng, tl, dt, ocfg.loss_scale, nb.out, nb.ws, stream=torch.cuda.current_stream())
            sumsq, norm, flag = nb.read()
            assert flag == 0 and abs(sumsq - info["sumsq"]) <= 1e-12 * info["sumsq"]
            st = zi.zi_adamw_step_streamed(eng, tl, dt, zcfg, nb.out, torch.cuda.current_stream())
            assert st == zi.ZI_OK
            stats = zi.zi_engine_last_stats(eng)
            g_host = placement != "lp_pinned"
            lp_host = placement in ("lp_pinned", "both_pinned", "all_pageable")
            assert stats.bytes_h2d == (12 + 2 * g_host) * sum(numel)
            assert stats.bytes_d2h == (12 + 2 * lp_host) * sum(numel)
            as_np = lambda x: x if isinstance(x, np.ndarray) else (x.numpy() if x.device.type == "cpu" else to_np(x))
            for e, (sp, sm, sv, sg, slp) in zip(exp, keep):
                got = (as_np(sp), as_np(sm), as_np(sv), as_np(slp).view(np.uint16))
                compare_state((e[0], e[1], e[2], e[4]), got, dt, f"{placement} ")
                assert np.array_equal(got[0].view(np.uint32), e[0].view(np.uint32))     # in fact bit-identical
    finally:
        zi.zi_engine_destroy(eng)


def test_streamed_norm_flags_and_mixed_residency():
    dt = zi.ZI_FP16
    eng = zi.zi_engine_create(0, 64 * 1024, 3)
    try:
        zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_RING_SLOTS, 3)
        sizes = [5 * 32768 + 77, 1000, 0, 40000, 3]
        gs = []
        for i, n in enumerate(sizes):
            g = np.empty(n, np.uint16)
            zi_synth.fill_normal_lp(g, n, 5 + i, zi_synth.STREAM_G, dt, std=50.0)
            gs.append(g)
        want, _ = oracle.grad_sumsq(gs, dt)
        # device, pinned, empty, ordinary, ordinary
        placed = [to_dev(gs[0]), _pinned16(gs[1]), None, gs[3].copy(), gs[4].copy()]
        tl = [(None, None, None, x, None, n) for x, n in zip(placed, sizes)]
        nb = NormBuffers()
        zi.zi_grad_norm_streamed(eng, tl, dt, 8.0, nb.out, nb.ws)
        sumsq, norm, flag = nb.read()
        assert flag == 0 and abs(sumsq - want) <= 1e-12 * want and abs(norm - np.sqrt(want) / 8.0) <= 1e-9 * norm
        placed[3][12345] = 0x7C00                     # +inf in an ordinary-memory tensor
        zi.zi_grad_norm_streamed(eng, tl, dt, 8.0, nb.out, nb.ws)
        assert nb.read()[2] == 1
        placed[3][12345] = 0
        p1 = _pinned16(gs[1])
        p1[999] = -1                                   # 0xFFFF: NaN in a pinned tensor's last element
        tl[1] = (None, None, None, p1, None, sizes[1])
        zi.zi_grad_norm_streamed(eng, tl, dt, 8.0, nb.out, nb.ws)
        assert nb.read()[2] == 1
        # all-empty list gives zeros
        zi.zi_grad_norm_streamed(eng, [], dt, 1.0, nb.out, nb.ws)
        assert nb.read() == (0.0, 0.0, 0)
        # ordinary-memory gradients without a ring are refused
        zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_RING_SLOTS, 0)
        with pytest.raises(zi.ZiError):
            zi.zi_grad_norm_streamed(eng, tl, dt, 8.0, nb.out, nb.ws)
    finally:
        zi.zi_engine_destroy(eng)


def _write_state_files(tmp, host, direct):
    """One file per array kind; tensor i of the list starts at a 4096-byte aligned offset."""
    offs, pos = [], 0
    for (p, m, v, g) in host:
        offs.append(pos)
        pos += (4 * p.size + 4095) // 4096 * 4096
    paths = [os.path.join(tmp, k + ".bin") for k in "pmv"]
    for w, path in enumerate(paths):
        with open(path, "wb") as f:
            for o, tensors in zip(offs, host):
                f.seek(o)
                f.write(tensors[w].tobytes())
            f.truncate(max(pos, 4096))
    flags = os.O_RDWR | (os.O_DIRECT if direct else 0)
    return [os.open(p, flags) for p in paths], offs, paths


@pytest.mark.parametrize("direct,host_g", [(False, False), (True, False), (True, True), (False, True)])
def test_state_in_files_through_the_pinned_ring(direct, host_g):
    """fp32 state in files (buffered and O_DIRECT descriptors): parallel reads into the pinned ring, the
    same device pipeline, parallel writes back.  Bit-identical to the resident step.  With host_g the
    gradients and the low-precision copy live in ordinary host memory and ride the ring as well."""
    w = zi_synth.workload("c4")
    eng = zi.zi_engine_create(0, 64 * 1024, 3)
    fds = []
    try:
        zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_COPY_THREADS, 4)
        zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_RING_SLOTS, 5)
        h = 128
        lists = [[9 * 16384 + 1236], [n for _ in range(2) for (_, n) in zi_synth.transformer_layer_shapes(h)]]
        for numel in lists:
            spec = zi_synth.StateSpec(777 + len(numel), zi.ZI_BF16, g_std=2e-3)
            host = [gen_numpy(spec, n, tensor=i) for i, n in enumerate(numel)]
            with tempfile.TemporaryDirectory(dir="/tmp") as tmp:
                fds, offs, paths = _write_state_files(tmp, host, direct)
                dg = [to_dev(t[3]) for t in host]
                dlp = [torch.zeros(t[3].size, dtype=torch.int16, device="cuda:0") for t in host]
                nb = NormBuffers()
                zi.zi_grad_norm([(None, None, None, g, None, g.numel()) for g in dg], zi.ZI_BF16, 1.0, nb.out, nb.ws)
                hlp = [np.zeros(t[3].size, np.uint16) for t in host]
                if host_g:
                    tl = [(fds[0], fds[1], fds[2], o, o, o, t[3], lp, t[3].size) for o, t, lp in zip(offs, host, hlp)]
                else:
                    tl = [(fds[0], fds[1], fds[2], o, o, o, g, lp, g.numel()) for o, g, lp in zip(offs, dg, dlp)]
                st = zi.zi_adamw_step_files(eng, tl, zi.ZI_BF16, zi_cfg(w), nb.out, torch.cuda.current_stream())
                assert st == zi.ZI_OK
                stats = zi.zi_engine_last_stats(eng)
                assert stats.bytes_h2d == (14 if host_g else 12) * sum(numel) == stats.bytes_d2h
                if host_g:
                    dlp = [to_dev(a) for a in hlp]
                for fd in fds:
                    os.close(fd)
                fds = []
                back = [np.fromfile(p, dtype=np.float32) for p in paths]
                for (p, m, v, g), o, lp in zip(host, offs, dlp):
                    dp, dm, dv, dgg = (to_dev(a) for a in (p, m, v, g))
                    rlp = torch.zeros(p.size, dtype=torch.int16, device="cuda:0")
                    zi.zi_adamw_step([(dp, dm, dv, dgg, rlp, p.size)], zi.ZI_BF16, zi_cfg(w), nb.out)
                    torch.cuda.synchronize()
                    for arr, ref in zip(back, (dp, dm, dv)):
                        got = arr[o // 4:o // 4 + p.size]
                        assert np.array_equal(got.view(np.uint32), to_np(ref).view(np.uint32))
                    assert torch.equal(lp, rlp)
    finally:
        for fd in fds:
            os.close(fd)
        zi.zi_engine_destroy(eng)


def test_file_step_argument_and_io_errors():
    n = 3 * 16384
    g = torch.zeros(n, dtype=torch.int16, device="cuda:0")
    lp = torch.zeros(n, dtype=torch.int16, device="cuda:0")
    cfg = zi.make_config(step=10)
    eng = zi.zi_engine_create(0, 64 * 1024, 3)
    with tempfile.TemporaryDirectory(dir="/tmp") as tmp:
        path = os.path.join(tmp, "s.bin")
        with open(path, "wb") as f:
            f.write(np.zeros(3 * n, np.float32).tobytes())
        fd = os.open(path, os.O_RDWR)
        fdro = os.open(path, os.O_RDONLY)
        fdd = os.open(path, os.O_RDWR | os.O_DIRECT)
        try:
            good = (fd, fd, fd, 0, 4 * n, 8 * n, g, lp, n)
            with pytest.raises(zi.ZiError) as e:                     # no ring yet
                zi.zi_adamw_step_files(eng, [good], zi.ZI_BF16, cfg)
            assert e.value.status == zi.ZI_ERR_INVALID_ARG
            zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_RING_SLOTS, 4)
            assert zi.zi_adamw_step_files(eng, [good], zi.ZI_BF16, cfg) == zi.ZI_OK
            assert zi.zi_adamw_step_files(eng, [], zi.ZI_BF16, cfg) == zi.ZI_OK
            for bad, status in (((-1, fd, fd, 0, 0, 0, g, lp, n), zi.ZI_ERR_INVALID_ARG),
                                ((987654, fd, fd, 0, 0, 0, g, lp, n), zi.ZI_ERR_INVALID_ARG),
                                ((fdro, fd, fd, 0, 4 * n, 8 * n, g, lp, n), zi.ZI_ERR_INVALID_ARG),
                                ((fd, fd, fd, 2, 4 * n, 8 * n, g, lp, n), zi.ZI_ERR_ALIGNMENT),
                                ((fdd, fd, fd, 512, 4 * n, 8 * n, g, lp, n), zi.ZI_ERR_ALIGNMENT),
                                ((fdd, fd, fd, 0, 4 * n, 8 * n, g[1:], lp[1:], n - 1), zi.ZI_ERR_ALIGNMENT),
                                ((fd, fd, fd, 0, 4 * n, 8 * n, None, lp, n), zi.ZI_ERR_INVALID_ARG),
                                ((fd, fd, fd, 0, 4 * n, 8 * n, g, lp, -5), zi.ZI_ERR_INVALID_ARG)):
                with pytest.raises(zi.ZiError) as e:
                    zi.zi_adamw_step_files(eng, [bad], zi.ZI_BF16, cfg)
                assert e.value.status == status, bad
            # the v region lies beyond the end of the file: a short read is an I/O error, not a crash
            with pytest.raises(zi.ZiError) as e:
                zi.zi_adamw_step_files(eng, [(fd, fd, fd, 0, 4 * n, 16 * n, g, lp, n)], zi.ZI_BF16, cfg)
            assert e.value.status == zi.ZI_ERR_IO and "reading" in e.value.message
            # the engine is still usable afterwards
            assert zi.zi_adamw_step_files(eng, [good], zi.ZI_BF16, cfg) == zi.ZI_OK
            assert zi.zi_engine_file_probe(eng, fd, -1, 4096 * 8) > 0
            with pytest.raises(zi.ZiError):
                zi.zi_engine_file_probe(eng, -1, -1, 4096)
            with pytest.raises(zi.ZiError):
                zi.zi_engine_file_probe(eng, fd, -1, 1000)
        finally:
            for d in (fd, fdro, fdd):
                os.close(d)
            zi.zi_engine_destroy(eng)


def test_copy_only_option_and_link_probe(engine):
    n = 8 * 16384
    w = zi_synth.workload("c2")
    host = gen_numpy(w["spec"], n)
    pp, pm, pv = (_pinned(a) for a in host[:3])
    g = to_dev(host[3])
    lp = torch.zeros(n, dtype=torch.int16, device="cuda:0")
    zi.zi_engine_set_option(engine, zi.ZI_OPT_SKIP_KERNEL, 1)
    try:
        zi.zi_adamw_step_streamed(engine, [(pp, pm, pv, g, lp, n)], zi.ZI_BF16, zi_cfg(w))
    finally:
        zi.zi_engine_set_option(engine, zi.ZI_OPT_SKIP_KERNEL, 0)
    # with the kernel removed the state makes the round trip unchanged
    assert np.array_equal(pp.numpy(), host[0]) and np.array_equal(pv.numpy(), host[2])
    assert zi.zi_engine_last_stats(engine).n_kernels == 0
    src = torch.zeros(1 << 20, dtype=torch.uint8, pin_memory=True)
    dst = torch.zeros(1 << 20, dtype=torch.uint8, pin_memory=True)
    for mode in (0, 1, 2):
        for piece, depth in ((0, 2), (4096, 0), (65536, 1), (1 << 18, 8)):
            assert zi.zi_engine_link_probe(engine, src, dst, 1 << 20, mode, piece, depth) > 0
    # what lands in host memory is the second half of the staging area: the probe moves real bytes
    with pytest.raises(zi.ZiError):
        zi.zi_engine_link_probe(engine, src, dst, 1 << 20, 2, 1 << 30, 2)          # piece beyond the staging memory
    with pytest.raises(zi.ZiError):
        zi.zi_engine_link_probe(engine, src, dst, 1 << 20, 2, 0, 9)
    with pytest.raises(zi.ZiError):
        zi.zi_engine_link_probe(engine, np.zeros(1 << 20, np.uint8), dst, 1 << 20, 0, 0, 2)   # pageable source


def test_pinned_allocator_round_trip():
    ptr = zi.zi_pinned_alloc(1 << 20)
    assert ptr and ptr % 256 == 0
    assert zi.zi_pinned_free(ptr) == zi.ZI_OK


def test_engine_create_destroy_cycle():
    e = zi.zi_engine_create(0, 4096, 2)
    assert zi.zi_engine_destroy(e) == zi.ZI_OK


# ------------------------------------------------------------------ gradient offload (device -> host)

def test_gradient_partitions_drain_while_the_producer_keeps_running():
    """Partitions of a gradient buffer are produced one after another on a producer stream (a dummy
    producer: repeated device copies into the partition) and handed to zi_grad_offload as soon as they
    are enqueued.  The calls return at once, the bytes arrive, and the total time shows that the drain
    of partition k overlapped the production of partition k + 1."""
    import time
    part = 1 << 27                      # 128 MiB per partition: ~2.4 ms on the link
    k_parts = 8
    dev = "cuda:0"
    src = torch.arange(part // 4, dtype=torch.int32, device=dev)
    gbuf = torch.zeros(k_parts * part // 4, dtype=torch.int32, device=dev)
    host = torch.zeros(k_parts * part // 4, dtype=torch.int32, pin_memory=True)
    producer = torch.cuda.Stream()
    eng = zi.zi_engine_create(0, 64 * 1024, 3)
    try:
        def produce(k, reps):
            view = gbuf[k * part // 4:(k + 1) * part // 4]
            with torch.cuda.stream(producer):
                for _ in range(reps):
                    view.copy_(src)          # the last copy leaves the final value
                view.add_(k)

        # calibrate: production alone, offload alone
        reps = 60
        torch.cuda.synchronize()
        t0 = time.perf_counter(); produce(0, reps); producer.synchronize(); t_prod = time.perf_counter() - t0
        t0 = time.perf_counter()
        zi.zi_grad_offload(eng, gbuf, host, part, producer)
        t_call = time.perf_counter() - t0
        zi.zi_grad_offload_wait(eng)
        t_copy = time.perf_counter() - t0
        progress(f"offload: producing a partition {t_prod * 1e3:.2f} ms, draining it {t_copy * 1e3:.2f} ms, "
                 f"the call itself {t_call * 1e6:.0f} us")
        gbuf.zero_(); host.zero_()
        torch.cuda.synchronize()

        t0 = time.perf_counter()
        calls = []
        for k in range(k_parts):
            produce(k, reps)
            c0 = time.perf_counter()
            zi.zi_grad_offload(eng, gbuf[k * part // 4:], host[k * part // 4:], part, producer)
            calls.append(time.perf_counter() - c0)
        producer.synchronize()
        t_produced = time.perf_counter() - t0
        zi.zi_grad_offload_wait(eng)
        t_all = time.perf_counter() - t0
        serial = k_parts * (t_prod + t_copy)
        progress(f"offload: {k_parts} partitions produced in {t_produced * 1e3:.1f} ms, all on the host after "
                 f"{t_all * 1e3:.1f} ms; one after the other would be {serial * 1e3:.1f} ms; slowest call "
                 f"{max(calls) * 1e6:.0f} us")
        assert max(calls) < 0.5 * min(t_prod, t_copy), "zi_grad_offload blocked"
        assert t_all < 0.8 * serial, "the drain did not overlap the producer"
        for k in range(k_parts):
            want = (torch.arange(part // 4, dtype=torch.int32) + k)
            assert torch.equal(host[k * part // 4:(k + 1) * part // 4], want), f"partition {k}"
        # argument checks: pageable destination, host source
        with pytest.raises(zi.ZiError):
            zi.zi_grad_offload(eng, gbuf, np.zeros(16, np.int32), 64, producer)
        with pytest.raises(zi.ZiError):
            zi.zi_grad_offload(eng, host, host, 64, producer)
        assert zi.zi_grad_offload(eng, gbuf, host, 0, producer) == zi.ZI_OK
    finally:
        zi.zi_engine_destroy(eng)


def test_offloaded_gradients_feed_the_streamed_norm_and_step_without_a_host_wait():
    """Gradients offloaded with zi_grad_offload are consumed from host memory by zi_grad_norm_streamed and
    zi_adamw_step_streamed on the same engine with no wait in between: the engine orders itself after the
    offload.  Results equal the oracle's."""
    w = zi_synth.workload("c3")
    dt = zi.ZI_FP16
    n = 5 * 16384 + 77
    p, m, v, g = gen_numpy(w["spec"], n)
    d_g = to_dev(g)
    hg = torch.zeros(n, dtype=torch.int16, pin_memory=True)
    pp, pm, pv = (_pinned(a) for a in (p, m, v))
    hlp = torch.zeros(n, dtype=torch.int16, pin_memory=True)
    eng = zi.zi_engine_create(0, 64 * 1024, 3)
    try:
        nb = NormBuffers()
        zi.zi_grad_offload(eng, d_g, hg, 2 * n, torch.cuda.current_stream())
        tl = [(pp, pm, pv, hg, hlp, n)]
        zi.zi_grad_norm_streamed(eng, tl, dt, w["loss_scale"], nb.out, nb.ws)
        st = zi.zi_adamw_step_streamed(eng, tl, dt, zi_cfg(w), nb.out)
        assert st == zi.ZI_OK
    finally:
        zi.zi_engine_destroy(eng)
    assert np.array_equal(hg.numpy().view(np.uint16), g)
    sumsq, flag = oracle.grad_sumsq([g], dt)
    lpe = np.zeros(n, np.uint16)
    oracle.adamw(p, m, v, g, lpe, dt, oracle_cfg(w), sumsq, flag)
    progress("offload -> streamed norm + step: " +
             compare_state((p, m, v, lpe), (pp.numpy(), pm.numpy(), pv.numpy(), hlp.numpy().view(np.uint16)), dt))


# ------------------------------------------------------ the step on the CPUs, link carries g and p_lp

@pytest.mark.parametrize("dt", [zi.ZI_BF16, zi.ZI_FP16])
@pytest.mark.parametrize("pinned", [True, False])
def test_cpu_step_with_device_gradients_and_copy(dt, pinned):
    """zi_adamw_step_cpu: state in host memory (pinned or ordinary), gradients and the copy on the device.
    Bit-identical to zi_adamw_step_streamed on the same values and to the oracle; the link carried 2 + 2
    bytes per element."""
    w = zi_synth.workload("c4" if dt == zi.ZI_BF16 else "c3")
    spec = zi_synth.StateSpec(777 + dt, dt, g_std=1e-3 if dt == zi.ZI_BF16 else 65.536)
    sizes = [3 * 16384 + 5, 100, 16384, 0, 7, 2 * 16384 - 1, 40_000]
    host = [gen_numpy(spec, n, tensor=i) for i, n in enumerate(sizes)]
    kw = dict(max_grad_norm=0.02, loss_scale=1.0 if dt == zi.ZI_BF16 else 65536.0)
    ocfg, zcfg = oracle_cfg(w, **kw), zi_cfg(w, **kw)
    sumsq, flag = oracle.grad_sumsq([h[3] for h in host], dt)
    exp = []
    for (p, m, v, g) in host:
        pe, me, ve, lpe = p.copy(), m.copy(), v.copy(), np.zeros(p.size, np.uint16)
        oracle.adamw(pe, me, ve, g, lpe, dt, ocfg, sumsq, flag)
        exp.append((pe, me, ve, lpe))
    d_g = [to_dev(h[3]) for h in host]
    nb = NormBuffers()
    tl_norm = [(None, None, None, g, None, g.numel()) for g in d_g]
    zi.zi_grad_norm(tl_norm, dt, kw["loss_scale"], nb.out, nb.ws)

    def host_state():
        if pinned:
            return [tuple(_pinned(a) for a in h[:3]) for h in host]
        return [tuple(torch.from_numpy(a.copy()) for a in h[:3]) for h in host]

    eng = zi.zi_engine_create(0, 64 * 1024, 3)
    try:
        zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_RING_SLOTS, 4)
        # reference: the GPU-side streamed step
        st_a = host_state()
        lp_a = [torch.zeros(n, dtype=torch.int16, device="cuda:0") for n in sizes]
        assert zi.zi_adamw_step_streamed(eng, [(a[0], a[1], a[2], g, lp, n) for a, g, lp, n in
                                               zip(st_a, d_g, lp_a, sizes)], dt, zcfg, nb.out) == zi.ZI_OK
        # the CPU placement
        st_b = host_state()
        lp_b = [torch.full((n,), 0x5555, dtype=torch.int16, device="cuda:0") for n in sizes]
        assert zi.zi_adamw_step_cpu(eng, [(b[0], b[1], b[2], g, lp, n) for b, g, lp, n in
                                          zip(st_b, d_g, lp_b, sizes)], dt, zcfg, nb.out, 4,
                                    torch.cuda.current_stream()) == zi.ZI_OK
        stats = zi.zi_engine_last_stats(eng)
        total = sum(sizes)
        assert stats.bytes_d2h == 2 * total == stats.bytes_h2d
        for i, n in enumerate(sizes):
            for x, y in zip(st_a[i], st_b[i]):
                assert np.array_equal(x.numpy().view(np.uint32), y.numpy().view(np.uint32)), f"tensor {i}"
            assert torch.equal(lp_a[i], lp_b[i]), f"tensor {i}: copy"
            got = (st_b[i][0].numpy(), st_b[i][1].numpy(), st_b[i][2].numpy(), to_np(lp_b[i]))
            compare_state(exp[i], got, dt, f"cpu step tensor {i} ")
        # overflow: nothing moves, nothing changes
        bad = d_g[0].clone()
        bad[11] = np.array([0x7F80 if dt == zi.ZI_BF16 else 0x7C00], np.uint16).view(np.int16)[0]
        zi.zi_grad_norm([(None, None, None, bad, None, bad.numel())], dt, kw["loss_scale"], nb.out, nb.ws)
        before = [x.clone() for x in st_b[0]]
        lp_before = lp_b[0].clone()
        assert zi.zi_adamw_step_cpu(eng, [(st_b[0][0], st_b[0][1], st_b[0][2], bad, lp_b[0], sizes[0])], dt, zcfg,
                                    nb.out, 2) == zi.ZI_SKIPPED_OVERFLOW
        assert all(torch.equal(x, y) for x, y in zip(before, st_b[0])) and torch.equal(lp_before, lp_b[0])
        assert zi.zi_engine_last_stats(eng).bytes_d2h == 0
        # everything in host memory: no ring needed, no link traffic
        zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_RING_SLOTS, 0)
        st_c = host_state()
        hg = [torch.from_numpy(h[3].view(np.int16).copy()) for h in host]
        hlp = [torch.zeros(n, dtype=torch.int16) for n in sizes]
        assert zi.zi_adamw_step_cpu(eng, [(c[0], c[1], c[2], g, lp, n) for c, g, lp, n in zip(st_c, hg, hlp, sizes)],
                                    dt, zcfg, None, 3) == zi.ZI_OK
        # (no norm result here: compare with the oracle without clipping)
        for i, (p, m, v, g) in enumerate(host):
            pe, me, ve, lpe = p.copy(), m.copy(), v.copy(), np.zeros(p.size, np.uint16)
            oracle.adamw(pe, me, ve, g, lpe, dt, ocfg, None, 0)
            compare_state((pe, me, ve, lpe), (st_c[i][0].numpy(), st_c[i][1].numpy(), st_c[i][2].numpy(),
                                              hlp[i].numpy().view(np.uint16)), dt, f"cpu step, all host, tensor {i} ")
        assert zi.zi_engine_last_stats(eng).bytes_d2h == 0 == zi.zi_engine_last_stats(eng).bytes_h2d
        # device gradients without a ring are refused
        with pytest.raises(zi.ZiError):
            zi.zi_adamw_step_cpu(eng, [(st_c[0][0], st_c[0][1], st_c[0][2], d_g[0], None, sizes[0])], dt, zcfg, None, 2)
    finally:
        zi.zi_engine_destroy(eng)
    progress(f"cpu step (dt={dt}, pinned={pinned}): equal to the streamed GPU step and to the oracle")


def test_many_small_offloads_reuse_the_event_ring_and_order_a_consumer_stream():
    """More offloads than the engine has events (the ring of 64 is reused), each behind its own producer
    write; a consumer stream ordered with zi_grad_offload_order then reads the host copy through a
    host-to-device copy without any host-side wait."""
    k, part = 150, 4096
    dev = "cuda:0"
    gbuf = torch.zeros(k * part, dtype=torch.int32, device=dev)
    host = torch.zeros(k * part, dtype=torch.int32, pin_memory=True)
    back = torch.zeros(k * part, dtype=torch.int32, device=dev)
    producer, consumer = torch.cuda.Stream(), torch.cuda.Stream()
    eng = zi.zi_engine_create(0, 64 * 1024, 3)
    try:
        for i in range(k):
            with torch.cuda.stream(producer):
                gbuf[i * part:(i + 1) * part] = i + 1
            zi.zi_grad_offload(eng, gbuf[i * part:], host[i * part:], 4 * part, producer)
        zi.zi_grad_offload_order(eng, consumer)
        with torch.cuda.stream(consumer):
            back.copy_(host, non_blocking=True)
        consumer.synchronize()
        want = torch.arange(1, k + 1, dtype=torch.int32, device=dev).repeat_interleave(part)
        assert torch.equal(back, want)
        assert zi.zi_grad_offload_wait(eng) == zi.ZI_OK and zi.zi_grad_offload_wait(eng) == zi.ZI_OK
        assert torch.equal(host.to(dev), want)
    finally:
        zi.zi_engine_destroy(eng)


def test_cpu_step_over_a_long_ragged_list():
    """More short tensors than one slot use packs (32 segments), zero-length entries and tensors without a
    copy: zi_adamw_step_cpu against the oracle."""
    dt = zi.ZI_BF16
    w = zi_synth.workload("c4")
    rng = np.random.default_rng(8)
    sizes = [int(x) for x in rng.integers(0, 3000, 90)] + [16384 * 2 + 9, 0, 5]
    spec = zi_synth.StateSpec(99, dt)
    host = [gen_numpy(spec, n, tensor=i) for i, n in enumerate(sizes)]
    ocfg, zcfg = oracle_cfg(w, max_grad_norm=0.0), zi_cfg(w, max_grad_norm=0.0)
    st = [tuple(torch.from_numpy(a.copy()) for a in h[:3]) for h in host]
    d_g = [to_dev(h[3]) for h in host]
    lps = [None if i % 7 == 3 else torch.zeros(n, dtype=torch.int16, device="cuda:0") for i, n in enumerate(sizes)]
    eng = zi.zi_engine_create(0, 64 * 1024, 3)
    try:
        zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_RING_SLOTS, 3)
        assert zi.zi_adamw_step_cpu(eng, [(s[0], s[1], s[2], g, lp, n) for s, g, lp, n in zip(st, d_g, lps, sizes)],
                                    dt, zcfg, None, 3) == zi.ZI_OK
        stats = zi.zi_engine_last_stats(eng)
        assert stats.bytes_d2h == 2 * sum(sizes)
        assert stats.bytes_h2d == 2 * sum(n for n, lp in zip(sizes, lps) if lp is not None)
    finally:
        zi.zi_engine_destroy(eng)
    for i, (p, m, v, g) in enumerate(host):
        lpe = np.zeros(p.size, np.uint16)
        oracle.adamw(p, m, v, g, lpe, dt, ocfg, None, 0)
        got = (st[i][0].numpy(), st[i][1].numpy(), st[i][2].numpy(), None if lps[i] is None else to_np(lps[i]))
        compare_state((p, m, v, None if lps[i] is None else lpe), got, dt, f"tensor {i} ")
