"""The five workloads at their full sizes, in the launch configuration bench.py times.

At these sizes the oracle verifies seeded sample ranges (both ends, tile / chunk / 2^32 boundaries,
random places) that it recomputes from regenerated inputs, plus properties that hold for every
element: the low-precision copy equals the round-to-nearest-even cast of the stored fp32 parameter
(checked with the tensor library's own converter over the whole array), and a skipped step leaves
every bit in place.
"""
import ctypes
import math
import os
import shutil
import tempfile

import numpy as np
import pytest
import torch

import oracle
import paper_2104_07857_amd as zi
import zi_synth
from gpu_util import (NormBuffers, TOL_NORM_REL, compare_state, device_range, device_state, fill_device_f32,
                      fill_device_lp,
                      gen_numpy, oracle_cfg, oracle_range, progress, sample_ranges, to_np, zi_cfg)

pytestmark = pytest.mark.gpu

WIDTH = 1 << 16


def _lp_torch(dt):
    return torch.bfloat16 if dt == zi.ZI_BF16 else torch.float16


def _copy_matches_cast_everywhere(p_dev, lp_dev, dt, block=1 << 28):
    n = p_dev.numel()
    for lo in range(0, n, block):
        hi = min(lo + block, n)
        want = p_dev[lo:hi].to(_lp_torch(dt)).view(torch.int16)
        if not torch.equal(want, lp_dev[lo:hi]):
            bad = int((want != lp_dev[lo:hi]).sum())
            raise AssertionError(f"low-precision copy differs from the cast of p in [{lo},{hi}): {bad} elements")


def test_c1_resident_1p3e9():
    w = zi_synth.workload("c1")
    n, dt, spec = w["numel"][0], w["lp_dtype"], w["spec"]
    progress(f"c1: generating {n} elements")
    p, m, v, g, lp = device_state(spec, n)
    nb = NormBuffers()
    tl = [(p, m, v, g, lp, n)]
    zi.zi_grad_norm(tl, dt, w["loss_scale"], nb.out, nb.ws)
    zi.zi_adamw_step(tl, dt, zi_cfg(w), nb.out)
    torch.cuda.synchronize()
    sumsq, norm, flag = nb.read()
    assert flag == 0
    # N(0, 1e-3) gradients; the generator truncates to bf16, which shrinks magnitudes by about 0.3%
    assert abs(norm - 1e-3 * math.sqrt(n)) < 1e-2 * 1e-3 * math.sqrt(n)
    progress(f"c1: stepped; norm {norm:.5f}")
    # Sample ranges: both ends, seeded random places, and the places where the kernel's tile numbering
    # changes regime: the end of the first XCD's share (128 tiles of 512 elements) and of the first run
    # of 8 x 128 tiles, the start of the last complete run, and the incomplete run behind it (whose
    # workgroups keep their own tiles).
    run = 8 * 128 * 512
    last_run = (((n + 511) // 512) // (8 * 128)) * run
    ranges = sample_ranges(n, WIDTH, extra_points=(4096 * 1000, n // 2, 1 << 30, 128 * 512, run, last_run - run,
                                                   last_run, last_run + 128 * 512),
                           count=10, seed=1)
    worst = ""
    for lo, hi in ranges:
        exp = oracle_range(spec, dt, oracle_cfg(w), lo, hi)
        worst = compare_state(exp, device_range(p, m, v, lp, lo, hi), dt, f"c1 [{lo},{hi}) ")
    _copy_matches_cast_everywhere(p, lp, dt)
    assert bool((v >= 0).all()) and not bool(torch.isnan(p).any())
    progress(f"c1: {len(ranges)} ranges of {WIDTH} verified; last: {worst}")


def test_resident_tensor_longer_than_2_pow_32_elements():
    """Maximum sizes: one resident tensor of 2^32 + 2^20 + 3 elements (69 GB of arrays).  Element indices
    pass 2^31 and 2^32 inside one launch of each kernel: an overflow planted beyond 2^32 must be seen and
    skip the step, and the step proper must match the oracle around both boundaries and at the ragged end."""
    w = zi_synth.workload("c1")
    dt, spec = w["lp_dtype"], w["spec"]
    n = (1 << 32) + (1 << 20) + 3
    progress(f"2^32+: generating {n} elements")
    p, m, v, g, lp = device_state(spec, n)
    nb = NormBuffers()
    tl = [(p, m, v, g, lp, n)]
    cfg = zi_cfg(w, max_grad_norm=1.0)
    ranges = sample_ranges(n, WIDTH, extra_points=(1 << 31, 1 << 32, (1 << 32) + (1 << 20)), count=6, seed=9)
    before = [device_range(p, m, v, lp, lo, hi) for lo, hi in ranges]

    j = (1 << 32) + 12345
    keep = int(g[j])
    g[j] = 0x7F80                                   # +inf in bf16, beyond index 2^32
    zi.zi_grad_norm(tl, dt, w["loss_scale"], nb.out, nb.ws)
    zi.zi_adamw_step(tl, dt, cfg, nb.out)
    torch.cuda.synchronize()
    assert nb.read()[2] == 1
    for (lo, hi), b in zip(ranges, before):
        for x, y in zip(b, device_range(p, m, v, lp, lo, hi)):
            assert np.array_equal(x.view(np.uint8), y.view(np.uint8)), f"skipped step changed [{lo},{hi})"
    progress("2^32+: overflow beyond 2^32 seen, nothing changed")

    g[j] = keep
    zi.zi_grad_norm(tl, dt, w["loss_scale"], nb.out, nb.ws)
    zi.zi_adamw_step(tl, dt, cfg, nb.out)
    torch.cuda.synchronize()
    sumsq, norm, flag = nb.read()
    assert flag == 0
    progress("2^32+: stepped; oracle sum of squares over 4.3e9 regenerated gradients ...")
    hg = np.empty(n, np.uint16)
    for lo in range(0, n, 1 << 30):
        spec.fill_g(hg[lo:], min(1 << 30, n - lo), 0, lo)
    osumsq, oflag = oracle.grad_sumsq([hg], dt)
    del hg
    onorm = math.sqrt(osumsq)
    assert oflag == 0 and abs(norm - onorm) <= TOL_NORM_REL * onorm          # every element was counted
    assert abs(onorm - 1e-3 * math.sqrt(n)) < 1e-2 * 1e-3 * math.sqrt(n)
    worst = ""
    for lo, hi in ranges:
        exp = oracle_range(spec, dt, oracle_cfg(w, max_grad_norm=1.0), lo, hi, sumsq=osumsq)
        worst = compare_state(exp, device_range(p, m, v, lp, lo, hi), dt, f"2^32+ [{lo},{hi}) ")
    _copy_matches_cast_everywhere(p, lp, dt)
    progress(f"2^32+: norm {norm:.4f} (clip active), {len(ranges)} ranges verified; last: {worst}")


def test_c3_loss_scaled_fp16_2e9_overflow_then_clip():
    w = zi_synth.workload("c3")
    n, dt, spec = w["numel"][0], w["lp_dtype"], w["spec"]
    progress(f"c3: generating {n} elements")
    hg = np.empty(n, np.uint16)
    spec.fill_g(hg, n)
    p = torch.empty(n, dtype=torch.float32, device="cuda:0")
    m = torch.empty_like(p)
    v = torch.empty_like(p)
    fill_device_f32(lambda b, c, f: spec.fill_p(b, c, 0, f), n, p)
    fill_device_f32(lambda b, c, f: spec.fill_m(b, c, 0, f), n, m)
    fill_device_f32(lambda b, c, f: spec.fill_v(b, c, 0, f), n, v)
    g = torch.from_numpy(hg.view(np.int16)).to("cuda:0")
    lp = torch.zeros(n, dtype=torch.int16, device="cuda:0")
    nb = NormBuffers()
    tl = [(p, m, v, g, lp, n)]

    # run A: +inf at a seeded index; the step must leave all four arrays bit-identical
    j = zi_synth.pick_index(spec.seed, 0x696E66, n)
    saved = int(g[j].item())
    g[j] = 0x7C00
    p0, m0, v0 = p.clone(), m.clone(), v.clone()
    zi.zi_grad_norm(tl, dt, w["loss_scale"], nb.out, nb.ws)
    zi.zi_adamw_step(tl, dt, zi_cfg(w), nb.out)
    torch.cuda.synchronize()
    assert nb.read()[2] == 1
    assert torch.equal(p.view(torch.int32), p0.view(torch.int32))
    assert torch.equal(m.view(torch.int32), m0.view(torch.int32))
    assert torch.equal(v.view(torch.int32), v0.view(torch.int32))
    assert not bool(lp.any())
    del p0, m0, v0
    progress(f"c3 run A: +inf at {j}, flag raised, state bit-identical")

    # run B: unscale, global norm, clip to 1, update
    g[j] = saved
    zi.zi_grad_norm(tl, dt, w["loss_scale"], nb.out, nb.ws)
    zi.zi_adamw_step(tl, dt, zi_cfg(w), nb.out)
    torch.cuda.synchronize()
    sumsq, norm, flag = nb.read()
    progress("c3 run B: stepped; oracle sum of squares over 2e9 elements ...")
    osumsq, oflag = oracle.grad_sumsq([hg], dt)
    onorm = math.sqrt(osumsq) / w["loss_scale"]
    assert flag == oflag == 0
    assert abs(norm - onorm) <= TOL_NORM_REL * onorm
    assert abs(onorm - 44.72) < 0.1                      # 1e-3 sqrt(2e9)
    s = oracle.scalars(oracle_cfg(w), osumsq)
    assert abs(s.clip - 1.0 / (onorm + 1e-6)) < 1e-12 and 0.0222 < s.clip < 0.0225
    ranges = sample_ranges(n, WIDTH, extra_points=(j, 1 << 30, n // 3), count=8, seed=3)
    worst = ""
    for lo, hi in ranges:
        exp = oracle_range(spec, dt, oracle_cfg(w), lo, hi, sumsq=osumsq, found_inf=0)
        worst = compare_state(exp, device_range(p, m, v, lp, lo, hi), dt, f"c3 [{lo},{hi}) ")
    _copy_matches_cast_everywhere(p, lp, dt)
    progress(f"c3 run B: norm {norm:.6f} (oracle {onorm:.6f}), clip {s.clip:.6f}; "
             f"{len(ranges)} ranges verified; last: {worst}")


class PinnedF32:
    """fp32 array in pinned host memory from the library's allocator, viewed as numpy."""

    def __init__(self, n):
        self.n = n
        self.ptr = zi.zi_pinned_alloc(4 * max(n, 1))
        self.np = np.ctypeslib.as_array((ctypes.c_float * max(n, 1)).from_address(self.ptr))[:n]

    def free(self):
        self.np = None
        zi.zi_pinned_free(self.ptr)


def _host_equals_device_everywhere(host: np.ndarray, dev_t: torch.Tensor, what: str, block=1 << 28):
    """Bit-for-bit comparison of a host fp32 array with a device tensor, over every element."""
    stage = torch.empty(block, dtype=torch.int32, pin_memory=True)
    hv = host.view(np.int32)
    dv = dev_t.view(torch.int32)
    for lo in range(0, host.size, block):
        c = min(block, host.size - lo)
        stage.numpy()[:c] = hv[lo:lo + c]
        if not torch.equal(stage[:c].to("cuda:0"), dv[lo:lo + c]):
            raise AssertionError(f"{what}: host and device results differ in [{lo},{lo + c})")


def _resident_twin(hp, hm, hv, g, n, dt, cfg):
    """The same state stepped by the resident call: device copies of the host arrays, stepped in HBM."""
    twin = []
    stage = torch.empty(1 << 28, dtype=torch.float32, pin_memory=True)
    for h in (hp, hm, hv):
        d = torch.empty(n, dtype=torch.float32, device="cuda:0")
        for lo in range(0, n, 1 << 28):
            c = min(1 << 28, n - lo)
            stage.numpy()[:c] = h[lo:lo + c]
            d[lo:lo + c].copy_(stage[:c])
        twin.append(d)
    lp2 = torch.zeros(n, dtype=torch.int16, device="cuda:0")
    zi.zi_adamw_step([(twin[0], twin[1], twin[2], g, lp2, n)], dt, cfg)
    torch.cuda.synchronize()
    return twin[0], twin[1], twin[2], lp2


def _c2_streamed_from_pinned_host(n):
    """Workload 2's recipe at n elements: fp32 p/m/v in page-locked host memory, bf16 gradients and the
    copy in HBM, 64 MiB chunks, three slots.  Skips (with the allocator's message) if the state cannot
    be page-locked on this host."""
    w = zi_synth.workload("c2")
    dt, spec = w["lp_dtype"], w["spec"]
    chunk = w["chunk_bytes"] // 4
    got = []
    try:
        progress(f"c2: pinning 3 x {4 * n / 1e9:.0f} GB")
        for _ in range(3):
            got.append(PinnedF32(n))
    except zi.ZiError as e:
        for a in got:
            a.free()
        assert e.status == zi.ZI_ERR_NOMEM
        pytest.skip(f"3 x {4 * n / 1e9:.0f} GB cannot be page-locked on this host: {e.message}")
    hp, hm, hv = got
    eng = None
    try:
        progress("c2: generating host state")
        piece = 1 << 30
        for lo in range(0, n, piece):
            c = min(piece, n - lo)
            spec.fill_p(hp.np[lo:lo + c], c, 0, lo)
            spec.fill_m(hm.np[lo:lo + c], c, 0, lo)
            spec.fill_v(hv.np[lo:lo + c], c, 0, lo)
            progress(f"c2: host state {lo + c}/{n}")
        g = torch.empty(n, dtype=torch.int16, device="cuda:0")
        fill_device_lp(lambda b, c, f: spec.fill_g(b, c, 0, f), n, g)
        lp = torch.zeros(n, dtype=torch.int16, device="cuda:0")
        progress("c2: resident twin of the same state")
        tp, tm, tv, tlp = _resident_twin(hp.np, hm.np, hv.np, g, n, dt, zi_cfg(w))
        progress("c2: gradients resident; streaming")
        eng = zi.zi_engine_create(0, w["chunk_bytes"], w["n_slots"])
        st = zi.zi_adamw_step_streamed(eng, [(hp.ptr, hm.ptr, hv.ptr, g, lp, n)], dt, zi_cfg(w), None,
                                       torch.cuda.current_stream())
        assert st == zi.ZI_OK
        stats = zi.zi_engine_last_stats(eng)
        assert stats.n_slot_uses == (n + chunk - 1) // chunk and stats.bytes_h2d == 12 * n == stats.bytes_d2h
        assert n != 8_000_000_000 or stats.n_slot_uses == 477
        progress(f"c2: streamed in {stats.seconds:.2f} s = {12 * n / stats.seconds / 1e9:.1f} GB/s per direction")
        # Reads, the update and writes of different chunks overlap: were they serialised, the rate per
        # direction could not exceed half of the slower one-way rate.
        nbytes = 1 << 30
        scratch = PinnedF32(nbytes // 4)
        try:
            one_way = min(nbytes / zi.zi_engine_link_probe(eng, hp.ptr, scratch.ptr, nbytes, mode)
                          for mode in (0, 1))
        finally:
            scratch.free()
        assert 12 * n / stats.seconds > 0.6 * one_way, "the pipeline does not overlap its two directions"
        tail0 = (n // chunk) * chunk
        ranges = sample_ranges(n, WIDTH, extra_points=(chunk, 2 * chunk, 3 * chunk, 100 * chunk, 1 << 32, tail0),
                               count=8, seed=2)
        worst = ""
        for lo, hi in ranges:
            exp = oracle_range(spec, dt, oracle_cfg(w), lo, hi)
            got = (hp.np[lo:hi].copy(), hm.np[lo:hi].copy(), hv.np[lo:hi].copy(), to_np(lp[lo:hi]))
            worst = compare_state(exp, got, dt, f"c2 [{lo},{hi}) ")
        # every element: what came back to the host is what the resident call computes, bit for bit
        _host_equals_device_everywhere(hp.np, tp, "c2 p")
        _host_equals_device_everywhere(hm.np, tm, "c2 m")
        _host_equals_device_everywhere(hv.np, tv, "c2 v")
        assert torch.equal(lp, tlp), "c2: low-precision copy differs from the resident call's"
        progress(f"c2: {len(ranges)} ranges verified by the oracle, all {n} elements equal to the resident step; "
                 f"last: {worst}")
    finally:
        if eng is not None:
            zi.zi_engine_destroy(eng)
        for a in (hp, hm, hv):
            a.free()


def test_c2_streamed_8e9_from_pinned_host():
    """Workload 2 exactly as stated: 8e9 elements = 96 GB of page-locked state.  Hosts whose driver caps
    page-locked memory below that cannot run it; the test then SKIPS with the allocator's message (the
    5e9-element test below and the 8e9-element test through the pinned ring are separate tests)."""
    _c2_streamed_from_pinned_host(zi_synth.workload("c2")["numel"][0])


def test_c2_recipe_at_5e9_from_pinned_host():
    """The same recipe at 5e9 elements (60 GB page-locked): crosses the 2^32-element boundary and ends
    in a partial chunk."""
    _c2_streamed_from_pinned_host(5_000_000_000)


def test_c2_full_8e9_in_ordinary_host_memory_through_the_pinned_ring():
    """The full host-resident workload: 8e9 elements = 96 GB of fp32 state in ordinary host memory, staged
    through a 6-slot pinned ring (1.1 GiB) by CPU threads, 477 chunks of 64 MiB per array."""
    w = zi_synth.workload("c2")
    n, dt, spec = w["numel"][0], w["lp_dtype"], w["spec"]
    chunk = w["chunk_bytes"] // 4
    import psutil
    avail = psutil.virtual_memory().available
    if avail < 120 * (1 << 30):
        pytest.skip(f"needs 96 GB of host memory for the state, {avail / 2**30:.0f} GiB available")
    progress(f"c2-ring: generating 3 x {4 * n / 1e9:.0f} GB of ordinary host memory")
    hp, hm, hv = (np.empty(n, np.float32) for _ in range(3))
    piece = 1 << 30
    for lo in range(0, n, piece):
        c = min(piece, n - lo)
        spec.fill_p(hp[lo:lo + c], c, 0, lo)
        spec.fill_m(hm[lo:lo + c], c, 0, lo)
        spec.fill_v(hv[lo:lo + c], c, 0, lo)
        if (lo // piece) % 2 == 1:
            progress(f"c2-ring: host state {lo + c}/{n}")
    g = torch.empty(n, dtype=torch.int16, device="cuda:0")
    fill_device_lp(lambda b, c, f: spec.fill_g(b, c, 0, f), n, g)
    lp = torch.zeros(n, dtype=torch.int16, device="cuda:0")
    eng = zi.zi_engine_create(0, w["chunk_bytes"], w["n_slots"])
    try:
        zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_COPY_THREADS, 7)
        zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_RING_SLOTS, 6)
        progress("c2-ring: streaming")
        st = zi.zi_adamw_step_streamed(eng, [(hp, hm, hv, g, lp, n)], dt, zi_cfg(w), None,
                                       torch.cuda.current_stream())
        assert st == zi.ZI_OK
        stats = zi.zi_engine_last_stats(eng)
        assert stats.n_slot_uses == 477 and stats.bytes_h2d == 12 * n == stats.bytes_d2h
        assert stats.bytes_staged_host == 24 * n
        progress(f"c2-ring: streamed in {stats.seconds:.2f} s = {12 * n / stats.seconds / 1e9:.1f} GB/s per direction")
    finally:
        zi.zi_engine_destroy(eng)
    tail0 = (n // chunk) * chunk
    ranges = sample_ranges(n, WIDTH, extra_points=(chunk, 2 * chunk, 6 * chunk, 7 * chunk, 1 << 32, tail0),
                           count=8, seed=5)
    worst = ""
    for lo, hi in ranges:
        exp = oracle_range(spec, dt, oracle_cfg(w), lo, hi)
        got = (hp[lo:hi].copy(), hm[lo:hi].copy(), hv[lo:hi].copy(), to_np(lp[lo:hi]))
        worst = compare_state(exp, got, dt, f"c2-ring [{lo},{hi}) ")
    stage = torch.empty(1 << 28, dtype=torch.float32, pin_memory=True)
    for lo in range(0, n, 1 << 28):
        c = min(1 << 28, n - lo)
        stage.numpy()[:c] = hp[lo:lo + c]
        want = stage[:c].to("cuda:0").to(torch.bfloat16).view(torch.int16)
        assert torch.equal(want, lp[lo:lo + c]), f"copy/cast mismatch in [{lo},{lo + c})"
    del stage
    # every element: the resident call on freshly regenerated copies of the inputs gives the same bits
    progress("c2-ring: resident twin from regenerated inputs")
    tp, tm, tv, _, tlp = device_state(spec, n)
    zi.zi_adamw_step([(tp, tm, tv, g, tlp, n)], dt, zi_cfg(w))
    torch.cuda.synchronize()
    _host_equals_device_everywhere(hp, tp, "c2-ring p")
    _host_equals_device_everywhere(hm, tm, "c2-ring m")
    _host_equals_device_everywhere(hv, tv, "c2-ring v")
    assert torch.equal(lp, tlp)
    progress(f"c2-ring: {len(ranges)} ranges verified by the oracle, all {n} elements equal to the resident step; "
             f"last: {worst}")


def test_file_tier_one_gibi_elements_direct_io():
    """State in files on the box's disk (3 x 4 GiB, O_DIRECT), 64 MiB chunks through a 6-slot pinned ring:
    sample ranges against the oracle, and the step's rate beside the storage probe's."""
    w = zi_synth.workload("c2")
    n, dt, spec = 1 << 30, w["lp_dtype"], w["spec"]
    chunk = w["chunk_bytes"] // 4
    eng = None
    fds = []
    with tempfile.TemporaryDirectory(dir="/tmp") as tmp:
        try:
            free = shutil.disk_usage(tmp).free
            if free < 20 * (1 << 30):
                pytest.skip(f"needs 16 GiB of disk under /tmp for the state files, {free / 2**30:.0f} GiB free")
            paths = [os.path.join(tmp, k + ".bin") for k in "pmv"]
            buf = np.empty(1 << 28, np.float32)
            for path, fill in zip(paths, (spec.fill_p, spec.fill_m, spec.fill_v)):
                with open(path, "wb") as f:
                    for lo in range(0, n, buf.size):
                        fill(buf, buf.size, 0, lo)
                        f.write(buf.tobytes())
                progress(f"file tier: wrote {path}")
            os.sync()
            fds = [os.open(p, os.O_RDWR | os.O_DIRECT) for p in paths]
            g = torch.empty(n, dtype=torch.int16, device="cuda:0")
            fill_device_lp(lambda b, c, f: spec.fill_g(b, c, 0, f), n, g)
            lp = torch.zeros(n, dtype=torch.int16, device="cuda:0")
            eng = zi.zi_engine_create(0, w["chunk_bytes"], w["n_slots"])
            zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_COPY_THREADS, 16)
            zi.zi_engine_set_option(eng, zi.ZI_OPT_HOST_RING_SLOTS, 6)
            nbytes = 4 * n
            rd = nbytes / zi.zi_engine_file_probe(eng, fds[0], -1, nbytes) / 1e9
            scratch = os.open(os.path.join(tmp, "scratch.bin"), os.O_RDWR | os.O_CREAT | os.O_DIRECT, 0o600)
            fds.append(scratch)
            wr = nbytes / zi.zi_engine_file_probe(eng, -1, scratch, nbytes) / 1e9
            both = nbytes / zi.zi_engine_file_probe(eng, fds[1], scratch, nbytes) / 1e9
            progress(f"file tier: storage probe read {rd:.2f} GB/s, write {wr:.2f} GB/s, both at once {both:.2f} GB/s each")
            st = zi.zi_adamw_step_files(eng, [(fds[0], fds[1], fds[2], 0, 0, 0, g, lp, n)], dt, zi_cfg(w), None,
                                        torch.cuda.current_stream())
            assert st == zi.ZI_OK
            stats = zi.zi_engine_last_stats(eng)
            assert stats.n_slot_uses == n // chunk and stats.bytes_h2d == 12 * n
            rate = 12 * n / stats.seconds / 1e9
            progress(f"file tier: step in {stats.seconds:.2f} s = {rate:.2f} GB/s read and {rate:.2f} GB/s written "
                     f"({rate / both:.2f} of the two-way probe)")
            for fd in fds:
                os.close(fd)
            fds = []
            maps = [np.memmap(p, dtype=np.float32, mode="r") for p in paths]
            ranges = sample_ranges(n, WIDTH, extra_points=(chunk, 5 * chunk, 6 * chunk), count=6, seed=7)
            worst = ""
            for lo, hi in ranges:
                exp = oracle_range(spec, dt, oracle_cfg(w), lo, hi)
                got = tuple(np.array(mm[lo:hi]) for mm in maps) + (to_np(lp[lo:hi]),)
                worst = compare_state(exp, got, dt, f"file tier [{lo},{hi}) ")
            for lo in range(0, n, 1 << 28):
                want = torch.from_numpy(np.array(maps[0][lo:lo + (1 << 28)])).to("cuda:0").to(torch.bfloat16)
                assert torch.equal(want.view(torch.int16), lp[lo:lo + (1 << 28)])
            del maps
            progress(f"file tier: {len(ranges)} ranges verified, copy consistent everywhere; last: {worst}")
        finally:
            for fd in fds:
                os.close(fd)
            if eng is not None:
                zi.zi_engine_destroy(eng)


def test_everything_offloaded_one_gibi_elements():
    """All five arrays in pinned host memory (16 GiB): norm reduced from host-resident gradients, then the
    step with gradients travelling in and the low-precision copy travelling out with each chunk."""
    w = zi_synth.workload("c2")
    n, dt, spec = 1 << 30, w["lp_dtype"], w["spec"]
    chunk = w["chunk_bytes"] // 4
    hp, hm, hv = PinnedF32(n), PinnedF32(n), PinnedF32(n)
    hg = torch.empty(n, dtype=torch.int16, pin_memory=True)
    hlp = torch.zeros(n, dtype=torch.int16, pin_memory=True)
    eng = None
    try:
        spec.fill_p(hp.np, n)
        spec.fill_m(hm.np, n)
        spec.fill_v(hv.np, n)
        spec.fill_g(hg, n)
        progress("offload: state, gradients and copy in pinned host memory")
        eng = zi.zi_engine_create(0, w["chunk_bytes"], w["n_slots"])
        tl = [(hp.ptr, hm.ptr, hv.ptr, hg, hlp, n)]
        nb = NormBuffers()
        cfg = dict(max_grad_norm=1.0)
        zi.zi_grad_norm_streamed(eng, tl, dt, 1.0, nb.out, nb.ws, stream=torch.cuda.current_stream())
        ns = zi.zi_engine_last_stats(eng)
        sumsq, norm, flag = nb.read()
        progress(f"offload: norm pass {ns.seconds * 1e3:.1f} ms = {2 * n / ns.seconds / 1e9:.1f} GB/s over the link")
        st = zi.zi_adamw_step_streamed(eng, tl, dt, zi_cfg(w, **cfg), nb.out, torch.cuda.current_stream())
        assert st == zi.ZI_OK
        stats = zi.zi_engine_last_stats(eng)
        assert stats.bytes_h2d == 14 * n == stats.bytes_d2h
        progress(f"offload: step in {stats.seconds:.3f} s = {14 * n / stats.seconds / 1e9:.1f} GB/s per direction")
        osumsq, oflag = oracle.grad_sumsq([hg.numpy().view(np.uint16)], dt)
        assert flag == oflag == 0 and abs(sumsq - osumsq) <= 1e-12 * osumsq
        assert oracle.scalars(oracle_cfg(w, **cfg), osumsq).clip < 0.04
        ranges = sample_ranges(n, WIDTH, extra_points=(chunk, 2 * chunk, 3 * chunk), count=6, seed=9)
        worst = ""
        lp_np = hlp.numpy().view(np.uint16)
        for lo, hi in ranges:
            exp = oracle_range(spec, dt, oracle_cfg(w, **cfg), lo, hi, sumsq=osumsq)
            got = (hp.np[lo:hi].copy(), hm.np[lo:hi].copy(), hv.np[lo:hi].copy(), lp_np[lo:hi].copy())
            worst = compare_state(exp, got, dt, f"offload [{lo},{hi}) ")
        want = torch.from_numpy(hp.np[:1 << 28]).to("cuda:0").to(torch.bfloat16).view(torch.int16).cpu()
        assert torch.equal(want, hlp[:1 << 28])
        progress(f"offload: norm {norm:.5f}; {len(ranges)} ranges verified; last: {worst}")
    finally:
        if eng is not None:
            zi.zi_engine_destroy(eng)
        for a in (hp, hm, hv):
            a.free()


def test_c4_ragged_transformer_layers_streamed_with_clip():
    w = zi_synth.workload("c4")
    numel, dt, spec = w["numel"], w["lp_dtype"], w["spec"]
    assert len(numel) == 48
    progress(f"c4: 48 tensors, {sum(numel)} elements, 144 pinned arrays")
    host, grads, lps, hgs = [], [], [], []
    eng = None
    try:
        for i, n in enumerate(numel):
            arrs = (PinnedF32(n), PinnedF32(n), PinnedF32(n))
            host.append(arrs)
            spec.fill_p(arrs[0].np, n, i)
            spec.fill_m(arrs[1].np, n, i)
            spec.fill_v(arrs[2].np, n, i)
            hg = np.empty(n, np.uint16)
            spec.fill_g(hg, n, i)
            hgs.append(hg)
            grads.append(torch.from_numpy(hg.view(np.int16)).to("cuda:0"))
            lps.append(torch.zeros(n, dtype=torch.int16, device="cuda:0"))
            if i % 12 == 11:
                progress(f"c4: layer {i // 12} generated")
        nb = NormBuffers()
        tl = [(a[0].ptr, a[1].ptr, a[2].ptr, g, lp, n) for a, g, lp, n in zip(host, grads, lps, numel)]
        zi.zi_grad_norm(tl, dt, w["loss_scale"], nb.out, nb.ws)
        eng = zi.zi_engine_create(0, w["chunk_bytes"], w["n_slots"])
        st = zi.zi_adamw_step_streamed(eng, tl, dt, zi_cfg(w), nb.out, torch.cuda.current_stream())
        assert st == zi.ZI_OK
        stats = zi.zi_engine_last_stats(eng)
        assert stats.n_slot_uses == 193 and stats.bytes_h2d == 12 * sum(numel)
        sumsq, norm, flag = nb.read()
        progress(f"c4: streamed in {stats.seconds:.2f} s; oracle sum of squares over 3.2e9 elements ...")
        osumsq, oflag = oracle.grad_sumsq(hgs, dt)
        onorm = math.sqrt(osumsq)
        assert flag == oflag == 0 and abs(norm - onorm) <= TOL_NORM_REL * onorm
        assert abs(onorm - 56.76) < 0.57                 # 1e-3 sqrt(3.22e9), bf16-truncated gradients
        ocfg = oracle_cfg(w)
        assert 0.0174 < oracle.scalars(ocfg, osumsq).clip < 0.0179
        worst = ""
        checked = 0
        chunk = w["chunk_bytes"] // 4
        for i, n in enumerate(numel):
            if n <= 4 * 8192:
                ranges = [(0, n)]                         # every small tensor in full
            elif i % 12 in (2, 10) and i // 12 in (0, 3):
                ranges = sample_ranges(n, WIDTH, extra_points=(chunk, n - chunk), count=2, seed=i)
            else:
                ranges = sample_ranges(n, 8192, count=0, seed=i)     # both ends of every large tensor
            for lo, hi in ranges:
                exp = oracle_range(spec, dt, ocfg, lo, hi, tensor=i, sumsq=osumsq)
                got = (host[i][0].np[lo:hi].copy(), host[i][1].np[lo:hi].copy(), host[i][2].np[lo:hi].copy(),
                       to_np(lps[i][lo:hi]))
                worst = compare_state(exp, got, dt, f"c4 tensor {i} [{lo},{hi}) ")
                checked += hi - lo
        progress(f"c4: norm {norm:.5f} (oracle {onorm:.5f}); {checked} elements verified over 48 tensors; "
                 f"last: {worst}")

        # The same list HBM-resident (long tensors get launches of their own, the 32 short ones share
        # one): every array must equal the streamed result bit for bit, over all 3.2e9 elements.
        progress("c4: the same list resident ...")
        res = []
        for i, n in enumerate(numel):
            dp, dm, dv = (torch.empty(n, dtype=torch.float32, device="cuda:0") for _ in range(3))
            fill_device_f32(lambda b, c, f: spec.fill_p(b, c, i, f), n, dp)
            fill_device_f32(lambda b, c, f: spec.fill_m(b, c, i, f), n, dm)
            fill_device_f32(lambda b, c, f: spec.fill_v(b, c, i, f), n, dv)
            res.append((dp, dm, dv, torch.zeros(n, dtype=torch.int16, device="cuda:0")))
        zi.zi_adamw_step([(r[0], r[1], r[2], g, r[3], n) for r, g, n in zip(res, grads, numel)], dt, zi_cfg(w), nb.out)
        torch.cuda.synchronize()
        for i, (r, arrs) in enumerate(zip(res, host)):
            for k in range(3):
                streamed = torch.from_numpy(arrs[k].np).to("cuda:0")
                assert torch.equal(streamed.view(torch.int32), r[k].view(torch.int32)), f"tensor {i} array {k}"
                del streamed
            assert torch.equal(r[3], lps[i]), f"tensor {i} copy"
        del res
        progress("c4: resident list equals the streamed result bit for bit over all 48 tensors")
    finally:
        if eng is not None:
            zi.zi_engine_destroy(eng)
        for arrs in host:
            for a in arrs:
                a.free()
