"""zi_grad_norm_noalloc (partials in the library's fixed device array) against zi_grad_norm."""
import ctypes
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2104_07857_amd as zi
import zi_synth
from gpu_util import NormBuffers, TOL_NORM_REL, progress, to_dev

pytestmark = pytest.mark.gpu


def _grads(n, dt, seed, std=1e-3):
    g = np.empty(n, np.uint16)
    zi_synth.fill_normal_lp(g, n, seed, zi_synth.STREAM_G, dt, std=std)
    return g


def _read(out):
    raw = out.cpu().numpy()
    return float(raw[0]), float(raw[1]), int(raw[2:3].view(np.uint32)[0])


def _both(tensors, dt, loss_scale):
    """(result of zi_grad_norm, result of zi_grad_norm_noalloc) on the same device gradients."""
    tl = zi.make_tensors([(None, None, None, d, None, d.numel()) for d in tensors])
    nb = NormBuffers()
    zi.zi_grad_norm(tl, dt, loss_scale, nb.out, nb.ws)
    torch.cuda.synchronize()
    ref = nb.read()
    out = torch.full((3,), float("nan"), dtype=torch.float64, device="cuda:0")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    zi.zi_grad_norm_noalloc(tl, dt, loss_scale, out, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return ref, _read(out)


def _agree(ref, got):
    assert got[2] == ref[2]                                       # flag: bit-exact
    if ref[2] == 0:
        assert abs(got[0] - ref[0]) <= 1e-12 * max(ref[0], 1e-300)
        assert abs(got[1] - ref[1]) <= TOL_NORM_REL * max(ref[1], 1e-300)


@pytest.mark.parametrize("dt", [zi.ZI_BF16, zi.ZI_FP16])
def test_two_calls_in_a_row_the_second_smaller(dt):
    """The second call reuses the array the first one filled: stale partials of the larger call must
    not leak into the smaller one's result."""
    std = 1e-3 if dt == zi.ZI_BF16 else 65.536
    big = [to_dev(_grads(n, dt, 700 + i, std)) for i, n in enumerate([(1 << 24) + 5, 1_000_003, 7, 16384 * 9 + 1])]
    small = [to_dev(_grads(n, dt, 800 + i, 50 * std)) for i, n in enumerate([4099, 1])]
    progress(f"no-alloc norm, dt={dt}: list of {sum(x.numel() for x in big)} elements, then {sum(x.numel() for x in small)}")
    ref, got = _both(big, dt, 4.0)
    _agree(ref, got)
    assert got[0] == ref[0]            # same block partition below the scratch limit: bit-identical sum
    want, wflag = oracle.grad_sumsq([x.cpu().numpy().view(np.uint16) for x in big], dt)
    assert wflag == got[2] == 0 and abs(got[1] - math.sqrt(want) / 4.0) <= TOL_NORM_REL * math.sqrt(want) / 4.0
    ref2, got2 = _both(small, dt, 4.0)
    _agree(ref2, got2)
    assert got2[0] == ref2[0]
    want2, _ = oracle.grad_sumsq([x.cpu().numpy().view(np.uint16) for x in small], dt)
    assert abs(got2[1] - math.sqrt(want2) / 4.0) <= TOL_NORM_REL * math.sqrt(want2) / 4.0
    # an inf in the second list, then a clean third call: the flag does not stick in the array
    bad = small[0].clone()
    bad[17] = np.array([0x7F80 if dt == zi.ZI_BF16 else 0x7C00], np.uint16).view(np.int16)[0]
    ref3, got3 = _both([bad, small[1]], dt, 4.0)
    assert ref3[2] == got3[2] == 1
    ref4, got4 = _both(small, dt, 4.0)
    assert got4 == got2 and ref4 == ref2
    # empty list: defined zeros
    _, got5 = _both([], dt, 1.0)
    assert got5 == (0.0, 0.0, 0)


def test_more_blocks_than_the_array_holds_and_the_list_limit():
    dt = zi.ZI_BF16
    n = 4096 * 4 * 16384            # a tensor that takes the per-tensor maximum of 4096 workgroups
    big = to_dev(_grads(n, dt, 6))
    progress("no-alloc norm: 5 x 4096 workgroups asked for, 16384 partials available")
    ref, got = _both([big] * 5, dt, 1.0)      # zi_grad_norm makes an intermediate pass; no-alloc uses fewer blocks
    _agree(ref, got)
    # then a small call right behind it
    ref2, got2 = _both([big[:1000]], dt, 1.0)
    _agree(ref2, got2)
    assert got2[0] == ref2[0]
    # more non-empty tensors than partials: refused before anything is launched
    out = torch.full((3,), 7.0, dtype=torch.float64, device="cuda:0")
    many = zi.make_tensors([(None, None, None, big[i:i + 1], None, 1) for i in range(zi.ZI_NOALLOC_MAX_PARTIALS + 1)])
    with pytest.raises(zi.ZiError) as e:
        zi.zi_grad_norm_noalloc(many, dt, 1.0, out)
    assert e.value.status == zi.ZI_ERR_UNSUPPORTED and "16384" in e.value.message
    torch.cuda.synchronize()
    assert out.cpu().tolist() == [7.0, 7.0, 7.0]
    # exactly at the limit it runs
    lim = zi.make_tensors([(None, None, None, big[i:i + 1], None, 1) for i in range(zi.ZI_NOALLOC_MAX_PARTIALS)])
    zi.zi_grad_norm_noalloc(lim, dt, 1.0, out)
    torch.cuda.synchronize()
    want, _ = oracle.grad_sumsq([big[:zi.ZI_NOALLOC_MAX_PARTIALS].cpu().numpy().view(np.uint16)], dt)
    assert abs(_read(out)[0] - want) <= 1e-12 * want


def test_captured_into_a_graph_with_the_step():
    """What the entry point is for: under stream capture nothing may allocate.  zi_grad_norm_noalloc and
    zi_adamw_step are captured once (after one eager call has looked up the array's address) and replayed
    three times with eager work in between; every replay equals the same number of eager steps."""
    from gpu_util import gen_numpy, zi_cfg
    w = zi_synth.workload("c4")
    dt = zi.ZI_BF16
    rng = np.random.default_rng(3)
    numel = [int(x) for x in rng.integers(1, 60_000, 40)] + [1_000_003]
    spec = zi_synth.StateSpec(77, dt, g_std=2e-3)
    host = [gen_numpy(spec, n, tensor=i) for i, n in enumerate(numel)]

    def device_copy():
        ts = [tuple(to_dev(a) for a in t) + (torch.zeros(t[0].size, dtype=torch.int16, device="cuda:0"),) for t in host]
        return ts, zi.make_tensors([t + (t[0].numel(),) for t in ts])

    cfg = zi_cfg(w)
    eager, eager_tl = device_copy()
    graphed, graphed_tl = device_copy()
    out_e = torch.zeros(4, dtype=torch.float64, device="cuda:0")
    out_g = torch.zeros(4, dtype=torch.float64, device="cuda:0")
    zi.zi_grad_norm_noalloc(eager_tl, dt, 1.0, out_e)            # first call on this device: not under capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        zi.zi_grad_norm_noalloc(graphed_tl, dt, 1.0, out_g, stream=side)
        zi.zi_adamw_step(graphed_tl, dt, cfg, out_g, stream=side)
        graph.capture_end()
    torch.cuda.synchronize()
    for a, b in zip(eager, graphed):
        assert torch.equal(a[0], b[0])                           # capture executed nothing
    for replay in range(3):
        graph.replay()
        torch.cuda.synchronize()
        zi.zi_grad_norm_noalloc(eager_tl, dt, 1.0, out_e)
        zi.zi_adamw_step(eager_tl, dt, cfg, out_e)
        torch.cuda.synchronize()
        assert torch.rand(1 << 18, device="cuda:0").sum().item() > 0          # unrelated eager work between replays
        assert _read(out_e) == _read(out_g), f"replay {replay}: norm result differs"
        for i, (a, b) in enumerate(zip(eager, graphed)):
            for x, y in zip(a, b):
                assert torch.equal(x, y), f"replay {replay}, tensor {i}"
