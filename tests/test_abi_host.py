"""Host-side checks of the C-ABI library: exports, argument validation, chunk planning (no GPU needed)."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2104_07857_amd as zi
import zi_synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = "".join(open(os.path.join(ROOT, "include", f)).read() for f in sorted(os.listdir(os.path.join(ROOT, "include")))
                   if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(zi_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    declared = _declared_functions()
    assert len(declared) >= 20
    L = ctypes.CDLL(zi.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), f"{name} declared in include/zi.h but not exported"
    assert sorted(zi.EXPORTS) == declared
    for name in declared:
        assert callable(getattr(zi, name)), f"binding lacks {name}"


def test_struct_layouts_match_the_header():
    assert ctypes.sizeof(zi.zi_norm_result) == 32
    assert ctypes.sizeof(zi.zi_tensor) == 48
    assert ctypes.sizeof(zi.zi_adamw_config) == 48
    assert ctypes.sizeof(zi.zi_chunk_segment) == 40
    assert ctypes.sizeof(zi.zi_stream_stats) == 56
    assert ctypes.sizeof(zi.zi_file_tensor) == 64
    assert zi.zi_norm_workspace_bytes(10 ** 10, 50) == 16384 * 16


def _arrays(n=64):
    return (np.zeros(n, np.float32), np.zeros(n, np.float32), np.zeros(n, np.float32),
            np.zeros(n, np.uint16), np.zeros(n, np.uint16))


@pytest.mark.parametrize("bad,status", [
    (dict(step=0), zi.ZI_ERR_INVALID_ARG), (dict(beta1=1.0), zi.ZI_ERR_INVALID_ARG),
    (dict(beta2=-0.5), zi.ZI_ERR_INVALID_ARG), (dict(eps=-1e-8), zi.ZI_ERR_INVALID_ARG),
    (dict(loss_scale=0.0), zi.ZI_ERR_INVALID_ARG), (dict(loss_scale=float("inf")), zi.ZI_ERR_INVALID_ARG),
    (dict(loss_scale=float("nan")), zi.ZI_ERR_INVALID_ARG), (dict(mode=3), zi.ZI_ERR_INVALID_ARG),
    (dict(lr=float("nan")), zi.ZI_ERR_INVALID_ARG), (dict(max_grad_norm=float("nan")), zi.ZI_ERR_INVALID_ARG)])
def test_step_rejects_bad_configurations_before_touching_anything(bad, status):
    p, m, v, g, lp = _arrays()
    with pytest.raises(zi.ZiError) as e:
        zi.zi_adamw_step([(p, m, v, g, lp)], zi.ZI_BF16, zi.make_config(**bad))
    assert e.value.status == status and e.value.message
    assert not p.any() and not lp.any()


def test_step_rejects_bad_tensors():
    p, m, v, g, lp = _arrays()
    cfg = zi.make_config()
    with pytest.raises(zi.ZiError) as e:
        zi.zi_adamw_step([(p, m, v, g, lp)], 7, cfg)
    assert e.value.status == zi.ZI_ERR_INVALID_ARG
    with pytest.raises(zi.ZiError) as e:
        zi.zi_adamw_step([(p, m, v, g, lp, -1)], zi.ZI_BF16, cfg)
    assert e.value.status == zi.ZI_ERR_INVALID_ARG
    with pytest.raises(zi.ZiError) as e:
        zi.zi_adamw_step([(p, None, v, g, lp, 64)], zi.ZI_BF16, cfg)
    assert e.value.status == zi.ZI_ERR_INVALID_ARG
    with pytest.raises(zi.ZiError) as e:
        zi.zi_adamw_step([(p.ctypes.data + 2, m, v, g, lp, 8)], zi.ZI_BF16, cfg)
    assert e.value.status == zi.ZI_ERR_ALIGNMENT
    with pytest.raises(zi.ZiError) as e:
        zi.zi_adamw_step([(p, m, v, g.ctypes.data + 1, lp, 8)], zi.ZI_BF16, cfg)
    assert e.value.status == zi.ZI_ERR_ALIGNMENT
    with pytest.raises(zi.ZiError) as e:
        zi.zi_adamw_step([(p, p, v, g, lp)], zi.ZI_BF16, cfg)
    assert e.value.status == zi.ZI_ERR_INVALID_ARG
    assert zi.lib().zi_adamw_step(None, 3, 0, ctypes.byref(cfg), None, None) == zi.ZI_ERR_INVALID_ARG
    assert zi.lib().zi_adamw_step(None, -1, 0, ctypes.byref(cfg), None, None) == zi.ZI_ERR_INVALID_ARG
    assert zi.lib().zi_adamw_step(None, 0, 0, None, None, None) == zi.ZI_ERR_INVALID_ARG
    # empty lists and empty tensors are valid and do nothing, even with no GPU
    assert zi.zi_adamw_step([], zi.ZI_BF16, cfg) == zi.ZI_OK
    assert zi.zi_adamw_step([(None, None, None, None, None, 0)], zi.ZI_FP16, cfg) == zi.ZI_OK


def test_norm_rejects_bad_arguments():
    g = np.zeros(64, np.uint16)
    out = np.zeros(4, np.float64)
    ws = np.zeros(zi.zi_norm_workspace_bytes() // 8, np.float64)
    t = [(None, None, None, g, None)]
    nb = ws.nbytes
    cases = [
        (dict(tensors=t, dt=9, loss_scale=1.0, d_out=out, d_workspace=ws, workspace_bytes=nb), zi.ZI_ERR_INVALID_ARG),
        (dict(tensors=t, dt=0, loss_scale=0.0, d_out=out, d_workspace=ws, workspace_bytes=nb), zi.ZI_ERR_INVALID_ARG),
        (dict(tensors=t, dt=0, loss_scale=1.0, d_out=None, d_workspace=ws, workspace_bytes=nb), zi.ZI_ERR_INVALID_ARG),
        (dict(tensors=t, dt=0, loss_scale=1.0, d_out=out.ctypes.data + 4, d_workspace=ws, workspace_bytes=nb),
         zi.ZI_ERR_ALIGNMENT),
        (dict(tensors=t, dt=0, loss_scale=1.0, d_out=out, d_workspace=None, workspace_bytes=nb), zi.ZI_ERR_INVALID_ARG),
        (dict(tensors=t, dt=0, loss_scale=1.0, d_out=out, d_workspace=ws.ctypes.data + 8, workspace_bytes=nb - 8),
         zi.ZI_ERR_ALIGNMENT),
        (dict(tensors=t, dt=0, loss_scale=1.0, d_out=out, d_workspace=ws, workspace_bytes=1024), zi.ZI_ERR_INVALID_ARG),
        (dict(tensors=[(None, None, None, None, None, 5)], dt=0, loss_scale=1.0, d_out=out, d_workspace=ws,
              workspace_bytes=nb), zi.ZI_ERR_INVALID_ARG),
        (dict(tensors=[(None, None, None, g.ctypes.data + 1, None, 5)], dt=0, loss_scale=1.0, d_out=out,
              d_workspace=ws, workspace_bytes=nb), zi.ZI_ERR_ALIGNMENT),
    ]
    for kw, status in cases:
        with pytest.raises(zi.ZiError) as e:
            zi.zi_grad_norm(**kw)
        assert e.value.status == status, kw


def test_engine_and_misc_argument_checks():
    for args in ((0, 0, 3), (0, 100, 3), (0, 256, 3), (0, 1 << 20, 1), (0, 1 << 20, 9), (-1, 1 << 20, 3)):
        with pytest.raises(zi.ZiError) as e:
            zi.zi_engine_create(*args)
        assert e.value.status == zi.ZI_ERR_INVALID_ARG
    assert zi.zi_engine_destroy(None) == zi.ZI_OK
    assert zi.zi_pinned_free(None) == zi.ZI_OK
    with pytest.raises(zi.ZiError):
        zi.zi_pinned_alloc(0)
    p, m, v, g, lp = _arrays()
    with pytest.raises(zi.ZiError) as e:
        zi.zi_adamw_step_streamed(None, [(p, m, v, g, lp)], zi.ZI_BF16, zi.make_config())
    assert e.value.status == zi.ZI_ERR_INVALID_ARG
    with pytest.raises(zi.ZiError) as e:
        zi.zi_adamw_step_files(None, [], zi.ZI_BF16, zi.make_config())
    assert e.value.status == zi.ZI_ERR_INVALID_ARG
    with pytest.raises(zi.ZiError):
        zi.zi_engine_file_probe(None, -1, -1, 4096)
    with pytest.raises(zi.ZiError):
        zi.zi_engine_last_stats(None)
    # the calls added around the streamed step refuse a missing engine the same way, before anything else
    for call in (lambda: zi.zi_grad_offload(None, p, m, 64),
                 lambda: zi.zi_grad_offload_wait(None),
                 lambda: zi.zi_grad_offload_order(None),
                 lambda: zi.zi_adamw_step_cpu(None, [(p, m, v, g, lp)], zi.ZI_BF16, zi.make_config(), None, 2),
                 lambda: zi.zi_engine_link_probe(None, p, m, 64, 0),
                 lambda: zi.zi_grad_norm_streamed(None, [(None, None, None, g, None, 64)], zi.ZI_BF16, 1.0, 8, 16, 1 << 20)):
        with pytest.raises(zi.ZiError) as e:
            call()
        assert e.value.status == zi.ZI_ERR_INVALID_ARG and "engine" in e.value.message
    # the no-allocation reduction validates like zi_grad_norm (no GPU here: the device query fails first)
    with pytest.raises(zi.ZiError) as e:
        zi.zi_grad_norm_noalloc([(None, None, None, g, None, 64)], zi.ZI_BF16, 1.0, 8)
    assert e.value.status in (zi.ZI_ERR_HIP, zi.ZI_ERR_INVALID_ARG)
    with pytest.raises(zi.ZiError):
        zi.zi_engine_set_option(None, 0, 1)
    buf = np.zeros(64, np.float32)
    for args in ((buf, buf, 256, 3), (None, buf, 256, 0), (buf, None, 256, 1), (buf, buf, 0, 0), (buf, buf, 100, 0)):
        with pytest.raises(zi.ZiError) as e:
            zi.zi_hbm_probe(*args)
        assert e.value.status == zi.ZI_ERR_INVALID_ARG
    with pytest.raises(zi.ZiError) as e:
        zi.zi_hbm_probe(buf.ctypes.data + 4, buf, 64, 0)
    assert e.value.status == zi.ZI_ERR_ALIGNMENT


def _check_plan(numel, chunk):
    segs, uses = zi.zi_plan_chunks(numel, chunk)
    covered = [0] * len(numel)
    per_use = {}
    last_use = -1
    for s in segs:
        assert 0 <= s.tensor < len(numel) and s.count > 0
        assert s.elem_offset == covered[s.tensor], "segments of a tensor are contiguous and in order"
        covered[s.tensor] += s.count
        assert s.slot_use >= last_use, "segments come sorted by slot use"
        last_use = s.slot_use
        per_use.setdefault(s.slot_use, []).append(s)
        assert s.slot_offset % 1024 == 0
        assert s.slot_offset + s.count <= chunk + 0 or (s.slot_offset == 0 and s.count <= chunk)
    assert covered == list(numel), "every element travels exactly once"
    assert sorted(per_use) == list(range(uses)), "slot uses are numbered without gaps"
    for u, ss in per_use.items():
        assert len(ss) <= 32
        spans = sorted((s.slot_offset, s.slot_offset + s.count + 8) for s in ss)
        for (a0, a1), (b0, b1) in zip(spans, spans[1:]):
            assert a1 <= b0, "packed segments (with their lead-in room) do not overlap"
        if len(ss) > 1:
            assert spans[-1][1] <= chunk
    return segs, uses


def test_chunk_plans_of_the_workloads():
    chunk = (64 << 20) // 4
    segs, uses = _check_plan([8_000_000_000], chunk)
    assert uses == 477 and segs[-1].count == 14_045_184 and segs[0].count == 16_777_216
    segs, uses = _check_plan(zi_synth.workload("c4")["numel"], chunk)
    assert uses == 4 * (12 + 4 + 16 + 16) + 1          # whole chunks of the 16 weights + one packed use
    assert sum(1 for s in segs if s.slot_use == uses - 1) == 32


def test_chunk_plans_of_awkward_lists():
    _check_plan([], 1024)
    _check_plan([0, 0], 1024)
    _check_plan([1], 1024)
    _check_plan([1023, 1024, 1025, 1, 0, 3000, 1017, 1016, 1015], 1024)
    _check_plan([5] * 100, 8192)                      # more small tensors than one launch takes
    _check_plan([10000, 3, 10000, 3, 9999, 17], 2048)
    rng = np.random.default_rng(0)
    for _ in range(50):
        k = int(rng.integers(1, 40))
        numel = [int(x) for x in rng.integers(0, 50000, k)]
        _check_plan(numel, int(rng.choice([1024, 2048, 8192, 16384])))
    for bad in (0, 63, 100, -1024, 1536):
        with pytest.raises(zi.ZiError):
            zi.zi_plan_chunks([10], bad)
    with pytest.raises(zi.ZiError):
        zi.zi_plan_chunks([-1], 64)
