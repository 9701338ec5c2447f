"""The seeded generators: reproducible, sliceable, right distributions and shapes."""
import os

import numpy as np
import pytest

import zi_synth as zs

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_constants.txt")


def _constants():
    out = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split()
            out[k] = v
    return out


def test_subranges_regenerate_exactly_and_threads_do_not_matter():
    n = 200_003
    a = np.empty(n, np.float32)
    zs.fill_normal_f32(a, n, 5, zs.STREAM_P, std=0.02)
    b = np.empty(n, np.float32)
    zs.fill_normal_f32(b, n, 5, zs.STREAM_P, std=0.02, nthreads=1)
    assert np.array_equal(a, b)
    for first, cnt in ((0, 1), (1, 1), (4095, 3), (12345, 70001), (n - 1, 1)):
        c = np.empty(cnt, np.float32)
        zs.fill_normal_f32(c, cnt, 5, zs.STREAM_P, first_index=first, std=0.02)
        assert np.array_equal(c, a[first:first + cnt])
    g = np.empty(n, np.uint16)
    zs.fill_normal_lp(g, n, 5, zs.STREAM_G, zs.FP16, std=65.536)
    h = np.empty(1001, np.uint16)
    zs.fill_normal_lp(h, 1001, 5, zs.STREAM_G, zs.FP16, first_index=777, std=65.536)
    assert np.array_equal(h, g[777:1778])


def test_streams_tensors_and_seeds_are_independent():
    n = 4096
    outs = []
    for seed, stream, tensor in ((1, 0, 0), (2, 0, 0), (1, 1, 0), (1, 0, 1)):
        a = np.empty(n, np.float32)
        zs.fill_normal_f32(a, n, seed, stream, tensor)
        outs.append(a)
    for i in range(len(outs)):
        for j in range(i + 1, len(outs)):
            assert abs(np.corrcoef(outs[i], outs[j])[0, 1]) < 0.08


def test_distributions_of_the_workload_recipe():
    n = 1 << 20
    w = zs.workload("c1")
    spec = w["spec"]
    p = np.empty(n, np.float32); spec.fill_p(p, n)
    m = np.empty(n, np.float32); spec.fill_m(m, n)
    v = np.empty(n, np.float32); spec.fill_v(v, n)
    g = np.empty(n, np.uint16); spec.fill_g(g, n)
    gf = (g.astype(np.uint32) << 16).view(np.float32)
    assert p.std() == pytest.approx(0.02, rel=5e-3) and abs(p.mean()) < 1e-4
    assert m.std() == pytest.approx(1e-4, rel=5e-3)
    assert (v >= 0).all() and np.sqrt((v.astype(np.float64) ** 2).mean()) == pytest.approx(1e-6, rel=5e-3)
    assert gf.std() == pytest.approx(1e-3, rel=1e-2) and np.isfinite(gf).all()
    w3 = zs.workload("c3")
    g3 = np.empty(n, np.uint16); w3["spec"].fill_g(g3, n)
    g3f = g3.view(np.float16).astype(np.float64)
    assert np.isfinite(g3f).all() and g3f.std() == pytest.approx(65.536, rel=1e-2)
    w0 = zs.workload("c0")
    z = np.ones(16, np.float32); w0["spec"].fill_m(z, 16)
    assert not z.any()


def test_workload_sizes_follow_the_paper_shapes():
    c = _constants()
    h = 8192
    shapes = zs.transformer_layer_shapes(h)
    assert len(shapes) == 12
    weights = sorted(n // (h * h) for _, n in shapes if n >= h * h)
    assert weights == sorted(int(x) for x in c["linear_shapes"].split(","))
    per_layer = sum(n for _, n in shapes)
    assert per_layer == 12 * h * h + 13 * h == 805_412_864
    assert per_layer // (h * h) == int(c["block_params_over_hd2"])
    w4 = zs.workload("c4")
    assert len(w4["numel"]) == 48 and sum(w4["numel"]) == 3_221_651_456
    assert zs.workload("c0")["numel"] == [1 << 20]
    assert zs.workload("c1")["numel"] == [1_300_000_000]
    assert zs.workload("c2")["numel"] == [8_000_000_000]
    assert zs.workload("c3")["numel"] == [2_000_000_000] and zs.workload("c3")["loss_scale"] == 65536.0
    # bytes the paper's accounting assigns to the step's state: fp32 p, m, v (+ fp32 g, which this path drops)
    assert int(c["optimizer_state_bytes_per_param"]) == 4 * 4
    assert int(c["model_state_bytes_per_param"]) == 2 + 2 + 4 * 4


def test_pick_index_is_seeded_and_in_range():
    a = zs.pick_index(3, 0x696E66, 2_000_000_000)
    assert a == zs.pick_index(3, 0x696E66, 2_000_000_000) and 0 <= a < 2_000_000_000
    assert a != zs.pick_index(4, 0x696E66, 2_000_000_000)
