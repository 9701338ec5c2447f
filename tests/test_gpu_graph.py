"""The resident path only enqueues kernels, so it can be captured into a HIP graph and replayed."""
import numpy as np
import pytest
import torch

import paper_2104_07857_amd as zi
import zi_synth
from gpu_util import NormBuffers, gen_numpy, to_dev, zi_cfg

pytestmark = pytest.mark.gpu


def test_norm_and_step_replay_from_a_captured_graph():
    """200 ragged tensors (a launch-bound list): capture zi_grad_norm + zi_adamw_step once, replay three
    times with eager work and synchronisations between the replays, and check every replay against the
    same number of eager steps on a copy of the state."""
    w = zi_synth.workload("c4")
    dt = zi.ZI_BF16
    rng = np.random.default_rng(0)
    numel = [int(x) for x in rng.integers(1, 40_000, 200)]
    spec = zi_synth.StateSpec(2024, dt, g_std=2e-3)
    host = [gen_numpy(spec, n, tensor=i) for i, n in enumerate(numel)]

    def device_copy():
        ts = [tuple(to_dev(a) for a in t) + (torch.zeros(t[0].size, dtype=torch.int16, device="cuda:0"),)
              for t in host]
        return ts, zi.make_tensors([t + (t[0].numel(),) for t in ts])

    cfg = zi_cfg(w)
    eager, eager_tl = device_copy()
    graphed, graphed_tl = device_copy()
    nb_e, nb_g = NormBuffers(), NormBuffers()

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        graph.capture_begin()
        zi.zi_grad_norm(graphed_tl, dt, 1.0, nb_g.out, nb_g.ws, stream=side)
        zi.zi_adamw_step(graphed_tl, dt, cfg, nb_g.out, stream=side)
        graph.capture_end()
    torch.cuda.synchronize()
    # capture must not have executed anything
    for a, b in zip(eager, graphed):
        assert torch.equal(a[0], b[0])

    for replay in range(3):
        graph.replay()
        zi.zi_grad_norm(eager_tl, dt, 1.0, nb_e.out, nb_e.ws)
        zi.zi_adamw_step(eager_tl, dt, cfg, nb_e.out)
        torch.cuda.synchronize()
        scratch = torch.rand(1 << 20, device="cuda:0").sum().item()     # unrelated eager work between replays
        assert scratch > 0
        assert nb_e.read() == nb_g.read(), f"replay {replay}: norm result differs"
        for i, (a, b) in enumerate(zip(eager, graphed)):
            for x, y in zip(a, b):
                assert torch.equal(x, y), f"replay {replay}, tensor {i}"
    assert not torch.equal(eager[0][0], to_dev(host[0][0]))      # the steps did change the state
