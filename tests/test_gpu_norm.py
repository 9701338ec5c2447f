"""Parity of zi_grad_norm (sum of squares, norm, overflow flag) with the CPU oracle."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2104_07857_amd as zi
import zi_synth
from gpu_util import NormBuffers, TOL_NORM_REL, progress, to_dev

pytestmark = pytest.mark.gpu

NORM_TILE = 16384


def _gpu_norm(gs, dt, loss_scale=1.0, nb=None):
    nb = nb or NormBuffers()
    devs = [g if isinstance(g, torch.Tensor) else to_dev(g) for g in gs]
    zi.zi_grad_norm([(None, None, None, d, None, d.numel()) for d in devs], dt, loss_scale, nb.out, nb.ws)
    torch.cuda.synchronize()
    return nb.read()


def _grads(n, dt, seed, std=1e-3):
    g = np.empty(n, np.uint16)
    zi_synth.fill_normal_lp(g, n, seed, zi_synth.STREAM_G, dt, std=std)
    return g


@pytest.mark.parametrize("dt", [zi.ZI_BF16, zi.ZI_FP16])
@pytest.mark.parametrize("n", [0, 1, 7, 8, 9, NORM_TILE - 1, NORM_TILE, NORM_TILE + 1, 4 * NORM_TILE + 3,
                               1_000_003, (1 << 24) + 5])
def test_single_tensor_sizes(n, dt):
    g = _grads(n, dt, 100 + n, std=1e-3 if dt == zi.ZI_BF16 else 65.536)
    want, wflag = oracle.grad_sumsq([g], dt)
    sumsq, norm, flag = _gpu_norm([g], dt, loss_scale=4.0)
    assert flag == wflag == 0
    assert abs(sumsq - want) <= 1e-12 * max(want, 1e-300)      # double accumulation on both sides
    assert abs(norm - math.sqrt(want) / 4.0) <= TOL_NORM_REL * max(math.sqrt(want) / 4.0, 1e-300)


def test_unaligned_views_and_lists():
    dt = zi.ZI_BF16
    base = to_dev(_grads(200_000, dt, 5))
    host = base.cpu().numpy().view(np.uint16)
    cuts = [(0, 0), (1, 1), (3, 50_001), (50_001, 50_001 + 7), (60_000, 199_999), (199_999, 200_000)]
    views = [base[a:b] for a, b in cuts]
    want, _ = oracle.grad_sumsq([host[a:b].copy() for a, b in cuts], dt)
    sumsq, norm, flag = _gpu_norm(views, dt)
    assert flag == 0 and abs(sumsq - want) <= 1e-12 * want
    # many tensors: more than one launch's table holds, and more partials than one finalize pass takes
    many = [base[i * 37:(i * 37) + 29] for i in range(300)]
    want, _ = oracle.grad_sumsq([host[i * 37:(i * 37) + 29].copy() for i in range(300)], dt)
    sumsq, _, _ = _gpu_norm(many, dt)
    assert abs(sumsq - want) <= 1e-12 * want
    # empty list: a defined zero result
    assert _gpu_norm([], dt) == (0.0, 0.0, 0)


def test_partial_budget_overflow_path():
    """A list whose block count exceeds the workspace's partial capacity forces intermediate finalizes."""
    dt = zi.ZI_BF16
    n = 4096 * 4 * NORM_TILE         # one tensor that takes the per-tensor maximum of 4096 blocks
    big = to_dev(_grads(n, dt, 6))
    host = big.cpu().numpy().view(np.uint16)
    one, _ = oracle.grad_sumsq([host], dt)
    sumsq, _, flag = _gpu_norm([big] * 5, dt)          # 5 x 4096 blocks > 16384 partials
    assert flag == 0 and abs(sumsq - 5 * one) <= 1e-12 * 5 * one


@pytest.mark.parametrize("dt,specials,finite_max", [
    (zi.ZI_BF16, [0x7F80, 0xFF80, 0x7FC0, 0x7F81, 0xFFFF], [0x7F7F, 0xFF7F]),
    (zi.ZI_FP16, [0x7C00, 0xFC00, 0x7E00, 0x7C01, 0xFFFF], [0x7BFF, 0xFBFF])])
def test_flag_is_bit_exact(dt, specials, finite_max):
    n = 3 * NORM_TILE + 5
    base = _grads(n, dt, 9)
    nb = NormBuffers()
    for s in specials:
        for pos in (0, 1, 7, 8, n - 1, n - 6, NORM_TILE, 2 * NORM_TILE + 17):
            g = base.copy()
            g[pos] = s
            assert _gpu_norm([g], dt, nb=nb)[2] == 1 == oracle.grad_sumsq([g], dt)[1], (hex(s), pos)
    # unaligned view with the special value in the scalar head and tail
    for pos in (0, 2, n - 4):
        g = base.copy()
        g[pos + 3] = specials[0]
        d = to_dev(g)
        assert _gpu_norm([d[3:]], dt, nb=nb)[2] == 1
    # the largest finite values are not an overflow; their squares stay finite in the double sum
    for s in finite_max:
        g = base.copy()
        g[11] = s
        want, wflag = oracle.grad_sumsq([g], dt)
        sumsq, _, flag = _gpu_norm([g], dt, nb=nb)
        assert flag == wflag == 0 and math.isfinite(sumsq) and abs(sumsq - want) <= 1e-12 * want
    assert _gpu_norm([base], dt, nb=nb)[2] == 0      # and the flag resets between calls


def test_constant_closed_form():
    g = torch.full((1 << 22,), 0x3E80, dtype=torch.int16, device="cuda:0")     # bf16 0.25
    sumsq, norm, flag = _gpu_norm([g], zi.ZI_BF16, loss_scale=2.0)
    assert sumsq == 0.0625 * (1 << 22) and norm == 0.25 * 2048 / 2.0 and flag == 0
    progress("norm closed form ok")


@pytest.mark.parametrize("n", [4, 1020, (1 << 20) + 4, 3 * (1 << 20) + 8 * 1000 + 4])
def test_hbm_probe_modes_do_what_they_say(n):
    # sizes: less than one lane group, a ragged single tile, one complete XCD run of 8 x 128 tiles plus
    # one vector, and several runs followed by an incomplete one
    a = torch.arange(n, dtype=torch.float32, device="cuda:0")
    b = torch.zeros(n + 4, dtype=torch.float32, device="cuda:0")
    ref = a.clone()
    zi.zi_hbm_probe(a, None, 4 * n, 0)
    torch.cuda.synchronize()
    assert torch.equal(a, ref)                       # a read leaves the buffer alone
    zi.zi_hbm_probe(a, b, 4 * n, 1)
    torch.cuda.synchronize()
    assert torch.equal(b[:n], ref) and not bool(b[n:].any())
    zi.zi_hbm_probe(a, None, 4 * n, 2)
    torch.cuda.synchronize()
    assert torch.equal(a, ref + 1.0)


def test_two_slices_combined_like_two_ranks_give_the_global_clip():
    """The sharded recipe on one GPU: each 'rank' reduces its slice, the 12 bytes are combined (sum, max) in
    device memory, zi_norm_refresh recomputes the norm, and each slice is stepped with the combined result:
    identical to stepping the whole tensor with its own norm."""
    from gpu_util import gen_numpy, zi_cfg
    w = zi_synth.workload("c4")
    dt = zi.ZI_BF16
    n, k = 300_001, 123_457
    p, m, v, g = gen_numpy(zi_synth.StateSpec(314, dt, g_std=2e-3), n)
    cfg = zi_cfg(w)
    whole = [to_dev(a) for a in (p, m, v, g)] + [torch.zeros(n, dtype=torch.int16, device="cuda:0")]
    nb = NormBuffers()
    zi.zi_grad_norm([tuple(whole) + (n,)], dt, 1.0, nb.out, nb.ws)
    zi.zi_adamw_step([tuple(whole) + (n,)], dt, cfg, nb.out)
    parts = [to_dev(a) for a in (p, m, v, g)] + [torch.zeros(n, dtype=torch.int16, device="cuda:0")]
    r0, r1 = NormBuffers(), NormBuffers()
    s0 = tuple(x[:k] for x in parts) + (k,)
    s1 = tuple(x[k:] for x in parts) + (n - k,)
    zi.zi_grad_norm([s0], dt, 1.0, r0.out, r0.ws)
    zi.zi_grad_norm([s1], dt, 1.0, r1.out, r1.ws)
    # the "all-reduce": sum of sumsq, max of the flag word, written back to both ranks' results
    total = r0.out[0] + r1.out[0]
    flag = torch.maximum(r0.out[2:3].view(torch.int64), r1.out[2:3].view(torch.int64))
    for r in (r0, r1):
        r.out[0] = total
        r.out[2:3].view(torch.int64).copy_(flag)
        zi.zi_norm_refresh(r.out, 1.0)
    zi.zi_adamw_step([s0], dt, cfg, r0.out)
    zi.zi_adamw_step([s1], dt, cfg, r1.out)
    torch.cuda.synchronize()
    assert abs(r0.read()[1] - nb.read()[1]) <= 1e-12 * nb.read()[1] and r0.read()[2] == 0
    for a, b in zip(whole, parts):
        assert torch.equal(a, b)
    with pytest.raises(zi.ZiError):
        zi.zi_norm_refresh(None, 1.0)
    with pytest.raises(zi.ZiError):
        zi.zi_norm_refresh(r0.out, 0.0)


@pytest.mark.parametrize("dt,expmask", [(zi.ZI_BF16, 0x7F80), (zi.ZI_FP16, 0x7C00)])
def test_every_finite_pattern_is_squared_exactly(dt, expmask):
    """All finite 16-bit patterns (subnormals, both zeros, the largest values: bf16 squares reach 1e77)
    in one tensor: squares are exact in double and the sum agrees with the oracle's compensated sum."""
    allp = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    finite = allp[(allp & expmask) != expmask]
    rng = np.random.default_rng(3)
    g = rng.permutation(np.tile(finite, 5))
    want, flag0 = oracle.grad_sumsq([g], dt)
    sumsq, _, flag = _gpu_norm([g], dt)
    assert flag == flag0 == 0
    assert math.isfinite(sumsq) and abs(sumsq - want) <= 1e-12 * want
    # one non-finite pattern anywhere raises the flag
    g2 = g.copy()
    g2[12345] = expmask
    assert _gpu_norm([g2], dt)[2] == 1
