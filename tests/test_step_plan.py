"""Host logic of the resident step's launch plan (no GPU): how many leading elements each tensor handles
one by one so that its vector body starts on 128-byte lines, and how tensors are grouped into launches."""
import ctypes

import numpy as np
import pytest

import paper_2104_07857_amd as zi

TILE = 512
BASE = 0x7F00_0000_0000          # made-up, 2 MiB aligned addresses: the plan never dereferences them
GAP = 1 << 36


def _tensor(n, offs=(0, 0, 0, 0, 0), k=0, lp=True):
    """Arrays that start offs[i] elements past aligned addresses."""
    a = [BASE + (5 * k + i) * GAP + offs[i] * (4 if i < 3 else 2) for i in range(5)]
    return (a[0], a[1], a[2], a[3], a[4] if lp else None, n)


def _line_aligned(t, head):
    fp = [(a + 4 * head) % 128 == 0 for a in t[:3]]
    lp = [(a + 2 * head) % 128 == 0 for a in t[3:5] if a is not None]
    return fp, lp


def test_aligned_arrays_start_at_once():
    items, launches = zi.zi_plan_step([_tensor(10 * TILE + 3)])
    assert launches == 1 and len(items) == 1
    it = items[0]
    assert (it.tensor, it.head, it.first_tile, it.launch, it.alone) == (0, 0, 0, 0, 1)
    assert it.n_tiles == 10                      # the 3 trailing elements ride with the first tile's lanes
    assert zi.zi_plan_step([_tensor(10 * TILE + 5)])[0][0].n_tiles == 11     # one more quad: a partial tile


@pytest.mark.parametrize("k", range(1, 64))
def test_common_offset_becomes_line_aligned(k):
    t = _tensor(100_000, (k,) * 5)
    items, _ = zi.zi_plan_step([t])
    head = items[0].head
    assert head == 64 - k
    fp, lp = _line_aligned(t, head)
    assert all(fp) and all(lp)


def test_unrelated_offsets_favour_the_fp32_arrays_and_keep_lane_alignment_where_possible():
    t = _tensor(100_000, (5, 5, 5, 2, 7))
    head = zi.zi_plan_step([t])[0][0].head
    assert all(_line_aligned(t, head)[0])        # p, m, v move 24 of the 28 bytes per element
    t = _tensor(100_000, (1, 2, 3, 0, 0))         # nothing in common: any head in 0..63 is legal
    assert 0 <= zi.zi_plan_step([t])[0][0].head < 64
    rng = np.random.default_rng(1)
    for _ in range(200):
        offs = tuple(int(x) for x in rng.integers(0, 64, 5))
        t = _tensor(int(rng.integers(1, 5000)), offs, lp=bool(rng.integers(0, 2)))
        it = zi.zi_plan_step([t])[0][0]
        assert 0 <= it.head <= min(63, t[5])
        body = t[5] - it.head
        assert it.n_tiles == max(1, -(-(body // 4) // (TILE // 4)))
        if len(set(o % 32 for o in offs[:3])) == 1:       # p, m, v share a phase: they end up line-aligned
            assert it.head == t[5] or all(_line_aligned(t, it.head)[0])


def test_head_never_exceeds_the_tensor():
    t = _tensor(5, (1,) * 5)
    it = zi.zi_plan_step([t])[0][0]
    assert it.head == 5 and it.n_tiles == 1


def test_long_tensors_are_launched_alone_and_short_ones_share():
    solo = 1 << 22
    lens = [1000, solo, 2000, solo - 2 * TILE, 3000] + [100] * 40 + [2 * solo, 0, 7]
    items, launches = zi.zi_plan_step([_tensor(n, k=i) for i, n in enumerate(lens)])
    by_tensor = {it.tensor: it for it in items}
    assert sorted(by_tensor) == [i for i, n in enumerate(lens) if n > 0]
    alone = [i for i, it in by_tensor.items() if it.alone]
    assert alone == [1, 45]                                    # exactly the tensors of >= 8192 tiles (2^22 elements)
    assert by_tensor[1].launch != by_tensor[45].launch
    shared = [it for it in items if not it.alone]
    assert len(shared) == 45
    per_launch = {}
    for it in shared:
        per_launch.setdefault(it.launch, []).append(it)
    assert sorted(len(v) for v in per_launch.values()) == [13, 32]       # 32 descriptors per launch
    assert launches == 4
    for group in per_launch.values():                          # tiles of a launch are numbered densely, in order
        nxt = 0
        for it in group:
            assert it.first_tile == nxt
            nxt += it.n_tiles


def test_argument_errors():
    with pytest.raises(zi.ZiError):
        zi.zi_plan_step([(BASE + 2, BASE + GAP, BASE + 2 * GAP, BASE + 3 * GAP, None, 10)])     # p not 4-byte aligned
    with pytest.raises(zi.ZiError):
        zi.zi_plan_step([(BASE, BASE, BASE + 2 * GAP, BASE + 3 * GAP, None, 10)])               # p aliases m
    assert zi.zi_plan_step([]) == ([], 0)
    assert ctypes.sizeof(zi.zi_step_plan_item) == 32
