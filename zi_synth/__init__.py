"""Seeded synthetic optimizer state (inputs only; none of the optimizer's arithmetic).

The arrays stand in for the model states of mixed-precision Adam training
(Section 3, "Memory for Model States": low-precision parameters and gradients,
fp32 momentum, variance and master parameters) at the Transformer shapes of
Section 3 (four linear layers per block: (hd,3hd), (hd,hd), (hd,4hd), (4hd,hd)).

Every value is a pure function of (seed, stream, tensor, index); sub-ranges of
huge arrays can be regenerated exactly.  Buffers are filled in place through
raw pointers, so pinned torch tensors and numpy arrays both work.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libzi_synth.so")

BF16 = 0
FP16 = 1

# stream ids of the four arrays of one tensor
STREAM_P, STREAM_M, STREAM_V, STREAM_G = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile gen.c into libzi_synth.so (gcc, OpenMP)."""
    src = os.path.join(_HERE, "gen.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        cmd = ["gcc", "-O2", "-fPIC", "-shared", "-fopenmp", "-mf16c", "-fno-fast-math",
               "-Wall", "-Wextra", "-o", _LIB_PATH, src, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB_PATH


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        L = ctypes.CDLL(_LIB_PATH)
        L.zs_fill_normal_f32.restype = ctypes.c_int
        L.zs_fill_normal_f32.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64, ctypes.c_uint32,
                                         ctypes.c_uint32, ctypes.c_int64, ctypes.c_double, ctypes.c_double,
                                         ctypes.c_int, ctypes.c_int]
        L.zs_fill_normal_lp.restype = ctypes.c_int
        L.zs_fill_normal_lp.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64, ctypes.c_uint32,
                                        ctypes.c_uint32, ctypes.c_int64, ctypes.c_double, ctypes.c_double,
                                        ctypes.c_int, ctypes.c_int]
        L.zs_normal_at.restype = ctypes.c_double
        L.zs_normal_at.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint64]
        L.zs_pick_index.restype = ctypes.c_uint64
        L.zs_pick_index.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64]
        L.zs_cpu_ok.restype = ctypes.c_int
        _lib = L
    return _lib


def _ptr(buf) -> int:
    """Raw address of a numpy array, a torch CPU tensor, or an int."""
    if isinstance(buf, int):
        return buf
    if isinstance(buf, np.ndarray):
        if not buf.flags["C_CONTIGUOUS"]:
            raise ValueError("buffer must be contiguous")
        return buf.ctypes.data
    if hasattr(buf, "data_ptr"):
        if buf.device.type != "cpu" or not buf.is_contiguous():
            raise ValueError("buffer must be a contiguous CPU tensor")
        return buf.data_ptr()
    raise TypeError(type(buf))


def fill_normal_f32(buf, n, seed, stream, tensor=0, first_index=0, mean=0.0, std=1.0,
                    take_abs=False, nthreads=0):
    """buf[i] = float32(mean + std * z(first_index + i)), |.| if take_abs."""
    rc = lib().zs_fill_normal_f32(_ptr(buf), int(n), int(seed), int(stream), int(tensor), int(first_index),
                                  float(mean), float(std), int(bool(take_abs)), int(nthreads))
    if rc != 0:
        raise ValueError(f"zs_fill_normal_f32 failed ({rc})")


def fill_normal_lp(buf, n, seed, stream, dtype, tensor=0, first_index=0, mean=0.0, std=1.0, nthreads=0):
    """Low-precision (bf16 or fp16 bit patterns, uint16) normal values."""
    rc = lib().zs_fill_normal_lp(_ptr(buf), int(n), int(seed), int(stream), int(tensor), int(first_index),
                                 float(mean), float(std), int(dtype), int(nthreads))
    if rc != 0:
        raise ValueError(f"zs_fill_normal_lp failed ({rc})")


def pick_index(seed, tag, n) -> int:
    return int(lib().zs_pick_index(int(seed), int(tag), int(n)))


def normal_at(seed, stream, tensor, index) -> float:
    return float(lib().zs_normal_at(int(seed), int(stream), int(tensor), int(index)))


# ----------------------------------------------------------------------------
# Workload recipes.  Each returns plain dicts of numbers; no optimizer maths.
# ----------------------------------------------------------------------------

HPARAMS = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)


def transformer_layer_shapes(h: int):
    """Element counts of the 12 tensors of one Transformer block at hidden size h.

    Four linear layers (3h x h, h x h, 4h x h, h x 4h) with their biases, and
    two LayerNorms (gamma, beta), in module order.
    """
    return [
        ("ln1.gamma", h), ("ln1.beta", h),
        ("attn.qkv.weight", 3 * h * h), ("attn.qkv.bias", 3 * h),
        ("attn.out.weight", h * h), ("attn.out.bias", h),
        ("ln2.gamma", h), ("ln2.beta", h),
        ("mlp.fc1.weight", 4 * h * h), ("mlp.fc1.bias", 4 * h),
        ("mlp.fc2.weight", 4 * h * h), ("mlp.fc2.bias", h),
    ]


class StateSpec:
    """Distribution of one state: which of p/m/v/g, with what std, for one workload."""

    def __init__(self, seed, lp_dtype, p_std=0.02, m_std=1e-4, v_std=1e-6, g_std=1e-3,
                 zero_moments=False):
        self.seed = seed
        self.lp_dtype = lp_dtype
        self.p_std, self.m_std, self.v_std, self.g_std = p_std, m_std, v_std, g_std
        self.zero_moments = zero_moments

    def fill_p(self, buf, n, tensor=0, first_index=0, nthreads=0):
        fill_normal_f32(buf, n, self.seed, STREAM_P, tensor, first_index, 0.0, self.p_std, False, nthreads)

    def fill_m(self, buf, n, tensor=0, first_index=0, nthreads=0):
        if self.zero_moments:
            ctypes.memset(_ptr(buf), 0, 4 * int(n))
        else:
            fill_normal_f32(buf, n, self.seed, STREAM_M, tensor, first_index, 0.0, self.m_std, False, nthreads)

    def fill_v(self, buf, n, tensor=0, first_index=0, nthreads=0):
        if self.zero_moments:
            ctypes.memset(_ptr(buf), 0, 4 * int(n))
        else:
            fill_normal_f32(buf, n, self.seed, STREAM_V, tensor, first_index, 0.0, self.v_std, True, nthreads)

    def fill_g(self, buf, n, tensor=0, first_index=0, nthreads=0):
        fill_normal_lp(buf, n, self.seed, STREAM_G, self.lp_dtype, tensor, first_index, 0.0, self.g_std, nthreads)


def workload(name: str):
    """The five workloads: sizes, dtype, step number, loss scale, clip, value recipe."""
    base_seed = 0x5EED0000
    if name == "c0":
        return dict(name=name, numel=[1 << 20], lp_dtype=BF16, step=1, loss_scale=1.0, max_grad_norm=0.0,
                    use_norm=False, streamed=False,
                    spec=StateSpec(base_seed + 0, BF16, zero_moments=True), **HPARAMS)
    if name == "c1":
        return dict(name=name, numel=[1_300_000_000], lp_dtype=BF16, step=10, loss_scale=1.0, max_grad_norm=0.0,
                    use_norm=False, streamed=False, spec=StateSpec(base_seed + 1, BF16), **HPARAMS)
    if name == "c2":
        return dict(name=name, numel=[8_000_000_000], lp_dtype=BF16, step=10, loss_scale=1.0, max_grad_norm=0.0,
                    use_norm=False, streamed=True, chunk_bytes=64 << 20, n_slots=3,
                    spec=StateSpec(base_seed + 2, BF16), **HPARAMS)
    if name == "c3":
        return dict(name=name, numel=[2_000_000_000], lp_dtype=FP16, step=10, loss_scale=65536.0,
                    max_grad_norm=1.0, use_norm=True, streamed=False,
                    spec=StateSpec(base_seed + 3, FP16, g_std=1e-3 * 65536.0), **HPARAMS)
    if name == "c4":
        h = 8192
        numel = [n for _ in range(4) for (_, n) in transformer_layer_shapes(h)]
        return dict(name=name, numel=numel, lp_dtype=BF16, step=100, loss_scale=1.0, max_grad_norm=1.0,
                    use_norm=True, streamed=True, chunk_bytes=64 << 20, n_slots=3,
                    spec=StateSpec(base_seed + 4, BF16), **HPARAMS)
    raise KeyError(name)
