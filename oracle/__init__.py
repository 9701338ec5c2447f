"""CPU oracle for the mixed-precision optimizer step — TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It wraps oracle/zi_oracle.c (plain single-threaded C) and shares
nothing with the HIP library.  See the header of zi_oracle.c for what is
computed and which passages of the paper fix it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libzi_oracle.so")

BF16 = 0
FP16 = 1
MODE_ADAMW = 0
MODE_ADAM_L2 = 1


def build(force: bool = False) -> str:
    """Compile zi_oracle.c with gcc: no contraction, no fast-math, hardware fmaf."""
    src = os.path.join(_HERE, "zi_oracle.c")
    hdr = os.path.join(_HERE, "zi_oracle.h")
    newest = max(os.path.getmtime(src), os.path.getmtime(hdr))
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < newest:
        cmd = ["gcc", "-O2", "-fPIC", "-shared", "-std=c11", "-ffp-contract=off", "-fno-fast-math",
               "-mfma", "-Wall", "-Wextra", "-o", _LIB_PATH, src, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB_PATH


class Config(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float), ("step", ctypes.c_int64),
                ("loss_scale", ctypes.c_float), ("max_grad_norm", ctypes.c_float), ("mode", ctypes.c_int32)]


class ScalarsOut(ctypes.Structure):
    _fields_ = [("bc1", ctypes.c_double), ("bc2", ctypes.c_double), ("norm", ctypes.c_double),
                ("clip", ctypes.c_double), ("omb1", ctypes.c_float), ("omb2", ctypes.c_float),
                ("step_size", ctypes.c_float), ("inv_sqrt_bc2", ctypes.c_float), ("decay", ctypes.c_float),
                ("gscale", ctypes.c_float)]


class SumsqState(ctypes.Structure):
    _fields_ = [("sum", ctypes.c_double), ("comp", ctypes.c_double), ("found_inf", ctypes.c_uint32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        L = ctypes.CDLL(_LIB_PATH)
        vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        L.zio_bf16_to_f32.restype = ctypes.c_float
        L.zio_bf16_to_f32.argtypes = [ctypes.c_uint16]
        L.zio_f16_to_f32.restype = ctypes.c_float
        L.zio_f16_to_f32.argtypes = [ctypes.c_uint16]
        L.zio_f32_to_bf16.restype = ctypes.c_uint16
        L.zio_f32_to_bf16.argtypes = [ctypes.c_float]
        L.zio_f32_to_f16.restype = ctypes.c_uint16
        L.zio_f32_to_f16.argtypes = [ctypes.c_float]
        L.zio_cast_array.restype = None
        L.zio_cast_array.argtypes = [vp, vp, i64, ci]
        L.zio_widen_array.restype = None
        L.zio_widen_array.argtypes = [vp, vp, i64, ci]
        L.zio_sumsq_init.restype = None
        L.zio_sumsq_init.argtypes = [ctypes.POINTER(SumsqState)]
        L.zio_sumsq_accumulate.restype = None
        L.zio_sumsq_accumulate.argtypes = [ctypes.POINTER(SumsqState), vp, i64, ci]
        L.zio_sumsq_value.restype = ctypes.c_double
        L.zio_sumsq_value.argtypes = [ctypes.POINTER(SumsqState)]
        L.zio_scalars.restype = ci
        L.zio_scalars.argtypes = [ctypes.POINTER(Config), ci, ctypes.c_double, ctypes.POINTER(ScalarsOut)]
        L.zio_adamw.restype = ci
        L.zio_adamw.argtypes = [vp, vp, vp, vp, vp, i64, ci, ctypes.POINTER(Config), ci, ctypes.c_double, ci]
        L.zio_cpu_ok.restype = ci
        if not L.zio_cpu_ok():
            raise RuntimeError("oracle needs a CPU with FMA")
        _lib = L
    return _lib


def config(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, step=1, loss_scale=1.0,
           max_grad_norm=0.0, mode=MODE_ADAMW) -> Config:
    return Config(lr, beta1, beta2, eps, weight_decay, int(step), loss_scale, max_grad_norm, int(mode))


def _chk(a: np.ndarray, dtype, name: str):
    if not isinstance(a, np.ndarray) or a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise TypeError(f"{name}: need a contiguous numpy array of {dtype}")
    return a.ctypes.data


def cast(x: np.ndarray, dtype: int) -> np.ndarray:
    """fp32 -> bf16/fp16 bit patterns (uint16), round to nearest even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, np.uint16)
    lib().zio_cast_array(x.ctypes.data, out.ctypes.data, x.size, dtype)
    return out


def widen(x: np.ndarray, dtype: int) -> np.ndarray:
    """bf16/fp16 bit patterns (uint16) -> fp32, exact."""
    x = np.ascontiguousarray(x, dtype=np.uint16)
    out = np.empty(x.shape, np.float32)
    lib().zio_widen_array(x.ctypes.data, out.ctypes.data, x.size, dtype)
    return out


def scalars(cfg: Config, sumsq=None) -> ScalarsOut:
    o = ScalarsOut()
    rc = lib().zio_scalars(ctypes.byref(cfg), 0 if sumsq is None else 1, 0.0 if sumsq is None else float(sumsq),
                           ctypes.byref(o))
    if rc != 0:
        raise ValueError("zio_scalars: bad configuration")
    return o


def grad_sumsq(grads, dtype: int):
    """Sum of squares (double) and non-finite flag over a list of uint16 gradient arrays, in list order."""
    st = SumsqState()
    lib().zio_sumsq_init(ctypes.byref(st))
    for g in grads:
        lib().zio_sumsq_accumulate(ctypes.byref(st), _chk(g, np.uint16, "g"), g.size, dtype)
    return float(lib().zio_sumsq_value(ctypes.byref(st))), int(st.found_inf)


def grad_norm(grads, dtype: int, loss_scale: float = 1.0):
    """(unscaled global L2 norm, found_inf)."""
    ss, flag = grad_sumsq(grads, dtype)
    return float(np.sqrt(ss) / float(np.float32(loss_scale))), flag


def adamw(p, m, v, g, p_lp, dtype: int, cfg: Config, sumsq=None, found_inf: int = 0) -> int:
    """One step in place on numpy arrays.  Returns 0 (updated) or 1 (skipped)."""
    n = p.size
    if not (m.size == n and v.size == n and g.size == n and (p_lp is None or p_lp.size == n)):
        raise ValueError("size mismatch")
    rc = lib().zio_adamw(_chk(p, np.float32, "p"), _chk(m, np.float32, "m"), _chk(v, np.float32, "v"),
                         _chk(g, np.uint16, "g"), None if p_lp is None else _chk(p_lp, np.uint16, "p_lp"),
                         n, dtype, ctypes.byref(cfg), 0 if sumsq is None else 1,
                         0.0 if sumsq is None else float(sumsq), int(found_inf))
    if rc < 0:
        raise ValueError("zio_adamw: bad argument")
    return rc


def step(tensors, dtype: int, cfg: Config, use_norm: bool):
    """The whole path over a list of (p, m, v, g, p_lp) numpy tuples.

    With use_norm: global norm and overflow flag over all gradients first, then
    unscale / clip / skip.  Returns dict(norm, found_inf, skipped, sumsq).
    """
    sumsq, flag = (None, 0)
    if use_norm:
        sumsq, flag = grad_sumsq([t[3] for t in tensors], dtype)
    skipped = 0
    for (p, m, v, g, p_lp) in tensors:
        skipped = adamw(p, m, v, g, p_lp, dtype, cfg, sumsq, flag)
    norm = None if sumsq is None else float(np.sqrt(sumsq) / float(cfg.loss_scale))
    return dict(norm=norm, found_inf=flag, skipped=bool(skipped), sumsq=sumsq)
