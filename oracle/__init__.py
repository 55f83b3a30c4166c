"""Python face of the CPU oracle (oracle/ma_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the host-baseline
leg of the benchmark.  The GPU library and its binding never import this package, and this
package imports nothing from them.  All arrays are numpy arrays on the host; 16-bit formats
travel as raw uint16 bit patterns.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_DT = {"f32": 0, "bf16": 1, "f16": 2}
_HERE = os.path.dirname(os.path.abspath(__file__))


class Hyper(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float),
                ("bias_correction", ctypes.c_int32)]


def _load():
    # MA_ORACLE_LIBRARY: an alternative build of the oracle.  tests/test_oracle_mutants.py points it
    # at deliberately broken builds to show that the pins notice each planted mistake.
    path = os.environ.get("MA_ORACLE_LIBRARY") or _build.build(force=False)
    lib = ctypes.CDLL(path)
    vp, sz, i32, i64, f32, f64 = (ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32,
                                  ctypes.c_int64, ctypes.c_float, ctypes.c_double)
    for name in ("ora_widen_bf16", "ora_widen_f16", "ora_round_bf16", "ora_round_f16"):
        getattr(lib, name).argtypes = [vp, vp, sz]
        getattr(lib, name).restype = None
    lib.ora_overflow_norm.argtypes = [vp, i32, sz, f32, i32, vp, vp]
    lib.ora_overflow_norm.restype = None
    lib.ora_clip_coef.argtypes = [f64, f64]
    lib.ora_clip_coef.restype = f32
    lib.ora_adamw_step.argtypes = [vp, vp, vp, vp, i32, vp, i32, sz, vp, i64, f32, f32, i32]
    lib.ora_adamw_step.restype = None
    lib.ora_step_scalars.argtypes = [vp, i64, f32, f32, vp]
    lib.ora_step_scalars.restype = None
    lib.ora_adamw_step_f64.argtypes = [vp, vp, vp, vp, i32, sz, vp, i64, f32, f32, vp, vp, vp]
    lib.ora_adamw_step_f64.restype = None
    lib.ora_optimizer_step.argtypes = [vp, vp, vp, vp, i32, vp, i32, sz, vp, i64, f32, f32, i32,
                                       vp, vp]
    lib.ora_optimizer_step.restype = i32
    lib.ora_grad_accumulate.argtypes = [vp, vp, i32, sz, i32]
    lib.ora_grad_accumulate.restype = None
    lib.ora_truncate_bf16.argtypes = [vp, vp, sz]
    lib.ora_truncate_bf16.restype = None
    lib.ora_adamw_step_bf16.argtypes = [vp, vp, vp, vp, i32, sz, vp, i64, f32, f32, i32]
    lib.ora_adamw_step_bf16.restype = None
    lib.ora_scaler_update.argtypes = [vp, vp, i32]
    lib.ora_scaler_update.restype = None
    lib.ora_optimizer_step_auto.argtypes = [vp, vp, vp, vp, i32, vp, i32, sz, vp, vp, vp, f32, i32, vp]
    lib.ora_optimizer_step_auto.restype = i32
    return lib


class ScalerCfg(ctypes.Structure):
    _fields_ = [("backoff", ctypes.c_float), ("growth", ctypes.c_float),
                ("min_scale", ctypes.c_float), ("max_scale", ctypes.c_float),
                ("window", ctypes.c_int32)]


class ScalerState(ctypes.Structure):
    _fields_ = [("scale", ctypes.c_float), ("good_steps", ctypes.c_int32),
                ("step", ctypes.c_int64), ("skipped", ctypes.c_int64)]


_lib = _load()


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _chk(a, dtype, name):
    if not isinstance(a, np.ndarray) or a.dtype != dtype or not a.flags["C_CONTIGUOUS"] or a.ndim != 1:
        raise TypeError("%s must be a contiguous 1-D numpy array of %s" % (name, dtype))


def _grad_dtype(gdt):
    return np.float32 if gdt == "f32" else np.uint16


def hyper(lr=1e-5, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, bias_correction=1):
    return Hyper(lr, beta1, beta2, eps, weight_decay, int(bias_correction))


def widen_bf16(bits):
    _chk(bits, np.uint16, "bits")
    out = np.empty(bits.shape, np.float32)
    _lib.ora_widen_bf16(_ptr(bits), _ptr(out), bits.size)
    return out


def widen_f16(bits):
    _chk(bits, np.uint16, "bits")
    out = np.empty(bits.shape, np.float32)
    _lib.ora_widen_f16(_ptr(bits), _ptr(out), bits.size)
    return out


def round_bf16(x):
    _chk(x, np.float32, "x")
    out = np.empty(x.shape, np.uint16)
    _lib.ora_round_bf16(_ptr(x), _ptr(out), x.size)
    return out


def round_f16(x):
    _chk(x, np.float32, "x")
    out = np.empty(x.shape, np.uint16)
    _lib.ora_round_f16(_ptr(x), _ptr(out), x.size)
    return out


def overflow_norm(grad, gdt, loss_scale=1.0, nthreads=1):
    """(overflow: bool, sumsq: float) of a raw gradient buffer (Sec. III-C flag; fp64 sum)."""
    _chk(grad, _grad_dtype(gdt), "grad")
    ov = ctypes.c_int32(0)
    ss = ctypes.c_double(0.0)
    _lib.ora_overflow_norm(_ptr(grad), _DT[gdt], grad.size, loss_scale, nthreads,
                           ctypes.byref(ov), ctypes.byref(ss))
    return bool(ov.value), ss.value


def clip_coef(sumsq, max_norm):
    return np.float32(_lib.ora_clip_coef(float(sumsq), float(max_norm)))


def step_scalars(h, step, loss_scale=1.0, clip=1.0):
    out = np.empty(9, np.float32)
    _lib.ora_step_scalars(ctypes.byref(h), int(step), loss_scale, clip, _ptr(out))
    return out


def adamw_step(p, m, v, grad, gdt, pdt, h, step, loss_scale=1.0, clip=1.0, nthreads=1,
               want_lp=True):
    """AdamW on fp32 p/m/v in place; returns the rounded low-precision copy of the new p."""
    for a, nm in ((p, "p"), (m, "m"), (v, "v")):
        _chk(a, np.float32, nm)
    _chk(grad, _grad_dtype(gdt), "grad")
    if not (p.size == m.size == v.size == grad.size):
        raise ValueError("size mismatch")
    p_lp = np.empty(p.shape, np.uint16) if want_lp else None
    _lib.ora_adamw_step(_ptr(p), _ptr(m), _ptr(v), _ptr(grad), _DT[gdt], _ptr(p_lp), _DT[pdt],
                        p.size, ctypes.byref(h), int(step), loss_scale, float(clip), nthreads)
    return p_lp


def adamw_step_f64(p, m, v, grad, gdt, h, step, loss_scale=1.0, clip=1.0):
    """The same step evaluated in fp64 from the textbook formula; inputs untouched."""
    for a, nm in ((p, "p"), (m, "m"), (v, "v")):
        _chk(a, np.float32, nm)
    _chk(grad, _grad_dtype(gdt), "grad")
    po, mo, vo = (np.empty(p.shape, np.float64) for _ in range(3))
    _lib.ora_adamw_step_f64(_ptr(p), _ptr(m), _ptr(v), _ptr(grad), _DT[gdt], p.size,
                            ctypes.byref(h), int(step), loss_scale, float(clip),
                            _ptr(po), _ptr(mo), _ptr(vo))
    return po, mo, vo


def optimizer_step(p, m, v, grad, gdt, p_lp, pdt, h, step, loss_scale=1.0, max_norm=0.0,
                   nthreads=1):
    """Scan, gate, update.  p/m/v/p_lp in place.  Returns (overflow, sumsq, clip)."""
    for a, nm in ((p, "p"), (m, "m"), (v, "v")):
        _chk(a, np.float32, nm)
    _chk(grad, _grad_dtype(gdt), "grad")
    _chk(p_lp, np.uint16, "p_lp")
    ss = ctypes.c_double(0.0)
    c = ctypes.c_float(0.0)
    ov = _lib.ora_optimizer_step(_ptr(p), _ptr(m), _ptr(v), _ptr(grad), _DT[gdt], _ptr(p_lp),
                                 _DT[pdt], p.size, ctypes.byref(h), int(step), loss_scale,
                                 float(max_norm), nthreads, ctypes.byref(ss), ctypes.byref(c))
    return bool(ov), ss.value, np.float32(c.value)


def grad_accumulate(acc, grad, gdt, first):
    """acc (fp32, in place) = grad if first else acc + grad, one fp32 addition per element."""
    _chk(acc, np.float32, "acc")
    _chk(grad, _grad_dtype(gdt), "grad")
    if acc.size != grad.size:
        raise ValueError("size mismatch")
    _lib.ora_grad_accumulate(_ptr(acc), _ptr(grad), _DT[gdt], acc.size, int(bool(first)))


def truncate_bf16(x):
    _chk(x, np.float32, "x")
    out = np.empty(x.shape, np.uint16)
    _lib.ora_truncate_bf16(_ptr(x), _ptr(out), x.size)
    return out


def adamw_step_bf16(p, m, v, grad, gdt, h, step, loss_scale=1.0, clip=1.0, nthreads=1):
    """AdamW with p, m, v held as bf16 bit patterns (uint16, in place), truncating stores."""
    for a, nm in ((p, "p"), (m, "m"), (v, "v")):
        _chk(a, np.uint16, nm)
    _chk(grad, _grad_dtype(gdt), "grad")
    if not (p.size == m.size == v.size == grad.size):
        raise ValueError("size mismatch")
    _lib.ora_adamw_step_bf16(_ptr(p), _ptr(m), _ptr(v), _ptr(grad), _DT[gdt], p.size,
                             ctypes.byref(h), int(step), loss_scale, float(clip), nthreads)


def scaler_cfg(backoff=0.5, growth=2.0, min_scale=1.0, max_scale=2.0 ** 24, window=1000):
    return ScalerCfg(backoff, growth, min_scale, max_scale, window)


def scaler_state(scale=65536.0, good_steps=0, step=0, skipped=0):
    return ScalerState(scale, good_steps, step, skipped)


def scaler_update(state, cfg, overflow):
    _lib.ora_scaler_update(ctypes.byref(state), ctypes.byref(cfg), int(bool(overflow)))


def optimizer_step_auto(p, m, v, grad, gdt, p_lp, pdt, h, state, cfg, max_norm=0.0, nthreads=1):
    """One iteration driven by the scaler state.  Returns (overflow, sumsq)."""
    for a, nm in ((p, "p"), (m, "m"), (v, "v")):
        _chk(a, np.float32, nm)
    _chk(grad, _grad_dtype(gdt), "grad")
    _chk(p_lp, np.uint16, "p_lp")
    ss = ctypes.c_double(0.0)
    ov = _lib.ora_optimizer_step_auto(_ptr(p), _ptr(m), _ptr(v), _ptr(grad), _DT[gdt], _ptr(p_lp),
                                      _DT[pdt], p.size, ctypes.byref(h), ctypes.byref(state),
                                      ctypes.byref(cfg), float(max_norm), nthreads, ctypes.byref(ss))
    return bool(ov), ss.value
