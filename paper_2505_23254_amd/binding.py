"""ctypes binding of libma_step.so (C ABI in include/ma.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.  torch is
used for device memory and the current HIP stream.  Importing this module fails loudly when the
library has not been built (python -m paper_2505_23254_amd.build, or __graft_entry__.build()).
"""
import ctypes
import os
import struct
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libma_step.so")

MA_F32, MA_BF16, MA_F16 = 0, 1, 2
_DT = {torch.float32: MA_F32, torch.bfloat16: MA_BF16, torch.float16: MA_F16}

MA_OK, MA_ERR_NULL, MA_ERR_DTYPE, MA_ERR_ALIGN, MA_ERR_ARG, MA_ERR_HIP, MA_ERR_FULL = 0, -1, -2, -3, -4, -5, -6
MA_POOL_EMBED, MA_POOL_FFN, MA_POOL_KV, MA_POOL_QO = 0, 1, 2, 3
MA_PINNED_PAGE, MA_PINNED_POW2 = 0, 1


class MaError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__("libma_step error %d: %s" % (code, message))
        self.code = code


class Hyper(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float),
                ("bias_correction", ctypes.c_int32)]


class Tensor(ctypes.Structure):
    _fields_ = [("p32", ctypes.c_void_p), ("m", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("grad", ctypes.c_void_p), ("p_lp", ctypes.c_void_p), ("n", ctypes.c_size_t)]


class TensorBF16(ctypes.Structure):
    _fields_ = [("p", ctypes.c_void_p), ("m", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("grad", ctypes.c_void_p), ("n", ctypes.c_size_t)]


class ScalerConfig(ctypes.Structure):
    _fields_ = [("backoff", ctypes.c_float), ("growth", ctypes.c_float),
                ("min_scale", ctypes.c_float), ("max_scale", ctypes.c_float),
                ("window", ctypes.c_int32)]


class ModelDims(ctypes.Structure):
    _fields_ = [(k, ctypes.c_uint64) for k in ("vocab", "hidden", "intermediate", "kv_dim", "q_dim")]


class PoolLayout(ctypes.Structure):
    _fields_ = [("count", ctypes.c_uint64 * 4), ("buffer_bytes", ctypes.c_uint64 * 4),
                ("offset", ctypes.c_uint64 * 4), ("total_bytes", ctypes.c_uint64),
                ("uniform_count", ctypes.c_uint64), ("uniform_buffer_bytes", ctypes.c_uint64),
                ("uniform_bytes", ctypes.c_uint64)]


class MultiPlanStruct(ctypes.Structure):
    _fields_ = [("table_dev", ctypes.c_void_p), ("entries", ctypes.c_uint64),
                ("total_elems", ctypes.c_uint64), ("norm_chunks", ctypes.c_uint64),
                ("step_chunks", ctypes.c_uint64), ("gdt", ctypes.c_int32), ("pdt", ctypes.c_int32),
                ("magic", ctypes.c_uint32), ("sdt", ctypes.c_uint32)]


class ArenaReport(ctypes.Structure):
    _fields_ = [("main_bytes", ctypes.c_uint64), ("side_bytes", ctypes.c_uint64),
                ("first_region_bytes", ctypes.c_uint64), ("blocks_created", ctypes.c_uint64),
                ("first_blocks_in_place", ctypes.c_uint64), ("second_blocks_in_place", ctypes.c_uint64),
                ("side_blocks_in_place", ctypes.c_uint64), ("regions_seen", ctypes.c_uint32),
                ("same_region_GBps", ctypes.c_float)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "%s is missing: build it first (python -m paper_2505_23254_amd.build). "
            "There is no fallback path." % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz, i32, i64, f32, f64 = (ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32,
                                  ctypes.c_int64, ctypes.c_float, ctypes.c_double)
    sig = {
        "ma_version": ([], ctypes.c_int),
        "ma_last_error": ([], ctypes.c_char_p),
        "ma_workspace_bytes": ([], sz),
        "ma_clip_coef": ([f64, f32], f32),
        "ma_step_scalars": ([vp, i64, f32, f32, vp], ctypes.c_int),
        "ma_plan_tensor": ([vp, i32, vp, vp, vp, vp, vp], ctypes.c_int),
        "ma_overflow_norm": ([vp, i32, sz, f32, vp, vp, sz, vp], ctypes.c_int),
        "ma_overflow_norm_static": ([vp, i32, sz, f32, vp, vp], ctypes.c_int),
        "ma_norm_combine": ([vp, sz, vp, vp], ctypes.c_int),
        "ma_adamw_step": ([vp, vp, vp, vp, i32, vp, i32, sz, vp, i64, f32, f32, vp], ctypes.c_int),
        "ma_adamw_step_gated": ([vp, vp, vp, vp, i32, vp, i32, sz, vp, i64, f32, vp, f32, vp],
                                ctypes.c_int),
        "ma_optimizer_step": ([vp, vp, vp, vp, i32, vp, i32, sz, vp, i64, f32, f32, vp, vp, sz, vp], ctypes.c_int),
        "ma_multi_optimizer_step": ([vp, vp, i64, f32, f32, vp, vp, sz, vp], ctypes.c_int),
        "ma_multi_table_bytes": ([sz], sz),
        "ma_multi_prepare": ([vp, sz, i32, i32, vp, sz, vp, vp], ctypes.c_int),
        "ma_multi_prepare_bf16": ([vp, sz, i32, vp, sz, vp, vp], ctypes.c_int),
        "ma_pool_layout_compute": ([vp, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32, vp],
                                   ctypes.c_int),
        "ma_pool_create": ([vp, vp], ctypes.c_int),
        "ma_pool_destroy": ([vp], None),
        "ma_pool_acquire": ([vp, ctypes.c_uint64, ctypes.c_int, vp, vp], ctypes.c_int),
        "ma_pool_lookup": ([vp, ctypes.c_uint64, vp, vp], ctypes.c_int),
        "ma_pool_release": ([vp, ctypes.c_uint64], ctypes.c_int),
        "ma_pool_in_use": ([vp, ctypes.c_int], ctypes.c_uint64),
        "ma_pinned_bytes": ([ctypes.c_uint64, ctypes.c_int], ctypes.c_uint64),
        "ma_pinned_alloc": ([sz, vp], ctypes.c_int),
        "ma_pinned_free": ([vp], ctypes.c_int),
        "ma_multi_overflow_norm": ([vp, f32, vp, vp, sz, vp], ctypes.c_int),
        "ma_multi_adamw_step": ([vp, vp, i64, f32, f32, vp], ctypes.c_int),
        "ma_multi_adamw_step_gated": ([vp, vp, i64, f32, vp, f32, vp], ctypes.c_int),
        "ma_adamw_step_bf16": ([vp, vp, vp, vp, i32, sz, vp, i64, f32, f32, vp], ctypes.c_int),
        "ma_adamw_step_bf16_gated": ([vp, vp, vp, vp, i32, sz, vp, i64, f32, vp, f32, vp],
                                     ctypes.c_int),
        "ma_grad_accumulate": ([vp, vp, i32, sz, ctypes.c_int, vp], ctypes.c_int),
        "ma_grad_accumulate_scan": ([vp, vp, i32, sz, ctypes.c_int, f32, vp, vp, vp, sz, vp], ctypes.c_int),
        "ma_scaler_init": ([vp, f32, i64, vp], ctypes.c_int),
        "ma_scaler_update": ([vp, vp, vp, vp], ctypes.c_int),
        "ma_overflow_norm_auto": ([vp, i32, sz, vp, vp, vp, sz, vp], ctypes.c_int),
        "ma_adamw_step_auto": ([vp, vp, vp, vp, i32, vp, i32, sz, vp, vp, vp, f32, vp],
                               ctypes.c_int),
        "ma_multi_overflow_norm_auto": ([vp, vp, vp, vp, sz, vp], ctypes.c_int),
        "ma_probe_update_mix": ([vp, vp, vp, vp, vp, sz, i32, vp], ctypes.c_int),
        "ma_probe_two_writes": ([vp, vp, sz, vp], ctypes.c_int),
        "ma_multi_adamw_step_auto": ([vp, vp, vp, vp, f32, vp], ctypes.c_int),
        "ma_arena_create": ([sz, sz, sz, sz, sz, vp], ctypes.c_int),
        "ma_arena_main": ([vp], vp),
        "ma_arena_side": ([vp], vp),
        "ma_arena_get_report": ([vp, vp], ctypes.c_int),
        "ma_arena_destroy": ([vp], ctypes.c_int),
    }
    for name, (args, res) in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = res
    return lib


lib = _load()


def _check(rc: int):
    if rc != MA_OK:
        raise MaError(rc, lib.ma_last_error().decode())


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _dev(t: Optional[torch.Tensor], name: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise TypeError("%s must live on the GPU" % name)
    if not t.is_contiguous():
        raise TypeError("%s must be contiguous" % name)
    return t.data_ptr()


def hyper(lr=1e-5, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, bias_correction=1) -> Hyper:
    return Hyper(lr, beta1, beta2, eps, weight_decay, int(bias_correction))


def version() -> int:
    return lib.ma_version()


def clip_coef(sumsq: float, max_norm: float) -> float:
    return lib.ma_clip_coef(float(sumsq), float(max_norm))


def step_scalars(h: Hyper, step: int, loss_scale: float = 1.0, clip: float = 1.0):
    """The nine fp32 scalars of one step (ma_step_scalars), as a list of Python floats."""
    out = (ctypes.c_float * 9)()
    _check(lib.ma_step_scalars(ctypes.byref(h), int(step), loss_scale, clip, out))
    return list(out)


def plan_tensor(p, m, v, g, lp, n: int, gdt: int):
    """ma_plan_tensor on raw addresses: (norm_items, step_items, norm_head, step_head, step_vec)."""
    t = Tensor(p, m, v, g, lp, n)
    ni, si = ctypes.c_uint64(), ctypes.c_uint64()
    nh, sh, sv = ctypes.c_uint32(), ctypes.c_uint32(), ctypes.c_uint32()
    _check(lib.ma_plan_tensor(ctypes.byref(t), gdt, ctypes.byref(ni), ctypes.byref(si),
                              ctypes.byref(nh), ctypes.byref(sh), ctypes.byref(sv)))
    return ni.value, si.value, nh.value, sh.value, sv.value


def workspace(device="cuda") -> torch.Tensor:
    """Device workspace for the scan calls (per-block partials)."""
    return torch.empty(lib.ma_workspace_bytes(), dtype=torch.uint8, device=device)


def new_result(count: int = 1, device="cuda") -> torch.Tensor:
    """`count` ma_norm_result slots (16 bytes each) as a float64 tensor of 2*count."""
    return torch.zeros(2 * count, dtype=torch.float64, device=device)


def read_result(res: torch.Tensor, index: int = 0):
    """Synchronising read-back of one ma_norm_result: (overflow: bool, sumsq: float)."""
    raw = res[2 * index:2 * index + 2].cpu().numpy().tobytes()
    ov, _, ss = struct.unpack("<iid", raw)
    return bool(ov), ss


def _slot(res: torch.Tensor, index: int) -> int:
    if res.dtype != torch.float64 or res.numel() < 2 * (index + 1):
        raise TypeError("result buffer must come from new_result()")
    return _dev(res, "result") + 16 * index


def overflow_norm(grad: torch.Tensor, loss_scale: float, out: torch.Tensor, ws: torch.Tensor,
                  index: int = 0, stream=None, n: Optional[int] = None) -> None:
    """ma_overflow_norm: scan `grad`, write slot `index` of `out`."""
    _check(lib.ma_overflow_norm(_dev(grad, "grad"), _DT[grad.dtype],
                                grad.numel() if n is None else n, loss_scale, _slot(out, index),
                                _dev(ws, "ws"), ws.numel() * ws.element_size(), _stream(stream)))


def overflow_norm_static(grad: torch.Tensor, loss_scale: float, out: torch.Tensor, index: int = 0,
                         stream=None, n: Optional[int] = None) -> None:
    """ma_overflow_norm_static: the scan with the library's own scratch (no workspace, no allocation)."""
    _check(lib.ma_overflow_norm_static(_dev(grad, "grad"), _DT[grad.dtype],
                                       grad.numel() if n is None else n, loss_scale, _slot(out, index),
                                       _stream(stream)))


def norm_combine(parts: torch.Tensor, count: int, out: torch.Tensor, index: int = 0,
                 stream=None) -> None:
    _check(lib.ma_norm_combine(_slot(parts, 0), count, _slot(out, index), _stream(stream)))


def _step_args(p, m, v, grad, p_lp):
    for t, nm in ((p, "p32"), (m, "m"), (v, "v")):
        if t.dtype != torch.float32:
            raise TypeError("%s must be float32" % nm)
    n = p.numel()
    if not (m.numel() == n and v.numel() == n and grad.numel() == n and
            (p_lp is None or p_lp.numel() == n)):
        raise ValueError("p32, m, v, grad and p_lp must have the same number of elements")
    pdt = _DT[p_lp.dtype] if p_lp is not None else MA_BF16
    return (_dev(p, "p32"), _dev(m, "m"), _dev(v, "v"), _dev(grad, "grad"), _DT[grad.dtype],
            _dev(p_lp, "p_lp"), pdt, n)


def adamw_step(p, m, v, grad, p_lp, h: Hyper, step: int, loss_scale: float = 1.0,
               clip: float = 1.0, stream=None) -> None:
    """ma_adamw_step on one flat sub-group (caller has already taken the gate)."""
    _check(lib.ma_adamw_step(*_step_args(p, m, v, grad, p_lp), ctypes.byref(h), int(step),
                             loss_scale, clip, _stream(stream)))


def adamw_step_gated(p, m, v, grad, p_lp, h: Hyper, step: int, loss_scale: float,
                     gate: torch.Tensor, max_norm: float, index: int = 0, stream=None) -> None:
    """ma_adamw_step_gated: the kernel reads slot `index` of `gate` on the device."""
    _check(lib.ma_adamw_step_gated(*_step_args(p, m, v, grad, p_lp), ctypes.byref(h), int(step),
                                   loss_scale, _slot(gate, index), max_norm, _stream(stream)))


def optimizer_step(p, m, v, grad, p_lp, h: Hyper, step: int, loss_scale: float, max_norm: float,
                   out: torch.Tensor, ws: torch.Tensor, index: int = 0, stream=None) -> None:
    """ma_optimizer_step: scan, gate and update of a flat sub-group in one call (two launches)."""
    _check(lib.ma_optimizer_step(*_step_args(p, m, v, grad, p_lp), ctypes.byref(h), int(step), loss_scale,
                                 max_norm, _slot(out, index), _dev(ws, "ws"), ws.numel() * ws.element_size(),
                                 _stream(stream)))


def read_result_raw(res: torch.Tensor, index: int = 0):
    """Synchronising read-back of one ma_norm_result as (overflow: int, sumsq: float)."""
    raw = res[2 * index:2 * index + 2].cpu().numpy().tobytes()
    ov, _, ss = struct.unpack("<iid", raw)
    return ov, ss


class MultiPlan:
    """A prepared tensor list (ma_multi_prepare).  Keeps the device table and the tensors alive."""

    def __init__(self, p: Sequence[torch.Tensor], m: Sequence[torch.Tensor],
                 v: Sequence[torch.Tensor], grad: Sequence[torch.Tensor],
                 p_lp: Optional[Sequence[torch.Tensor]], stream=None):
        count = len(p)
        if not (len(m) == count and len(v) == count and len(grad) == count and
                (p_lp is None or len(p_lp) == count)) or count == 0:
            raise ValueError("lists must be non-empty and of equal length")
        gdt = _DT[grad[0].dtype]
        pdt = _DT[p_lp[0].dtype] if p_lp is not None else MA_BF16
        arr = (Tensor * count)()
        for i in range(count):
            lp = p_lp[i] if p_lp is not None else None
            if _DT[grad[i].dtype] != gdt or (lp is not None and _DT[lp.dtype] != pdt):
                raise TypeError("all tensors of a list share one gradient and one p_lp dtype")
            pp, pm, pv, pg, _, pl, _, n = _step_args(p[i], m[i], v[i], grad[i], lp)
            arr[i] = Tensor(pp, pm, pv, pg, pl, n)
        self._keep = (list(p), list(m), list(v), list(grad), list(p_lp) if p_lp is not None else None)
        self.table = torch.empty(lib.ma_multi_table_bytes(count), dtype=torch.uint8,
                                 device=p[0].device)
        self.plan = MultiPlanStruct()
        _check(lib.ma_multi_prepare(arr, count, gdt, pdt, self.table.data_ptr(),
                                    self.table.numel(), _stream(stream), ctypes.byref(self.plan)))

    @property
    def total(self) -> int:
        return int(self.plan.total_elems)


class MultiPlanBF16(MultiPlan):
    """A prepared tensor list whose p, m, v are bfloat16 tensors (ma_multi_prepare_bf16)."""

    def __init__(self, p: Sequence[torch.Tensor], m: Sequence[torch.Tensor],
                 v: Sequence[torch.Tensor], grad: Sequence[torch.Tensor], stream=None):
        count = len(p)
        if not (len(m) == count and len(v) == count and len(grad) == count) or count == 0:
            raise ValueError("lists must be non-empty and of equal length")
        gdt = _DT[grad[0].dtype]
        arr = (TensorBF16 * count)()
        for i in range(count):
            if _DT[grad[i].dtype] != gdt:
                raise TypeError("all tensors of a list share one gradient dtype")
            pp, pm, pv, pg, _, n = _bf16_state_args(p[i], m[i], v[i], grad[i])
            arr[i] = TensorBF16(pp, pm, pv, pg, n)
        self._keep = (list(p), list(m), list(v), list(grad), None)
        self.table = torch.empty(lib.ma_multi_table_bytes(count), dtype=torch.uint8,
                                 device=p[0].device)
        self.plan = MultiPlanStruct()
        _check(lib.ma_multi_prepare_bf16(arr, count, gdt, self.table.data_ptr(), self.table.numel(),
                                         _stream(stream), ctypes.byref(self.plan)))


def multi_overflow_norm(plan: MultiPlan, loss_scale: float, out: torch.Tensor, ws: torch.Tensor,
                        index: int = 0, stream=None) -> None:
    _check(lib.ma_multi_overflow_norm(ctypes.byref(plan.plan), loss_scale, _slot(out, index),
                                      _dev(ws, "ws"), ws.numel() * ws.element_size(),
                                      _stream(stream)))


def multi_adamw_step(plan: MultiPlan, h: Hyper, step: int, loss_scale: float = 1.0,
                     clip: float = 1.0, stream=None) -> None:
    _check(lib.ma_multi_adamw_step(ctypes.byref(plan.plan), ctypes.byref(h), int(step), loss_scale,
                                   clip, _stream(stream)))


def multi_adamw_step_gated(plan: MultiPlan, h: Hyper, step: int, loss_scale: float,
                           gate: torch.Tensor, max_norm: float, index: int = 0,
                           stream=None) -> None:
    _check(lib.ma_multi_adamw_step_gated(ctypes.byref(plan.plan), ctypes.byref(h), int(step),
                                         loss_scale, _slot(gate, index), max_norm, _stream(stream)))


def multi_optimizer_step(plan: MultiPlan, h: Hyper, step: int, loss_scale: float, max_norm: float,
                         out: torch.Tensor, ws: torch.Tensor, index: int = 0, stream=None) -> None:
    """ma_multi_optimizer_step: scan, gate and update of a prepared tensor list in one call."""
    _check(lib.ma_multi_optimizer_step(ctypes.byref(plan.plan), ctypes.byref(h), int(step), loss_scale,
                                       max_norm, _slot(out, index), _dev(ws, "ws"),
                                       ws.numel() * ws.element_size(), _stream(stream)))


# ---- half-precision optimizer states ---------------------------------------------------------

def _bf16_state_args(p, m, v, grad):
    for t, nm in ((p, "p"), (m, "m"), (v, "v")):
        if t.dtype != torch.bfloat16:
            raise TypeError("%s must be bfloat16" % nm)
    n = p.numel()
    if not (m.numel() == n and v.numel() == n and grad.numel() == n):
        raise ValueError("p, m, v and grad must have the same number of elements")
    return _dev(p, "p"), _dev(m, "m"), _dev(v, "v"), _dev(grad, "grad"), _DT[grad.dtype], n


def adamw_step_bf16(p, m, v, grad, h: Hyper, step: int, loss_scale: float = 1.0,
                    clip: float = 1.0, stream=None) -> None:
    """ma_adamw_step_bf16: p, m, v held in bf16 and stored back by truncation."""
    _check(lib.ma_adamw_step_bf16(*_bf16_state_args(p, m, v, grad), ctypes.byref(h), int(step),
                                  loss_scale, clip, _stream(stream)))


def adamw_step_bf16_gated(p, m, v, grad, h: Hyper, step: int, loss_scale: float,
                          gate: torch.Tensor, max_norm: float, index: int = 0, stream=None) -> None:
    _check(lib.ma_adamw_step_bf16_gated(*_bf16_state_args(p, m, v, grad), ctypes.byref(h),
                                        int(step), loss_scale, _slot(gate, index), max_norm,
                                        _stream(stream)))


# ---- gradient accumulation ---------------------------------------------------------------------

def grad_accumulate(acc32: torch.Tensor, grad: torch.Tensor, first: bool, stream=None) -> None:
    """ma_grad_accumulate: acc32 = grad if first else acc32 + grad (fp32 flat buffer)."""
    if acc32.dtype != torch.float32:
        raise TypeError("acc32 must be float32")
    if acc32.numel() != grad.numel():
        raise ValueError("acc32 and grad must have the same number of elements")
    _check(lib.ma_grad_accumulate(_dev(acc32, "acc32"), _dev(grad, "grad"), _DT[grad.dtype],
                                  grad.numel(), int(bool(first)), _stream(stream)))


def grad_accumulate_scan(acc32: torch.Tensor, grad: torch.Tensor, first: bool, loss_scale: float,
                         out: torch.Tensor, ws: torch.Tensor, index: int = 0,
                         scaler: Optional[torch.Tensor] = None, stream=None) -> None:
    """ma_grad_accumulate_scan: accumulate, and scan the new contents of acc32 in the same pass."""
    if acc32.dtype != torch.float32:
        raise TypeError("acc32 must be float32")
    if acc32.numel() != grad.numel():
        raise ValueError("acc32 and grad must have the same number of elements")
    _check(lib.ma_grad_accumulate_scan(_dev(acc32, "acc32"), _dev(grad, "grad"), _DT[grad.dtype],
                                       grad.numel(), int(bool(first)), loss_scale,
                                       None if scaler is None else _scaler(scaler), _slot(out, index),
                                       _dev(ws, "ws"), ws.numel() * ws.element_size(), _stream(stream)))


# ---- dynamic loss scale on the device ------------------------------------------------------------

def scaler_config(backoff=0.5, growth=2.0, min_scale=1.0, max_scale=2.0 ** 24,
                  window=1000) -> ScalerConfig:
    return ScalerConfig(backoff, growth, min_scale, max_scale, int(window))


def new_scaler(scale: float, applied_steps: int = 0, device="cuda", stream=None) -> torch.Tensor:
    """One ma_scaler_state (24 bytes) in device memory, as an int64 tensor of 3."""
    st = torch.zeros(3, dtype=torch.int64, device=device)
    _check(lib.ma_scaler_init(_dev(st, "scaler"), scale, int(applied_steps), _stream(stream)))
    return st


def read_scaler(st: torch.Tensor):
    """Synchronising read-back: (scale, good_steps, step, skipped)."""
    return struct.unpack("<fiqq", st.cpu().numpy().tobytes())


def _scaler(st: torch.Tensor) -> int:
    if st.dtype != torch.int64 or st.numel() < 3:
        raise TypeError("scaler state must come from new_scaler()")
    return _dev(st, "scaler")


def scaler_update(st: torch.Tensor, gate: torch.Tensor, cfg: ScalerConfig, index: int = 0,
                  stream=None) -> None:
    _check(lib.ma_scaler_update(_scaler(st), _slot(gate, index), ctypes.byref(cfg), _stream(stream)))


def overflow_norm_auto(grad: torch.Tensor, scaler: torch.Tensor, out: torch.Tensor,
                       ws: torch.Tensor, index: int = 0, stream=None) -> None:
    _check(lib.ma_overflow_norm_auto(_dev(grad, "grad"), _DT[grad.dtype], grad.numel(),
                                     _scaler(scaler), _slot(out, index), _dev(ws, "ws"),
                                     ws.numel() * ws.element_size(), _stream(stream)))


def adamw_step_auto(p, m, v, grad, p_lp, h: Hyper, scaler: torch.Tensor, gate: torch.Tensor,
                    max_norm: float, index: int = 0, stream=None) -> None:
    _check(lib.ma_adamw_step_auto(*_step_args(p, m, v, grad, p_lp), ctypes.byref(h),
                                  _scaler(scaler), _slot(gate, index), max_norm, _stream(stream)))


def multi_overflow_norm_auto(plan: MultiPlan, scaler: torch.Tensor, out: torch.Tensor,
                             ws: torch.Tensor, index: int = 0, stream=None) -> None:
    _check(lib.ma_multi_overflow_norm_auto(ctypes.byref(plan.plan), _scaler(scaler),
                                           _slot(out, index), _dev(ws, "ws"),
                                           ws.numel() * ws.element_size(), _stream(stream)))


def multi_adamw_step_auto(plan: MultiPlan, h: Hyper, scaler: torch.Tensor, gate: torch.Tensor,
                          max_norm: float, index: int = 0, stream=None) -> None:
    _check(lib.ma_multi_adamw_step_auto(ctypes.byref(plan.plan), ctypes.byref(h), _scaler(scaler),
                                        _slot(gate, index), max_norm, _stream(stream)))


# ---- measurement aids ---------------------------------------------------------------------------------

def probe_update_mix(a, b, c, d16, e16=None, stream=None) -> None:
    """ma_probe_update_mix over the buffers of a state (contents destroyed): 14 B in / 14 B out per
    element for 4-byte a, b, c (e16 required), 8 in / 6 out for 2-byte a, b, c."""
    n, eb = a.numel(), a.element_size()
    if not (b.numel() == n and c.numel() == n and d16.numel() == n and (e16 is None or e16.numel() == n)):
        raise ValueError("the buffers must have the same number of elements")
    if eb not in (2, 4) or b.element_size() != eb or c.element_size() != eb or d16.element_size() != 2 or \
            (eb == 4 and (e16 is None or e16.element_size() != 2)):
        raise TypeError("a, b, c hold 4-byte (with a 2-byte e16) or 2-byte elements, d16 2-byte elements")
    _check(lib.ma_probe_update_mix(_dev(a, "a"), _dev(b, "b"), _dev(c, "c"), _dev(d16, "d16"),
                                   _dev(e16, "e16"), n, eb, _stream(stream)))


def probe_two_writes(x: torch.Tensor, y: torch.Tensor, stream=None) -> None:
    """ma_probe_two_writes over two equally large device buffers (contents destroyed)."""
    nb = x.numel() * x.element_size()
    if y.numel() * y.element_size() != nb:
        raise ValueError("the two buffers must be equally large")
    _check(lib.ma_probe_two_writes(_dev(x, "x"), _dev(y, "y"), nb, _stream(stream)))


# ---- host side: parameter buffer pool and pinned sizes ------------------------------------------------

def pool_layout(vocab: int, hidden: int, intermediate: int, kv_dim: int, q_dim: int,
                blocks_in_flight: int = 1, elem_bytes: int = 2, partitions: int = 1,
                align: int = 1) -> PoolLayout:
    """ma_pool_layout_compute: sizes of the adaptive and of the uniform parameter buffer pool."""
    dims = ModelDims(vocab, hidden, intermediate, kv_dim, q_dim)
    out = PoolLayout()
    _check(lib.ma_pool_layout_compute(ctypes.byref(dims), blocks_in_flight, elem_bytes, partitions,
                                      align, ctypes.byref(out)))
    return out


class BufferPool:
    """ma_pool_*: hands out byte offsets into one monolithic allocation, keyed by the caller."""

    def __init__(self, layout: PoolLayout):
        self._h = ctypes.c_void_p()
        _check(lib.ma_pool_create(ctypes.byref(layout), ctypes.byref(self._h)))

    def acquire(self, key: int, kind: int):
        off, nb = ctypes.c_uint64(), ctypes.c_uint64()
        _check(lib.ma_pool_acquire(self._h, key, kind, ctypes.byref(off), ctypes.byref(nb)))
        return off.value, nb.value

    def lookup(self, key: int):
        off, nb = ctypes.c_uint64(), ctypes.c_uint64()
        _check(lib.ma_pool_lookup(self._h, key, ctypes.byref(off), ctypes.byref(nb)))
        return off.value, nb.value

    def release(self, key: int) -> None:
        _check(lib.ma_pool_release(self._h, key))

    def in_use(self, kind: int) -> int:
        return lib.ma_pool_in_use(self._h, kind)

    def close(self) -> None:
        if self._h:
            lib.ma_pool_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        self.close()


def pinned_bytes(request: int, policy: int = MA_PINNED_PAGE) -> int:
    return lib.ma_pinned_bytes(request, policy)


def pinned_alloc(nbytes: int) -> int:
    """ma_pinned_alloc: address of page-locked host memory of exactly the page-rounded size."""
    p = ctypes.c_void_p()
    _check(lib.ma_pinned_alloc(nbytes, ctypes.byref(p)))
    return p.value


def pinned_free(ptr: int) -> None:
    _check(lib.ma_pinned_free(ptr))


class _RawDeviceBytes:
    """A device address range offered to torch through the CUDA array interface."""

    def __init__(self, ptr: int, nbytes: int, owner):
        self.owner = owner
        self.__cuda_array_interface__ = {"shape": (nbytes,), "typestr": "|u1", "data": (ptr, False),
                                         "version": 3, "strides": None}


class Arena:
    """ma_arena_create: `main_bytes` (+ `side_bytes`) of device memory stitched from physical blocks so
    that the first `first_region_bytes` of main, the rest of main and the side part lie in three
    different HBM regions.  `.main` / `.side` are uint8 tensors over the two parts (views: they do not
    own the memory; call close() only after the last use of them)."""

    def __init__(self, main_bytes: int, first_region_bytes: int, side_bytes: int = 0,
                 block_bytes: int = 0, max_transient_bytes: int = 0):
        h = ctypes.c_void_p()
        _check(lib.ma_arena_create(main_bytes, first_region_bytes, side_bytes, block_bytes,
                                   max_transient_bytes, ctypes.byref(h)))
        self._h = h
        try:
            rep = ArenaReport()
            _check(lib.ma_arena_get_report(h, ctypes.byref(rep)))
            self.report = {k: getattr(rep, k) for k, _ in ArenaReport._fields_}
            self.main = torch.as_tensor(_RawDeviceBytes(lib.ma_arena_main(h), main_bytes, self), device="cuda")
            self.side = (torch.as_tensor(_RawDeviceBytes(lib.ma_arena_side(h), side_bytes, self), device="cuda")
                         if side_bytes else None)
        except Exception:
            lib.ma_arena_destroy(h)      # nothing refers to the range yet
            self._h = None
            raise

    def close(self):
        if self._h:
            torch.cuda.synchronize()
            self.main = self.side = None
            _check(lib.ma_arena_destroy(self._h))
            self._h = None
