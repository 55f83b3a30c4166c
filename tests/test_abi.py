"""The C-ABI library loads, exports every symbol the public header declares, and rejects bad
arguments before anything reaches the device (no GPU needed: these calls launch nothing)."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2505_23254_amd import binding as ma

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "ma.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ma_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert len(names) >= 12
    raw = ctypes.CDLL(ma.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), n


def test_sizes_and_version():
    assert ma.version() >= 100
    assert ma.lib.ma_workspace_bytes() % 16 == 0 and ma.lib.ma_workspace_bytes() >= 4096 * 16
    assert ma.lib.ma_multi_table_bytes(10) == 10 * ma.lib.ma_multi_table_bytes(1)
    assert ctypes.sizeof(ma.Hyper) == 24 and ctypes.sizeof(ma.Tensor) == 48
    assert ctypes.sizeof(ma.MultiPlanStruct) == 56


def test_host_clip_coef_matches_oracle():
    for ss in (0.0, 1e-12, 0.25, 1.0, 100.0, 1.23456789e7, 1e30):
        for mn in (1.0, 0.1, 3.0, 0.0, -1.0):
            assert np.float32(ma.clip_coef(ss, mn)) == oracle.clip_coef(ss, float(np.float32(mn)))


H = ma.hyper()
A = 0x10000  # a fake, suitably aligned "device" address; never dereferenced on these paths


def _step(**kw):
    a = dict(p=A, m=A, v=A, g=A, gdt=ma.MA_BF16, lp=A, pdt=ma.MA_BF16, n=16, h=ctypes.byref(H),
             step=1, scale=1.0, clip=1.0)
    a.update(kw)
    return ma.lib.ma_adamw_step(a["p"], a["m"], a["v"], a["g"], a["gdt"], a["lp"], a["pdt"], a["n"],
                                a["h"], a["step"], a["scale"], a["clip"], None)


def test_step_argument_errors():
    assert _step(step=0) == ma.MA_ERR_ARG and b"step" in ma.lib.ma_last_error()
    assert _step(clip=0.0) == ma.MA_ERR_ARG
    assert _step(clip=1.5) == ma.MA_ERR_ARG
    assert _step(scale=0.0) == ma.MA_ERR_ARG
    assert _step(scale=float("inf")) == ma.MA_ERR_ARG
    assert _step(gdt=7) == ma.MA_ERR_DTYPE
    assert _step(pdt=ma.MA_F32) == ma.MA_ERR_DTYPE
    assert _step(h=None) == ma.MA_ERR_NULL
    assert _step(p=None) == ma.MA_ERR_NULL
    assert _step(g=None) == ma.MA_ERR_NULL
    assert _step(p=A + 2) == ma.MA_ERR_ALIGN
    assert _step(g=A + 1) == ma.MA_ERR_ALIGN
    assert _step(lp=A + 1) == ma.MA_ERR_ALIGN
    for bad in (dict(lr=-1.0), dict(beta1=1.0), dict(beta2=-0.1), dict(eps=0.0),
                dict(weight_decay=-1.0), dict(lr=float("nan"))):
        h = ma.hyper(**bad)
        assert _step(h=ctypes.byref(h)) == ma.MA_ERR_ARG
    assert _step(n=0) == ma.MA_OK          # empty sub-group: nothing to do, nothing launched


def test_scan_argument_errors():
    f = ma.lib.ma_overflow_norm
    ws = ma.lib.ma_workspace_bytes()
    assert f(A, ma.MA_BF16, 8, 1.0, None, A, ws, None) == ma.MA_ERR_NULL
    assert f(A, ma.MA_BF16, 8, 1.0, A, None, ws, None) == ma.MA_ERR_NULL
    assert f(A, ma.MA_BF16, 8, 1.0, A, A, ws - 1, None) == ma.MA_ERR_ARG
    assert f(A, 9, 8, 1.0, A, A, ws, None) == ma.MA_ERR_DTYPE
    assert f(A, ma.MA_F16, 8, -2.0, A, A, ws, None) == ma.MA_ERR_ARG
    assert f(None, ma.MA_F16, 8, 1.0, A, A, ws, None) == ma.MA_ERR_NULL
    assert f(A + 1, ma.MA_F16, 8, 1.0, A, A, ws, None) == ma.MA_ERR_ALIGN
    assert f(A, ma.MA_F16, 8, 1.0, A + 4, A, ws, None) == ma.MA_ERR_ALIGN
    assert ma.lib.ma_norm_combine(A, 0, A + 64, None) == ma.MA_ERR_ARG
    assert ma.lib.ma_norm_combine(A, 4, A + 16, None) == ma.MA_ERR_ARG     # out inside parts
    assert ma.lib.ma_norm_combine(None, 4, A, None) == ma.MA_ERR_NULL


def test_multi_argument_errors():
    arr = (ma.Tensor * 2)(ma.Tensor(A, A, A, A, A, 8), ma.Tensor(A, A, A, A + 1, A, 8))
    plan = ma.MultiPlanStruct()
    prep = ma.lib.ma_multi_prepare
    assert prep(arr, 2, ma.MA_BF16, ma.MA_BF16, A, 160, None, ctypes.byref(plan)) == ma.MA_ERR_ALIGN
    assert b"tensor 1" in ma.lib.ma_last_error()
    assert prep(arr, 1, ma.MA_BF16, ma.MA_BF16, A, 10, None, ctypes.byref(plan)) == ma.MA_ERR_ARG
    assert prep(arr, 0, ma.MA_BF16, ma.MA_BF16, A, 160, None, ctypes.byref(plan)) == ma.MA_ERR_ARG
    assert prep(None, 1, ma.MA_BF16, ma.MA_BF16, A, 160, None, ctypes.byref(plan)) == ma.MA_ERR_NULL
    assert prep(arr, 1, ma.MA_BF16, ma.MA_F32, A, 160, None, ctypes.byref(plan)) == ma.MA_ERR_DTYPE
    mixed = (ma.Tensor * 2)(ma.Tensor(A, A, A, A, A, 8), ma.Tensor(A, A, A, A, None, 8))
    assert prep(mixed, 2, ma.MA_BF16, ma.MA_BF16, A, 160, None, ctypes.byref(plan)) == ma.MA_ERR_ARG
    # a plan that did not come from ma_multi_prepare is refused
    assert ma.lib.ma_multi_adamw_step(ctypes.byref(plan), ctypes.byref(H), 1, 1.0, 1.0, None) == ma.MA_ERR_ARG
    assert ma.lib.ma_multi_overflow_norm(ctypes.byref(plan), 1.0, A, A, 1 << 20, None) == ma.MA_ERR_ARG
    assert ma.lib.ma_multi_adamw_step_gated(None, ctypes.byref(H), 1, 1.0, A, 1.0, None) == ma.MA_ERR_NULL
