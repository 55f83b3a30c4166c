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
    assert ma.lib.ma_multi_table_bytes(10) - ma.lib.ma_multi_table_bytes(1) == 9 * 80    # one 80-byte row per tensor
    assert ma.lib.ma_multi_table_bytes(1) == 64 + 80                                     # after a 64-byte head
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
    # the variant with library-owned scratch checks the same arguments, and its size limit, first
    g = ma.lib.ma_overflow_norm_static
    assert g(A, ma.MA_BF16, 8, 1.0, None, None) == ma.MA_ERR_NULL
    assert g(None, ma.MA_BF16, 8, 1.0, A, None) == ma.MA_ERR_NULL
    assert g(A, 9, 8, 1.0, A, None) == ma.MA_ERR_DTYPE
    assert g(A + 1, ma.MA_F16, 8, 1.0, A, None) == ma.MA_ERR_ALIGN
    assert g(A, ma.MA_F16, 8, 0.0, A, None) == ma.MA_ERR_ARG
    assert g(A, ma.MA_F16, (1 << 38) + 1, 1.0, A, None) == ma.MA_ERR_ARG and b"maximum" in ma.lib.ma_last_error()
    assert ma.lib.ma_norm_combine(A, 0, A + 64, None) == ma.MA_ERR_ARG
    assert ma.lib.ma_norm_combine(A, 4, A + 16, None) == ma.MA_ERR_ARG     # out inside parts
    assert ma.lib.ma_norm_combine(None, 4, A, None) == ma.MA_ERR_NULL


def test_multi_argument_errors():
    arr = (ma.Tensor * 2)(ma.Tensor(A, A, A, A, A, 8), ma.Tensor(A, A, A, A + 1, A, 8))
    plan = ma.MultiPlanStruct()
    prep = ma.lib.ma_multi_prepare
    assert prep(arr, 2, ma.MA_BF16, ma.MA_BF16, A, 224, None, ctypes.byref(plan)) == ma.MA_ERR_ALIGN
    assert b"tensor 1" in ma.lib.ma_last_error()
    assert prep(arr, 1, ma.MA_BF16, ma.MA_BF16, A, 10, None, ctypes.byref(plan)) == ma.MA_ERR_ARG
    assert prep(arr, 0, ma.MA_BF16, ma.MA_BF16, A, 224, None, ctypes.byref(plan)) == ma.MA_ERR_ARG
    assert prep(None, 1, ma.MA_BF16, ma.MA_BF16, A, 224, None, ctypes.byref(plan)) == ma.MA_ERR_NULL
    assert prep(arr, 1, ma.MA_BF16, ma.MA_F32, A, 224, None, ctypes.byref(plan)) == ma.MA_ERR_DTYPE
    mixed = (ma.Tensor * 2)(ma.Tensor(A, A, A, A, A, 8), ma.Tensor(A, A, A, A, None, 8))
    assert prep(mixed, 2, ma.MA_BF16, ma.MA_BF16, A, 224, None, ctypes.byref(plan)) == ma.MA_ERR_ARG
    # a plan that did not come from ma_multi_prepare is refused
    assert ma.lib.ma_multi_adamw_step(ctypes.byref(plan), ctypes.byref(H), 1, 1.0, 1.0, None) == ma.MA_ERR_ARG
    assert ma.lib.ma_multi_overflow_norm(ctypes.byref(plan), 1.0, A, A, 1 << 20, None) == ma.MA_ERR_ARG
    assert ma.lib.ma_multi_adamw_step_gated(None, ctypes.byref(H), 1, 1.0, A, 1.0, None) == ma.MA_ERR_NULL


def test_multi_bf16_argument_errors():
    arr = (ma.TensorBF16 * 2)(ma.TensorBF16(A, A, A, A, 8), ma.TensorBF16(A, A + 1, A, A, 8))
    plan = ma.MultiPlanStruct()
    prep = ma.lib.ma_multi_prepare_bf16
    assert ctypes.sizeof(ma.TensorBF16) == 40
    assert prep(arr, 2, ma.MA_BF16, A, 224, None, ctypes.byref(plan)) == ma.MA_ERR_ALIGN
    assert b"tensor 1" in ma.lib.ma_last_error()
    assert prep(arr, 1, 9, A, 224, None, ctypes.byref(plan)) == ma.MA_ERR_DTYPE
    assert prep(None, 1, ma.MA_BF16, A, 224, None, ctypes.byref(plan)) == ma.MA_ERR_NULL
    assert prep(arr, 1, ma.MA_BF16, A, 8, None, ctypes.byref(plan)) == ma.MA_ERR_ARG
    assert prep(arr, 1, ma.MA_BF16, A, 224, None, None) == ma.MA_ERR_NULL
    nul = (ma.TensorBF16 * 1)(ma.TensorBF16(A, None, A, A, 8))
    assert prep(nul, 1, ma.MA_BF16, A, 224, None, ctypes.byref(plan)) == ma.MA_ERR_NULL
    # a plan with an unknown state dtype is refused
    good = ma.MultiPlanStruct(A, 1, 8, 1, 1, ma.MA_BF16, ma.MA_BF16, 0x4D415450, 7)
    assert ma.lib.ma_multi_adamw_step(ctypes.byref(good), ctypes.byref(H), 1, 1.0, 1.0, None) == ma.MA_ERR_ARG


def test_host_step_scalars_match_oracle_bit_for_bit():
    import itertools
    for lr, b1, b2, eps, wd, bc in itertools.product((1e-5, 3e-2, 0.0), (0.9, 0.0, 0.8), (0.999, 0.95),
                                                     (1e-8, 1e-3), (0.01, 0.0), (1, 0)):
        for step, scale, clip in ((1, 1.0, 1.0), (100, 65536.0, 0.37), (10 ** 6, 3.0, 1e-3), (7, 0.5, 1.0)):
            got = np.array(ma.step_scalars(ma.hyper(lr, b1, b2, eps, wd, bc), step, scale, clip), np.float32)
            ref = oracle.step_scalars(oracle.hyper(lr, b1, b2, eps, wd, bc), step, scale, clip)
            assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), (lr, b1, b2, eps, wd, bc, step)


def sweep_steps(count=4000, seed=5):
    """Update numbers for the bias-correction sweeps: the small ones, decades up to 10^6 and their
    neighbours, and seeded log-uniform draws in between."""
    rng = np.random.default_rng(seed)
    t = set(range(1, 300)) | {10 ** k + d for k in range(2, 7) for d in (-1, 0, 1)} | {2 ** k for k in range(1, 21)}
    t |= set(int(x) for x in np.exp(rng.uniform(np.log(300), np.log(2e6), count)).astype(np.int64))
    return sorted(t)


SWEEP_BETAS = ((0.9, 0.999), (0.8, 0.95), (0.99, 0.9999))


def test_host_bias_corrections_match_the_oracle_over_a_sweep_of_update_numbers():
    """lr / (1 - beta1^t) and 1 / sqrt(1 - beta2^t): the library's integer power against the oracle's
    library pow, as fp32 bit patterns, over thousands of update numbers."""
    steps = sweep_steps()
    assert len(steps) > 3000 and {1, 2, 1000, 10 ** 5, 10 ** 6} <= set(steps)
    for b1, b2 in SWEEP_BETAS:
        for lr in (1e-3, 3.7e-5):
            h, ho = ma.hyper(lr, b1, b2, 1e-8, 0.01, 1), oracle.hyper(lr, b1, b2, 1e-8, 0.01, 1)
            for t in steps:
                got = np.array(ma.step_scalars(h, t), np.float32)
                ref = oracle.step_scalars(ho, t)
                assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), (b1, b2, lr, t)


def _model_plan(p, m, v, g, lp, n, gbytes, norm_chunk_bytes, step_chunk_elems):
    """Independent model of the work split, from the contract in the header."""
    norm_head = ((16 - g % 16) % 16) // gbytes
    norm_items = 1 if n <= norm_head else -(-(n - norm_head) // (norm_chunk_bytes // gbytes))
    h = ((16 - p % 16) % 16) // 4
    ok = all((a + h * eb) % (4 * eb) == 0 for a, eb in ((m, 4), (v, 4), (g, gbytes)) + (((lp, 2),) if lp else ()))
    if ok:
        step_items = 1 if n <= h else -(-(n - h) // step_chunk_elems)
        return norm_items, step_items, norm_head, h, 1
    return norm_items, -(-n // step_chunk_elems), norm_head, 0, 0


def test_work_split_of_a_tensor():
    # the two work-item sizes are read off two calls, then every alignment class is checked
    base = 0x7F0000000000
    big = 1 << 40
    ni, si, *_ = ma.plan_tensor(base, base, base, base, base, big, ma.MA_BF16)
    norm_chunk_bytes, step_chunk_elems = 2 * big // ni, big // si
    assert norm_chunk_bytes % (256 * 16) == 0 and step_chunk_elems % 1024 == 0
    rng = np.random.default_rng(3)
    for gdt, gb in ((ma.MA_BF16, 2), (ma.MA_F16, 2), (ma.MA_F32, 4)):
        for trial in range(400):
            k = int(rng.integers(0, 8))
            same = trial % 2 == 0
            offs = [k] * 5 if same else [int(x) for x in rng.integers(0, 8, 5)]
            p, m, v = (base + 4 * o for o in offs[:3])
            g = base + gb * offs[3]
            lp = (base + 2 * offs[4]) if trial % 5 else None
            n = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 4095, 4096, 4097, 16384, 16385, 100003, 2 ** 31 + 5]))
            got = ma.plan_tensor(p, m, v, g, lp, n, gdt)
            want = _model_plan(p, m, v, g, lp or 0, n, gb, norm_chunk_bytes, step_chunk_elems)
            assert got == want, (offs, n, gdt, got, want)
            if same:
                assert got[4] == 1 and got[3] == (4 - k % 4) % 4
    assert ma.plan_tensor(base, base, base, base, base, 0, ma.MA_BF16) == (0, 0, 0, 0, 0)


def test_bf16_state_and_accumulate_argument_errors():
    f = ma.lib.ma_adamw_step_bf16
    hb = ctypes.byref(H)
    assert f(A, A, A, A, ma.MA_BF16, 16, hb, 0, 1.0, 1.0, None) == ma.MA_ERR_ARG
    assert f(A, A, A, A, ma.MA_BF16, 16, hb, 1, 1.0, 0.0, None) == ma.MA_ERR_ARG
    assert f(A, A, A, A, 5, 16, hb, 1, 1.0, 1.0, None) == ma.MA_ERR_DTYPE
    assert f(None, A, A, A, ma.MA_BF16, 16, hb, 1, 1.0, 1.0, None) == ma.MA_ERR_NULL
    assert f(A + 1, A, A, A, ma.MA_BF16, 16, hb, 1, 1.0, 1.0, None) == ma.MA_ERR_ALIGN
    assert f(A, A, A + 1, A, ma.MA_BF16, 16, hb, 1, 1.0, 1.0, None) == ma.MA_ERR_ALIGN
    assert f(A, A, A, A + 2, ma.MA_F32, 16, hb, 1, 1.0, 1.0, None) == ma.MA_ERR_ALIGN
    assert f(A, A, A, A, ma.MA_BF16, 0, hb, 1, 1.0, 1.0, None) == ma.MA_OK
    fg = ma.lib.ma_adamw_step_bf16_gated
    assert fg(A, A, A, A, ma.MA_BF16, 16, hb, 1, 1.0, None, 1.0, None) == ma.MA_ERR_NULL
    assert fg(A, A, A, A, ma.MA_BF16, 16, hb, 1, 1.0, A + 4, 1.0, None) == ma.MA_ERR_ALIGN
    assert fg(A, A, A, A, ma.MA_BF16, 16, hb, 1, 1.0, A, float("nan"), None) == ma.MA_ERR_ARG
    acc = ma.lib.ma_grad_accumulate
    assert acc(None, A, ma.MA_BF16, 8, 1, None) == ma.MA_ERR_NULL
    assert acc(A, None, ma.MA_BF16, 8, 1, None) == ma.MA_ERR_NULL
    assert acc(A + 2, A, ma.MA_BF16, 8, 1, None) == ma.MA_ERR_ALIGN
    assert acc(A, A + 1, ma.MA_F16, 8, 0, None) == ma.MA_ERR_ALIGN
    assert acc(A, A + 2, ma.MA_F32, 8, 0, None) == ma.MA_ERR_ALIGN
    assert acc(A, A, 4, 8, 0, None) == ma.MA_ERR_DTYPE
    assert acc(A, A, ma.MA_BF16, 0, 0, None) == ma.MA_OK
    fused = ma.lib.ma_grad_accumulate_scan
    ws = ma.lib.ma_workspace_bytes()
    assert fused(A, A, ma.MA_BF16, 8, 0, 1.0, None, None, A, ws, None) == ma.MA_ERR_NULL       # out_dev
    assert fused(A, A, ma.MA_BF16, 8, 0, 1.0, None, A, None, ws, None) == ma.MA_ERR_NULL       # ws
    assert fused(A, A, ma.MA_BF16, 8, 0, 1.0, None, A, A, ws - 16, None) == ma.MA_ERR_ARG
    assert fused(A, A, ma.MA_BF16, 8, 0, 0.0, None, A, A, ws, None) == ma.MA_ERR_ARG           # scale
    assert fused(A, A, ma.MA_BF16, 8, 0, 0.0, A + 4, A, A, ws, None) == ma.MA_ERR_ALIGN        # scaler
    assert fused(None, A, ma.MA_BF16, 8, 0, 1.0, None, A, A, ws, None) == ma.MA_ERR_NULL
    assert fused(A, A + 1, ma.MA_BF16, 8, 0, 1.0, None, A, A, ws, None) == ma.MA_ERR_ALIGN
    assert fused(A, A, 6, 8, 0, 1.0, None, A, A, ws, None) == ma.MA_ERR_DTYPE


def test_scaler_argument_errors():
    assert ctypes.sizeof(ma.ScalerConfig) == 20
    init, upd = ma.lib.ma_scaler_init, ma.lib.ma_scaler_update
    assert init(None, 1.0, 0, None) == ma.MA_ERR_NULL
    assert init(A + 4, 1.0, 0, None) == ma.MA_ERR_ALIGN
    assert init(A, 0.0, 0, None) == ma.MA_ERR_ARG
    assert init(A, float("inf"), 0, None) == ma.MA_ERR_ARG
    assert init(A, 1.0, -1, None) == ma.MA_ERR_ARG
    good = ma.scaler_config()
    assert upd(None, A, ctypes.byref(good), None) == ma.MA_ERR_NULL
    assert upd(A, None, ctypes.byref(good), None) == ma.MA_ERR_NULL
    assert upd(A, A, None, None) == ma.MA_ERR_NULL
    assert upd(A + 4, A, ctypes.byref(good), None) == ma.MA_ERR_ALIGN
    for bad in (dict(backoff=0.0), dict(backoff=1.0), dict(growth=0.5), dict(growth=float("inf")),
                dict(min_scale=0.0), dict(min_scale=4.0, max_scale=2.0), dict(max_scale=float("inf")),
                dict(window=0)):
        c = ma.scaler_config(**bad)
        assert upd(A, A, ctypes.byref(c), None) == ma.MA_ERR_ARG, bad
    ws = ma.lib.ma_workspace_bytes()
    na = ma.lib.ma_overflow_norm_auto
    assert na(A, ma.MA_F16, 8, None, A, A, ws, None) == ma.MA_ERR_NULL
    assert na(A, ma.MA_F16, 8, A + 4, A, A, ws, None) == ma.MA_ERR_ALIGN
    assert na(A, ma.MA_F16, 8, A, None, A, ws, None) == ma.MA_ERR_NULL
    sa = ma.lib.ma_adamw_step_auto
    hb = ctypes.byref(H)
    assert sa(A, A, A, A, ma.MA_F16, A, ma.MA_BF16, 8, hb, None, A, 1.0, None) == ma.MA_ERR_NULL
    assert sa(A, A, A, A, ma.MA_F16, A, ma.MA_BF16, 8, hb, A, None, 1.0, None) == ma.MA_ERR_NULL
    assert sa(A, A, A, A, ma.MA_F16, A, ma.MA_BF16, 8, None, A, A, 1.0, None) == ma.MA_ERR_NULL
    assert sa(A, A, A, A, ma.MA_F16, A, ma.MA_F32, 8, hb, A, A, 1.0, None) == ma.MA_ERR_DTYPE
    plan = ma.MultiPlanStruct()
    assert ma.lib.ma_multi_overflow_norm_auto(ctypes.byref(plan), A, A, A, ws, None) == ma.MA_ERR_ARG
    assert ma.lib.ma_multi_adamw_step_auto(ctypes.byref(plan), hb, A, A, 1.0, None) == ma.MA_ERR_ARG


def test_region_window_placement():
    """Host logic of the HBM placement helper: the traffic midpoint of a state lands on the boundary
    between the first two 96 GiB regions; very large states are centred on the middle region."""
    from paper_2505_23254_amd import hbm, synth
    G = hbm.GIB
    mid = hbm.DeviceArena._midpoint
    assert mid(120 * G, None) == 60 * G
    # p, m, v (read + written) then g, p_lp (one direction): half of 28 units lies 6/8 into m
    n = 1 << 30
    tr = synth.flat_traffic(n)
    assert [w for _, w in tr] == [2.0, 2.0, 2.0, 1.0, 1.0]
    assert sum(b for b, _ in tr) == synth.flat_state_bytes(n)
    assert mid(synth.flat_state_bytes(n), tr) == 4 * n + 3 * n
    shapes = synth.llama3_8b_shapes()
    assert synth.list_state_bytes(shapes, "streams") == synth.flat_state_bytes(8_030_257_152)
    assert synth.list_state_bytes(shapes, "tensor") >= 14 * 8_030_257_152
    assert synth.list_traffic(shapes, "tensor") is None

    class Fake(hbm.DeviceArena):
        def __init__(self, nbytes):
            self.buf = np.empty(0)
            self._n = nbytes

        @property
        def nbytes(self):
            return self._n

        def window(self, nbytes, traffic=None):      # same arithmetic, returns the start offset
            self.buf = _Span(self._n)
            return super().window(nbytes, traffic)

    class _Span:
        def __init__(self, n):
            self.n = n

        def numel(self):
            return self.n

        def __getitem__(self, sl):
            return sl.start, sl.stop

    a = Fake(283 * G)
    s, e = a.window(120 * G)
    assert (s, e) == (36 * G, 156 * G)
    s, e = a.window(200 * G)                           # larger than two regions: centred on 144 GiB
    assert (s + e) // 2 == 144 * G
    s, e = a.window(280 * G)
    assert s >= 0 and e <= 283 * G
    with pytest.raises(ValueError):
        a.window(284 * G)


def test_header_is_plain_c_and_layouts_match_the_binding(tmp_path):
    """include/ma.h compiles as C99 and as C++ with every warning an error, and each struct the
    binding mirrors has the size and field offsets the C compiler gives it."""
    import subprocess
    mirrors = {"ma_hyper": ma.Hyper, "ma_tensor": ma.Tensor, "ma_tensor_bf16": ma.TensorBF16,
               "ma_scaler_config": ma.ScalerConfig, "ma_model_dims": ma.ModelDims,
               "ma_pool_layout": ma.PoolLayout, "ma_multi_plan": ma.MultiPlanStruct}
    lines = ['#include "ma.h"', "#include <stdio.h>", "#include <stddef.h>", "int main(void) {"]
    for cname, cls in mirrors.items():
        lines.append('  printf("%s size %%zu\\n", sizeof(%s));' % (cname, cname))
        for field, _ in cls._fields_:
            lines.append('  printf("%s %s %%zu\\n", offsetof(%s, %s));' % (cname, field, cname, field))
    for cname in ("ma_norm_result", "ma_scaler_state"):
        lines.append('  printf("%s size %%zu\\n", sizeof(%s));' % (cname, cname))
    lines += ["  return 0;", "}"]
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines) + "\n")
    inc = os.path.join(ROOT, "include")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Wpedantic", "-Werror", "-I", inc, str(src), "-o", str(exe)],
                   check=True, capture_output=True)
    cpp = tmp_path / "layout.cpp"
    cpp.write_text(src.read_text())
    subprocess.run(["g++", "-std=c++11", "-Wall", "-Wextra", "-Wpedantic", "-Werror", "-fsyntax-only", "-I", inc, str(cpp)],
                   check=True, capture_output=True)
    got = {}
    for line in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n"):
        if line:
            a, b, c = line.split()
            got[(a, b)] = int(c)
    for cname, cls in mirrors.items():
        assert got[(cname, "size")] == ctypes.sizeof(cls), cname
        for field, _ in cls._fields_:
            assert got[(cname, field)] == getattr(cls, field).offset, (cname, field)
    assert got[("ma_norm_result", "size")] == 16 and got[("ma_scaler_state", "size")] == 24


def test_a_plain_c_program_links_and_calls_the_host_side(tmp_path):
    """A C99 translation unit that includes only include/ma.h links against the library and calls
    its host-side entry points (nothing here needs a GPU)."""
    import subprocess
    src = tmp_path / "host_calls.c"
    src.write_text(r'''
#include "ma.h"
#include <stdio.h>
int main(void) {
  ma_model_dims d = {152064u, 3584u, 18944u, 512u, 3584u};   /* Qwen2.5-7B shapes */
  ma_pool_layout lay;
  int rc = ma_pool_layout_compute(&d, 1u, 2u, 1u, 1u, &lay);
  ma_hyper h = {1e-5f, 0.9f, 0.999f, 1e-8f, 0.01f, 1};
  float sc[9];
  int rc2 = ma_step_scalars(&h, 100, 1.0f, 1.0f, sc);
  int rc3 = ma_step_scalars(&h, 0, 1.0f, 1.0f, sc);           /* step < 1: an argument error */
  printf("%d %d %d %llu %llu %.9g %.9g %d\n", ma_version() >= 100, rc, rc2,
         (unsigned long long)lay.total_bytes, (unsigned long long)lay.uniform_bytes,
         (double)ma_clip_coef(100.0, 1.0f), (double)sc[0], rc3);
  printf("%s\n", ma_last_error());
  return 0;
}
''')
    exe = tmp_path / "host_calls"
    libdir = os.path.dirname(ma.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"), str(src),
                    "-L", libdir, "-l:" + os.path.basename(ma.LIB_PATH), "-Wl,-rpath," + libdir, "-o", str(exe)],
                   check=True, capture_output=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    f = out[0].split()
    assert f[:3] == ["1", "0", "0"]
    lay = ma.pool_layout(152064, 3584, 18944, 512, 3584, 1, 2)
    assert int(f[3]) == lay.total_bytes and int(f[4]) == lay.uniform_bytes
    assert abs(float(f[5]) - 0.1) < 1e-7 and np.float32(float(f[6])) == np.float32(0.9)
    assert int(f[7]) == ma.MA_ERR_ARG and "step" in out[1]


def test_gpu_tests_refuse_a_substituted_oracle(tmp_path):
    """With MA_ORACLE_LIBRARY set every GPU-marked test fails in its set-up, before it touches a GPU."""
    import shutil
    import subprocess
    import sys
    alt = tmp_path / "liboracle_copy.so"
    shutil.copy(os.path.join(ROOT, "oracle", "liboracle.so"), alt)
    env = dict(os.environ, MA_ORACLE_LIBRARY=str(alt))
    r = subprocess.run([sys.executable, "-m", "pytest", "tests/test_zz_no_alloc.py", "-m", "gpu", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True)
    assert r.returncode != 0 and "MA_ORACLE_LIBRARY is set" in r.stdout


def test_overlapping_buffers_are_rejected():
    """Byte ranges that share a byte: MA_ERR_ARG before anything is launched (fake addresses)."""
    B = 0x100000
    ok = dict(p=B, m=B + 0x1000, v=B + 0x2000, g=B + 0x3000, lp=B + 0x4000, n=1024)      # 4 KiB apart: disjoint
    assert _step(**dict(ok, step=0)) == ma.MA_ERR_ARG and b"step" in ma.lib.ma_last_error()  # still the first error
    for bad in (dict(m=B + 0xFFC), dict(v=B), dict(g=B + 0x2800), dict(lp=B + 0x37FE), dict(p=B + 0x4000 + 2044)):
        assert _step(**dict(ok, **bad)) == ma.MA_ERR_ARG, bad
        assert b"overlap" in ma.lib.ma_last_error()
    # the same through a tensor list: inside one tensor, and between two tensors
    plan = ma.MultiPlanStruct()
    prep = ma.lib.ma_multi_prepare
    inside = (ma.Tensor * 1)(ma.Tensor(B, B + 0x1000, B + 0x2000, B + 0x3000, B + 0x2F00, 1024))
    assert prep(inside, 1, ma.MA_BF16, ma.MA_BF16, A, 224, None, ctypes.byref(plan)) == ma.MA_ERR_ARG
    assert b"overlap" in ma.lib.ma_last_error()
    C = B + 0x10000
    across = (ma.Tensor * 2)(ma.Tensor(B, B + 0x1000, B + 0x2000, B + 0x3000, B + 0x4000, 1024),
                             ma.Tensor(C, C + 0x1000, B + 0x1800, C + 0x3000, C + 0x4000, 1024))
    assert prep(across, 2, ma.MA_BF16, ma.MA_BF16, A, 224, None, ctypes.byref(plan)) == ma.MA_ERR_ARG
    assert b"tensor 0" in ma.lib.ma_last_error() and b"tensor 1" in ma.lib.ma_last_error()
    # accumulation
    assert ma.lib.ma_grad_accumulate(B, B + 2048, ma.MA_BF16, 1024, 1, None) == ma.MA_ERR_ARG
    assert b"overlap" in ma.lib.ma_last_error()


def test_probe_argument_errors():
    f, g = ma.lib.ma_probe_update_mix, ma.lib.ma_probe_two_writes
    assert f(A, A, A, A, A, 1 << 20, 3, None) == ma.MA_ERR_ARG
    assert f(A, A, None, A, A, 1 << 20, 4, None) == ma.MA_ERR_NULL
    assert f(A, A, A, A, None, 1 << 20, 4, None) == ma.MA_ERR_NULL          # the 16-bit output is needed with 4-byte states
    assert f(A, A + 4, A, A, A, 1 << 20, 4, None) == ma.MA_ERR_ALIGN
    assert f(A, A, A, A, A, 100, 4, None) == ma.MA_ERR_ARG
    assert g(A, None, 1 << 20, None) == ma.MA_ERR_NULL
    assert g(A, A + 8, 1 << 20, None) == ma.MA_ERR_ALIGN
    assert g(A, A, 1024, None) == ma.MA_ERR_ARG


def test_arena_argument_errors():
    """ma_arena_create turns down what it cannot build before it touches the device."""
    f = ma.lib.ma_arena_create
    h = ctypes.c_void_p()
    GIB = 1 << 30
    assert f(GIB, GIB // 2, 0, 0, 0, None) == ma.MA_ERR_NULL
    assert f(0, 0, 0, 0, 0, ctypes.byref(h)) == ma.MA_ERR_ARG
    assert f(GIB, 2 * GIB, 0, 0, 0, ctypes.byref(h)) == ma.MA_ERR_ARG and b"first_region_bytes" in ma.lib.ma_last_error()
    assert f(GIB, 0, 0, 3 << 20, 0, ctypes.byref(h)) == ma.MA_ERR_ARG          # block below 64 MiB
    assert f(GIB, 0, 0, (64 << 20) + 4096, 0, ctypes.byref(h)) == ma.MA_ERR_ARG  # not a multiple of 2 MiB
    assert h.value is None
    assert ma.lib.ma_arena_destroy(None) == ma.MA_OK
    assert ma.lib.ma_arena_main(None) is None and ma.lib.ma_arena_side(None) is None
    assert ma.lib.ma_arena_get_report(None, None) == ma.MA_ERR_NULL
