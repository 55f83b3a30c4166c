"""GPU parity at the edges: the fp32-subnormal range (denormals are preserved on both sides, so the
match is bit for bit) and the device-side bias corrections over thousands of update numbers."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_23254_amd import synth
from tests.test_abi import SWEEP_BETAS, sweep_steps

pytestmark = pytest.mark.gpu

ma = None


@pytest.fixture(scope="module", autouse=True)
def _lib():
    global ma
    from paper_2505_23254_amd import binding
    ma = binding
    assert torch.cuda.is_available()
    yield


def _dev16(bits, gdt):
    t = torch.from_numpy(bits.view(np.int16).copy()).cuda()
    return t.view(torch.bfloat16 if gdt == "bf16" else torch.float16)


def _bits(t):
    return t.detach().cpu().contiguous().view(torch.int32 if t.element_size() == 4 else torch.int16).numpy()


def _equal_bits(name, got, ref, what):
    a, b = _bits(got), ref.view(np.int32 if ref.itemsize == 4 else np.int16)
    bad = np.nonzero(a != b)[0]
    assert bad.size == 0, "%s %s: %d of %d differ, first at %d: gpu %#x oracle %#x" % (
        what, name, bad.size, a.size, bad[0], int(a[bad[0]]) & 0xFFFFFFFF, int(b[bad[0]]) & 0xFFFFFFFF)


@pytest.mark.parametrize("pdt", ["bf16", "f16"])
@pytest.mark.parametrize("case", synth.EXTREME_CASES)
def test_flat_step_in_the_subnormal_range_is_bit_exact(case, pdt):
    """v, g * gscale, m (and for one case eps and the whole denominator) in the fp32-subnormal range,
    fp16-subnormal gradients at loss scale 1: scan, then the update, against the oracle bit for bit."""
    n = 50_003                                             # several work items and a ragged tail
    p, m, v, g, gdt, scale, clip, eps = synth.extreme_case(case, n)
    h_ref = oracle.hyper(1e-3, 0.9, 0.999, eps, 0.1, 1)
    h = ma.hyper(1e-3, 0.9, 0.999, eps, 0.1, 1)
    dp, dm, dv = (torch.from_numpy(x.copy()).cuda() for x in (p, m, v))
    dg = _dev16(g, gdt)
    dlp = torch.zeros(n, dtype=torch.bfloat16 if pdt == "bf16" else torch.float16, device="cuda")
    ov_ref, ss_ref = oracle.overflow_norm(g, gdt, scale)
    lp = oracle.adamw_step(p, m, v, g, gdt, pdt, h_ref, 7, scale, clip)
    ws, res = ma.workspace(), ma.new_result()
    ma.overflow_norm(dg, scale, res, ws)
    ma.adamw_step(dp, dm, dv, dg, dlp, h, 7, scale, clip)
    ov, ss = ma.read_result(res)
    assert ov == ov_ref == False
    assert ss_ref > 0 and abs(ss - ss_ref) <= 1e-12 * ss_ref       # fp64 on both sides: tiny squares survive
    for name, got, ref in (("p", dp, p), ("m", dm, m), ("v", dv, v), ("p_lp", dlp, lp)):
        _equal_bits(name, got, ref, case)
    if case == "subnormal":                                         # the new moments really are subnormal
        tiny = float(np.finfo(np.float32).tiny)
        for x in (m, v):
            assert np.count_nonzero((np.abs(x) < tiny) & (x != 0)) > n // 2


@pytest.mark.parametrize("case", ["subnormal", "subnormal_eps", "f16_subnormal_grads"])
def test_list_step_in_the_subnormal_range_is_bit_exact(case):
    """The same ranges through the tensor-list kernels: ragged tensors packed back to back (most of
    them misaligned), one scan and one gated update launch; the gate passes (tiny norm, no clip)."""
    sizes = [4099, 1, 12_288, 70_001, 5, 33_000, 8191]
    n = sum(sizes)
    p, m, v, g, gdt, scale, _, eps = synth.extreme_case(case, n, seed=1)
    h_ref, h = oracle.hyper(1e-3, 0.9, 0.999, eps, 0.1, 1), ma.hyper(1e-3, 0.9, 0.999, eps, 0.1, 1)
    dp, dm, dv = (torch.from_numpy(x.copy()).cuda() for x in (p, m, v))
    dg, dlp = _dev16(g, gdt), torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    offs = np.concatenate([[0], np.cumsum(sizes)])
    cut = lambda t: [t[a:b] for a, b in zip(offs[:-1], offs[1:])]
    plan = ma.MultiPlan(cut(dp), cut(dm), cut(dv), cut(dg), cut(dlp))
    lp = np.zeros(n, np.uint16)
    ov_ref, ss_ref, c_ref = oracle.optimizer_step(p, m, v, g, gdt, lp, "bf16", h_ref, 3, scale, 1.0)
    assert not ov_ref and c_ref == 1.0
    ws, res = ma.workspace(), ma.new_result()
    ma.multi_overflow_norm(plan, scale, res, ws)
    ma.multi_adamw_step_gated(plan, h, 3, scale, res, 1.0)
    ov, ss = ma.read_result(res)
    assert not ov and abs(ss - ss_ref) <= 1e-12 * ss_ref
    for name, got, ref in (("p", dp, p), ("m", dm, m), ("v", dv, v), ("p_lp", dlp, lp)):
        _equal_bits(name, got, ref, case)


def test_bf16_state_step_in_the_subnormal_range_is_bit_exact():
    """States held in bf16 and stored by truncation, with subnormal patterns in p, m, v and g."""
    n = 70_001                                             # several 16,384-element work items and a ragged tail
    p, m, v, g, gdt, scale, clip, eps = synth.extreme_case("subnormal", n, seed=2)
    bp, bm, bv = ((x.view(np.uint32) >> 16).astype(np.uint16) for x in (p, m, v))      # inputs: upper halves
    h_ref, h = oracle.hyper(1e-3, 0.9, 0.999, eps, 0.1, 1), ma.hyper(1e-3, 0.9, 0.999, eps, 0.1, 1)
    dp, dm, dv, dg = (_dev16(x, "bf16") for x in (bp, bm, bv, g))
    oracle.adamw_step_bf16(bp, bm, bv, g, gdt, h_ref, 5, scale, clip)
    ma.adamw_step_bf16(dp, dm, dv, dg, h, 5, scale, clip)
    for name, got, ref in (("p", dp, bp), ("m", dm, bm), ("v", dv, bv)):
        _equal_bits(name, got, ref, "bf16 states")
    assert np.count_nonzero(((bm & 0x7F80) == 0) & ((bm & 0x7F) != 0)) > n // 4


def test_device_side_bias_corrections_over_a_sweep_of_update_numbers():
    """ma_adamw_step_auto derives lr / (1 - beta1^t) and 1 / sqrt(1 - beta2^t) on the device from the
    update number in device memory.  Sweep: thousands of t (1, 2, the decades up to 10^6 and their
    neighbours, seeded draws between) x three (beta1, beta2) pairs, 64 elements each, against the
    oracle (library pow on the host) bit for bit.  Half of the elements have p = 0 and no decay term, so
    that p' is the single rounded product -step_size * u: a change of step_size or of the second
    scalar (through the denominator) by one unit in the last place shows in several elements."""
    steps = sweep_steps()
    n = 64
    rng = np.random.default_rng(77)
    p0 = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    p0[::2] = 0.0
    m0 = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    v0 = (rng.standard_normal(n) ** 2 * 1e-4).astype(np.float32)
    g = synth.bits16(torch.from_numpy((rng.standard_normal(n) * 1e-2).astype(np.float32)).to(torch.bfloat16))
    dg = _dev16(g, "bf16")
    d0 = [torch.from_numpy(x).cuda() for x in (p0, m0, v0)]
    dp, dm, dv = (torch.empty_like(x) for x in d0)
    dlp = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    ws, res = ma.workspace(), ma.new_result()
    ma.overflow_norm(dg, 1.0, res, ws)                     # clean gate; max_norm 0: no clipping
    scaler = ma.new_scaler(1.0, 0)
    out = torch.empty(len(steps), 3, n, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    # sensitivity of the check itself, shown on the oracle: lr one unit in the last place larger moves
    # step_size by about one unit, and the outputs notice
    ha, hb = oracle.hyper(1e-3, 0.9, 0.999, 1e-8, 0.0, 1), oracle.hyper(float(np.nextafter(np.float32(1e-3), np.float32(1))), 0.9, 0.999, 1e-8, 0.0, 1)
    pa, pb = p0.copy(), p0.copy()
    oracle.adamw_step(pa, m0.copy(), v0.copy(), g, "bf16", "bf16", ha, 1000)
    oracle.adamw_step(pb, m0.copy(), v0.copy(), g, "bf16", "bf16", hb, 1000)
    assert np.count_nonzero(pa != pb) >= 8
    for b1, b2 in SWEEP_BETAS:
        h, h_ref = ma.hyper(1e-3, b1, b2, 1e-8, 0.0, 1), oracle.hyper(1e-3, b1, b2, 1e-8, 0.0, 1)
        for k, t in enumerate(steps):
            for dst, src in zip((dp, dm, dv), d0):
                dst.copy_(src)
            ma._check(ma.lib.ma_scaler_init(scaler.data_ptr(), 1.0, t - 1, stream))
            ma.adamw_step_auto(dp, dm, dv, dg, dlp, h, scaler, res, 0.0)
            out[k, 0].copy_(dp)
            out[k, 1].copy_(dm)
            out[k, 2].copy_(dv)
        got = out.cpu().numpy()
        for k, t in enumerate(steps):
            p, m, v = p0.copy(), m0.copy(), v0.copy()
            oracle.adamw_step(p, m, v, g, "bf16", "bf16", h_ref, t)
            for name, a, b in (("p", got[k, 0], p), ("m", got[k, 1], m), ("v", got[k, 2], v)):
                assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), (b1, b2, t, name)
