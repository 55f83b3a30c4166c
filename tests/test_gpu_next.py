"""GPU parity for the rows beyond the basic step: gradient accumulation into the fp32 flat buffer
(Sec. III-C), the step with bf16 states stored by truncation (Extended Experiments, bf16
half-precision optimizer) and the dynamic loss scale kept on the device (Sec. III-C).  Same bar as
the basic step: integer / bit-pattern results exact, fp32 within 2 ulp, sumsq within 1e-5."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_23254_amd import synth
from tests._util import (MAX_ULP, SUMSQ_RTOL, assert_state_close, host_f32, host_grad, oracle_hyper,
                         ulp_distance)
from tests.test_oracle_next import _parse_cases

pytestmark = pytest.mark.gpu

ma = None
TORCH_DT = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}


@pytest.fixture(scope="module", autouse=True)
def _lib():
    global ma
    from paper_2505_23254_amd import binding
    ma = binding
    assert torch.cuda.is_available()
    yield


def _hyper(cfg):
    return ma.hyper(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, cfg.weight_decay, 1)


def _host_state(st, pdt="bf16"):
    return dict(p=host_f32(st.p), m=host_f32(st.m), v=host_f32(st.v), lp=synth.bits16(st.p_lp), pdt=pdt)


def _micro_grad(n, seed, gdt, scale, device="cuda"):
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    x = torch.empty(n, dtype=torch.float32, device=device).normal_(0.0, 1e-3, generator=gen) * scale
    return x.to(TORCH_DT[gdt])


# ---- gradient accumulation --------------------------------------------------------------------------

ACC_SIZES = [0, 1, 3, 4, 5, 1023, 1024, 4095, 4096, 4097, 8191, 8192, 8193, 12287, 12288, 12289, 16385, 100_003,
             (1 << 20) + 7]


@pytest.mark.parametrize("gdt", ["bf16", "f16", "f32"])
def test_accumulate_micro_batches(gdt):
    """Four micro-batches into the fp32 flat buffer: bit-identical to the oracle after each one
    (one IEEE fp32 addition per element); the first call overwrites whatever the buffer held."""
    for n in ACC_SIZES:
        acc = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
        ref = np.full(n, np.nan, np.float32)
        for k in range(4):
            g = _micro_grad(n, 1000 + 13 * k + n % 11, gdt, 64.0)
            g_host = host_grad(g)
            oracle.grad_accumulate(ref, g_host, gdt, first=(k == 0))
            ma.grad_accumulate(acc, g, first=(k == 0))
            assert np.array_equal(host_f32(acc).view(np.uint32), ref.view(np.uint32)), (n, k)
            assert np.array_equal(host_grad(g), g_host)


@pytest.mark.parametrize("off_acc,off_g", [(1, 1), (3, 3), (1, 2), (0, 1), (2, 0), (0, 4)])
def test_accumulate_misaligned(off_acc, off_g):
    n = 20_011
    base = torch.zeros(n + 8, dtype=torch.float32, device="cuda")
    gbase = _micro_grad(n + 8, 5, "bf16", 1.0)
    acc, g = base[off_acc:off_acc + n], gbase[off_g:off_g + n]
    ref = np.zeros(n, np.float32)
    for k in range(3):
        oracle.grad_accumulate(ref, host_grad(g), "bf16", first=False)
        ma.grad_accumulate(acc, g, first=False)
    assert np.array_equal(host_f32(acc).view(np.uint32), ref.view(np.uint32))
    full = host_f32(base)
    assert not full[:off_acc].any() and not full[off_acc + n:].any()      # nothing outside the view


def test_accumulated_fp32_buffer_feeds_scan_and_step():
    """The whole chain of Sec. III-C / IV-A: accumulate fp16 micro-batches into the fp32 buffer,
    scan it with Algorithm 1's fp32 mask fused with the norm, gate, update."""
    n, S, micro = 250_003, 4096.0, 3
    cfg = synth.FlatConfig("t", n, seed=17, m_std=1e-4, v_std=1e-8, step=9, max_norm=0.02)
    st = synth.make_flat(cfg, device="cuda")
    ref = _host_state(st)
    acc = torch.empty(n, dtype=torch.float32, device="cuda")
    acc_ref = np.empty(n, np.float32)
    for k in range(micro):
        g = _micro_grad(n, 300 + k, "f16", S)
        oracle.grad_accumulate(acc_ref, host_grad(g), "f16", first=(k == 0))
        ma.grad_accumulate(acc, g, first=(k == 0))
    ov_ref, ss_ref, c_ref = oracle.optimizer_step(ref["p"], ref["m"], ref["v"], acc_ref, "f32",
                                                  ref["lp"], "bf16", oracle_hyper(cfg), 9, S, cfg.max_norm)
    ws, res = ma.workspace(), ma.new_result(2)
    ma.overflow_norm(acc, S, res, ws)
    ma.adamw_step_gated(st.p, st.m, st.v, acc, st.p_lp, _hyper(cfg), 9, S, res, cfg.max_norm)
    ov, ss = ma.read_result(res)
    assert not ov and not ov_ref and c_ref < 1
    assert abs(ss - ss_ref) <= SUMSQ_RTOL * ss_ref and abs(ss - ss_ref) <= 1e-12 * ss_ref
    assert_state_close(_host_state(st), ref, "accumulated")
    # two fp16 values that are finite on their own but overflow the fp32 sum cannot exist (fp16
    # max is 65504), so an overflow enters the buffer only through an inf/NaN micro-batch entry:
    g = _micro_grad(n, 999, "f16", S)
    g.view(torch.int16)[n - 3] = 0x7C00
    ma.grad_accumulate(acc, g, first=False)
    ma.overflow_norm(acc, S, res, ws, index=1)
    assert ma.read_result(res, 1)[0] is True


# ---- bf16 optimizer states stored by truncation --------------------------------------------------------

def _bf16_state(cfg, n):
    """p, m, v as bf16 device tensors (truncated views of the fp32 synthetic state) + host copies."""
    st = synth.make_flat(cfg, device="cuda", n=n)
    shift = lambda t: (t.view(torch.int32) >> 16).to(torch.int16).view(torch.bfloat16).contiguous()
    p, m, v = shift(st.p), shift(st.m), shift(st.v)
    return st, p, m, v


# a work item of this variant is 16,384 elements (256 lanes x 8 groups x 8 elements)
BF_SIZES = [0, 1, 3, 4, 5, 7, 8, 9, 15, 16, 17, 1023, 1024, 4096, 4097, 8191, 8192, 8193, 12287, 12288, 12289, 16383,
            16384, 16385, 24577, 32767, 32768, 32769, 49153, 100_003, (1 << 20) + 5]


@pytest.mark.parametrize("gdt,scale,clip", [("bf16", 1.0, 1.0), ("bf16", 1.0, 0.3), ("f16", 1024.0, 0.5),
                                            ("f32", 8.0, 0.7)])
def test_bf16_state_step_sizes(gdt, scale, clip):
    for n in BF_SIZES:
        cfg = synth.FlatConfig("t", n, seed=200 + n % 89, gdt="bf16" if gdt == "f32" else gdt,
                               loss_scale=scale, m_std=1e-3, v_std=1e-6, step=7, lr=1e-2, weight_decay=0.1,
                               eps=1e-6)
        st, p, m, v = _bf16_state(cfg, n)
        if gdt == "f32":                  # fp32 gradients: the accumulated flat buffer as input
            st.g = st.g.to(torch.float32) * 1.0001
        g_host = host_grad(st.g)
        rp, rm, rv = synth.bits16(p), synth.bits16(m), synth.bits16(v)
        moved_from = rp.copy()
        oracle.adamw_step_bf16(rp, rm, rv, g_host, gdt, oracle_hyper(cfg), 7, scale, clip)
        ma.adamw_step_bf16(p, m, v, st.g, _hyper(cfg), 7, scale, clip)
        # fp32 arithmetic agrees bit for bit, hence so do the truncated patterns
        assert np.array_equal(synth.bits16(p), rp), n
        assert np.array_equal(synth.bits16(m), rm), n
        assert np.array_equal(synth.bits16(v), rv), n
        assert np.array_equal(host_grad(st.g), g_host)
        if n > 1000:
            assert (rp != moved_from).mean() > 0.5      # the step is large enough to be visible in bf16


def test_bf16_state_step_gated_and_skip():
    n = 70_003
    cfg = synth.FlatConfig("t", n, seed=23, m_std=1e-3, v_std=1e-6, step=4, lr=1e-2, max_norm=0.05)
    st, p, m, v = _bf16_state(cfg, n)
    g_host = host_grad(st.g)
    rp, rm, rv = synth.bits16(p), synth.bits16(m), synth.bits16(v)
    ov_ref, ss_ref = oracle.overflow_norm(g_host, "bf16")
    c_ref = oracle.clip_coef(ss_ref, float(np.float32(cfg.max_norm)))
    assert not ov_ref and c_ref < 1
    oracle.adamw_step_bf16(rp, rm, rv, g_host, "bf16", oracle_hyper(cfg), 4, 1.0, float(c_ref))
    ws, res = ma.workspace(), ma.new_result()
    ma.overflow_norm(st.g, 1.0, res, ws)
    ma.adamw_step_bf16_gated(p, m, v, st.g, _hyper(cfg), 4, 1.0, res, cfg.max_norm)
    assert np.array_equal(synth.bits16(p), rp) and np.array_equal(synth.bits16(m), rm)
    assert np.array_equal(synth.bits16(v), rv)
    # overflow: untouched
    st.g.view(torch.int16)[n // 3] = 0x7F80
    ma.overflow_norm(st.g, 1.0, res, ws)
    ma.adamw_step_bf16_gated(p, m, v, st.g, _hyper(cfg), 5, 1.0, res, cfg.max_norm)
    assert ma.read_result(res)[0] is True
    assert np.array_equal(synth.bits16(p), rp) and np.array_equal(synth.bits16(m), rm)
    assert np.array_equal(synth.bits16(v), rv)


def test_bf16_state_misaligned():
    n = 30_001
    cfg = synth.FlatConfig("t", n + 16, seed=29, m_std=1e-3, v_std=1e-6, step=2, lr=1e-2)
    st, P, M, V = _bf16_state(cfg, n + 16)
    for offs in [(1, 1, 1, 1), (3, 3, 3, 3), (1, 2, 3, 0), (0, 0, 0, 2), (4, 4, 4, 4), (7, 7, 7, 7), (8, 8, 8, 8),
                 (5, 5, 5, 1), (0, 0, 0, 4), (8, 0, 0, 0)]:
        p, m, v, g = (t[o:o + n] for t, o in zip((P, M, V, st.g), offs))
        rp, rm, rv = synth.bits16(p), synth.bits16(m), synth.bits16(v)
        edges = [synth.bits16(t) for t in (P, M, V)]
        oracle.adamw_step_bf16(rp, rm, rv, host_grad(g), "bf16", oracle_hyper(cfg), 2, 1.0, 1.0)
        ma.adamw_step_bf16(p, m, v, g, _hyper(cfg), 2)
        for t, r, full, e, o in zip((p, m, v), (rp, rm, rv), (P, M, V), edges, offs):
            assert np.array_equal(synth.bits16(t), r), offs
            now = synth.bits16(full)
            assert np.array_equal(now[:o], e[:o]) and np.array_equal(now[o + n:], e[o + n:])


def test_truncation_of_special_values():
    """Patterns whose truncation is delicate: largest finite stays finite (no rounding up to inf),
    inf stays inf, NaN with payload only in the dropped half stays NaN.  With lr = 0, beta1 = 0 and a
    gradient chosen so that m' = g exactly, m carries fp32 values we control into the store."""
    # m' = 0*m + 1*g with fp32 gradients: any fp32 pattern reaches the truncating store of m
    pats = np.array([0x3F80FFFF, 0xBF80FFFF, 0x7F7FFFFF, 0x0001FFFF, 0x00008000, 0x7F800000,
                     0xFF800000, 0x7F800001, 0xFFC12345, 0x80000000, 0x3F808000], np.uint32)
    n = pats.size
    g = torch.from_numpy(pats.view(np.float32).copy()).cuda()
    z = lambda: torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    p, m, v = z(), z(), z()
    h = ma.hyper(lr=0.0, beta1=0.0, beta2=0.0, weight_decay=0.0)
    ma.adamw_step_bf16(p, m, v, g, h, 1)
    got = synth.bits16(m)
    want = oracle.truncate_bf16(pats.view(np.float32).copy())
    nan = np.isnan(pats.view(np.float32)) | (pats == 0x80000000)      # (+0) + (-0) = +0, not g
    is_nan16 = lambda b: ((b & 0x7F80) == 0x7F80) & ((b & 0x007F) != 0)
    assert np.array_equal(got[~nan], want[~nan])
    really_nan = np.isnan(pats.view(np.float32))
    assert np.all(is_nan16(got[really_nan])) and np.all(is_nan16(want[really_nan]))
    rp, rm, rv = (np.zeros(n, np.uint16) for _ in range(3))
    oracle.adamw_step_bf16(rp, rm, rv, pats.view(np.float32).copy(), "f32",
                           oracle.hyper(lr=0.0, beta1=0.0, beta2=0.0, weight_decay=0.0), 1)
    # NaNs produced by the arithmetic itself (inf/inf, 0*inf) may differ in sign and payload between
    # the two machines; their class may not
    for dev, ref in ((m, rm), (v, rv), (p, rp)):
        d = synth.bits16(dev)
        dn = is_nan16(d)
        assert np.array_equal(dn, is_nan16(ref))
        assert np.array_equal(d[~dn], ref[~dn])


# ---- dynamic loss scale on the device ------------------------------------------------------------------

def _set_gate(res, overflow, sumsq=1.0):
    raw = np.zeros(2, np.float64)
    raw.view(np.int32)[0] = int(overflow)
    raw[1] = sumsq
    res.copy_(torch.from_numpy(raw))


def test_scaler_policy_hand_worked_sequences(golden_dir):
    for c in _parse_cases(golden_dir + "/loss_scale_sequence.txt"):
        st = ma.new_scaler(c["scale0"])
        cfg = ma.scaler_config(*c["cfg"])
        res = ma.new_result()
        assert ma.read_scaler(st) == (c["scale0"], 0, 0, 0)
        for flag, scale, good, step, skipped in c["rows"]:
            _set_gate(res, flag)
            ma.scaler_update(st, res, cfg)
            assert ma.read_scaler(st) == (scale, good, step, skipped), (c["name"], flag)


@pytest.mark.parametrize("gdt", ["f16", "bf16"])
def test_auto_iterations_track_the_oracle(gdt):
    """Twelve iterations driven entirely from device state (scale, update number, gate): planted
    overflows skip and halve the scale, clean steps apply update number step+1 with the bias
    corrections evaluated on the device, growth after three clean steps.  No host round trip is
    needed between the calls of an iteration; the test reads back only to compare."""
    n = 60_001
    S0 = 2048.0
    cfg = synth.FlatConfig("t", n, seed=31, gdt=gdt, m_std=1e-4, v_std=1e-8, max_norm=0.02)
    st = synth.make_flat(cfg, device="cuda")
    ref = _host_state(st)
    h_ref, h = oracle_hyper(cfg), _hyper(cfg)
    state_ref, cfg_ref = oracle.scaler_state(scale=S0, step=41), oracle.scaler_cfg(window=3)
    scaler, scfg = ma.new_scaler(S0, 41), ma.scaler_config(window=3)
    ws, res = ma.workspace(), ma.new_result()
    bad_iters = {1, 2, 7}
    for it in range(12):
        scale_now = state_ref.scale
        g = _micro_grad(n, 400 + it, gdt, scale_now)
        if it in bad_iters:
            bits = synth.NONFINITE_BITS[gdt][it % 5]
            g.view(torch.int16)[(it * 7919) % n] = bits - 0x10000 if bits >= 0x8000 else bits
        g_host = host_grad(g)
        ov_ref, ss_ref = oracle.optimizer_step_auto(ref["p"], ref["m"], ref["v"], g_host, gdt, ref["lp"],
                                                    "bf16", h_ref, state_ref, cfg_ref, cfg.max_norm)
        ma.overflow_norm_auto(g, scaler, res, ws)
        ma.adamw_step_auto(st.p, st.m, st.v, g, st.p_lp, h, scaler, res, cfg.max_norm)
        ma.scaler_update(scaler, res, scfg)
        ov, ss = ma.read_result(res)
        assert ov == ov_ref == (it in bad_iters), it
        if not ov:
            assert abs(ss - ss_ref) <= SUMSQ_RTOL * ss_ref and abs(ss - ss_ref) <= 1e-12 * ss_ref
        assert ma.read_scaler(scaler) == (state_ref.scale, state_ref.good_steps, state_ref.step,
                                          state_ref.skipped), it
        assert_state_close(_host_state(st), ref, "iteration %d" % it)
    assert state_ref.skipped == 3 and state_ref.step == 41 + 9


def test_auto_long_trajectory_without_host_round_trips():
    """300 iterations enqueued back to back with no synchronisation in between: scale, update number and
    gate live on the device the whole time.  Overflows are planted at fixed iterations, so the oracle's
    trajectory (run first) tells which scale each iteration's gradient carries; at the end the state,
    the scale, the counters and the last result equal the oracle's.  The scale grows (window 4) until
    the fp16 gradients overflow by themselves, falls, and grows again, many times."""
    n, iters = 20_011, 300
    S0 = 4096.0
    cfg = synth.FlatConfig("t", n, seed=131, gdt="f16", m_std=1e-4, v_std=1e-8, max_norm=0.05)
    st = synth.make_flat(cfg, device="cuda")
    ref = _host_state(st)
    h_ref, h = oracle_hyper(cfg), _hyper(cfg)
    state_ref, cfg_ref = oracle.scaler_state(scale=S0, step=0), oracle.scaler_cfg(window=4)
    bad = {it for it in range(iters) if it % 23 == 5 or it % 57 == 11}
    base = _micro_grad(n, 977, "f16", 1.0).to(torch.float32)                  # one direction, re-scaled per iteration
    grads, last = [], None
    for it in range(iters):
        g = (base * (state_ref.scale * (1.0 + 0.01 * (it % 7)))).to(torch.float16)
        if it in bad:
            g.view(torch.int16)[(it * 7919) % n] = 0x7C00                        # +inf
        grads.append(g)
        last = oracle.optimizer_step_auto(ref["p"], ref["m"], ref["v"], host_grad(g), "f16", ref["lp"], "bf16",
                                          h_ref, state_ref, cfg_ref, cfg.max_norm)
    # besides the planted ones the growing scale runs into the fp16 range on its own, as in training
    assert state_ref.skipped > len(bad) and state_ref.step == iters - state_ref.skipped and state_ref.step > 200
    scaler, scfg = ma.new_scaler(S0, 0), ma.scaler_config(window=4)
    ws, res = ma.workspace(), ma.new_result()
    torch.cuda.synchronize()
    for it in range(iters):                                                     # nothing below waits for the device
        ma.overflow_norm_auto(grads[it], scaler, res, ws)
        ma.adamw_step_auto(st.p, st.m, st.v, grads[it], st.p_lp, h, scaler, res, cfg.max_norm)
        ma.scaler_update(scaler, res, scfg)
    ov, ss = ma.read_result(res)
    assert ov == last[0] and (ov or abs(ss - last[1]) <= 1e-12 * last[1])
    assert ma.read_scaler(scaler) == (state_ref.scale, state_ref.good_steps, state_ref.step, state_ref.skipped)
    got = _host_state(st)
    assert_state_close(got, ref, "after %d iterations" % iters)
    for k in ("p", "m", "v"):
        assert np.array_equal(got[k].view(np.uint32), ref[k].view(np.uint32)), k


def test_auto_equals_host_driven_gated_step():
    """The device-evaluated bias corrections equal the host's: an auto step is bit-identical to the
    gated step given the same scale and update number, at small and large update numbers."""
    n = 33_333
    for applied in (0, 1, 99, 9_999, 1_000_000):
        cfg = synth.FlatConfig("t", n, seed=37, gdt="f16", loss_scale=512.0, m_std=1e-4, v_std=1e-8,
                               max_norm=0.03)
        a = synth.make_flat(cfg, device="cuda")
        b = synth.make_flat(cfg, device="cuda")
        ws, res = ma.workspace(), ma.new_result()
        scaler = ma.new_scaler(512.0, applied)
        ma.overflow_norm_auto(a.g, scaler, res, ws)
        ma.adamw_step_auto(a.p, a.m, a.v, a.g, a.p_lp, _hyper(cfg), scaler, res, cfg.max_norm)
        ra = ma.read_result(res)
        ma.overflow_norm(b.g, 512.0, res, ws)
        ma.adamw_step_gated(b.p, b.m, b.v, b.g, b.p_lp, _hyper(cfg), applied + 1, 512.0, res, cfg.max_norm)
        assert ra == ma.read_result(res)
        for x, y in ((a.p, b.p), (a.m, b.m), (a.v, b.v)):
            assert ulp_distance(host_f32(x), host_f32(y)).max() <= MAX_ULP
            assert host_f32(x).tobytes() == host_f32(y).tobytes(), applied
        assert synth.bits16(a.p_lp).tobytes() == synth.bits16(b.p_lp).tobytes()


def test_multi_auto_iteration():
    shapes = synth.scaled_shapes(synth.llama3_8b_shapes(), 16384, ragged=True)
    cfg = synth.FlatConfig("t", 0, seed=43, gdt="f16", loss_scale=256.0, m_std=1e-4, v_std=1e-8,
                           max_norm=0.05)
    ls = synth.make_list(shapes, cfg, device="cuda")
    fl = ls.flat
    ref = dict(p=host_f32(fl.p), m=host_f32(fl.m), v=host_f32(fl.v), lp=synth.bits16(fl.p_lp), pdt="bf16")
    plan = ma.MultiPlan(ls.p, ls.m, ls.v, ls.g, ls.p_lp)
    scaler, scfg = ma.new_scaler(256.0, 10), ma.scaler_config(window=100)
    state_ref, cfg_ref = oracle.scaler_state(scale=256.0, step=10), oracle.scaler_cfg(window=100)
    ws, res = ma.workspace(), ma.new_result()
    # the oracle walks the tensors of the list; padding between tensors belongs to no tensor
    ss_ref = 0.0
    for g in ls.g:
        ov, ss = oracle.overflow_norm(host_grad(g), "f16", 256.0)
        assert not ov
        ss_ref += ss
    c_ref = oracle.clip_coef(ss_ref, float(np.float32(cfg.max_norm)))
    refs = []
    for i in range(len(shapes)):
        r = dict(p=host_f32(ls.p[i]), m=host_f32(ls.m[i]), v=host_f32(ls.v[i]), pdt="bf16")
        r["lp"] = oracle.adamw_step(r["p"], r["m"], r["v"], host_grad(ls.g[i]), "f16", "bf16",
                                    oracle_hyper(cfg), 11, 256.0, float(c_ref))
        refs.append(r)
    oracle.scaler_update(state_ref, cfg_ref, 0)
    ma.multi_overflow_norm_auto(plan, scaler, res, ws)
    ma.multi_adamw_step_auto(plan, _hyper(cfg), scaler, res, cfg.max_norm)
    ma.scaler_update(scaler, res, scfg)
    ov, ss = ma.read_result(res)
    assert not ov and abs(ss - ss_ref) <= 1e-12 * ss_ref
    assert ma.read_scaler(scaler) == (256.0, 1, 11, 0)
    for i in range(len(shapes)):
        got = dict(p=host_f32(ls.p[i]), m=host_f32(ls.m[i]), v=host_f32(ls.v[i]), lp=synth.bits16(ls.p_lp[i]))
        assert_state_close(got, refs[i], "tensor %d" % i)
    # an overflow skips the list and halves the scale
    before = host_f32(fl.p).tobytes()
    ls.g[3].view(torch.int16)[1] = 0x7E00
    ma.multi_overflow_norm_auto(plan, scaler, res, ws)
    ma.multi_adamw_step_auto(plan, _hyper(cfg), scaler, res, cfg.max_norm)
    ma.scaler_update(scaler, res, scfg)
    assert ma.read_result(res)[0] is True
    assert ma.read_scaler(scaler) == (128.0, 0, 11, 1)
    assert host_f32(fl.p).tobytes() == before


# ---- the whole iteration as one captured graph ----------------------------------------------------------

def test_auto_iteration_replays_as_a_graph():
    """Scan, gated update and loss-scale update read everything that changes from iteration to
    iteration (scale, update number, gate) from device memory, so ONE captured graph serves every
    iteration.  Replays are interleaved with eager work and synchronisations, include a skipped
    iteration, and are checked against the oracle after every replay."""
    n = 150_001
    S0 = 1024.0
    cfg = synth.FlatConfig("t", n, seed=91, gdt="f16", m_std=1e-4, v_std=1e-8, max_norm=0.05)
    st = synth.make_flat(cfg, device="cuda")
    ref = _host_state(st)
    h_ref, h = oracle_hyper(cfg), _hyper(cfg)
    state_ref, cfg_ref = oracle.scaler_state(scale=S0, step=7), oracle.scaler_cfg(window=2)
    scaler, scfg = ma.new_scaler(S0, 7), ma.scaler_config(window=2)
    ws, res = ma.workspace(), ma.new_result()
    g_in = torch.zeros(n, dtype=torch.float16, device="cuda")     # the graph reads its gradient here

    def iteration():
        ma.overflow_norm_auto(g_in, scaler, res, ws)
        ma.adamw_step_auto(st.p, st.m, st.v, g_in, st.p_lp, h, scaler, res, cfg.max_norm)
        ma.scaler_update(scaler, res, scfg)

    # one eager iteration first (also initialises everything the library caches per process)
    def feed(it, bad):
        g = _micro_grad(n, 700 + it, "f16", state_ref.scale)
        if bad:
            g.view(torch.int16)[it * 31 % n] = 0x7C00
        g_in.copy_(g)
        return host_grad(g)

    def check(it, g_host, expect_overflow):
        ov_ref, ss_ref = oracle.optimizer_step_auto(ref["p"], ref["m"], ref["v"], g_host, "f16", ref["lp"],
                                                    "bf16", h_ref, state_ref, cfg_ref, cfg.max_norm)
        torch.cuda.synchronize()
        ov, ss = ma.read_result(res)
        assert ov == ov_ref == expect_overflow, it
        if not ov:
            assert abs(ss - ss_ref) <= 1e-12 * ss_ref
        assert ma.read_scaler(scaler) == (state_ref.scale, state_ref.good_steps, state_ref.step,
                                          state_ref.skipped), it
        assert_state_close(_host_state(st), ref, "graph iteration %d" % it)

    gh = feed(0, False)
    iteration()
    check(0, gh, False)

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    gh = feed(1, False)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        iteration()
    torch.cuda.synchronize()
    # capturing does not execute: the state is still that of iteration 0
    assert ma.read_scaler(scaler)[2] == 8
    for it in range(1, 9):
        bad = it in (3, 6)
        gh = feed(it, bad)
        graph.replay()
        check(it, gh, bad)
        # eager work of the program between replays
        _ = (st.p[:1000] * 2).sum().item()
    assert state_ref.skipped == 2


def test_list_iteration_replays_as_a_graph():
    """The same for a tensor list (about 1000 work items): ONE captured graph serves every iteration,
    skipped ones included, and the counters at the head of the plan's table read zero after every
    replay."""
    shapes = synth.scaled_shapes(synth.llama3_8b_shapes(), 2048, ragged=True)
    cfg = synth.FlatConfig("t", 0, seed=93, gdt="bf16", loss_scale=1.0, m_std=1e-4, v_std=1e-8, max_norm=0.1)
    ls = synth.make_list(shapes, cfg, device="cuda")
    plan = ma.MultiPlan(ls.p, ls.m, ls.v, ls.g, ls.p_lp)
    assert plan.plan.step_chunks >= 512
    h_ref, h = oracle_hyper(cfg), _hyper(cfg)
    scaler, scfg = ma.new_scaler(1.0, 3), ma.scaler_config(window=1000)
    ws, res = ma.workspace(), ma.new_result()
    refs = [dict(p=host_f32(ls.p[i]), m=host_f32(ls.m[i]), v=host_f32(ls.v[i]), lp=synth.bits16(ls.p_lp[i]),
                 pdt="bf16") for i in range(len(shapes))]

    def iteration():
        ma.multi_overflow_norm_auto(plan, scaler, res, ws)
        ma.multi_adamw_step_auto(plan, h, scaler, res, cfg.max_norm)
        ma.scaler_update(scaler, res, scfg)

    def feed(it, bad):
        gen = torch.Generator(device="cuda")
        gen.manual_seed(900 + it)
        synth._fill_grad(ls.flat.g, 1e-3, 1.0, gen)
        if bad:
            ls.g[it % len(shapes)].view(torch.int16)[0] = 0x7F81
        return [host_grad(g) for g in ls.g]

    applied = 3
    scale = 1.0

    def check(it, g_hosts, bad):
        nonlocal applied, scale
        torch.cuda.synchronize()
        ov, ss = ma.read_result(res)
        assert ov == bad, it
        assert plan.table[:64].view(torch.int32).cpu().tolist() == [0] * 16, it
        if bad:
            scale = max(scale * 0.5, 1.0)
        else:
            ss_ref = sum(oracle.overflow_norm(g, "bf16", scale)[1] for g in g_hosts)
            assert abs(ss - ss_ref) <= 1e-12 * ss_ref
            c_ref = oracle.clip_coef(ss_ref, float(np.float32(cfg.max_norm)))
            applied += 1
            for r, g in zip(refs, g_hosts):
                r["lp"] = oracle.adamw_step(r["p"], r["m"], r["v"], g, "bf16", "bf16", h_ref, applied, scale,
                                            float(c_ref), nthreads=8)
        assert ma.read_scaler(scaler)[2] == applied, it
        for i in range(len(shapes)):
            got = dict(p=host_f32(ls.p[i]), m=host_f32(ls.m[i]), v=host_f32(ls.v[i]), lp=synth.bits16(ls.p_lp[i]))
            assert_state_close(got, refs[i], "graph iteration %d, tensor %d" % (it, i))

    gh = feed(0, False)
    iteration()
    check(0, gh, False)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        iteration()
    torch.cuda.synchronize()
    for it in range(1, 6):
        bad = it == 3
        gh = feed(it, bad)
        graph.replay()
        check(it, gh, bad)
        _ = (ls.flat.p[:1000] * 2).sum().item()      # eager work of the program between replays


def test_multi_list_with_bf16_states():
    """A ragged miniature of the 8B-shaped list with p, m, v held in bf16: one scan launch, one gated
    update launch over the prepared list, against the oracle tensor by tensor; then an overflow."""
    shapes = synth.scaled_shapes(synth.llama3_8b_shapes(), 4096, ragged=True)
    cfg = synth.FlatConfig("t", 0, seed=53, m_std=1e-3, v_std=1e-6, step=6, lr=1e-2, weight_decay=0.1,
                           eps=1e-6, max_norm=0.05)
    for align in (64, 1):
        ls = synth.make_list(shapes, cfg, device="cuda", align_elems=align)
        shift = lambda t: (t.view(torch.int32) >> 16).to(torch.int16).view(torch.bfloat16).contiguous()
        fp, fm, fv = shift(ls.flat.p), shift(ls.flat.m), shift(ls.flat.v)
        offs = [t.data_ptr() // 4 - ls.flat.p.data_ptr() // 4 for t in ls.p]
        cut = lambda buf: [buf[o:o + n] for o, (_, n) in zip(offs, shapes)]
        P, M, V = cut(fp), cut(fm), cut(fv)
        g_hosts = [host_grad(g) for g in ls.g]
        ss_ref = 0.0
        for g in g_hosts:
            ov, ss = oracle.overflow_norm(g, "bf16")
            assert not ov
            ss_ref += ss
        c_ref = oracle.clip_coef(ss_ref, float(np.float32(cfg.max_norm)))
        assert c_ref < 1
        refs = []
        for i in range(len(shapes)):
            rp, rm, rv = synth.bits16(P[i]), synth.bits16(M[i]), synth.bits16(V[i])
            oracle.adamw_step_bf16(rp, rm, rv, g_hosts[i], "bf16", oracle_hyper(cfg), 6, 1.0, float(c_ref))
            refs.append((rp, rm, rv))
        plan = ma.MultiPlanBF16(P, M, V, ls.g)
        assert plan.total == sum(n for _, n in shapes) and plan.plan.sdt == ma.MA_BF16
        ws, res = ma.workspace(), ma.new_result()
        ma.multi_overflow_norm(plan, 1.0, res, ws)
        ma.multi_adamw_step_gated(plan, _hyper(cfg), 6, 1.0, res, cfg.max_norm)
        ov, ss = ma.read_result(res)
        assert not ov and abs(ss - ss_ref) <= 1e-12 * ss_ref
        for i in range(len(shapes)):
            for t, r in zip((P[i], M[i], V[i]), refs[i]):
                assert np.array_equal(synth.bits16(t), r), (align, i, shapes[i])
        # the ungated call with the host's coefficient does the same on a second copy
        before = [synth.bits16(t) for t in (fp, fm, fv)]
        ls.g[5].view(torch.int16)[0] = 0x7F80
        ma.multi_overflow_norm(plan, 1.0, res, ws)
        ma.multi_adamw_step_gated(plan, _hyper(cfg), 7, 1.0, res, cfg.max_norm)
        assert ma.read_result(res)[0] is True
        for t, b in zip((fp, fm, fv), before):
            assert np.array_equal(synth.bits16(t), b)


@pytest.mark.parametrize("gdt", ["bf16", "f16", "f32"])
def test_accumulate_fused_with_scan(gdt):
    """The last micro-batch accumulated and scanned in one pass: the buffer equals the oracle's, and
    {overflow, sumsq} equals the oracle's scan of the accumulated fp32 buffer; also through views
    that force the scalar path, with a device-resident scale, and with planted non-finite values."""
    ws = ma.workspace()
    S = 256.0
    for n in [0, 1, 3, 5, 1023, 4096, 4097, 8193, 100_003, (1 << 20) + 7]:
        for off_acc, off_g in ((0, 0), (1, 1), (1, 2)):
            base = torch.zeros(n + 4, dtype=torch.float32, device="cuda")
            acc = base[off_acc:off_acc + n]
            ref = np.zeros(n, np.float32)
            res = ma.new_result(2)
            for k in range(3):
                gfull = _micro_grad(n + 4, 2000 + 7 * k + n % 13, gdt, S)
                g = gfull[off_g:off_g + n]
                oracle.grad_accumulate(ref, host_grad(g), gdt, first=(k == 0))
                if k < 2:
                    ma.grad_accumulate(acc, g, first=(k == 0))
                else:
                    ma.grad_accumulate_scan(acc, g, False, S, res, ws)
            assert np.array_equal(host_f32(acc).view(np.uint32), ref.view(np.uint32)), (n, off_acc, off_g)
            ov_ref, ss_ref = oracle.overflow_norm(ref, "f32", S)
            ov, ss = ma.read_result(res)
            assert ov == ov_ref == False
            assert abs(ss - ss_ref) <= 1e-12 * max(ss_ref, 1e-300), (n, ss, ss_ref)
            # the stand-alone scan of the same buffer agrees (same kernels' arithmetic, other order)
            ma.overflow_norm(acc, S, res, ws, index=1)
            assert abs(ma.read_result(res, 1)[1] - ss) <= 1e-12 * max(ss, 1e-300)
    # one micro-batch per iteration: the overwrite itself is fused with the scan (its own tile size)
    for n in [0, 1, 5, 4097, 12287, 12288, 12289, 24577, 100_003]:
        for off_acc, off_g in ((0, 0), (1, 1), (2, 1)):
            acc = torch.full((n + 4,), float("nan"), dtype=torch.float32, device="cuda")[off_acc:off_acc + n]
            g = _micro_grad(n + 4, 3000 + n % 17, gdt, S)[off_g:off_g + n]
            res = ma.new_result()
            ma.grad_accumulate_scan(acc, g, True, S, res, ws)
            ref = np.full(n, np.nan, np.float32)
            oracle.grad_accumulate(ref, host_grad(g), gdt, first=True)
            assert np.array_equal(host_f32(acc).view(np.uint32), ref.view(np.uint32)), (n, off_acc, off_g)
            ov_ref, ss_ref = oracle.overflow_norm(ref, "f32", S)
            ov, ss = ma.read_result(res)
            assert ov == ov_ref == False and abs(ss - ss_ref) <= 1e-12 * max(ss_ref, 1e-300), (n, ss, ss_ref)
    # `first` with scan, scale taken from device memory, and an overflow entering with the micro-batch
    n = 50_001
    acc = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    g = _micro_grad(n, 77, gdt, S)
    scaler = ma.new_scaler(S, 0)
    res = ma.new_result(2)
    ma.grad_accumulate_scan(acc, g, True, 1.0, res, ws, scaler=scaler)
    ref = np.full(n, np.nan, np.float32)
    oracle.grad_accumulate(ref, host_grad(g), gdt, first=True)
    ov_ref, ss_ref = oracle.overflow_norm(ref, "f32", S)
    ov, ss = ma.read_result(res)
    assert not ov and not ov_ref and abs(ss - ss_ref) <= 1e-12 * ss_ref
    if gdt != "f32":
        bits = synth.NONFINITE_BITS[gdt][1]
        g.view(torch.int16)[n - 2] = bits - 0x10000
    else:
        g[n - 2] = float("-inf")
    ma.grad_accumulate_scan(acc, g, False, S, res, ws, index=1)
    assert ma.read_result(res, 1)[0] is True
    oracle.grad_accumulate(ref, host_grad(g), gdt, first=False)
    assert oracle.overflow_norm(ref, "f32", S)[0] is True
    assert np.array_equal(host_f32(acc).view(np.uint32), ref.view(np.uint32))


def test_multi_list_with_fp32_gradients():
    """The tensor list fed from an accumulated fp32 gradient buffer (Algorithm 1's own dtype): one
    scan launch with the 0x7F800000 mask, one gated update launch, fp16 parameter copies."""
    shapes = synth.scaled_shapes(synth.llama3_8b_shapes(), 8192, ragged=True)
    cfg = synth.FlatConfig("t", 0, seed=57, m_std=1e-4, v_std=1e-8, step=12, pdt="f16", max_norm=0.03)
    S = 32.0
    for align in (64, 1):
        ls = synth.make_list(shapes, cfg, device="cuda", align_elems=align)
        total = ls.flat.p.numel()
        g32_flat = (ls.flat.g.to(torch.float32) * (S * 1.0003)).contiguous()
        offs = [t.data_ptr() // 4 - ls.flat.p.data_ptr() // 4 for t in ls.p]
        G32 = [g32_flat[o:o + n] for o, (_, n) in zip(offs, shapes)]
        ss_ref, refs = 0.0, []
        for g in G32:
            ov, ss = oracle.overflow_norm(host_f32(g), "f32", S)
            assert not ov
            ss_ref += ss
        c_ref = oracle.clip_coef(ss_ref, float(np.float32(cfg.max_norm)))
        assert c_ref < 1
        for i in range(len(shapes)):
            r = dict(p=host_f32(ls.p[i]), m=host_f32(ls.m[i]), v=host_f32(ls.v[i]), pdt="f16")
            r["lp"] = oracle.adamw_step(r["p"], r["m"], r["v"], host_f32(G32[i]), "f32", "f16",
                                        oracle_hyper(cfg), 12, S, float(c_ref))
            refs.append(r)
        plan = ma.MultiPlan(ls.p, ls.m, ls.v, G32, ls.p_lp)
        ws, res = ma.workspace(), ma.new_result()
        ma.multi_overflow_norm(plan, S, res, ws)
        ma.multi_adamw_step_gated(plan, _hyper(cfg), 12, S, res, cfg.max_norm)
        ov, ss = ma.read_result(res)
        assert not ov and abs(ss - ss_ref) <= 1e-12 * ss_ref
        for i in range(len(shapes)):
            got = dict(p=host_f32(ls.p[i]), m=host_f32(ls.m[i]), v=host_f32(ls.v[i]),
                       lp=synth.bits16(ls.p_lp[i]))
            assert_state_close(got, refs[i], "tensor %d" % i)
        G32[11][0] = float("inf")
        ma.multi_overflow_norm(plan, S, res, ws)
        assert ma.read_result(res)[0] is True


def test_randomised_bf16_states_and_accumulation():
    """Seeded random cases for the two rows beyond the basic step: 80 bf16-state steps (sizes 0..3e5,
    each buffer at its own element offset, all gradient dtypes, random hyper-parameters, gated) and
    80 accumulation sequences (1 to 5 micro-batches, the last one fused with the scan); bit patterns
    against the oracle."""
    rng = np.random.default_rng(777)
    ws = ma.workspace()

    def view(t, n, o):
        base = torch.zeros(n + 16, dtype=t.dtype, device="cuda")
        base[o:o + n].copy_(t)
        return base[o:o + n]

    for case in range(80):
        n = int(rng.choice([rng.integers(0, 40), rng.integers(40, 9000), rng.integers(9000, 300000)]))
        gdt = str(rng.choice(["bf16", "f16", "f32"]))
        S = float(2.0 ** rng.integers(0, 14)) if gdt != "f32" else 1.0
        cfg = synth.FlatConfig("z", n, seed=int(rng.integers(1 << 30)), gdt="bf16" if gdt == "f32" else gdt,
                               loss_scale=S, m_std=1e-3, v_std=1e-6, step=int(rng.integers(1, 200)),
                               lr=float(10 ** rng.uniform(-4, -1)), weight_decay=float(rng.choice([0.0, 0.1])),
                               eps=float(10 ** rng.uniform(-8, -4)), max_norm=float(rng.choice([0.0, 0.05, 5.0])))
        st, p, m, v = _bf16_state(cfg, n)
        g = st.g if gdt != "f32" else st.g.to(torch.float32) * 1.3
        same = rng.random() < 0.5
        o0 = int(rng.integers(0, 17))
        p, m, v, g = (view(t, n, o0 if same else int(rng.integers(0, 17))) for t in (p, m, v, g))
        rp, rm, rv = synth.bits16(p), synth.bits16(m), synth.bits16(v)
        g_host = host_grad(g)
        ov_ref, ss_ref = oracle.overflow_norm(g_host, gdt, S)
        c_ref = oracle.clip_coef(ss_ref, float(np.float32(cfg.max_norm)))
        oracle.adamw_step_bf16(rp, rm, rv, g_host, gdt, oracle_hyper(cfg), cfg.step, S, float(c_ref))
        res = ma.new_result()
        ma.overflow_norm(g, S, res, ws)
        ma.adamw_step_bf16_gated(p, m, v, g, _hyper(cfg), cfg.step, S, res, cfg.max_norm)
        what = "bf16-state case %d: n=%d gdt=%s %r" % (case, n, gdt, cfg)
        assert ma.read_result(res)[0] is False and not ov_ref, what
        for t, r in ((p, rp), (m, rm), (v, rv)):
            assert np.array_equal(synth.bits16(t), r), what

    for case in range(80):
        n = int(rng.choice([rng.integers(0, 40), rng.integers(40, 9000), rng.integers(9000, 300000)]))
        gdt = str(rng.choice(["bf16", "f16", "f32"]))
        S = float(2.0 ** rng.integers(0, 14))
        micro = int(rng.integers(1, 6))
        acc = view(torch.full((n,), float("nan"), dtype=torch.float32, device="cuda"), n, int(rng.integers(0, 9)))
        ref = np.full(n, np.nan, np.float32)
        res = ma.new_result()
        for k in range(micro):
            g = view(_micro_grad(n, int(rng.integers(1 << 30)), gdt, S), n, int(rng.integers(0, 9)))
            oracle.grad_accumulate(ref, host_grad(g), gdt, first=(k == 0))
            if k < micro - 1:
                ma.grad_accumulate(acc, g, first=(k == 0))
            else:
                ma.grad_accumulate_scan(acc, g, k == 0, S, res, ws)
        what = "accumulation case %d: n=%d gdt=%s micro=%d" % (case, n, gdt, micro)
        assert np.array_equal(host_f32(acc).view(np.uint32), ref.view(np.uint32)), what
        ov_ref, ss_ref = oracle.overflow_norm(ref, "f32", S)
        ov, ss = ma.read_result(res)
        assert ov == ov_ref is False and abs(ss - ss_ref) <= 1e-11 * max(ss_ref, 1e-300), what


def test_whole_iteration_accumulate_check_step():
    """The order of Sec. IV-A at list scale: micro-batch gradients accumulate into the fp32 flat gradient
    buffer, the fused check runs inside the last accumulation pass (no separate scan), and the gated
    multi-tensor step takes that buffer as its fp32 gradient.  Three iterations: one micro-batch; three
    with an infinity in the second (the step is skipped, the state stays as it is, the update number
    does not advance); two, clean again.  Every element against the oracle's chain of the same calls."""
    shapes = [("a", 64 * 1000), ("b", 4096 * 37), ("c", 64), ("d", 128 * 4097), ("e", 64 * 333)]
    cfg = synth.FlatConfig("iteration", 0, seed=11, m_std=1e-4, v_std=1e-8, step=7, max_norm=1.0, gdt="f32")
    ls = synth.make_list(shapes, cfg, device="cuda", layout="streams")
    n = ls.total
    assert ls.flat.g.numel() == n and ls.flat.g.dtype == torch.float32       # one flat buffer, no padding
    plan = ma.MultiPlan(ls.p, ls.m, ls.v, ls.g, ls.p_lp)
    ws, res = ma.workspace(), ma.new_result()
    ref = _host_state(ls.flat)
    acc_ref = np.full(n, np.nan, np.float32)
    S, t = 256.0, cfg.step
    for it, (micro, poison) in enumerate([(1, False), (3, True), (2, False)]):
        for k in range(micro):
            g = _micro_grad(n, 5000 + 10 * it + k, "bf16", S)
            if poison and k == 1:
                g.view(torch.int16)[n - 12345] = 0x7F80                      # +inf in one micro-batch
            oracle.grad_accumulate(acc_ref, host_grad(g), "bf16", first=(k == 0))
            if k < micro - 1:
                ma.grad_accumulate(ls.flat.g, g, first=(k == 0))
            else:
                ma.grad_accumulate_scan(ls.flat.g, g, k == 0, S, res, ws)
        ma.multi_adamw_step_gated(plan, _hyper(cfg), t, S, res, cfg.max_norm)
        ov_ref, ss_ref = oracle.overflow_norm(acc_ref, "f32", S)
        ov, ss = ma.read_result(res)
        what = "iteration %d (%d micro-batches)" % (it, micro)
        assert ov == ov_ref == poison, what
        assert np.array_equal(host_f32(ls.flat.g).view(np.uint32), acc_ref.view(np.uint32)), what
        if not poison:
            assert abs(ss - ss_ref) <= 1e-11 * ss_ref, what
            c_ref = oracle.clip_coef(ss_ref, float(np.float32(cfg.max_norm)))
            assert np.float32(ma.clip_coef(ss, cfg.max_norm)) == c_ref
            ref["lp"] = oracle.adamw_step(ref["p"], ref["m"], ref["v"], acc_ref, "f32", "bf16", oracle_hyper(cfg),
                                          t, S, float(c_ref))
            t += 1
        got = _host_state(ls.flat)
        assert_state_close(got, ref, what)
        for k in ("p", "m", "v"):                                            # in fact bit for bit
            assert np.array_equal(got[k].view(np.uint32), ref[k].view(np.uint32)), what + " " + k
    assert t == cfg.step + 2
