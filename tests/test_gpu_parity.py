"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs, element by element.  Sizes span several work items and ragged tails; the bar is: flag and
skip exact, p_lp bit-exact given the same fp32 p, p/m/v within 2 ulp, sumsq within 1e-5."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_23254_amd import synth
from tests._util import (GDT_NAME, MAX_ULP, SUMSQ_RTOL, assert_state_close, host_f32, host_grad,
                         oracle_hyper, round_lp, ulp_distance)

pytestmark = pytest.mark.gpu

ma = None


@pytest.fixture(scope="module", autouse=True)
def _lib():
    global ma
    from paper_2505_23254_amd import binding
    ma = binding
    assert torch.cuda.is_available()
    yield


def _hyper(cfg):
    return ma.hyper(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, cfg.weight_decay, 1)


def _host_state(st, pdt):
    return dict(p=host_f32(st.p), m=host_f32(st.m), v=host_f32(st.v), lp=synth.bits16(st.p_lp), pdt=pdt)


SIZES = [0, 1, 3, 4, 5, 63, 64, 65, 1023, 1024, 2047, 2048, 2049, 4097, 8191, 100_003, 1 << 20]


@pytest.mark.parametrize("gdt,pdt", [("bf16", "bf16"), ("f16", "bf16"), ("bf16", "f16"), ("f16", "f16")])
def test_flat_scan_and_step_sizes(gdt, pdt):
    """Config 1 (t = 1, zero moments, no clipping) and the same at t = 100 with non-zero moments,
    at sizes from empty to 2^20 including every ragged-tail class."""
    ws = ma.workspace()
    for n in SIZES:
        for variant in range(2):
            cfg = synth.FlatConfig("t", n, seed=100 + n % 97, gdt=gdt, pdt=pdt,
                                   loss_scale=1.0 if gdt == "bf16" else 1024.0)
            if variant:
                cfg.m_std, cfg.v_std, cfg.step = 1e-4, 1e-8, 100
            st = synth.make_flat(cfg, device="cuda")
            g_host = host_grad(st.g)
            ref = _host_state(st, pdt)
            clip = 1.0 if not variant else 0.25
            # oracle
            ov_ref, ss_ref = oracle.overflow_norm(g_host, gdt, cfg.loss_scale)
            ref["lp"] = oracle.adamw_step(ref["p"], ref["m"], ref["v"], g_host, gdt, pdt,
                                          oracle_hyper(cfg), cfg.step, cfg.loss_scale, clip)
            # HIP path
            res = ma.new_result()
            ma.overflow_norm(st.g, cfg.loss_scale, res, ws)
            ma.adamw_step(st.p, st.m, st.v, st.g, st.p_lp, _hyper(cfg), cfg.step, cfg.loss_scale, clip)
            ov, ss = ma.read_result(res)
            assert ov == ov_ref == False
            assert abs(ss - ss_ref) <= SUMSQ_RTOL * ss_ref, (n, ss, ss_ref)
            if n:
                assert abs(ss - ss_ref) <= 1e-12 * ss_ref      # fp64 accumulation on both sides
            assert_state_close(_host_state(st, pdt), ref, "n=%d variant=%d" % (n, variant))
            assert np.array_equal(host_grad(st.g), g_host)      # the gradient is read-only


def test_config1_exact_shape():
    cfg = synth.config("c1")
    st = synth.make_flat(cfg, device="cuda")
    g_host = host_grad(st.g)
    ref = _host_state(st, "bf16")
    ov_ref, ss_ref, c_ref = oracle.optimizer_step(ref["p"], ref["m"], ref["v"], g_host, "bf16",
                                                  ref["lp"], "bf16", oracle_hyper(cfg), 1, 1.0, 0.0)
    ws, res = ma.workspace(), ma.new_result()
    ma.overflow_norm(st.g, 1.0, res, ws)
    ma.adamw_step_gated(st.p, st.m, st.v, st.g, st.p_lp, _hyper(cfg), 1, 1.0, res, 0.0)
    ov, ss = ma.read_result(res)
    assert (ov, ov_ref) == (False, False) and c_ref == 1.0
    assert abs(ss - ss_ref) <= 1e-12 * ss_ref
    got = _host_state(st, "bf16")
    assert_state_close(got, ref, "c1")
    # same operation order on both sides: in fact bit-identical
    for k in ("p", "m", "v"):
        assert np.array_equal(got[k].view(np.uint32), ref[k].view(np.uint32)), k
    assert np.array_equal(got["lp"], ref["lp"])


@pytest.mark.parametrize("gdt", ["bf16", "f16"])
def test_gated_step_with_clipping(gdt):
    n = 300_007
    S = 1.0 if gdt == "bf16" else 65536.0
    cfg = synth.FlatConfig("t", n, seed=5, gdt=gdt, m_std=1e-4, v_std=1e-8, step=100,
                           loss_scale=S, max_norm=0.01)
    st = synth.make_flat(cfg, device="cuda")
    g_host = host_grad(st.g)
    ref = _host_state(st, "bf16")
    ov_ref, ss_ref, c_ref = oracle.optimizer_step(ref["p"], ref["m"], ref["v"], g_host, gdt,
                                                  ref["lp"], "bf16", oracle_hyper(cfg), 100, S,
                                                  cfg.max_norm)
    assert not ov_ref and c_ref < 1.0
    ws, res = ma.workspace(), ma.new_result()
    ma.overflow_norm(st.g, S, res, ws)
    ma.adamw_step_gated(st.p, st.m, st.v, st.g, st.p_lp, _hyper(cfg), 100, S, res, cfg.max_norm)
    ov, ss = ma.read_result(res)
    assert not ov and abs(ss - ss_ref) <= 1e-12 * ss_ref
    # the host helper and the device gate derive the same coefficient as the oracle
    assert np.float32(ma.clip_coef(ss, cfg.max_norm)) == c_ref
    assert_state_close(_host_state(st, "bf16"), ref, "gated")


@pytest.mark.parametrize("gdt", ["bf16", "f16"])
def test_overflow_is_found_everywhere_and_skips_the_step(gdt):
    """A single inf/NaN at the first element, the last, inside the ragged tail, at work-item and
    block boundaries: flag = 1 and the gated step leaves p, m, v, p_lp bit-unchanged."""
    n = 70_001
    cfg = synth.FlatConfig("t", n, seed=9, gdt=gdt, m_std=1e-4, v_std=1e-8, step=3)
    ws = ma.workspace()
    positions = [0, 1, 7, 8, 2047, 2048, 8191, 8192, 16383, 16384, 65535, 65536, n - 2, n - 1]
    for k, pos in enumerate(positions):
        st = synth.make_flat(cfg, device="cuda")
        bits = synth.NONFINITE_BITS[gdt][k % 5]
        st.g.view(torch.int16)[pos] = bits - 0x10000 if bits >= 0x8000 else bits
        before = _host_state(st, "bf16")
        g_host = host_grad(st.g)
        assert oracle.overflow_norm(g_host, gdt)[0] is True
        res = ma.new_result()
        ma.overflow_norm(st.g, 1.0, res, ws)
        ma.adamw_step_gated(st.p, st.m, st.v, st.g, st.p_lp, _hyper(cfg), 3, 1.0, res, 1.0)
        assert ma.read_result(res)[0] is True, pos
        after = _host_state(st, "bf16")
        for key in ("p", "m", "v", "lp"):
            assert after[key].tobytes() == before[key].tobytes(), (pos, key)


@pytest.mark.parametrize("gdt", ["bf16", "f16"])
def test_flag_on_every_16_bit_pattern(gdt):
    """All finite patterns together give 0; every pattern with an all-ones exponent, alone among
    zeros, gives 1 (the exponent-mask rule of Algorithm 1 at the gradient's own width)."""
    mask = 0x7F80 if gdt == "bf16" else 0x7C00
    tdt = torch.bfloat16 if gdt == "bf16" else torch.float16
    allp = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    finite = allp[(allp & mask) != mask]
    bad = allp[(allp & mask) == mask]
    ws, res = ma.workspace(), ma.new_result()
    g = torch.from_numpy(finite.view(np.int16)).cuda().view(tdt)
    ma.overflow_norm(g, 1.0, res, ws)
    assert ma.read_result(res)[0] is False and oracle.overflow_norm(finite, gdt)[0] is False
    n = 5000
    buf = torch.zeros(n, dtype=torch.int16, device="cuda")
    out = ma.new_result(len(bad))
    for k, b in enumerate(bad.tolist()):
        pos = (k * 37) % n
        buf[pos] = b - 0x10000 if b >= 0x8000 else b
        ma.overflow_norm(buf.view(tdt), 1.0, out, ws, index=k)
        buf[pos] = 0
    flags = out.cpu().numpy().view(np.int32)[0::4]
    assert np.all(flags == 1)


@pytest.mark.parametrize("pdt", ["bf16", "f16"])
def test_low_precision_cast_on_rounding_critical_patterns(pdt):
    """With lr = 0 the step returns p unchanged, so p_lp = RNE(p) for any p we choose: every
    upper half combined with the lower halves that decide rounding, including inf and NaN."""
    hi = np.arange(65536, dtype=np.uint32) << 16
    lows = [0x0000, 0x0001, 0x0FFF, 0x1000, 0x1001, 0x1FFF, 0x2000, 0x3000, 0x7FFF, 0x8000, 0x8001, 0xFFFF]
    bits = np.concatenate([hi | lo for lo in lows])
    n = bits.size
    p = torch.from_numpy(bits.view(np.float32).copy()).cuda()
    m = torch.zeros(n, device="cuda")
    v = torch.ones(n, device="cuda")
    g = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    lp = torch.zeros(n, dtype=torch.bfloat16 if pdt == "bf16" else torch.float16, device="cuda")
    h = ma.hyper(lr=0.0, weight_decay=0.0)
    ref_p, ref_m, ref_v = bits.view(np.float32).copy(), np.zeros(n, np.float32), np.ones(n, np.float32)
    oracle.adamw_step(ref_p, ref_m, ref_v, np.zeros(n, np.uint16), "bf16", pdt,
                      oracle.hyper(lr=0.0, weight_decay=0.0), 1)
    ma.adamw_step(p, m, v, g, lp, h, 1)
    p_out = host_f32(p)
    # finite non-zero p really is unchanged (inf turns into NaN through 0*inf, -0 into +0: on
    # both sides), so the cast sees exactly the patterns chosen above
    keep = np.isfinite(bits.view(np.float32)) & ((bits & 0x7FFFFFFF) != 0)
    assert np.array_equal(p_out.view(np.uint32)[keep], bits[keep])
    assert ulp_distance(p_out, ref_p).max() == 0
    assert np.array_equal(np.isnan(p_out), np.isnan(ref_p))
    assert np.array_equal(synth.bits16(lp), round_lp(p_out, pdt))
    # a parameter pushed past the largest finite value becomes inf and is cast to inf
    p2 = torch.tensor([3.4e38, -3.4e38, 1.0], device="cuda")
    g2 = torch.tensor([-1.0, 1.0, 1.0], dtype=torch.bfloat16, device="cuda")
    m2, v2 = torch.zeros(3, device="cuda"), torch.zeros(3, device="cuda")
    lp2 = torch.zeros(3, dtype=lp.dtype, device="cuda")
    ma.adamw_step(p2, m2, v2, g2, lp2, ma.hyper(lr=3e38, weight_decay=0.0), 1)
    inf_bits = (0x7F80, 0xFF80) if pdt == "bf16" else (0x7C00, 0xFC00)
    assert torch.isinf(p2[:2]).all() and tuple(synth.bits16(lp2)[:2].tolist()) == inf_bits


def test_scan_is_deterministic_and_chunking_invariant():
    n = 3_000_001
    cfg = synth.FlatConfig("t", n, seed=21)
    st = synth.make_flat(cfg, device="cuda")
    ws, res = ma.workspace(), ma.new_result(8)
    for k in range(4):
        ma.overflow_norm(st.g, 1.0, res, ws, index=k)
    raw = res.cpu().numpy().view(np.uint64).reshape(-1, 2)
    assert np.all(raw[:4] == raw[0])                    # bit-identical run to run
    # the flag and the sum of any partition of the buffer agree with the whole
    cuts = [0, 1, 4097, 1_000_003, 2_500_000, n]
    parts = ma.new_result(len(cuts) - 1)
    for k in range(len(cuts) - 1):
        ma.overflow_norm(st.g[cuts[k]:cuts[k + 1]], 1.0, parts, ws, index=k)
    ma.norm_combine(parts, len(cuts) - 1, res, index=5)
    ov, ss = ma.read_result(res, 5)
    ov0, ss0 = ma.read_result(res, 0)
    assert ov == ov0 == False and abs(ss - ss0) <= 1e-13 * ss0


@pytest.mark.parametrize("offsets", [(1, 1, 1, 1, 1), (3, 3, 3, 3, 3), (2, 2, 2, 6, 10),
                                     (1, 2, 3, 0, 1), (0, 0, 0, 1, 0), (0, 0, 0, 0, 3)])
def test_misaligned_views(offsets):
    """Slices at odd element offsets: equal offsets reach the 4-wide path after a head of up to
    three elements, unequal ones take the scalar path; results are the same either way."""
    n = 50_021
    cfg = synth.FlatConfig("t", n + 16, seed=33, m_std=1e-4, v_std=1e-8, step=7, gdt="f16",
                           loss_scale=256.0)
    st = synth.make_flat(cfg, device="cuda")
    op, om, ov_, og, ol = offsets
    p, m, v = st.p[op:op + n], st.m[om:om + n], st.v[ov_:ov_ + n]
    g, lp = st.g[og:og + n], st.p_lp[ol:ol + n]
    ref = dict(p=host_f32(p), m=host_f32(m), v=host_f32(v), lp=synth.bits16(lp), pdt="bf16")
    g_host = host_grad(g)
    edge = dict(p=host_f32(st.p), m=host_f32(st.m), v=host_f32(st.v), lp=synth.bits16(st.p_lp))
    ov_ref, ss_ref = oracle.overflow_norm(g_host, "f16", 256.0)
    ref["lp"] = oracle.adamw_step(ref["p"], ref["m"], ref["v"], g_host, "f16", "bf16",
                                  oracle_hyper(cfg), 7, 256.0, 0.5)
    ws, res = ma.workspace(), ma.new_result()
    ma.overflow_norm(g, 256.0, res, ws)
    ma.adamw_step(p, m, v, g, lp, _hyper(cfg), 7, 256.0, 0.5)
    ov, ss = ma.read_result(res)
    assert ov == ov_ref and abs(ss - ss_ref) <= 1e-12 * ss_ref
    got = dict(p=host_f32(p), m=host_f32(m), v=host_f32(v), lp=synth.bits16(lp))
    assert_state_close(got, ref, "offsets %s" % (offsets,))
    # nothing outside the slices was touched
    for key, off, full in (("p", op, st.p), ("m", om, st.m), ("v", ov_, st.v)):
        now = host_f32(full)
        assert np.array_equal(now[:off], edge[key][:off]) and np.array_equal(now[off + n:], edge[key][off + n:])
    now = synth.bits16(st.p_lp)
    assert np.array_equal(now[:ol], edge["lp"][:ol]) and np.array_equal(now[ol + n:], edge["lp"][ol + n:])


def test_no_low_precision_copy():
    n = 10_001
    cfg = synth.FlatConfig("t", n, seed=41, m_std=1e-4, v_std=1e-8, step=2)
    st = synth.make_flat(cfg, device="cuda")
    ref = _host_state(st, "bf16")
    lp_before = synth.bits16(st.p_lp)
    oracle.adamw_step(ref["p"], ref["m"], ref["v"], host_grad(st.g), "bf16", "bf16", oracle_hyper(cfg), 2)
    ma.adamw_step(st.p, st.m, st.v, st.g, None, _hyper(cfg), 2)
    for k, t in (("p", st.p), ("m", st.m), ("v", st.v)):
        assert ulp_distance(host_f32(t), ref[k]).max() <= MAX_ULP
    assert np.array_equal(synth.bits16(st.p_lp), lp_before)


def test_fp32_gradients():
    n = 123_457
    cfg = synth.FlatConfig("t", n, seed=43, m_std=1e-4, v_std=1e-8, step=11)
    st = synth.make_flat(cfg, device="cuda")
    g32 = st.g.to(torch.float32) * 1.0001
    g_host = host_f32(g32)
    ref = _host_state(st, "bf16")
    ov_ref, ss_ref = oracle.overflow_norm(g_host, "f32", 2.0)
    ref["lp"] = oracle.adamw_step(ref["p"], ref["m"], ref["v"], g_host, "f32", "bf16",
                                  oracle_hyper(cfg), 11, 2.0, 0.75)
    ws, res = ma.workspace(), ma.new_result(2)
    ma.overflow_norm(g32, 2.0, res, ws)
    ma.adamw_step(st.p, st.m, st.v, g32, st.p_lp, _hyper(cfg), 11, 2.0, 0.75)
    ov, ss = ma.read_result(res)
    assert ov == ov_ref == False and abs(ss - ss_ref) <= 1e-12 * ss_ref
    assert_state_close(_host_state(st, "bf16"), ref, "fp32 grads")
    g32[n // 2] = float("nan")
    ma.overflow_norm(g32, 2.0, res, ws, index=1)
    assert ma.read_result(res, 1)[0] is True


@pytest.mark.parametrize("align_elems,layout", [(64, "streams"), (1, "streams"), (64, "tensor")])
def test_multi_tensor_list_miniature(align_elems, layout):
    """A 1/4096-scale Llama-3-8B-shaped list (290 tensors, ragged sizes): one scan launch, one
    gated update launch, compared tensor by tensor with the oracle run on the same list."""
    shapes = synth.scaled_shapes(synth.llama3_8b_shapes(), 4096, ragged=True)
    cfg = synth.FlatConfig("t", 0, seed=51, m_std=1e-4, v_std=1e-8, step=100, max_norm=0.05)
    ls = synth.make_list(shapes, cfg, device="cuda", align_elems=align_elems, layout=layout)
    refs, g_hosts = [], []
    for i in range(len(shapes)):
        refs.append(dict(p=host_f32(ls.p[i]), m=host_f32(ls.m[i]), v=host_f32(ls.v[i]),
                         lp=synth.bits16(ls.p_lp[i]), pdt="bf16"))
        g_hosts.append(host_grad(ls.g[i]))
    # oracle: global norm over the whole list (sum of per-tensor fp64 sums, list order), one clip
    ss_ref = 0.0
    for g in g_hosts:
        ov, ss = oracle.overflow_norm(g, "bf16")
        assert not ov
        ss_ref += ss
    c_ref = oracle.clip_coef(ss_ref, float(np.float32(cfg.max_norm)))
    assert c_ref < 1
    for r, g in zip(refs, g_hosts):
        r["lp"] = oracle.adamw_step(r["p"], r["m"], r["v"], g, "bf16", "bf16", oracle_hyper(cfg), 100,
                                    1.0, float(c_ref))
    plan = ma.MultiPlan(ls.p, ls.m, ls.v, ls.g, ls.p_lp)
    assert plan.total == sum(n for _, n in shapes)
    ws, res = ma.workspace(), ma.new_result()
    ma.multi_overflow_norm(plan, 1.0, res, ws)
    ma.multi_adamw_step_gated(plan, _hyper(cfg), 100, 1.0, res, cfg.max_norm)
    ov, ss = ma.read_result(res)
    assert not ov and abs(ss - ss_ref) <= 1e-12 * ss_ref
    assert np.float32(ma.clip_coef(ss, cfg.max_norm)) == c_ref
    for i in range(len(shapes)):
        got = dict(p=host_f32(ls.p[i]), m=host_f32(ls.m[i]), v=host_f32(ls.v[i]), lp=synth.bits16(ls.p_lp[i]))
        assert_state_close(got, refs[i], "tensor %d (%s)" % (i, shapes[i][0]))
    # overflow in one small tensor gates the whole list: not one byte of the allocation changes
    ls.g[7].view(torch.int16)[0] = 0x7FC0
    whole = ls.flat.arena if layout == "streams" else ls.arena
    before = whole.cpu().numpy().tobytes()
    ma.multi_overflow_norm(plan, 1.0, res, ws)
    ma.multi_adamw_step_gated(plan, _hyper(cfg), 101, 1.0, res, cfg.max_norm)
    assert ma.read_result(res)[0] is True
    assert whole.cpu().numpy().tobytes() == before


def test_multi_ungated_equals_gated_with_same_clip():
    shapes = [("a", 5000), ("b", 1), ("c", 0), ("d", 4096), ("e", 12345)]
    cfg = synth.FlatConfig("t", 0, seed=61, m_std=1e-4, v_std=1e-8, step=5, gdt="f16", pdt="f16",
                           loss_scale=128.0)
    la = synth.make_list(shapes, cfg, device="cuda")
    lb = synth.make_list(shapes, cfg, device="cuda")
    pa = ma.MultiPlan(la.p, la.m, la.v, la.g, la.p_lp)
    pb = ma.MultiPlan(lb.p, lb.m, lb.v, lb.g, lb.p_lp)
    ws, res = ma.workspace(), ma.new_result()
    ma.multi_overflow_norm(pa, 128.0, res, ws)
    _, ss = ma.read_result(res)
    c = ma.clip_coef(ss, 0.02)
    assert c < 1
    ma.multi_adamw_step_gated(pa, _hyper(cfg), 5, 128.0, res, 0.02)
    ma.multi_adamw_step(pb, _hyper(cfg), 5, 128.0, c)
    for x, y in ((la.flat.p, lb.flat.p), (la.flat.m, lb.flat.m), (la.flat.v, lb.flat.v)):
        assert host_f32(x).tobytes() == host_f32(y).tobytes()
    assert synth.bits16(la.flat.p_lp).tobytes() == synth.bits16(lb.flat.p_lp).tobytes()


def test_sub_group_streaming_miniature():
    """A 14B-class-shaped list at 1/4096 scale, processed as 4 equal flat sub-groups cut without
    regard to tensor boundaries: four scans, one combine, four gated updates on one stream --
    against the oracle run on the whole flat buffer with the global norm."""
    shapes = synth.scaled_shapes(synth.qwen14b_class_shapes(), 4096, ragged=False)
    cfg = synth.FlatConfig("t", 0, seed=71, m_std=1e-4, v_std=1e-8, step=100, max_norm=0.05)
    ls = synth.make_list(shapes, cfg, device="cuda", align_elems=1)
    fl = ls.flat
    total = fl.p.numel()
    assert total % 4 == 0
    ref = dict(p=host_f32(fl.p), m=host_f32(fl.m), v=host_f32(fl.v), lp=synth.bits16(fl.p_lp), pdt="bf16")
    g_host = host_grad(fl.g)
    sub = total // 4
    ss_ref = 0.0
    for k in range(4):
        ss_ref += oracle.overflow_norm(g_host[k * sub:(k + 1) * sub], "bf16")[1]
    c_ref = oracle.clip_coef(ss_ref, float(np.float32(cfg.max_norm)))
    ref["lp"] = oracle.adamw_step(ref["p"], ref["m"], ref["v"], g_host, "bf16", "bf16",
                                  oracle_hyper(cfg), 100, 1.0, float(c_ref))
    ws, parts, res = ma.workspace(), ma.new_result(4), ma.new_result()
    for k in range(4):
        ma.overflow_norm(fl.g[k * sub:(k + 1) * sub], 1.0, parts, ws, index=k)
    ma.norm_combine(parts, 4, res)
    for k in range(4):
        s = slice(k * sub, (k + 1) * sub)
        ma.adamw_step_gated(fl.p[s], fl.m[s], fl.v[s], fl.g[s], fl.p_lp[s], _hyper(cfg), 100, 1.0,
                            res, cfg.max_norm)
    ov, ss = ma.read_result(res)
    assert not ov and abs(ss - ss_ref) <= 1e-12 * ss_ref
    got = dict(p=host_f32(fl.p), m=host_f32(fl.m), v=host_f32(fl.v), lp=synth.bits16(fl.p_lp))
    assert_state_close(got, ref, "sub-groups")


def test_parameter_groups_share_one_global_norm():
    """Two parameter groups of one model, as fine-tuning recipes have them: the matrices with weight
    decay, the norm vectors without and at another learning rate.  Each group is a prepared list of
    its own; their scans are combined into ONE global norm (the clip coefficient is a property of the
    whole gradient), and each group's gated step reads that result with its own hyper-parameters.  An
    overflow in the small group skips both."""
    shapes = synth.scaled_shapes(synth.llama3_8b_shapes(), 2048, ragged=True)
    cfg = synth.FlatConfig("groups", 0, seed=81, m_std=1e-4, v_std=1e-8, step=42, max_norm=0.05)
    ls = synth.make_list(shapes, cfg, device="cuda")
    small = [i for i, (name, _) in enumerate(shapes) if "norm" in name]  # the norm vectors
    large = [i for i in range(len(shapes)) if i not in small]
    assert small and large
    pick = lambda lst, idx: [lst[i] for i in idx]
    hy = {"large": dict(lr=1e-5, wd=0.01), "small": dict(lr=3e-5, wd=0.0)}
    groups = {"large": large, "small": small}
    plans = {k: ma.MultiPlan(*(pick(x, idx) for x in (ls.p, ls.m, ls.v, ls.g, ls.p_lp))) for k, idx in groups.items()}
    refs = {i: dict(p=host_f32(ls.p[i]), m=host_f32(ls.m[i]), v=host_f32(ls.v[i]), lp=synth.bits16(ls.p_lp[i]),
                    pdt="bf16") for i in range(len(shapes))}
    # oracle: per-group sums in list order, added in group order; one clip coefficient for all
    ss_groups = [sum(oracle.overflow_norm(host_grad(ls.g[i]), "bf16")[1] for i in groups[k]) for k in ("large", "small")]
    ss_ref = ss_groups[0] + ss_groups[1]
    c_ref = oracle.clip_coef(ss_ref, float(np.float32(cfg.max_norm)))
    assert c_ref < 1
    for k, idx in groups.items():
        h = oracle.hyper(hy[k]["lr"], cfg.beta1, cfg.beta2, cfg.eps, hy[k]["wd"], 1)
        for i in idx:
            r = refs[i]
            r["lp"] = oracle.adamw_step(r["p"], r["m"], r["v"], host_grad(ls.g[i]), "bf16", "bf16", h, 42, 1.0, float(c_ref))
    ws, parts, res = ma.workspace(), ma.new_result(2), ma.new_result()
    for j, k in enumerate(("large", "small")):
        ma.multi_overflow_norm(plans[k], 1.0, parts, ws, index=j)
    ma.norm_combine(parts, 2, res)
    for k in ("large", "small"):
        ma.multi_adamw_step_gated(plans[k], ma.hyper(hy[k]["lr"], cfg.beta1, cfg.beta2, cfg.eps, hy[k]["wd"], 1),
                                  42, 1.0, res, cfg.max_norm)
    ov, ss = ma.read_result(res)
    assert not ov and abs(ss - ss_ref) <= 1e-12 * ss_ref
    assert np.float32(ma.clip_coef(ss, cfg.max_norm)) == c_ref
    for i in range(len(shapes)):
        got = dict(p=host_f32(ls.p[i]), m=host_f32(ls.m[i]), v=host_f32(ls.v[i]), lp=synth.bits16(ls.p_lp[i]))
        assert_state_close(got, refs[i], "tensor %d (%s)" % (i, shapes[i][0]))
    # an overflow in one norm vector: the combined result gates BOTH groups
    ls.g[small[0]].view(torch.int16)[0] = 0x7F81                         # a NaN pattern of bf16
    before = ls.flat.arena.cpu().numpy().tobytes()
    for j, k in enumerate(("large", "small")):
        ma.multi_overflow_norm(plans[k], 1.0, parts, ws, index=j)
    ma.norm_combine(parts, 2, res)
    for k in ("large", "small"):
        ma.multi_adamw_step_gated(plans[k], ma.hyper(hy[k]["lr"], cfg.beta1, cfg.beta2, cfg.eps, hy[k]["wd"], 1),
                                  43, 1.0, res, cfg.max_norm)
    assert ma.read_result(res)[0] is True
    assert ls.flat.arena.cpu().numpy().tobytes() == before


def test_several_steps_track_the_oracle():
    """Ten consecutive steps with fresh gradients: the two trajectories stay within the bar at
    every step (they are bit-identical as long as the clip coefficients agree)."""
    n = 40_003
    cfg = synth.FlatConfig("t", n, seed=81, m_std=0, v_std=0, max_norm=0.5)
    st = synth.make_flat(cfg, device="cuda")
    ref = _host_state(st, "bf16")
    ws, res = ma.workspace(), ma.new_result()
    gen = torch.Generator(device="cuda")
    gen.manual_seed(82)
    for t in range(1, 11):
        st.g.copy_(torch.randn(n, device="cuda", generator=gen) * 1e-2)
        g_host = host_grad(st.g)
        oracle.optimizer_step(ref["p"], ref["m"], ref["v"], g_host, "bf16", ref["lp"], "bf16",
                              oracle_hyper(cfg), t, 1.0, cfg.max_norm)
        ma.overflow_norm(st.g, 1.0, res, ws)
        ma.adamw_step_gated(st.p, st.m, st.v, st.g, st.p_lp, _hyper(cfg), t, 1.0, res, cfg.max_norm)
        assert_state_close(_host_state(st, "bf16"), ref, "step %d" % t)


def test_two_sub_groups_on_two_streams():
    """The library keeps no state of its own between calls: two sub-groups, each with its own
    workspace and result slot, stepped concurrently on two non-default streams (three iterations,
    calls interleaved) end exactly where the oracle puts each of them."""
    sizes = (2_000_003, 1_500_001)
    cfgs = [synth.FlatConfig("s%d" % k, n, seed=60 + k, gdt=("bf16", "f16")[k], m_std=1e-4, v_std=1e-8,
                             step=10, loss_scale=(1.0, 1024.0)[k], max_norm=(0.02, 0.5)[k])
            for k, n in enumerate(sizes)]
    sts = [synth.make_flat(c, device="cuda") for c in cfgs]
    refs = [_host_state(st, "bf16") for st in sts]
    g_hosts = [host_grad(st.g) for st in sts]
    for k, c in enumerate(cfgs):
        for it in range(3):
            ov, _, _ = oracle.optimizer_step(refs[k]["p"], refs[k]["m"], refs[k]["v"], g_hosts[k], c.gdt,
                                             refs[k]["lp"], "bf16", oracle_hyper(c), 10 + it, c.loss_scale,
                                             c.max_norm)
            assert not ov
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    wss = [ma.workspace(), ma.workspace()]
    ress = [ma.new_result(), ma.new_result()]
    for it in range(3):
        for k, (c, st) in enumerate(zip(cfgs, sts)):
            ma.overflow_norm(st.g, c.loss_scale, ress[k], wss[k], stream=streams[k])
        for k, (c, st) in enumerate(zip(cfgs, sts)):
            ma.adamw_step_gated(st.p, st.m, st.v, st.g, st.p_lp, _hyper(c), 10 + it, c.loss_scale, ress[k],
                                c.max_norm, stream=streams[k])
    torch.cuda.synchronize()
    for k, st in enumerate(sts):
        assert_state_close(_host_state(st, "bf16"), refs[k], "stream %d" % k)


def test_four_host_threads_on_four_streams():
    """The entry points may be called from several host threads at once (the error message is per
    thread, the per-device caches are guarded): four threads, each with its own sub-group, stream,
    workspace and result slot, run 20 iterations of scan + gated step concurrently, one of them through
    the whole-step call and one through a prepared list; every sub-group ends where the oracle puts it."""
    import threading
    sizes = (300_007, 1_000_003, 65_536, 2_000_001)
    cfgs = [synth.FlatConfig("t%d" % k, n, seed=160 + k, gdt=("bf16", "f16", "bf16", "f16")[k], m_std=1e-4,
                             v_std=1e-8, step=3, loss_scale=(1.0, 256.0, 1.0, 1024.0)[k], max_norm=(0.02, 0.5, 0.0, 0.1)[k])
            for k, n in enumerate(sizes)]
    sts = [synth.make_flat(c, device="cuda") for c in cfgs]
    refs = [_host_state(st, "bf16") for st in sts]
    iters = 20
    for k, c in enumerate(cfgs):
        g = host_grad(sts[k].g)
        for it in range(iters):
            ov, _, _ = oracle.optimizer_step(refs[k]["p"], refs[k]["m"], refs[k]["v"], g, c.gdt, refs[k]["lp"], "bf16",
                                             oracle_hyper(c), 3 + it, c.loss_scale, c.max_norm)
            assert not ov
    plan = ma.MultiPlan([sts[3].p], [sts[3].m], [sts[3].v], [sts[3].g], [sts[3].p_lp])
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in sizes]
    wss = [ma.workspace() for _ in sizes]
    ress = [ma.new_result() for _ in sizes]
    errors, start = [], threading.Barrier(len(sizes))

    def work(k):
        try:
            c, st = cfgs[k], sts[k]
            start.wait()
            for it in range(iters):
                if k == 2:
                    ma.optimizer_step(st.p, st.m, st.v, st.g, st.p_lp, _hyper(c), 3 + it, c.loss_scale, c.max_norm,
                                      ress[k], wss[k], stream=streams[k])
                elif k == 3:
                    ma.multi_overflow_norm(plan, c.loss_scale, ress[k], wss[k], stream=streams[k])
                    ma.multi_adamw_step_gated(plan, _hyper(c), 3 + it, c.loss_scale, ress[k], c.max_norm, stream=streams[k])
                else:
                    ma.overflow_norm(st.g, c.loss_scale, ress[k], wss[k], stream=streams[k])
                    ma.adamw_step_gated(st.p, st.m, st.v, st.g, st.p_lp, _hyper(c), 3 + it, c.loss_scale, ress[k],
                                        c.max_norm, stream=streams[k])
        except Exception as e:      # noqa: BLE001 - reported by the main thread
            errors.append((k, repr(e)))

    threads = [threading.Thread(target=work, args=(k,)) for k in range(len(sizes))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for k, st in enumerate(sts):
        assert_state_close(_host_state(st, "bf16"), refs[k], "thread %d" % k)


def test_multi_list_repeated_launches():
    """A 1/512-scale 8B-shaped list (about 4000 work items), four iterations on one plan, the third
    one skipped by an overflow: every element is updated exactly once per applied iteration and the
    counters at the head of the plan's table read zero after every launch.  (Lists of this size keep
    fixed shares; tests/test_gpu_fullsize.py has the same at a size that draws late items on demand.)"""
    shapes = synth.scaled_shapes(synth.llama3_8b_shapes(), 512, ragged=True)
    cfg = synth.FlatConfig("t", 0, seed=77, m_std=1e-4, v_std=1e-8, step=100, max_norm=0.3)
    ls = synth.make_list(shapes, cfg, device="cuda", align_elems=1)
    refs = [dict(p=host_f32(ls.p[i]), m=host_f32(ls.m[i]), v=host_f32(ls.v[i]), lp=synth.bits16(ls.p_lp[i]),
                 pdt="bf16") for i in range(len(shapes))]
    g_hosts = [host_grad(g) for g in ls.g]
    ss_ref = sum(oracle.overflow_norm(g, "bf16")[1] for g in g_hosts)
    c_ref = oracle.clip_coef(ss_ref, float(np.float32(cfg.max_norm)))
    plan = ma.MultiPlan(ls.p, ls.m, ls.v, ls.g, ls.p_lp)
    assert plan.plan.step_chunks > 3000
    ws, res = ma.workspace(), ma.new_result()
    head = lambda: plan.table[:64].view(torch.int32).cpu().tolist()
    assert head() == [0] * 16
    step = 100
    for it in range(4):
        if it == 2:       # an overflow: the launch returns before any block touches the counters
            keep = ls.g[3].view(torch.int16)[5].item()
            ls.g[3].view(torch.int16)[5] = 0x7F80
        ma.multi_overflow_norm(plan, 1.0, res, ws)
        ma.multi_adamw_step_gated(plan, _hyper(cfg), step, 1.0, res, cfg.max_norm)
        ov, ss = ma.read_result(res)
        assert head() == [0] * 16, it
        if it == 2:
            assert ov
            ls.g[3].view(torch.int16)[5] = keep
            continue
        assert not ov and abs(ss - ss_ref) <= 1e-12 * ss_ref
        for r, g in zip(refs, g_hosts):
            r["lp"] = oracle.adamw_step(r["p"], r["m"], r["v"], g, "bf16", "bf16", oracle_hyper(cfg), step,
                                        1.0, float(c_ref), nthreads=8)
        step += 1
        for i in range(len(shapes)):
            got = dict(p=host_f32(ls.p[i]), m=host_f32(ls.m[i]), v=host_f32(ls.v[i]), lp=synth.bits16(ls.p_lp[i]))
            assert_state_close(got, refs[i], "iteration %d, tensor %d (%s)" % (it, i, shapes[i][0]))


def test_randomised_sizes_alignments_and_hyper_parameters():
    """150 seeded random cases of the flat scan + gated update: sizes from 0 to 4e5, every buffer at
    its own element offset from an aligned base (0..8), all gradient and copy dtypes, hyper-parameters
    over several decades, loss scales 1..65536, with and without clipping.  p, m, v must equal the
    oracle's bit for bit (and the copy with them); the sum of squares to 1e-11 (fp64 on both sides,
    different summation order)."""
    rng = np.random.default_rng(20250527)
    ws = ma.workspace()
    for case in range(150):
        n = int(rng.choice([rng.integers(0, 64), rng.integers(64, 5000), rng.integers(5000, 40000),
                            rng.integers(40000, 400000)]))
        gdt = str(rng.choice(["bf16", "f16", "f32"]))
        pdt = str(rng.choice(["bf16", "f16"]))
        offs = [int(rng.integers(0, 9)) for _ in range(5)]
        if rng.random() < 0.5:
            offs = [offs[0]] * 5
        S = float(2.0 ** rng.integers(0, 17)) if gdt != "f32" else 1.0
        cfg = synth.FlatConfig("z", n, seed=int(rng.integers(1 << 30)), gdt="bf16" if gdt == "f32" else gdt, pdt=pdt,
                               loss_scale=S, m_std=float(10 ** rng.uniform(-6, -2)),
                               v_std=float(10 ** rng.uniform(-10, -4)), g_std=float(10 ** rng.uniform(-6, -1)),
                               step=int(rng.choice([1, 2, 7, 100, 100000])), lr=float(10 ** rng.uniform(-6, -1)),
                               beta1=float(rng.choice([0.0, 0.5, 0.9, 0.99])),
                               beta2=float(rng.choice([0.0, 0.9, 0.999, 0.9999])), eps=float(10 ** rng.uniform(-10, -3)),
                               weight_decay=float(rng.choice([0.0, 0.01, 0.3])),
                               max_norm=float(rng.choice([0.0, 0.01, 1.0, 100.0])))
        st = synth.make_flat(cfg, device="cuda", n=n)

        def view(t, o):
            base = torch.zeros(n + 16, dtype=t.dtype, device="cuda")
            base[o:o + n].copy_(t)
            return base[o:o + n]

        g = st.g if gdt != "f32" else st.g.to(torch.float32) * 1.7
        p, m, v, g, lp = (view(t, o) for t, o in zip((st.p, st.m, st.v, g, st.p_lp), offs))
        ref = dict(p=host_f32(p), m=host_f32(m), v=host_f32(v), lp=synth.bits16(lp), pdt=pdt)
        ov_ref, ss_ref, _ = oracle.optimizer_step(ref["p"], ref["m"], ref["v"], host_grad(g), gdt, ref["lp"], pdt,
                                                  oracle_hyper(cfg), cfg.step, S, cfg.max_norm)
        res = ma.new_result()
        ma.overflow_norm(g, S, res, ws)
        ma.adamw_step_gated(p, m, v, g, lp, _hyper(cfg), cfg.step, S, res, cfg.max_norm)
        ov, ss = ma.read_result(res)
        what = "case %d: n=%d gdt=%s pdt=%s offsets=%s %r" % (case, n, gdt, pdt, offs, cfg)
        assert ov == ov_ref is False, what
        assert abs(ss - ss_ref) <= 1e-11 * ss_ref, what
        got = dict(p=host_f32(p), m=host_f32(m), v=host_f32(v), lp=synth.bits16(lp))
        for k in ("p", "m", "v"):
            assert np.array_equal(got[k].view(np.uint32), ref[k].view(np.uint32)), (k, what)
        assert np.array_equal(got["lp"], ref["lp"]), what


def test_list_of_twenty_thousand_tiny_tensors():
    """Many small tensors (0 to 300 elements each, packed back to back, so nearly every one starts off
    the packet grid): one work item per tensor, a table of 20,000 rows searched on the scalar unit.
    Since the tensors tile the flat buffers without gaps the oracle runs once over the flat state."""
    rng = np.random.default_rng(777)
    sizes = rng.integers(0, 301, 20_000).tolist()
    sizes[17] = 5000                                                  # and one that spans two work items
    shapes = [("t%d" % i, int(k)) for i, k in enumerate(sizes)]
    cfg = synth.FlatConfig("tiny", 0, seed=91, m_std=1e-4, v_std=1e-8, step=12, max_norm=0.05, gdt="f16",
                           loss_scale=64.0)
    ls = synth.make_list(shapes, cfg, device="cuda", align_elems=1)
    fl = ls.flat
    total = sum(sizes)
    assert fl.p.numel() == total
    ref = dict(p=host_f32(fl.p), m=host_f32(fl.m), v=host_f32(fl.v), lp=synth.bits16(fl.p_lp), pdt="bf16")
    g_host = host_grad(fl.g)
    ov_ref, ss_ref = oracle.overflow_norm(g_host, "f16", 64.0)
    c_ref = oracle.clip_coef(ss_ref, float(np.float32(cfg.max_norm)))
    assert not ov_ref and c_ref < 1
    ref["lp"] = oracle.adamw_step(ref["p"], ref["m"], ref["v"], g_host, "f16", "bf16", oracle_hyper(cfg), 12, 64.0,
                                  float(c_ref))
    plan = ma.MultiPlan(ls.p, ls.m, ls.v, ls.g, ls.p_lp)
    assert plan.total == total and plan.plan.entries == sum(1 for k in sizes if k > 0)
    ws, res = ma.workspace(), ma.new_result()
    ma.multi_overflow_norm(plan, 64.0, res, ws)
    ma.multi_adamw_step_gated(plan, _hyper(cfg), 12, 64.0, res, cfg.max_norm)
    ov, ss = ma.read_result(res)
    assert not ov and abs(ss - ss_ref) <= 1e-11 * ss_ref          # per-tensor partial sums: another order than the oracle's
    assert np.float32(ma.clip_coef(ss, cfg.max_norm)) == c_ref
    got = dict(p=host_f32(fl.p), m=host_f32(fl.m), v=host_f32(fl.v), lp=synth.bits16(fl.p_lp))
    assert_state_close(got, ref, "20,000 tiny tensors")
    for k in ("p", "m", "v"):
        assert np.array_equal(got[k].view(np.uint32), ref[k].view(np.uint32)), k
    # the whole-step call over the same plan, and a NaN in a one-element tensor skipping everything
    ma.multi_optimizer_step(plan, _hyper(cfg), 13, 64.0, cfg.max_norm, res, ws)
    ref["lp"] = oracle.adamw_step(ref["p"], ref["m"], ref["v"], g_host, "f16", "bf16", oracle_hyper(cfg), 13, 64.0,
                                  float(c_ref))
    assert_state_close(dict(p=host_f32(fl.p), m=host_f32(fl.m), v=host_f32(fl.v), lp=synth.bits16(fl.p_lp)), ref,
                       "second step, one call")
    one = next(i for i, k in enumerate(sizes) if k == 1)
    ls.g[one].view(torch.int16)[0] = 0x7E00
    before = fl.arena.cpu().numpy().tobytes()
    ma.multi_optimizer_step(plan, _hyper(cfg), 14, 64.0, cfg.max_norm, res, ws)
    assert ma.read_result(res)[0] is True and fl.arena.cpu().numpy().tobytes() == before


def test_randomised_tensor_lists():
    """40 seeded random tensor lists: 1 to 40 tensors of 0 to 60,000 elements, each of the five buffers
    of each tensor at its own element offset (so rows with every combination of packet-path and
    scalar-path alignment meet in one launch), both gradient dtypes, with the parameter copy or
    without; p, m, v and the copy bit for bit against the oracle run tensor by tensor."""
    rng = np.random.default_rng(4242)
    ws = ma.workspace()
    tensors = elements = 0
    for case in range(40):
        count = int(rng.integers(1, 41))
        gdt = str(rng.choice(["bf16", "f16", "f32"]))
        pdt = str(rng.choice(["bf16", "f16"]))
        with_lp = bool(rng.random() < 0.8)
        S = float(2.0 ** rng.integers(0, 12)) if gdt != "f32" else 1.0
        cfg = synth.FlatConfig("z", 0, seed=int(rng.integers(1 << 30)), gdt="bf16" if gdt == "f32" else gdt, pdt=pdt,
                               loss_scale=S, m_std=1e-4, v_std=1e-8, step=int(rng.integers(1, 50)),
                               lr=float(10 ** rng.uniform(-5, -2)), max_norm=float(rng.choice([0.0, 0.05, 10.0])))
        P, M, V, G, L = [], [], [], [], []
        for k in range(count):
            n = int(rng.choice([0, rng.integers(1, 9), rng.integers(9, 5000), rng.integers(5000, 60000)]))
            st = synth.make_flat(synth.FlatConfig(**{**cfg.__dict__, "seed": cfg.seed + k, "n": n}), device="cuda", n=n)
            same = rng.random() < 0.5
            o0 = int(rng.integers(0, 9))

            def view(t):
                o = o0 if same else int(rng.integers(0, 9))
                base = torch.zeros(n + 16, dtype=t.dtype, device="cuda")
                base[o:o + n].copy_(t)
                return base[o:o + n]

            g = st.g if gdt != "f32" else st.g.to(torch.float32) * 0.9
            for lst, t in ((P, st.p), (M, st.m), (V, st.v), (G, g), (L, st.p_lp)):
                lst.append(view(t))
        refs = [dict(p=host_f32(P[k]), m=host_f32(M[k]), v=host_f32(V[k]), lp=synth.bits16(L[k]), pdt=pdt)
                for k in range(count)]
        g_hosts = [host_grad(g) for g in G]
        ss_ref = sum(oracle.overflow_norm(g, gdt, S)[1] for g in g_hosts)
        c_ref = oracle.clip_coef(ss_ref, float(np.float32(cfg.max_norm)))
        for r, g in zip(refs, g_hosts):
            new_lp = oracle.adamw_step(r["p"], r["m"], r["v"], g, gdt, pdt, oracle_hyper(cfg), cfg.step, S, float(c_ref))
            if with_lp:
                r["lp"] = new_lp
        plan = ma.MultiPlan(P, M, V, G, L if with_lp else None)
        res = ma.new_result()
        ma.multi_overflow_norm(plan, S, res, ws)
        ma.multi_adamw_step_gated(plan, _hyper(cfg), cfg.step, S, res, cfg.max_norm)
        ov, ss = ma.read_result(res)
        what = "case %d: %d tensors, gdt=%s pdt=%s copy=%s" % (case, count, gdt, pdt, with_lp)
        assert not ov and abs(ss - ss_ref) <= 1e-11 * max(ss_ref, 1e-300), what
        assert np.float32(ma.clip_coef(ss, cfg.max_norm)) == c_ref, what
        for k in range(count):
            for name, t in (("p", P[k]), ("m", M[k]), ("v", V[k])):
                assert np.array_equal(host_f32(t).view(np.uint32), refs[k][name].view(np.uint32)), (what, k, name)
            assert np.array_equal(synth.bits16(L[k]), refs[k]["lp"]), (what, k, "copy")
        tensors += count
        elements += plan.total
    assert tensors > 400 and elements > 3_000_000       # the draw really covers what the docstring says
