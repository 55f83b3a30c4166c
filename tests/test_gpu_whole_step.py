"""GPU parity of the whole step in one call (ma_optimizer_step, ma_multi_optimizer_step: scan launch +
update launch that adds up the scan's partials itself) against the oracle's scan + gate + update, and
bit for bit against the separate calls."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2505_23254_amd import synth
from tests._util import SUMSQ_RTOL, assert_state_close, host_f32, host_grad, oracle_hyper

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


SIZES = [0, 1, 3, 4, 5, 63, 1023, 4095, 4096, 4097, 8191, 100_003, 1 << 20, (1 << 20) + 7, 3_000_001, 20_000_003]


@pytest.mark.parametrize("gdt,pdt", [("bf16", "bf16"), ("f16", "f16"), ("f16", "bf16")])
def test_whole_step_sizes(gdt, pdt):
    """Empty to 2e7 elements (one partial to the scan's full grid of partials, ragged tails), with
    clipping, two steps in a row on one workspace that starts out filled with garbage."""
    ws = ma.workspace()
    ws.fill_(0xA5)
    S = 1.0 if gdt == "bf16" else 1024.0
    for n in SIZES:
        cfg = synth.FlatConfig("t", n, seed=200 + n % 89, gdt=gdt, pdt=pdt, loss_scale=S, m_std=1e-4, v_std=1e-8,
                               step=100, max_norm=0.01)
        st = synth.make_flat(cfg, device="cuda")
        g_host = host_grad(st.g)
        ref = _host_state(st, pdt)
        res = ma.new_result()
        for step in (100, 101):
            ov_ref, ss_ref, c_ref = oracle.optimizer_step(ref["p"], ref["m"], ref["v"], g_host, gdt, ref["lp"], pdt,
                                                          oracle_hyper(cfg), step, S, cfg.max_norm)
            ma.optimizer_step(st.p, st.m, st.v, st.g, st.p_lp, _hyper(cfg), step, S, cfg.max_norm, res, ws)
            ov, ss = ma.read_result_raw(res)
            assert ov == 0 and not ov_ref, (n, ov)
            if n:
                assert abs(ss - ss_ref) <= SUMSQ_RTOL * ss_ref, (n, ss, ss_ref)
                # both sides accumulate in fp64; beyond 1e7 terms the oracle's index-order sum itself
                # carries a few 1e-12 of rounding
                assert abs(ss - ss_ref) <= (1e-12 if n <= 10 ** 7 else 1e-11) * ss_ref, (n, ss, ss_ref)
                assert np.float32(ma.clip_coef(ss, cfg.max_norm)) == c_ref
            else:
                assert ss == 0.0
            assert_state_close(_host_state(st, pdt), ref, "n=%d step=%d" % (n, step))
            assert np.array_equal(host_grad(st.g), g_host)


@pytest.mark.parametrize("n", [5, (1 << 20) + 5, 30_000_001])
def test_whole_step_equals_the_separate_calls_bit_for_bit(n):
    cfg = synth.FlatConfig("t", n, seed=7, m_std=1e-4, v_std=1e-8, step=50, max_norm=0.02)
    a, b = synth.make_flat(cfg, device="cuda"), synth.make_flat(cfg, device="cuda")
    ws, ra, rb = ma.workspace(), ma.new_result(), ma.new_result()
    ma.optimizer_step(a.p, a.m, a.v, a.g, a.p_lp, _hyper(cfg), 50, 1.0, cfg.max_norm, ra, ws)
    ma.overflow_norm(b.g, 1.0, rb, ws)
    ma.adamw_step_gated(b.p, b.m, b.v, b.g, b.p_lp, _hyper(cfg), 50, 1.0, rb, cfg.max_norm)
    torch.cuda.synchronize()
    assert torch.equal(ra.view(torch.int64), rb.view(torch.int64))         # the 16 result bytes
    for x, y in ((a.p, b.p), (a.m, b.m), (a.v, b.v)):
        assert torch.equal(x.view(torch.int32), y.view(torch.int32))
    assert torch.equal(a.p_lp.view(torch.int16), b.p_lp.view(torch.int16))


@pytest.mark.parametrize("gdt", ["bf16", "f16"])
def test_whole_step_skips_on_overflow(gdt):
    n = 700_001
    cfg = synth.FlatConfig("t", n, seed=11, gdt=gdt, m_std=1e-4, v_std=1e-8, max_norm=1.0,
                           loss_scale=1.0 if gdt == "bf16" else 512.0)
    ws, res = ma.workspace(), ma.new_result()
    for pos in (0, 4095, 4096, n // 2, n - 1):
        st = synth.make_flat(cfg, device="cuda")
        for k, bits in enumerate(synth.NONFINITE_BITS[gdt]):
            keep = [t.clone() for t in (st.p, st.m, st.v, st.p_lp)]
            st.g.view(torch.int16)[pos] = bits - 0x10000 if bits >= 0x8000 else bits
            assert oracle.overflow_norm(host_grad(st.g), gdt, cfg.loss_scale)[0] is True
            ma.optimizer_step(st.p, st.m, st.v, st.g, st.p_lp, _hyper(cfg), 3, cfg.loss_scale, 1.0, res, ws)
            assert ma.read_result_raw(res)[0] == 1, (pos, k)
            for a, b in zip(keep, (st.p, st.m, st.v, st.p_lp)):
                assert torch.equal(a.view(torch.int16), b.view(torch.int16))


@pytest.mark.parametrize("offsets", [(1, 1, 1, 1, 1), (3, 3, 3, 3, 3), (2, 2, 2, 6, 10), (0, 1, 0, 0, 0), (1, 0, 2, 3, 5)])
def test_whole_step_on_misaligned_views(offsets):
    n = 50_000
    cfg = synth.FlatConfig("t", n + 16, seed=13, gdt="f16", pdt="f16", loss_scale=256.0, m_std=1e-4, v_std=1e-8,
                           max_norm=0.05)
    st = synth.make_flat(cfg, device="cuda")
    p, m, v, g, lp = (t[o:o + n] for t, o in zip((st.p, st.m, st.v, st.g, st.p_lp), offsets))
    ref = dict(p=host_f32(p), m=host_f32(m), v=host_f32(v), lp=synth.bits16(lp), pdt="f16")
    g_host = host_grad(g)
    oracle.optimizer_step(ref["p"], ref["m"], ref["v"], g_host, "f16", ref["lp"], "f16", oracle_hyper(cfg), 9, 256.0, 0.05)
    edge = [t.clone() for t in (st.p, st.m, st.v, st.p_lp)]
    ws, res = ma.workspace(), ma.new_result()
    ma.optimizer_step(p, m, v, g, lp, _hyper(cfg), 9, 256.0, 0.05, res, ws)
    assert ma.read_result_raw(res)[0] == 0
    got = dict(p=host_f32(p), m=host_f32(m), v=host_f32(v), lp=synth.bits16(lp))
    assert_state_close(got, ref, str(offsets))
    for t, e, o in zip((st.p, st.m, st.v, st.p_lp), edge, offsets[:3] + offsets[4:]):      # nothing outside the views
        assert torch.equal(t[:o].view(torch.int16), e[:o].view(torch.int16))
        assert torch.equal(t[o + n:].view(torch.int16), e[o + n:].view(torch.int16))


def test_whole_step_two_streams_and_a_graph():
    """Forty calls in a row on two streams with a workspace each, then one captured call replayed three
    times with eager work between the replays; every result against the oracle."""
    n = 300_003
    cfgs = [synth.FlatConfig("t", n, seed=21 + k, m_std=1e-4, v_std=1e-8, max_norm=0.05) for k in range(2)]
    sts = [synth.make_flat(c, device="cuda") for c in cfgs]
    refs = [_host_state(s, "bf16") for s in sts]
    gh = [host_grad(s.g) for s in sts]
    wss, ress = [ma.workspace() for _ in range(2)], [ma.new_result() for _ in range(2)]
    streams = [torch.cuda.Stream() for _ in range(2)]
    torch.cuda.synchronize()
    for step in range(1, 41):
        for k in range(2):
            with torch.cuda.stream(streams[k]):
                ma.optimizer_step(sts[k].p, sts[k].m, sts[k].v, sts[k].g, sts[k].p_lp, _hyper(cfgs[k]), step, 1.0,
                                  0.05, ress[k], wss[k])
    torch.cuda.synchronize()
    for k in range(2):
        for step in range(1, 41):
            oracle.optimizer_step(refs[k]["p"], refs[k]["m"], refs[k]["v"], gh[k], "bf16", refs[k]["lp"], "bf16",
                                  oracle_hyper(cfgs[k]), step, 1.0, 0.05)
        assert ma.read_result_raw(ress[k])[0] == 0
        assert_state_close(_host_state(sts[k], "bf16"), refs[k], "stream %d after 40 calls" % k)
    st, ref, cfg, ws, res = sts[0], refs[0], cfgs[0], wss[0], ress[0]
    graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        ma.optimizer_step(st.p, st.m, st.v, st.g, st.p_lp, _hyper(cfg), 41, 1.0, 0.05, res, ws)
    torch.cuda.synchronize()
    for it in range(3):
        graph.replay()
        torch.cuda.synchronize()
        oracle.optimizer_step(ref["p"], ref["m"], ref["v"], gh[0], "bf16", ref["lp"], "bf16", oracle_hyper(cfg), 41, 1.0, 0.05)
        assert_state_close(_host_state(st, "bf16"), ref, "replay %d" % it)
        _ = (st.p[:1000] * 2).sum().item()


@pytest.mark.parametrize("align_elems", [64, 1])
def test_whole_step_over_a_tensor_list(align_elems):
    """ma_multi_optimizer_step on a miniature of the 8B list (ragged tensors, packed back to back when
    align_elems = 1): against the oracle, bit for bit against the separate list calls, and skipped as a
    whole when one tensor holds a NaN."""
    shapes = synth.scaled_shapes(synth.llama3_8b_shapes(), 2000, ragged=True)
    cfg = synth.FlatConfig("t", 0, seed=41, m_std=1e-4, v_std=1e-8, step=7, max_norm=0.05)
    a = synth.make_list(shapes, cfg, device="cuda", align_elems=align_elems)
    b = synth.make_list(shapes, cfg, device="cuda", align_elems=align_elems)
    pa, pb = ma.MultiPlan(a.p, a.m, a.v, a.g, a.p_lp), ma.MultiPlan(b.p, b.m, b.v, b.g, b.p_lp)
    ws, ra, rb = ma.workspace(), ma.new_result(), ma.new_result()
    refs = [dict(p=host_f32(a.p[i]), m=host_f32(a.m[i]), v=host_f32(a.v[i]), lp=synth.bits16(a.p_lp[i]), pdt="bf16")
            for i in range(len(shapes))]
    g_hosts = [host_grad(g) for g in a.g]
    ss_ref = sum(oracle.overflow_norm(g, "bf16", 1.0)[1] for g in g_hosts)
    c_ref = oracle.clip_coef(ss_ref, cfg.max_norm)
    assert c_ref < 1
    ma.multi_optimizer_step(pa, _hyper(cfg), 7, 1.0, cfg.max_norm, ra, ws)
    ma.multi_overflow_norm(pb, 1.0, rb, ws)
    ma.multi_adamw_step_gated(pb, _hyper(cfg), 7, 1.0, rb, cfg.max_norm)
    torch.cuda.synchronize()
    assert torch.equal(ra.view(torch.int64), rb.view(torch.int64))
    ov, ss = ma.read_result_raw(ra)
    assert ov == 0 and abs(ss - ss_ref) <= 1e-12 * ss_ref and np.float32(ma.clip_coef(ss, cfg.max_norm)) == c_ref
    for i in range(len(shapes)):
        refs[i]["lp"] = oracle.adamw_step(refs[i]["p"], refs[i]["m"], refs[i]["v"], g_hosts[i], "bf16", "bf16",
                                          oracle_hyper(cfg), 7, 1.0, float(c_ref))
        got = dict(p=host_f32(a.p[i]), m=host_f32(a.m[i]), v=host_f32(a.v[i]), lp=synth.bits16(a.p_lp[i]))
        assert_state_close(got, refs[i], "tensor %d" % i)
        for x, y in ((a.p[i], b.p[i]), (a.m[i], b.m[i]), (a.v[i], b.v[i])):
            assert torch.equal(x.view(torch.int32), y.view(torch.int32))
    keep = a.flat.p.clone()
    a.g[17].view(torch.int16)[3] = 0x7FC0
    ma.multi_optimizer_step(pa, _hyper(cfg), 8, 1.0, cfg.max_norm, ra, ws)
    assert ma.read_result_raw(ra)[0] == 1
    assert torch.equal(keep.view(torch.int32), a.flat.p.view(torch.int32))


def test_whole_step_argument_errors_come_before_any_launch():
    ws, res = ma.workspace(), ma.new_result()
    cfg = synth.FlatConfig("t", 4096, seed=1)
    st = synth.make_flat(cfg, device="cuda")
    res.fill_(7.0)
    torch.cuda.synchronize()
    for kw in (dict(step=0), dict(ws=ws[:1024])):
        with pytest.raises(ma.MaError) as e:
            ma.optimizer_step(st.p, st.m, st.v, st.g, st.p_lp, _hyper(cfg), kw.get("step", 1), 1.0, 1.0, res,
                              kw.get("ws", ws))
        assert e.value.code == ma.MA_ERR_ARG
    with pytest.raises(ma.MaError) as e:            # p_lp overlapping the gradient
        ma.optimizer_step(st.p, st.m, st.v, st.g, st.g.view(torch.bfloat16), _hyper(cfg), 1, 1.0, 1.0, res, ws)
    assert e.value.code == ma.MA_ERR_ARG and "overlap" in str(e.value)
    torch.cuda.synchronize()
    assert res.tolist() == [7.0, 7.0]               # nothing ran
