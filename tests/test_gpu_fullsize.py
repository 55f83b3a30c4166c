"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

Flat configurations up to 10^8 elements, the 8B-shaped list (8.03e9 elements, in the layout and
placement the benchmark times) and all four sub-groups of the 14B-class list (12.57e9 elements) are
compared with the oracle on EVERY element (the large ones in slabs streamed through the host).  The
8B list in its other layout, a flat sub-group just beyond 2^31 elements, and the 8.03e9-element
bf16-state and accumulation workloads are compared on samples the oracle can compute one by one --
the first and last 65,536 elements of every tensor, both sides of every sub-group cut and of element
2^32, and seeded random blocks -- while the overflow flag and the sum of squares are checked over
ALL elements.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_23254_amd import hbm, synth
from tests._util import SUMSQ_RTOL, FullCompare, assert_state_close, host_f32, host_grad, oracle_hyper

pytestmark = pytest.mark.gpu

EDGE = 65_536
THREADS = 16
SLAB = 1 << 27          # elements per slab of a full comparison
ma = None


@pytest.fixture(scope="module", autouse=True)
def _lib():
    global ma
    from paper_2505_23254_amd import binding
    ma = binding
    assert torch.cuda.is_available()
    yield
    torch.cuda.empty_cache()


@pytest.fixture(autouse=True)
def _release_hbm():
    """Hand cached blocks back between tests: the large cases need most of the device."""
    import gc
    gc.collect()
    torch.cuda.empty_cache()
    yield
    gc.collect()
    torch.cuda.empty_cache()


def _need_gib(gib):
    free, _ = torch.cuda.mem_get_info()
    if free < gib * 2 ** 30:
        pytest.skip("needs %.0f GiB of free HBM, device has %.0f" % (gib, free / 2 ** 30))


def _hyper(cfg):
    return ma.hyper(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, cfg.weight_decay, 1)


def _oracle_norm_all(g: torch.Tensor, gdt: str, scale: float, piece: int = 1 << 28):
    """Oracle flag and sum of squares over a whole device gradient, streamed through the host."""
    ov, ss = False, 0.0
    for a in range(0, g.numel(), piece):
        o, s = oracle.overflow_norm(host_grad(g[a:a + piece]), gdt, scale, nthreads=THREADS)
        ov, ss = ov or o, ss + s
    return ov, ss


def _merge(ranges, n):
    out = []
    for a, b in sorted((max(0, a), min(n, b)) for a, b in ranges):
        if a >= b:
            continue
        if out and a <= out[-1][1]:
            out[-1][1] = max(out[-1][1], b)
        else:
            out.append([a, b])
    return out


def _gather(t: torch.Tensor, ranges):
    return torch.cat([t[a:b] for a, b in ranges])


def _sample_state(fl, ranges, pdt):
    return dict(p=host_f32(_gather(fl.p, ranges)), m=host_f32(_gather(fl.m, ranges)),
                v=host_f32(_gather(fl.v, ranges)), lp=synth.bits16(_gather(fl.p_lp, ranges)), pdt=pdt)


def _checksums(fl):
    return [int(t.view(torch.int32 if t.element_size() == 4 else torch.int16).sum(dtype=torch.int64))
            for t in (fl.p, fl.m, fl.v, fl.p_lp)]


@pytest.mark.parametrize("name", ["c2", "c3a"])
def test_flat_configs_elementwise(name):
    cfg = synth.config(name)
    st = synth.make_flat(cfg, device="cuda")
    g_host = host_grad(st.g)
    ref = dict(p=host_f32(st.p), m=host_f32(st.m), v=host_f32(st.v), lp=synth.bits16(st.p_lp), pdt="bf16")
    ov_ref, ss_ref, c_ref = oracle.optimizer_step(ref["p"], ref["m"], ref["v"], g_host, cfg.gdt, ref["lp"],
                                                  "bf16", oracle_hyper(cfg), cfg.step, cfg.loss_scale,
                                                  cfg.max_norm, nthreads=THREADS)
    assert not ov_ref and 0.05 < c_ref < 0.2          # norm ~ 10: clipping really bites
    ws, res = ma.workspace(), ma.new_result()
    ma.overflow_norm(st.g, cfg.loss_scale, res, ws)
    ma.adamw_step_gated(st.p, st.m, st.v, st.g, st.p_lp, _hyper(cfg), cfg.step, cfg.loss_scale, res,
                        cfg.max_norm)
    ov, ss = ma.read_result(res)
    assert not ov and abs(ss - ss_ref) <= SUMSQ_RTOL * ss_ref
    assert np.float32(ma.clip_coef(ss, cfg.max_norm)) == c_ref
    got = dict(p=host_f32(st.p), m=host_f32(st.m), v=host_f32(st.v), lp=synth.bits16(st.p_lp))
    assert_state_close(got, ref, name)


def test_fp16_overflow_variant_skips_at_full_size():
    cfg = synth.config("c3b")
    st = synth.make_flat(cfg, device="cuda")
    assert len(st.inject_idx) == 17
    assert oracle.overflow_norm(host_grad(st.g), "f16", cfg.loss_scale, nthreads=THREADS)[0] is True
    keep = [t.clone() for t in (st.p, st.m, st.v, st.p_lp)]
    ws, res = ma.workspace(), ma.new_result()
    ma.overflow_norm(st.g, cfg.loss_scale, res, ws)
    ma.adamw_step_gated(st.p, st.m, st.v, st.g, st.p_lp, _hyper(cfg), cfg.step, cfg.loss_scale, res,
                        cfg.max_norm)
    assert ma.read_result(res)[0] is True
    for a, b in zip(keep, (st.p, st.m, st.v, st.p_lp)):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def _list_ranges(shapes, total, seed, n_random):
    ranges, off = [], 0
    for _, n in shapes:
        ranges += [(off, off + EDGE), (off + n - EDGE, off + n)]
        off += n
    rng = np.random.default_rng(seed)
    for a in rng.integers(0, total - EDGE, n_random).tolist():
        ranges.append((a, a + EDGE))
    return ranges


def _tensor_ranges(shapes, seed, n_random):
    """Per tensor: first and last EDGE elements; plus seeded random blocks inside random tensors."""
    per = [[(0, EDGE), (n - EDGE, n)] for _, n in shapes]
    rng = np.random.default_rng(seed)
    sizes = np.array([n for _, n in shapes], dtype=np.float64)
    for i in rng.choice(len(shapes), n_random, p=sizes / sizes.sum()).tolist():
        n = shapes[i][1]
        a = int(rng.integers(0, max(1, n - EDGE)))
        per[i].append((a, a + EDGE))
    return [_merge(r, shapes[i][1]) for i, r in enumerate(per)]


def _gather_list(tensors, per):
    return torch.cat([t[a:b] for t, r in zip(tensors, per) for a, b in r])


def _sample_list(ls, per, pdt):
    return dict(p=host_f32(_gather_list(ls.p, per)), m=host_f32(_gather_list(ls.m, per)),
                v=host_f32(_gather_list(ls.v, per)), lp=synth.bits16(_gather_list(ls.p_lp, per)), pdt=pdt)


def _checksums_list(ls):
    out = []
    for lst in (ls.p, ls.m, ls.v, ls.p_lp):
        out.append(sum(int(t.view(torch.int32 if t.element_size() == 4 else torch.int16).sum(dtype=torch.int64))
                       for t in lst))
    return out


def _parts_and_traffic(shapes):
    parts = synth.list_state_parts(shapes)
    return parts[0], synth.list_traffic(shapes)[:4], parts[1]


def test_llama3_8b_list_every_element():
    """The benchmark workload itself, as the benchmark lays it out and places it (flat streams cut from
    a range that the library's placement helper maps from physical blocks of known HBM region:
    p | m | v | g across the boundary between two regions, the copy in a third): 290 tensors,
    8,030,257,152 elements, one scan launch and one gated update launch.  Flag and sum over all
    elements, and EVERY element of p, m, v and the bf16 copy against the oracle: each work item is
    processed exactly once, whichever block draws it."""
    _need_gib(250)
    shapes = synth.llama3_8b_shapes()
    cfg = synth.FlatConfig("llama3_8b", 0, seed=3, m_std=1e-4, v_std=1e-8, step=100, max_norm=1.0)
    # the benchmark's arena, with less room to spare: the copy of the state before the step must fit too
    arena = hbm.StitchedArena(ma.Arena, half_bytes=64 * hbm.GIB, side_bytes=16 * hbm.GIB)
    try:
        print("stitched arena:", arena.report)
        main, side = arena.split_window(*_parts_and_traffic(shapes))
        ls = synth.make_list(shapes, cfg, device="cuda", layout="streams", arena=(main, side))
        n = ls.total
        assert n == 8_030_257_152 and ls.flat.p.numel() == n          # no padding between the views
        base = arena.arena.main.data_ptr()
        assert ls.flat.p.data_ptr() - base < arena.half < ls.flat.m.data_ptr() + 4 * n - base   # the boundary falls into m
        assert ls.flat.p_lp.data_ptr() == arena.arena.side.data_ptr()                          # the copy lies in the side part
        keep = [torch.empty(n, dtype=torch.float32, device="cuda") for _ in range(3)]           # the state before the step
        for dst, src in zip(keep, (ls.flat.p, ls.flat.m, ls.flat.v)):
            dst.copy_(src)
        full = FullCompare(SLAB, "bf16", "bf16", THREADS)
        ov_ref, ss_ref = full.norm(ls.flat.g, 1.0)
        c_ref = oracle.clip_coef(ss_ref, 1.0)
        assert not ov_ref and 0.005 < c_ref < 0.02         # norm ~ 90
        plan = ma.MultiPlan(ls.p, ls.m, ls.v, ls.g, ls.p_lp)
        assert plan.plan.step_chunks >= 65536              # late work items are drawn on demand at this size
        ws, res = ma.workspace(), ma.new_result()
        ma.multi_overflow_norm(plan, 1.0, res, ws)
        ma.multi_adamw_step_gated(plan, _hyper(cfg), 100, 1.0, res, 1.0)
        ov, ss = ma.read_result(res)
        assert not ov and abs(ss - ss_ref) <= SUMSQ_RTOL * ss_ref
        assert np.float32(ma.clip_coef(ss, 1.0)) == c_ref
        assert plan.table[:64].view(torch.int32).cpu().tolist() == [0] * 16
        full.step(keep, ls.flat.g, (ls.flat.p, ls.flat.m, ls.flat.v, ls.flat.p_lp), oracle_hyper(cfg), 100, 1.0,
                  float(c_ref), "8B list")
        assert full.elements == n
        print("8B list: %d elements compared, %d slabs not bit-identical" % (full.elements, full.inexact_slabs))
        # one NaN in a norm vector: the whole list is skipped, checked over every byte via checksums
        sums = _checksums_list(ls)
        ls.g[8].view(torch.int16)[4095] = 0x7FC0
        ma.multi_overflow_norm(plan, 1.0, res, ws)
        ma.multi_adamw_step_gated(plan, _hyper(cfg), 101, 1.0, res, 1.0)
        assert ma.read_result(res)[0] is True
        assert _checksums_list(ls) == sums
    finally:                      # the range is unmapped whatever happened; nothing touches its views afterwards
        torch.cuda.synchronize()
        arena.release()


@pytest.mark.parametrize("layout", ["tensor"])
def test_llama3_8b_list_sampled(layout):
    """The same list in its other layout ("tensor": the five buffers of a tensor adjacent), on
    samples: tensor edges and seeded random blocks; flag and sum over all elements."""
    _need_gib(135)
    shapes = synth.llama3_8b_shapes()
    cfg = synth.FlatConfig("llama3_8b", 0, seed=3, m_std=1e-4, v_std=1e-8, step=100, max_norm=1.0)
    # placed as the benchmark places it: cut from a whole-device allocation, traffic split evenly
    # over two HBM regions
    device_arena = hbm.DeviceArena("cuda", reserve_gib=12)      # the checks below need temporaries
    window = device_arena.window(synth.list_state_bytes(shapes, layout), synth.list_traffic(shapes, layout))
    ls = synth.make_list(shapes, cfg, device="cuda", layout=layout, arena=window)
    assert ls.arena.data_ptr() == window.data_ptr()
    assert ls.total == 8_030_257_152
    if layout == "streams":
        assert ls.flat.p.numel() == ls.total               # no padding between the views
    per = _tensor_ranges(shapes, 17, 1200)
    before = _sample_list(ls, per, "bf16")
    g_s = host_grad(_gather_list(ls.g, per))
    ov_ref, ss_ref = False, 0.0
    for g in ls.g:                                         # flag and sum over ALL elements
        o, s_ = _oracle_norm_all(g, "bf16", 1.0)
        ov_ref, ss_ref = ov_ref or o, ss_ref + s_
    c_ref = oracle.clip_coef(ss_ref, 1.0)
    assert not ov_ref and 0.005 < c_ref < 0.02         # norm ~ 90
    before["lp"] = oracle.adamw_step(before["p"], before["m"], before["v"], g_s, "bf16", "bf16",
                                     oracle_hyper(cfg), 100, 1.0, float(c_ref), nthreads=THREADS)
    plan = ma.MultiPlan(ls.p, ls.m, ls.v, ls.g, ls.p_lp)
    ws, res = ma.workspace(), ma.new_result()
    ma.multi_overflow_norm(plan, 1.0, res, ws)
    ma.multi_adamw_step_gated(plan, _hyper(cfg), 100, 1.0, res, 1.0)
    ov, ss = ma.read_result(res)
    assert not ov and abs(ss - ss_ref) <= SUMSQ_RTOL * ss_ref
    assert np.float32(ma.clip_coef(ss, 1.0)) == c_ref
    assert_state_close(_sample_list(ls, per, "bf16"), before, "8B list sample (%s)" % layout)
    # one NaN in a norm vector: the whole list is skipped, checked over every byte via checksums
    sums = _checksums_list(ls)
    ls.g[8].view(torch.int16)[4095] = 0x7FC0
    ma.multi_overflow_norm(plan, 1.0, res, ws)
    ma.multi_adamw_step_gated(plan, _hyper(cfg), 101, 1.0, res, 1.0)
    assert ma.read_result(res)[0] is True
    assert _checksums_list(ls) == sums


def test_14b_class_four_sub_groups():
    """12,567,592,960 elements as 4 equal flat sub-groups (3,141,898,240 each, beyond 2^31) cut
    without regard to tensor boundaries.  First iteration: 4 scans, 1 combine, 4 gated updates back to
    back on one stream, as the benchmark enqueues them, compared on samples.  Second iteration: the
    same launches, each sub-group's update followed by a comparison of EVERY element of that sub-group
    with the oracle.  Third iteration: the sub-groups as one-tensor lists, on samples."""
    _need_gib(250)
    shapes = synth.qwen14b_class_shapes()
    total = sum(n for _, n in shapes)
    cfg = synth.FlatConfig("qwen14b_4sub", 0, seed=4, m_std=1e-4, v_std=1e-8, step=100, max_norm=1.0)
    # placed as the benchmark places it: in the library-built arena, p | m | v | g around the boundary
    # between two HBM regions, the copy in a third
    arena = hbm.StitchedArena(ma.Arena)
    try:
        print("stitched arena:", arena.report)
        where = arena.split_window(synth.flat_state_parts(total)[0], synth.flat_traffic(total)[:4],
                                   synth.flat_state_parts(total)[1])
        _four_sub_groups(synth.make_flat(cfg, device="cuda", n=total, arena=where), shapes, total, cfg)
    finally:                      # the range is unmapped whatever happened; nothing touches its views afterwards
        torch.cuda.synchronize()
        arena.release()


def _four_sub_groups(fl, shapes, total, cfg):
    sub = total // 4
    assert sub == 3_141_898_240
    ranges = _list_ranges(shapes, total, 19, 600)
    for k in range(1, 4):
        ranges.append((k * sub - EDGE, k * sub + EDGE))
    ranges = _merge(ranges, total)
    before = _sample_state(fl, ranges, "bf16")
    g_s = host_grad(_gather(fl.g, ranges))
    ss_ref = 0.0
    for k in range(4):
        ov_k, ss_k = _oracle_norm_all(fl.g[k * sub:(k + 1) * sub], "bf16", 1.0)
        assert not ov_k
        ss_ref += ss_k
    c_ref = oracle.clip_coef(ss_ref, 1.0)
    before["lp"] = oracle.adamw_step(before["p"], before["m"], before["v"], g_s, "bf16", "bf16",
                                     oracle_hyper(cfg), 100, 1.0, float(c_ref), nthreads=THREADS)
    ws, parts, res = ma.workspace(), ma.new_result(4), ma.new_result()
    for k in range(4):
        ma.overflow_norm(fl.g[k * sub:(k + 1) * sub], 1.0, parts, ws, index=k)
    ma.norm_combine(parts, 4, res)
    for k in range(4):
        s = slice(k * sub, (k + 1) * sub)
        ma.adamw_step_gated(fl.p[s], fl.m[s], fl.v[s], fl.g[s], fl.p_lp[s], _hyper(cfg), 100, 1.0, res, 1.0)
    ov, ss = ma.read_result(res)
    assert not ov and abs(ss - ss_ref) <= SUMSQ_RTOL * ss_ref
    assert np.float32(ma.clip_coef(ss, 1.0)) == c_ref
    assert_state_close(_sample_state(fl, ranges, "bf16"), before, "14B sub-groups sample")
    # second iteration: every element of every sub-group
    full = FullCompare(SLAB, "bf16", "bf16", THREADS)
    keep = [torch.empty(sub, dtype=torch.float32, device="cuda") for _ in range(3)]
    for k in range(4):
        ma.overflow_norm(fl.g[k * sub:(k + 1) * sub], 1.0, parts, ws, index=k)
    ma.norm_combine(parts, 4, res)
    for k in range(4):
        s = slice(k * sub, (k + 1) * sub)
        for dst, src in zip(keep, (fl.p[s], fl.m[s], fl.v[s])):
            dst.copy_(src)
        ma.adamw_step_gated(fl.p[s], fl.m[s], fl.v[s], fl.g[s], fl.p_lp[s], _hyper(cfg), 101, 1.0, res, 1.0)
        full.step(keep, fl.g[s], (fl.p[s], fl.m[s], fl.v[s], fl.p_lp[s]), oracle_hyper(cfg), 101, 1.0,
                  float(c_ref), "14B sub-group %d" % k)
    assert ma.read_result(res) == (False, ss)
    assert full.elements == total
    print("14B sub-groups: %d elements compared, %d slabs not bit-identical" % (full.elements, full.inexact_slabs))
    del keep, full
    torch.cuda.empty_cache()
    before["lp"] = oracle.adamw_step(before["p"], before["m"], before["v"], g_s, "bf16", "bf16",
                                     oracle_hyper(cfg), 101, 1.0, float(c_ref), nthreads=THREADS)
    assert_state_close(_sample_state(fl, ranges, "bf16"), before, "14B sub-groups sample, second iteration")
    # a third iteration with every sub-group prepared as a one-tensor list (the form in which a flat
    # sub-group gets its late work items drawn on demand)
    plans = []
    for k in range(4):
        s = slice(k * sub, (k + 1) * sub)
        plans.append(ma.MultiPlan([fl.p[s]], [fl.m[s]], [fl.v[s]], [fl.g[s]], [fl.p_lp[s]]))
    before["lp"] = oracle.adamw_step(before["p"], before["m"], before["v"], g_s, "bf16", "bf16",
                                     oracle_hyper(cfg), 102, 1.0, float(c_ref), nthreads=THREADS)
    for k in range(4):
        ma.multi_overflow_norm(plans[k], 1.0, parts, ws, index=k)
    ma.norm_combine(parts, 4, res)
    for k in range(4):
        ma.multi_adamw_step_gated(plans[k], _hyper(cfg), 102, 1.0, res, 1.0)
    ov, ss2 = ma.read_result(res)
    assert not ov and ss2 == ss
    assert_state_close(_sample_state(fl, ranges, "bf16"), before, "14B sub-groups as one-tensor lists")


def test_flat_sub_group_beyond_2_to_31():
    """n = 2^31 + 5: 64-bit indexing, ragged tail of one element group plus one."""
    _need_gib(40)
    n = (1 << 31) + 5
    cfg = synth.FlatConfig("big", n, seed=6, m_std=1e-4, v_std=1e-8, step=9, gdt="f16", loss_scale=512.0,
                           max_norm=2.0)
    fl = synth.make_flat(cfg, device="cuda")
    rng = np.random.default_rng(23)
    ranges = [(0, EDGE), (n - EDGE, n), ((1 << 31) - EDGE, (1 << 31) + 5), ((1 << 30) - 999, (1 << 30) + 999)]
    ranges += [(a, a + 4099) for a in rng.integers(0, n - 5000, 300).tolist()]
    ranges = _merge(ranges, n)
    before = _sample_state(fl, ranges, "bf16")
    g_s = host_grad(_gather(fl.g, ranges))
    ov_ref, ss_ref = _oracle_norm_all(fl.g, "f16", 512.0)
    c_ref = oracle.clip_coef(ss_ref, 2.0)
    assert not ov_ref and c_ref < 1
    before["lp"] = oracle.adamw_step(before["p"], before["m"], before["v"], g_s, "f16", "bf16",
                                     oracle_hyper(cfg), 9, 512.0, float(c_ref), nthreads=THREADS)
    ws, res = ma.workspace(), ma.new_result(2)
    ma.overflow_norm(fl.g, 512.0, res, ws)
    ma.adamw_step_gated(fl.p, fl.m, fl.v, fl.g, fl.p_lp, _hyper(cfg), 9, 512.0, res, 2.0)
    ov, ss = ma.read_result(res)
    assert not ov and abs(ss - ss_ref) <= SUMSQ_RTOL * ss_ref
    assert_state_close(_sample_state(fl, ranges, "bf16"), before, "2^31+5")
    # an inf in the very last element is seen
    fl.g.view(torch.int16)[n - 1] = 0x7C00
    ma.overflow_norm(fl.g, 512.0, res, ws, index=1)
    assert ma.read_result(res, 1)[0] is True


N_8B = 8_030_257_152


def _random_ranges(n, seed, count):
    rng = np.random.default_rng(seed)
    r = [(0, EDGE), (n - EDGE, n), ((1 << 32) - EDGE, (1 << 32) + EDGE)]
    r += [(a, a + EDGE) for a in rng.integers(0, n - EDGE, count).tolist()]
    return _merge(r, n)


def test_bf16_states_8b_sampled():
    """The bf16-state benchmark workload: one flat sub-group of 8,030,257,152 elements with p, m, v
    held in bf16 (Extended Experiments), scan then gated truncating update; sampled blocks bit-exact,
    flag and sum of squares over all elements."""
    _need_gib(80)
    n = N_8B
    cfg = synth.FlatConfig("bf16_states_8b", n, seed=5, m_std=1e-4, v_std=1e-8, step=100, max_norm=1.0)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(cfg.seed)
    p, m, v, g = (torch.empty(n, dtype=torch.bfloat16, device="cuda") for _ in range(4))
    for t, std in ((p, cfg.p_std), (m, cfg.m_std), (v, cfg.v_std), (g, cfg.g_std)):
        synth._fill_grad(t, std, 1.0, gen)
    v.abs_()
    ranges = _random_ranges(n, 29, 900)
    rp, rm, rv = (synth.bits16(_gather(t, ranges)) for t in (p, m, v))
    g_s = host_grad(_gather(g, ranges))
    ov_ref, ss_ref = _oracle_norm_all(g, "bf16", 1.0)
    c_ref = oracle.clip_coef(ss_ref, 1.0)
    assert not ov_ref and 0.005 < c_ref < 0.02
    oracle.adamw_step_bf16(rp, rm, rv, g_s, "bf16", oracle_hyper(cfg), 100, 1.0, float(c_ref), nthreads=THREADS)
    ws, res = ma.workspace(), ma.new_result()
    ma.overflow_norm(g, 1.0, res, ws)
    ma.adamw_step_bf16_gated(p, m, v, g, _hyper(cfg), 100, 1.0, res, 1.0)
    ov, ss = ma.read_result(res)
    assert not ov and abs(ss - ss_ref) <= SUMSQ_RTOL * ss_ref
    assert np.float32(ma.clip_coef(ss, 1.0)) == c_ref
    for name, t, ref in (("p", p, rp), ("m", m, rm), ("v", v, rv)):
        got = synth.bits16(_gather(t, ranges))
        assert np.array_equal(got, ref), "%s: %d of %d sampled patterns differ" % (name, (got != ref).sum(), ref.size)
    assert np.array_equal(host_grad(_gather(g, ranges)), g_s)        # gradients are read-only
    # an overflow anywhere skips the whole sub-group
    sums = [int(t.view(torch.int16).sum(dtype=torch.int64)) for t in (p, m, v)]
    g.view(torch.int16)[n - 3] = 0x7F80
    ma.overflow_norm(g, 1.0, res, ws)
    ma.adamw_step_bf16_gated(p, m, v, g, _hyper(cfg), 101, 1.0, res, 1.0)
    assert ma.read_result(res)[0] is True
    assert [int(t.view(torch.int16).sum(dtype=torch.int64)) for t in (p, m, v)] == sums


def test_accumulate_8b_sampled():
    """The accumulation benchmark workload: three bf16 micro-batch gradients of 8,030,257,152 elements
    into the fp32 flat buffer (overwrite, add, add fused with the scan); sampled blocks bit-exact,
    flag and sum of squares against the oracle's scan of the whole accumulated buffer."""
    _need_gib(60)
    n = N_8B
    S = 1024.0
    acc = torch.empty(n, dtype=torch.float32, device="cuda")
    acc[:EDGE] = float("nan")                                # whatever the buffer held is overwritten
    g = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(31)
    ranges = _random_ranges(n, 37, 900)
    ref = np.zeros(sum(b - a for a, b in ranges), np.float32)
    ws, res = ma.workspace(), ma.new_result()
    for k in range(3):
        synth._fill_grad(g, 1e-3, S, gen)
        oracle.grad_accumulate(ref, host_grad(_gather(g, ranges)), "bf16", first=(k == 0))
        if k < 2:
            ma.grad_accumulate(acc, g, first=(k == 0))
        else:
            ma.grad_accumulate_scan(acc, g, False, S, res, ws)
    assert np.array_equal(host_f32(_gather(acc, ranges)).view(np.uint32), ref.view(np.uint32))
    ov_ref, ss_ref = _oracle_norm_all(acc, "f32", S, piece=1 << 27)
    ov, ss = ma.read_result(res)
    assert not ov and not ov_ref
    assert abs(ss - ss_ref) <= SUMSQ_RTOL * ss_ref
    assert abs(ss / n - 3e-6) < 1e-8                         # three N(0, 1e-3) draws: variance 3e-6 each
    # a NaN arriving with the next micro-batch is seen by the fused scan
    g.view(torch.int16)[n - 1] = 0x7FC1
    ma.grad_accumulate_scan(acc, g, False, S, res, ws)
    assert ma.read_result(res)[0] is True


def test_flat_fp32_states_beyond_2_to_32():
    """One flat call on 8,030,257,155 elements (element indices beyond 2^32, a ragged tail of three):
    scan, gated update with fp16 gradients and an fp16 copy; sampled blocks on both sides of element
    2^32, flag and sum over all elements."""
    _need_gib(135)
    n = N_8B + 3
    cfg = synth.FlatConfig("flat8b", n, seed=8, m_std=1e-4, v_std=1e-8, step=12, gdt="f16", pdt="f16",
                           loss_scale=4096.0, max_norm=1.0)
    fl = synth.make_flat(cfg, device="cuda")
    ranges = _random_ranges(n, 41, 500)
    before = _sample_state(fl, ranges, "f16")
    g_s = host_grad(_gather(fl.g, ranges))
    ov_ref, ss_ref = _oracle_norm_all(fl.g, "f16", 4096.0)
    c_ref = oracle.clip_coef(ss_ref, 1.0)
    assert not ov_ref and c_ref < 0.02
    before["lp"] = oracle.adamw_step(before["p"], before["m"], before["v"], g_s, "f16", "f16",
                                     oracle_hyper(cfg), 12, 4096.0, float(c_ref), nthreads=THREADS)
    ws, res = ma.workspace(), ma.new_result(2)
    ma.overflow_norm(fl.g, 4096.0, res, ws)
    ma.adamw_step_gated(fl.p, fl.m, fl.v, fl.g, fl.p_lp, _hyper(cfg), 12, 4096.0, res, 1.0)
    ov, ss = ma.read_result(res)
    assert not ov and abs(ss - ss_ref) <= SUMSQ_RTOL * ss_ref
    assert np.float32(ma.clip_coef(ss, 1.0)) == c_ref
    assert_state_close(_sample_state(fl, ranges, "f16"), before, "flat 8B + 3")
    # a NaN just beyond element 2^32 is seen
    fl.g.view(torch.int16)[(1 << 32) + 1] = 0x7E00
    ma.overflow_norm(fl.g, 4096.0, res, ws, index=1)
    assert ma.read_result(res, 1)[0] is True


def test_list_with_late_items_drawn_on_demand_eager_and_graph():
    """A 1/24-scale 8B-shaped list (3.3e8 elements, about 82,000 work items): large enough that the
    update kernel hands the last part of every XCD's share out on demand.  One eager iteration, then
    ONE captured graph (scan, gated update, loss-scale update, all reading their inputs on the
    device) replayed twice, the first replay skipped by a NaN.  After every iteration EVERY element
    of every tensor is compared with the oracle: each work item is processed exactly once whichever
    block draws it; and the counters at the head of the plan's table read zero again (a stale
    counter would leave late items of the next launch undone)."""
    _need_gib(20)
    shapes = synth.scaled_shapes(synth.llama3_8b_shapes(), 24, ragged=True)
    cfg = synth.FlatConfig("t", 0, seed=95, m_std=1e-4, v_std=1e-8, max_norm=1.0)
    ls = synth.make_list(shapes, cfg, device="cuda", align_elems=1)
    plan = ma.MultiPlan(ls.p, ls.m, ls.v, ls.g, ls.p_lp)
    assert plan.plan.step_chunks >= 65536
    h_ref, h = oracle_hyper(cfg), _hyper(cfg)
    scaler, scfg = ma.new_scaler(1.0, 41), ma.scaler_config(window=1000)
    ws, res = ma.workspace(), ma.new_result()
    refs = [dict(p=host_f32(ls.p[i]), m=host_f32(ls.m[i]), v=host_f32(ls.v[i]), lp=synth.bits16(ls.p_lp[i]),
                 pdt="bf16") for i in range(len(shapes))]
    head = lambda: plan.table[:64].view(torch.int32).cpu().tolist()
    assert head() == [0] * 16

    def iteration():
        ma.multi_overflow_norm_auto(plan, scaler, res, ws)
        ma.multi_adamw_step_auto(plan, h, scaler, res, cfg.max_norm)
        ma.scaler_update(scaler, res, scfg)

    def feed(it, bad):
        gen = torch.Generator(device="cuda")
        gen.manual_seed(950 + it)
        synth._fill_grad(ls.flat.g, 1e-3, 1.0, gen)
        if bad:
            ls.g[-1].view(torch.int16)[-1] = 0x7FC0       # the very last element of the list
        return [host_grad(g) for g in ls.g]

    applied = 41

    def check(it, g_hosts, bad):
        nonlocal applied
        torch.cuda.synchronize()
        ov, ss = ma.read_result(res)
        assert ov == bad, it
        assert head() == [0] * 16, it
        if not bad:
            ss_ref = sum(oracle.overflow_norm(g, "bf16", 1.0, nthreads=THREADS)[1] for g in g_hosts)
            assert abs(ss - ss_ref) <= SUMSQ_RTOL * ss_ref
            c_ref = oracle.clip_coef(ss_ref, 1.0)
            assert np.float32(ma.clip_coef(ss, 1.0)) == c_ref
            applied += 1
            for r, g in zip(refs, g_hosts):
                r["lp"] = oracle.adamw_step(r["p"], r["m"], r["v"], g, "bf16", "bf16", h_ref, applied, 1.0,
                                            float(c_ref), nthreads=THREADS)
        assert ma.read_scaler(scaler)[2] == applied, it
        for i in range(len(shapes)):
            got = dict(p=host_f32(ls.p[i]), m=host_f32(ls.m[i]), v=host_f32(ls.v[i]), lp=synth.bits16(ls.p_lp[i]))
            assert_state_close(got, refs[i], "iteration %d, tensor %d (%s)" % (it, i, shapes[i][0]))

    gh = feed(0, False)
    iteration()
    check(0, gh, False)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        iteration()
    torch.cuda.synchronize()
    for it in range(1, 3):
        bad = it == 1
        gh = feed(it, bad)
        graph.replay()
        check(it, gh, bad)
        _ = (ls.flat.p[:1000] * 2).sum().item()      # eager work of the program between replays


def test_bf16_state_list_with_late_items_drawn_on_demand():
    """The same size class for a list whose p, m, v are held in bf16 (1/6-scale 8B shapes, 1.34e9
    elements, work items of 16,384 elements): two iterations on one plan, every truncated pattern of
    every tensor against the oracle, counters back at zero."""
    _need_gib(32)
    shapes = synth.scaled_shapes(synth.llama3_8b_shapes(), 6, ragged=True)
    cfg = synth.FlatConfig("t", 0, seed=97, m_std=1e-3, v_std=1e-6, lr=1e-2, weight_decay=0.1, eps=1e-6,
                           max_norm=1.0)
    ls = synth.make_list(shapes, cfg, device="cuda", align_elems=1)
    shift = lambda t: (t.view(torch.int32) >> 16).to(torch.int16).view(torch.bfloat16).contiguous()
    fp, fm, fv = shift(ls.flat.p), shift(ls.flat.m), shift(ls.flat.v)
    offs = [t.data_ptr() // 4 - ls.flat.p.data_ptr() // 4 for t in ls.p]
    cut = lambda buf: [buf[o:o + n] for o, (_, n) in zip(offs, shapes)]
    P, M, V = cut(fp), cut(fm), cut(fv)
    grads = list(ls.g)
    del ls.p, ls.m, ls.v, ls.p_lp
    ls.flat.p = ls.flat.m = ls.flat.v = ls.flat.p_lp = None      # the fp32 originals are no longer needed
    torch.cuda.empty_cache()
    plan = ma.MultiPlanBF16(P, M, V, grads)
    assert plan.plan.step_chunks >= 65536 and plan.plan.sdt == ma.MA_BF16
    refs = [(synth.bits16(P[i]), synth.bits16(M[i]), synth.bits16(V[i])) for i in range(len(shapes))]
    g_hosts = [host_grad(g) for g in grads]
    ss_ref = sum(oracle.overflow_norm(g, "bf16", 1.0, nthreads=THREADS)[1] for g in g_hosts)
    c_ref = oracle.clip_coef(ss_ref, 1.0)
    assert c_ref < 1
    ws, res = ma.workspace(), ma.new_result()
    for step in (5, 6):
        ma.multi_overflow_norm(plan, 1.0, res, ws)
        ma.multi_adamw_step_gated(plan, _hyper(cfg), step, 1.0, res, cfg.max_norm)
        ov, ss = ma.read_result(res)
        assert not ov and abs(ss - ss_ref) <= SUMSQ_RTOL * ss_ref
        assert plan.table[:64].view(torch.int32).cpu().tolist() == [0] * 16
        for i in range(len(shapes)):
            rp, rm, rv = refs[i]
            oracle.adamw_step_bf16(rp, rm, rv, g_hosts[i], "bf16", oracle_hyper(cfg), step, 1.0, float(c_ref),
                                   nthreads=THREADS)
            for name, t, r in (("p", P[i], rp), ("m", M[i], rm), ("v", V[i], rv)):
                got = synth.bits16(t)
                assert np.array_equal(got, r), "step %d tensor %d (%s) %s: %d patterns differ" % (
                    step, i, shapes[i][0], name, int((got != r).sum()))
