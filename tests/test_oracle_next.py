"""Pins for the oracle functions beyond the basic step: gradient accumulation into the fp32 flat
buffer (Sec. III-C), the step with bf16 states stored by truncation (Extended Experiments), and the
dynamic loss scale (Sec. III-C)."""
import numpy as np
import pytest

import oracle
from paper_2505_23254_amd import synth


def _grad(n, seed, gdt, scale=1.0):
    cfg = synth.FlatConfig("t", n, seed=seed, gdt=gdt, loss_scale=scale)
    return synth.bits16(synth.make_flat(cfg).g)


@pytest.mark.parametrize("gdt", ["bf16", "f16"])
def test_accumulate_is_one_ieee_addition(gdt):
    n = 20_001
    widen = oracle.widen_bf16 if gdt == "bf16" else oracle.widen_f16
    acc = np.full(n, np.float32(123.0))
    ref = None
    for k in range(4):
        g = _grad(n, 50 + k, gdt, 64.0)
        gw = widen(g)
        ref = gw.copy() if k == 0 else (ref + gw).astype(np.float32)   # numpy fp32 add is IEEE
        oracle.grad_accumulate(acc, g, gdt, first=(k == 0))
        assert np.array_equal(acc.view(np.uint32), ref.view(np.uint32))
    # against exact arithmetic: each partial sum is the correctly rounded sum of its two operands
    a = np.array([1.0, 1.0, 16777216.0, -0.0], np.float32)
    g = np.array([0x3380, 0x3300, 0x3F80, 0x8000], np.uint16)     # bf16: 2^-24, 2^-25, 1.0, -0
    oracle.grad_accumulate(a, g, "bf16", first=False)
    assert a[0] == np.float32(1.0) and a[1] == np.float32(1.0)    # 1 + 2^-24 is a tie: even is 1.0
    assert a[2] == np.float32(16777216.0)                          # 2^24 + 1 ties to even 2^24
    assert np.signbit(a[3])                                        # -0 + -0 = -0
    # fp32 gradients accumulate too; `first` overwrites whatever was there, including NaN
    acc = np.full(5, np.nan, np.float32)
    g32 = np.array([1, -2, 3.5, 0, 1e-40], np.float32)
    oracle.grad_accumulate(acc, g32, "f32", first=True)
    assert np.array_equal(acc, g32)


def test_truncation_hand_values_and_properties():
    cases = [(0x3F80FFFF, 0x3F80), (0xBF80FFFF, 0xBF80), (0x3F800000, 0x3F80), (0x7F7FFFFF, 0x7F7F),
             (0x00008000, 0x0000), (0x0001FFFF, 0x0001), (0x7F800000, 0x7F80), (0xFF800000, 0xFF80),
             (0x7F800001, 0x7FC0), (0xFFC12345, 0xFFC1), (0x80000000, 0x8000)]
    for src, want in cases:
        x = np.array([src], np.uint32).view(np.float32)
        assert int(oracle.truncate_bf16(x)[0]) == want, hex(src)
    rng = np.random.default_rng(5)
    bits = rng.integers(0, 1 << 32, 500_000, dtype=np.uint64).astype(np.uint32)
    x = bits.view(np.float32)
    t = oracle.truncate_bf16(x)
    fin = np.isfinite(x)
    assert np.array_equal(t[fin], (bits[fin] >> 16).astype(np.uint16))     # plain shift
    y = oracle.widen_bf16(t)
    assert np.all(np.abs(y[fin]) <= np.abs(x[fin]))                          # toward zero
    assert np.array_equal(np.signbit(y[fin]), np.signbit(x[fin]))
    nxt = oracle.widen_bf16((t[fin] + 1).astype(np.uint16))                  # next pattern away from 0
    ok = ~np.isfinite(nxt) | (np.abs(x[fin]) < np.abs(nxt))
    assert np.all(ok)                                                         # less than one step away
    assert np.array_equal(oracle.truncate_bf16(y[fin]), t[fin])               # idempotent
    assert np.all(np.isnan(y[np.isnan(x)]))


@pytest.mark.parametrize("gdt,scale,clip", [("bf16", 1.0, 1.0), ("bf16", 1.0, 0.3), ("f16", 1024.0, 0.5)])
def test_bf16_state_step_is_widen_fp32_step_truncate(gdt, scale, clip):
    n = 30_000
    cfg = synth.FlatConfig("t", n, seed=60, gdt=gdt, loss_scale=scale, m_std=1e-3, v_std=1e-6)
    st = synth.make_flat(cfg)
    g = synth.bits16(st.g)
    shift = lambda a: (a.view(np.uint32) >> 16).astype(np.uint16)
    p = shift(st.p.numpy()); m = shift(st.m.numpy()); v = shift(st.v.numpy())
    h = oracle.hyper(lr=1e-2, weight_decay=0.1, eps=1e-6)
    # composition written with library pieces: widen by shift, the fp32 oracle step, shift back
    up = lambda a: (a.astype(np.uint32) << 16).view(np.float32)
    pf, mf, vf = up(p), up(m), up(v)
    oracle.adamw_step(pf, mf, vf, g, gdt, "bf16", h, 7, scale, clip, want_lp=False)
    oracle.adamw_step_bf16(p, m, v, g, gdt, h, 7, scale, clip)
    assert np.array_equal(p, shift(pf)) and np.array_equal(m, shift(mf)) and np.array_equal(v, shift(vf))
    # threads do not matter
    p2, m2, v2 = shift(st.p.numpy()), shift(st.m.numpy()), shift(st.v.numpy())
    oracle.adamw_step_bf16(p2, m2, v2, g, gdt, h, 7, scale, clip, nthreads=4)
    assert np.array_equal(p, p2) and np.array_equal(m, m2) and np.array_equal(v, v2)
    # with lr large enough the parameters do move, and the moments track the fp32 ones to 2^-7
    assert (p != shift(st.p.numpy())).mean() > 0.5
    np.testing.assert_allclose(up(m), mf, rtol=2.0 ** -7, atol=0)


def _parse_cases(path):
    cases, cur = [], None
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        a = line.split()
        if a[0] == "case":
            cur = dict(name=a[1], scale0=float(a[2]), cfg=(float(a[3]), float(a[4]), float(a[5]), float(a[6]), int(a[7])), rows=[])
            cases.append(cur)
        else:
            cur["rows"].append((int(a[0]), float(a[2]), int(a[3]), int(a[4]), int(a[5])))
    return cases


def test_loss_scale_policy_hand_worked(golden_dir):
    cases = _parse_cases(golden_dir + "/loss_scale_sequence.txt")
    assert len(cases) == 4
    for c in cases:
        st = oracle.scaler_state(scale=c["scale0"])
        cfg = oracle.scaler_cfg(*c["cfg"])
        for flag, scale, good, step, skipped in c["rows"]:
            oracle.scaler_update(st, cfg, flag)
            assert (st.scale, st.good_steps, st.step, st.skipped) == (scale, good, step, skipped), (c["name"], flag)


def test_loss_scale_closed_forms():
    cfg = oracle.scaler_cfg(window=10 ** 9)
    st = oracle.scaler_state(scale=2.0 ** 20)
    for k in range(1, 25):
        oracle.scaler_update(st, cfg, 1)
        assert st.scale == max(2.0 ** (20 - k), 1.0) and st.step == 0 and st.skipped == k
    cfg = oracle.scaler_cfg(window=5)
    st = oracle.scaler_state(scale=1.0)
    for k in range(1, 101):
        oracle.scaler_update(st, cfg, 0)
        assert st.scale == min(2.0 ** (k // 5), 2.0 ** 24) and st.step == k and st.good_steps == k % 5


def test_auto_iteration_skips_and_backs_off_then_steps():
    n = 5000
    cfg_s = synth.FlatConfig("t", n, seed=70, gdt="f16", loss_scale=1024.0, m_std=1e-4, v_std=1e-8)
    st = synth.make_flat(cfg_s)
    p, m, v = st.p.numpy().copy(), st.m.numpy().copy(), st.v.numpy().copy()
    g = synth.bits16(st.g)
    lp = oracle.round_bf16(p)
    h = oracle.hyper()
    state, cfg = oracle.scaler_state(scale=1024.0, step=41), oracle.scaler_cfg(window=2)
    bad = g.copy()
    bad[n // 2] = 0x7C00
    keep = (p.copy(), m.copy(), v.copy(), lp.copy())
    ov, _ = oracle.optimizer_step_auto(p, m, v, bad, "f16", lp, "bf16", h, state, cfg, 1.0)
    assert ov and (state.scale, state.step, state.skipped, state.good_steps) == (512.0, 41, 1, 0)
    assert all(a.tobytes() == b.tobytes() for a, b in zip(keep, (p, m, v, lp)))
    # the caller now produces gradients at the lower scale: here the same values, halved (exact)
    g_half = (g.view(np.float16).astype(np.float32) * 0.5).astype(np.float16).view(np.uint16)
    pa, ma, va, lpa = (a.copy() for a in keep)
    ov, ss = oracle.optimizer_step_auto(p, m, v, g_half, "f16", lp, "bf16", h, state, cfg, 1.0)
    assert not ov and (state.scale, state.step, state.good_steps) == (512.0, 42, 1)
    ov2, ss2, c2 = oracle.optimizer_step(pa, ma, va, g_half, "f16", lpa, "bf16", h, 42, 512.0, 1.0)
    assert ss == ss2 and np.array_equal(p, pa) and np.array_equal(lp, lpa)
    oracle.optimizer_step_auto(p, m, v, g_half, "f16", lp, "bf16", h, state, cfg, 1.0)
    assert (state.scale, state.step, state.good_steps) == (1024.0, 43, 0)
