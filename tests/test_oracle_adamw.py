"""Pins for the oracle's AdamW step and the skip-on-overflow gate.

The paper prints no update formula (Sec. II-A names bias correction and decoupled weight
decay only), so the fp32 oracle is pinned against what the mathematics fixes: the first-step
closed form, degenerate hyper-parameters, exact symmetries, an fp64 evaluation of the
textbook formula written separately inside the oracle, and a library AdamW run in fp64 with
hyper-parameters chosen so that every term (decay, eps, both bias corrections) moves the
result far above fp32 rounding.  The gate is pinned by the invariant of Sec. III-C: a step
that sees any inf/NaN changes nothing.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_23254_amd import synth

EPS32 = float(np.finfo(np.float32).eps)


def _state(n, seed, gdt="bf16", m_std=1e-4, v_std=1e-8, g_std=1e-3, scale=1.0):
    cfg = synth.FlatConfig("t", n, seed=seed, gdt=gdt, m_std=m_std, v_std=v_std, g_std=g_std,
                           loss_scale=scale)
    st = synth.make_flat(cfg)
    return (st.p.numpy().copy(), st.m.numpy().copy(), st.v.numpy().copy(), synth.bits16(st.g))


def _widen(bits, gdt):
    return (oracle.widen_bf16 if gdt == "bf16" else oracle.widen_f16)(bits).astype(np.float64)


@pytest.mark.parametrize("gdt", ["bf16", "f16"])
def test_first_step_closed_form(gdt):
    # t = 1, m = v = 0:  m' = (1-b1) g,  v' = (1-b2) g^2,
    # p' = p - lr*wd*p - lr * g / (|g| + eps)     (both bias corrections cancel exactly)
    p, m, v, g = _state(20000, 21, gdt=gdt, m_std=0, v_std=0)
    h = oracle.hyper(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-4, weight_decay=0.1)
    gd = _widen(g, gdt)
    p0 = p.astype(np.float64)
    oracle.adamw_step(p, m, v, g, gdt, "bf16", h, step=1)
    lr, wd, eps = float(np.float32(1e-3)), float(np.float32(0.1)), float(np.float32(1e-4))
    b1, b2 = float(np.float32(0.9)), float(np.float32(0.999))
    want = p0 - lr * wd * p0 - lr * gd / (np.abs(gd) + eps)
    assert np.max(np.abs(p - want)) <= 4 * EPS32 * np.max(np.abs(p0))
    np.testing.assert_allclose(m, (1 - b1) * gd, rtol=4 * EPS32, atol=0)
    np.testing.assert_allclose(v, (1 - b2) * gd * gd, rtol=4 * EPS32, atol=1e-45)
    # the update really is O(lr): the closed form is not satisfied by "p unchanged"
    assert np.median(np.abs(p - p0)) > 0.5 * lr


def test_first_step_sign_limit():
    # |g| >> eps: the Adam part tends to -lr*sign(g)
    p, m, v, g = _state(4096, 22, m_std=0, v_std=0, g_std=1.0)
    h = oracle.hyper(lr=1e-2, eps=1e-8, weight_decay=0.0)
    gd = _widen(g, "bf16")
    p0 = p.astype(np.float64)
    oracle.adamw_step(p, m, v, g, "bf16", "bf16", h, step=1)
    big = np.abs(gd) > 1e-3
    assert np.allclose((p - p0)[big], -float(np.float32(1e-2)) * np.sign(gd[big]), rtol=1e-4)


def test_zero_gradient_is_pure_decay():
    p, m, v, _ = _state(5000, 23)
    g = np.zeros(5000, np.uint16)
    h = oracle.hyper(lr=1e-2, weight_decay=0.1, eps=1e-8)
    p0, m0, v0 = p.copy(), m.copy(), v.copy()
    m[:] = 0
    oracle.adamw_step(p, m, v, g, "bf16", "bf16", h, step=7)
    d = np.float32(np.float64(np.float32(1e-2)) * np.float64(np.float32(0.1)))
    assert np.all(m == 0)
    np.testing.assert_allclose(v, np.float32(0.999) * v0, rtol=EPS32)
    np.testing.assert_allclose(p, p0.astype(np.float64) * (1 - float(d)), rtol=2 * EPS32)


def test_zero_lr_freezes_p_but_moments_advance():
    p, m, v, g = _state(5000, 24)
    h = oracle.hyper(lr=0.0)
    p0, m0, v0 = p.copy(), m.copy(), v.copy()
    lp = oracle.adamw_step(p, m, v, g, "bf16", "bf16", h, step=3)
    assert np.array_equal(p.view(np.uint32), p0.view(np.uint32))
    assert not np.array_equal(m, m0) and not np.array_equal(v, v0)
    assert np.array_equal(lp, oracle.round_bf16(p0))


def test_no_momentum_no_decay_reduces_to_normalised_gradient():
    # beta1 = beta2 = 0, wd = 0: p' = p - lr * g / (|g| + eps), m' = g, v' = g^2, any t
    p, m, v, g = _state(5000, 25)
    h = oracle.hyper(lr=1e-3, beta1=0.0, beta2=0.0, eps=1e-5, weight_decay=0.0)
    gd = _widen(g, "bf16")
    p0 = p.astype(np.float64)
    oracle.adamw_step(p, m, v, g, "bf16", "bf16", h, step=9)
    lr, eps = float(np.float32(1e-3)), float(np.float32(1e-5))
    assert np.max(np.abs(p - (p0 - lr * gd / (np.abs(gd) + eps)))) <= 4 * EPS32 * np.max(np.abs(p0))
    assert np.array_equal(m, gd.astype(np.float32))
    np.testing.assert_allclose(v, gd * gd, rtol=EPS32, atol=1e-45)


def test_bias_correction_switch():
    p, m, v, g = _state(3000, 26)
    h1 = oracle.hyper(bias_correction=1)
    h0 = oracle.hyper(bias_correction=0)
    s1 = oracle.step_scalars(h1, 10)
    s0 = oracle.step_scalars(h0, 10)
    b1, b2, lr = float(np.float32(0.9)), float(np.float32(0.999)), float(np.float32(1e-5))
    assert s1[5] == np.float32(lr / (1 - b1 ** 10)) and s0[5] == np.float32(lr)
    assert s1[6] == np.float32(1 / np.sqrt(1 - b2 ** 10)) and s0[6] == np.float32(1.0)
    assert s1[2] == np.float32(1 - b1) and s1[3] == np.float32(1 - b2)
    assert s1[7] == np.float32(lr * float(np.float32(0.01)))
    # t -> infinity: bias correction fades, both switches agree
    pa, ma, va = p.copy(), m.copy(), v.copy()
    pb, mb, vb = p.copy(), m.copy(), v.copy()
    oracle.adamw_step(pa, ma, va, g, "bf16", "bf16", h1, step=10 ** 6)
    oracle.adamw_step(pb, mb, vb, g, "bf16", "bf16", h0, step=10 ** 6)
    assert np.array_equal(pa, pb)


def test_unscale_and_clip_scalar():
    h = oracle.hyper()
    assert oracle.step_scalars(h, 1, loss_scale=65536.0, clip=0.5)[8] == np.float32(0.5 / 65536.0)
    # a gradient stored at scale S with clip c gives the same step as the unscaled gradient
    # times c stored at scale 1, when both multiplications are exact (powers of two)
    rng = np.random.default_rng(3)
    base = (rng.standard_normal(2048) * 1e-3).astype(np.float16)
    p, m, v, _ = _state(2048, 27)
    pa, ma, va = p.copy(), m.copy(), v.copy()
    pb, mb, vb = p.copy(), m.copy(), v.copy()
    g_scaled = (base.astype(np.float32) * 1024.0).astype(np.float16)
    g_pre = (base.astype(np.float32) * 0.5).astype(np.float16)
    keep = (g_pre.astype(np.float32) * 2.0 == base.astype(np.float32))       # no underflow in 0.5x
    oracle.adamw_step(pa, ma, va, g_scaled.view(np.uint16), "f16", "f16", h, 5, 1024.0, 0.5)
    oracle.adamw_step(pb, mb, vb, g_pre.view(np.uint16), "f16", "f16", h, 5, 1.0, 1.0)
    assert keep.sum() > 1500
    assert np.array_equal(pa[keep], pb[keep]) and np.array_equal(ma[keep], mb[keep])


def test_exact_symmetries():
    p, m, v, g = _state(4000, 28)
    h = oracle.hyper(lr=1e-3, eps=1e-6, weight_decay=0.05)
    pa, ma, va = p.copy(), m.copy(), v.copy()
    lpa = oracle.adamw_step(pa, ma, va, g, "bf16", "bf16", h, 4)
    # negate p, m, g: p', m' negate, v' unchanged (round-to-nearest is symmetric)
    pb, mb, vb = -p, -m, v.copy()
    lpb = oracle.adamw_step(pb, mb, vb, g ^ 0x8000, "bf16", "bf16", h, 4)
    assert np.array_equal(pb, -pa) and np.array_equal(mb, -ma) and np.array_equal(vb, va)
    assert np.array_equal(lpb, lpa ^ 0x8000)
    # scale m and g by 4 (exact): m' scales by 4, v' by 16 -- with beta only, no eps involvement
    pc, mc, vc = p.copy(), (m * 4).astype(np.float32), (v * 16).astype(np.float32)
    g4 = oracle.round_bf16((oracle.widen_bf16(g) * 4).astype(np.float32))
    oracle.adamw_step(pc, mc, vc, g4, "bf16", "bf16", h, 4)
    assert np.array_equal(mc, ma * 4) and np.array_equal(vc, va * 16)


@pytest.mark.parametrize("gdt,scale,clip", [("bf16", 1.0, 1.0), ("f16", 65536.0, 0.37), ("bf16", 1.0, 0.1)])
def test_fp32_step_is_bounded_by_fp64_evaluation(gdt, scale, clip):
    p, m, v, g = _state(50000, 29, gdt=gdt, scale=scale)
    h = oracle.hyper(lr=1e-3, eps=1e-6, weight_decay=0.05)
    p64, m64, v64 = oracle.adamw_step_f64(p, m, v, g, gdt, h, 100, scale, clip)
    p0, m0 = p.astype(np.float64), m.astype(np.float64)
    oracle.adamw_step(p, m, v, g, gdt, "bf16", h, 100, scale, clip)
    gd = _widen(g, gdt) * clip / scale
    # m' and v' are two-term sums: error <= a few ulp of the larger term (m' may cancel, so the
    # bound is on the terms, not on the result)
    mterms = np.abs(0.9 * m0) + np.abs(0.1 * gd)
    assert np.all(np.abs(m - m64) <= 4 * EPS32 * mterms + 1e-45)
    assert np.all(np.abs(v - v64) <= 4 * EPS32 * np.abs(v64) + 1e-45)
    # p' = q - step*m'/d: rounding of q and of p' (<= 1 ulp of p each), the error of m' carried
    # through step/d, and a few relative roundings of the quotient chain
    bc1, bc2 = 1 - float(np.float32(0.9)) ** 100, 1 - float(np.float32(0.999)) ** 100
    d = np.sqrt(v64 / bc2) + float(np.float32(1e-6))
    carried = float(np.float32(1e-3)) / bc1 / d * (4 * EPS32 * mterms)
    upd = np.abs(p64 - p0)
    assert np.all(np.abs(p - p64) <= 2 * EPS32 * np.abs(p0) + carried + 8 * EPS32 * upd + 1e-45)
    assert np.median(upd) > 100 * EPS32 * np.median(np.abs(p0))   # the bound is not vacuous


@pytest.mark.parametrize("wd,eps,lr", [(0.1, 1e-3, 1e-2), (0.0, 1e-8, 1e-3), (0.3, 1e-5, 3e-2)])
def test_trajectory_against_library_adamw_in_fp64(wd, eps, lr):
    """Five steps from non-zero moments at t = 3..7, compared with torch.optim.AdamW on fp64
    tensors.  Hyper-parameters are large on purpose: with lr*wd ~ 1e-3 and eps comparable to
    sqrt(v), a misplaced eps, decay on the wrong p, a missing or swapped bias correction or
    swapped betas each move p by far more than the tolerance."""
    n = 4000
    p, m, v, _ = _state(n, 31, m_std=1e-3, v_std=1e-6)
    h = oracle.hyper(lr=lr, beta1=0.8, beta2=0.95, eps=eps, weight_decay=wd)
    f = lambda x: float(np.float32(x))
    tp = torch.tensor(p.astype(np.float64), requires_grad=True)
    opt = torch.optim.AdamW([tp], lr=f(lr), betas=(f(0.8), f(0.95)), eps=f(eps), weight_decay=f(wd),
                            foreach=False, fused=False, amsgrad=False, maximize=False)
    opt.state[tp] = {"step": torch.tensor(2.0), "exp_avg": torch.tensor(m.astype(np.float64)),
                     "exp_avg_sq": torch.tensor(v.astype(np.float64))}
    rng = np.random.default_rng(33)
    for t in range(3, 8):
        g = oracle.round_bf16((rng.standard_normal(n) * 1e-3).astype(np.float32))
        clip = 0.5 if t % 2 else 1.0
        p_before = p.astype(np.float64)
        tp_before = tp.detach().clone().numpy()
        oracle.adamw_step(p, m, v, g, "bf16", "bf16", h, t, 1.0, clip)
        tp.grad = torch.tensor(_widen(g, "bf16") * clip)
        opt.step()
        d_or = p.astype(np.float64) - p_before
        d_lib = tp.detach().numpy() - tp_before
        # per-step update agrees to fp32 rounding of p plus a relative 1e-5 of the update
        assert np.all(np.abs(d_or - d_lib) <= 2 * EPS32 * np.abs(p_before) + 1e-5 * np.abs(d_lib))
        assert np.median(np.abs(d_lib)) > 100 * EPS32 * np.median(np.abs(p_before))
        np.testing.assert_allclose(m, opt.state[tp]["exp_avg"].numpy(), rtol=1e-4, atol=1e-9)
        np.testing.assert_allclose(v, opt.state[tp]["exp_avg_sq"].numpy(), rtol=1e-4, atol=1e-12)
    np.testing.assert_allclose(p, tp.detach().numpy(), rtol=1e-5, atol=1e-7)


@pytest.mark.parametrize("pdt", ["bf16", "f16"])
def test_low_precision_copy_is_the_rounded_new_p(pdt):
    p, m, v, g = _state(30000, 35)
    h = oracle.hyper()
    lp = oracle.adamw_step(p, m, v, g, "bf16", pdt, h, 2)
    rnd = oracle.round_bf16 if pdt == "bf16" else oracle.round_f16
    assert np.array_equal(lp, rnd(p))


def test_threads_do_not_change_the_step():
    p, m, v, g = _state(100_003, 36)
    h = oracle.hyper()
    pa, ma, va = p.copy(), m.copy(), v.copy()
    la = oracle.adamw_step(pa, ma, va, g, "bf16", "bf16", h, 2)
    lb = oracle.adamw_step(p, m, v, g, "bf16", "bf16", h, 2, nthreads=5)
    assert np.array_equal(pa, p) and np.array_equal(ma, m) and np.array_equal(va, v)
    assert np.array_equal(la, lb)


@pytest.mark.parametrize("gdt", ["bf16", "f16"])
def test_any_nonfinite_gradient_skips_the_step(gdt):
    n = 10_000
    p, m, v, g = _state(n, 37, gdt=gdt, scale=65536.0 if gdt == "f16" else 1.0)
    h = oracle.hyper()
    lp0 = oracle.round_bf16(p)
    for pos in (0, n - 1, 4321):
        for bits in synth.NONFINITE_BITS[gdt]:
            gg = g.copy()
            gg[pos] = bits
            pa, ma, va, lpa = p.copy(), m.copy(), v.copy(), lp0.copy()
            ov, _, _ = oracle.optimizer_step(pa, ma, va, gg, gdt, lpa, "bf16", h, 5,
                                             65536.0 if gdt == "f16" else 1.0, 1.0)
            assert ov is True
            assert pa.tobytes() == p.tobytes() and ma.tobytes() == m.tobytes()
            assert va.tobytes() == v.tobytes() and lpa.tobytes() == lp0.tobytes()
    # the clean gradient does step, with the clip the norm implies
    pa, ma, va, lpa = p.copy(), m.copy(), v.copy(), lp0.copy()
    S = 65536.0 if gdt == "f16" else 1.0
    ov, ss, c = oracle.optimizer_step(pa, ma, va, g, gdt, lpa, "bf16", h, 5, S, 0.01)
    assert ov is False and c == oracle.clip_coef(ss, float(np.float32(0.01))) and c < 1
    pb, mb, vb = p.copy(), m.copy(), v.copy()
    lpb = oracle.adamw_step(pb, mb, vb, g, gdt, "bf16", h, 5, S, float(c))
    assert np.array_equal(pa, pb) and np.array_equal(lpa, lpb) and not np.array_equal(pa, p)


def test_8b_shaped_list_matches_printed_buffer_size(golden_dir):
    vals = {}
    with open(golden_dir + "/flat_buffer_size.txt") as f:
        for line in f:
            if not line.startswith("#") and line.strip():
                k, x = line.split()
                vals[k] = float(x)
    total = sum(n for _, n in synth.llama3_8b_shapes())
    assert total == 8_030_257_152
    assert abs(total * 4 / 2 ** 30 - vals["flat_buffer_gib"]) < 0.01
    assert abs(total * 4 * 2.25 / 2 ** 30 - vals["peak_during_check_gib"]) < 0.02
    assert sum(n for _, n in synth.qwen14b_class_shapes()) == 12_567_592_960


# ---- every rounding of the step, re-derived in exact rational arithmetic ------------------------
# Each fp32 operation of the step returns the representable value nearest to the exact result (ties
# to the even significand), subnormal results included; an addition exists only as the tail of a
# fused multiply-add, which rounds once.  Below, the exact result of every operation is a Fraction
# and `_rnd32` is that rounding written from its definition, so the comparison does not depend on
# the host's floating-point unit, its flush-to-zero switches or its library.
from fractions import Fraction
from math import isqrt


def _rnd32(x: Fraction) -> Fraction:
    if x == 0:
        return x
    a = abs(x)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1                                   # now 2^e <= a < 2^(e+1)
    q = Fraction(2) ** (max(e, -126) - 23)       # spacing of fp32 values around a (subnormal: 2^-149)
    k, r = divmod(a, q)
    if 2 * r > q or (2 * r == q and k % 2 == 1):
        k += 1
    assert k * q < Fraction(2) ** 128            # the cases below stay finite
    return k * q if x > 0 else -(k * q)


def _sqrt32(x: Fraction) -> Fraction:
    """Correctly rounded square root of an fp32 value: integer square root with 80 extra bits and a
    sticky half-unit (the root of an fp32 value is never a rounding midpoint)."""
    if x == 0:
        return x
    t = 200
    n = x * Fraction(4) ** t
    assert n.denominator == 1
    s = isqrt(n.numerator)
    exact = s * s == n.numerator
    return _rnd32(Fraction(s, 2 ** t) if exact else Fraction(2 * s + 1, 2 ** (t + 1)))


@pytest.mark.parametrize("case", synth.EXTREME_CASES)
def test_every_rounding_against_exact_rational_arithmetic(case):
    n, step = 1200, 7
    p, m, v, g, gdt, scale, clip, eps = synth.extreme_case(case, n)
    if gdt == "bf16":
        w = (g.astype(np.uint32) << 16).view(np.float32)
        assert case != "subnormal" or np.count_nonzero((g & 0x7F80) == 0) > n // 4     # bf16 subnormal patterns occur
    else:
        w = g.view(np.float16).astype(np.float32)
        assert np.count_nonzero((g & 0x7C00) == 0) > n // 2                             # fp16 subnormal patterns
    h = oracle.hyper(lr=1e-3, beta1=0.9, beta2=0.999, eps=eps, weight_decay=0.1)
    s = [Fraction(float(x)) for x in oracle.step_scalars(h, step, scale, clip)]
    b1, b2, omb1, omb2, eps_, step_size, isb2, decay, gscale = s
    assert eps_ > 0
    want = []
    for i in range(n):
        P, M, V, W = (Fraction(float(x[i])) for x in (p, m, v, w))
        G = _rnd32(W * gscale)
        M1 = _rnd32(b1 * M + _rnd32(omb1 * G))
        V1 = _rnd32(b2 * V + _rnd32(omb2 * _rnd32(G * G)))
        D = _rnd32(_sqrt32(V1) * isb2 + eps_)
        U = _rnd32(M1 / D)
        Q = _rnd32(-decay * P + P)
        want.append((float(_rnd32(-step_size * U + Q)), float(M1), float(V1)))
    want = np.array(want, np.float64)
    lp = oracle.adamw_step(p, m, v, g, gdt, "bf16", h, step, scale, clip)
    for k, (name, got) in enumerate((("p", p), ("m", m), ("v", v))):
        bad = np.nonzero(got.astype(np.float64) != want[:, k])[0]
        assert bad.size == 0, "%s[%d]: oracle %r, exact %r" % (name, bad[0], got[bad[0]], want[bad[0], k])
    assert np.array_equal(lp, oracle.round_bf16(p))
    if case.startswith("subnormal"):     # the case really lives where it claims to
        tiny = float(np.finfo(np.float32).tiny)
        assert np.count_nonzero((np.abs(m) < tiny) & (m != 0)) > n // 2
    if case == "subnormal":
        tiny = float(np.finfo(np.float32).tiny)
        assert np.count_nonzero((np.abs(v) < tiny) & (v != 0)) > n // 2
