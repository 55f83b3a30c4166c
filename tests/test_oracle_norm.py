"""Pins for the oracle's overflow flag and sum of squares.

Flag: the oracle classifies the widened value (isinf or isnan).  It is pinned against the
exponent-mask rule of Algorithm 1 (Sec. IV-D) on every 16-bit pattern of both gradient
formats, against the fp32 patterns of tests/golden/fp32_overflow_patterns.txt, and against
the unfused library chain that Sec. III-C describes (isinf().any() or isnan().any()).
Sum of squares: exact rational arithmetic on small inputs, closed forms, scale invariance.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from paper_2505_23254_amd import synth

MASK = {"bf16": 0x7F80, "f16": 0x7C00}


@pytest.mark.parametrize("gdt", ["bf16", "f16"])
def test_flag_equals_exponent_mask_rule_on_every_pattern(gdt):
    for b in range(65536):
        g = np.array([b], np.uint16)
        ov, _ = oracle.overflow_norm(g, gdt)
        assert ov == ((b & MASK[gdt]) == MASK[gdt]), hex(b)


def test_flag_on_printed_fp32_mask(golden_dir):
    rows = 0
    with open(golden_dir + "/fp32_overflow_patterns.txt") as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            a = line.split()
            bits, want = int(a[0], 16), bool(int(a[1]))
            assert want == ((bits & 0x7F800000) == 0x7F800000)   # the fixture obeys Algorithm 1
            g = np.array([bits], np.uint32).view(np.float32)
            ov, _ = oracle.overflow_norm(g, "f32")
            assert ov == want, a
            rows += 1
    assert rows >= 15


@pytest.mark.parametrize("gdt", ["bf16", "f16"])
@pytest.mark.parametrize("n", [1, 2, 7, 64, 1000, 4097])
def test_single_planted_value_is_found_anywhere(gdt, n):
    cfg = synth.FlatConfig("t", n, seed=3, gdt=gdt)
    base = synth.bits16(synth.make_flat(cfg).g)
    assert oracle.overflow_norm(base, gdt)[0] is False
    for pos in sorted({0, n - 1, n // 2, n // 3}):
        for bits in synth.NONFINITE_BITS[gdt]:
            g = base.copy()
            g[pos] = bits
            assert oracle.overflow_norm(g, gdt)[0] is True
            assert oracle.overflow_norm(g, gdt, nthreads=3)[0] is True


@pytest.mark.parametrize("gdt", ["bf16", "f16"])
def test_flag_equals_unfused_library_chain(gdt):
    # Sec. III-C: the baseline decides the same thing with isinf().any() then isnan().any().
    tdt = torch.bfloat16 if gdt == "bf16" else torch.float16
    rng = np.random.default_rng(5)
    for trial in range(200):
        n = int(rng.integers(1, 300))
        bits = rng.integers(0, 65536, n, dtype=np.uint32).astype(np.uint16)
        if trial % 2 == 0:                       # make half the trials finite-only
            bits = np.where((bits & MASK[gdt]) == MASK[gdt], bits & 0x3FFF, bits).astype(np.uint16)
        t = torch.from_numpy(bits.view(np.int16)).view(tdt)
        want = bool(torch.isinf(t).any() or torch.isnan(t).any())
        assert oracle.overflow_norm(bits, gdt)[0] == want


def _exact_sumsq(bits, gdt, scale):
    widen = oracle.widen_bf16 if gdt == "bf16" else oracle.widen_f16
    vals = widen(bits)
    tot = Fraction(0)
    for x in vals.tolist():
        q = Fraction(x) / Fraction(scale)
        tot += q * q
    return tot


@pytest.mark.parametrize("gdt,scale", [("bf16", 1.0), ("f16", 65536.0), ("bf16", 3.0), ("f16", 1000.0)])
def test_sumsq_against_exact_rational_sum(gdt, scale):
    cfg = synth.FlatConfig("t", 513, seed=11, gdt=gdt, loss_scale=scale)
    bits = synth.bits16(synth.make_flat(cfg).g)
    ov, ss = oracle.overflow_norm(bits, gdt, loss_scale=scale)
    exact = _exact_sumsq(bits, gdt, scale)
    assert not ov
    assert abs(Fraction(ss) - exact) <= exact * Fraction(1, 10 ** 13)
    _, ss3 = oracle.overflow_norm(bits, gdt, loss_scale=scale, nthreads=3)
    assert abs(Fraction(ss3) - exact) <= exact * Fraction(1, 10 ** 13)


def test_sumsq_closed_forms():
    one_bf16, one_f16 = 0x3F80, 0x3C00
    for n in (1, 5, 1000, 65537):
        assert oracle.overflow_norm(np.full(n, one_bf16, np.uint16), "bf16")[1] == float(n)
        assert oracle.overflow_norm(np.full(n, one_f16, np.uint16), "f16")[1] == float(n)
    # sum_{k=1..K} (k/64)^2 = K(K+1)(2K+1)/6/4096, every term exact in fp16 and in fp64
    K = 2000
    vals = (np.arange(1, K + 1) / 64.0).astype(np.float16)
    got = oracle.overflow_norm(vals.view(np.uint16), "f16")[1]
    assert got == K * (K + 1) * (2 * K + 1) / 6 / 4096
    # scaled by a power of two: sum (g/S)^2 = sum g^2 / S^2 exactly
    got = oracle.overflow_norm(vals.view(np.uint16), "f16", loss_scale=8.0)[1]
    assert got == K * (K + 1) * (2 * K + 1) / 6 / 4096 / 64
    # signs do not matter, empty input sums to zero without overflow
    neg = (-np.arange(1, K + 1) / 64.0).astype(np.float16)
    assert oracle.overflow_norm(neg.view(np.uint16), "f16")[1] == K * (K + 1) * (2 * K + 1) / 6 / 4096
    assert oracle.overflow_norm(np.zeros(0, np.uint16), "bf16") == (False, 0.0)


def test_sumsq_matches_fsum_and_statistics():
    import math
    cfg = synth.FlatConfig("t", 200_000, seed=13, gdt="bf16")
    bits = synth.bits16(synth.make_flat(cfg).g)
    vals = oracle.widen_bf16(bits).astype(np.float64)
    want = math.fsum((vals * vals).tolist())
    _, got = oracle.overflow_norm(bits, "bf16")
    assert abs(got - want) <= 1e-12 * want
    # N(0, sigma^2): sumsq = n sigma^2 (1 +- a few sqrt(2/n)); bf16 rounding adds ~1e-5 relative
    n, sigma = bits.size, cfg.g_std
    assert abs(got / (n * sigma * sigma) - 1.0) < 5 * math.sqrt(2.0 / n) + 1e-3


def test_loss_scale_invariance_fp16():
    # the same underlying gradient stored at two power-of-two scales gives the same sumsq
    rng = np.random.default_rng(17)
    base = (rng.standard_normal(4096) * 1e-3).astype(np.float32)
    s1, s2 = 1024.0, 65536.0
    g1 = (base * s1).astype(np.float16)
    g2 = (g1.astype(np.float32) * (s2 / s1)).astype(np.float16)   # exact: power-of-two factor
    a = oracle.overflow_norm(g1.view(np.uint16), "f16", loss_scale=s1)[1]
    b = oracle.overflow_norm(g2.view(np.uint16), "f16", loss_scale=s2)[1]
    assert a == b


def test_clip_coef():
    assert oracle.clip_coef(100.0, 1.0) == np.float32(1.0 / (10.0 + 1e-6))
    assert oracle.clip_coef(0.25, 1.0) == np.float32(1.0)       # norm 0.5 < max_norm
    assert oracle.clip_coef(4.0, 1.0) == np.float32(1.0 / (2.0 + 1e-6))
    assert oracle.clip_coef(1e30, 0.0) == np.float32(1.0)       # disabled
    assert oracle.clip_coef(1e30, -1.0) == np.float32(1.0)
    assert oracle.clip_coef(0.0, 1.0) == np.float32(1.0)
