"""Pins for the oracle's widening and round-to-nearest-even narrowing.

The oracle rounds from the definition (nearest representable value, ties to even, in fp64
arithmetic).  It is pinned here against things that are not that code: hand-worked ties
(tests/golden/rne_ties.txt), the integer add-and-shift rule, and the converters of two
libraries (torch for bf16, numpy for fp16) over every pattern family where a rounding
mistake could hide.
"""
import numpy as np
import pytest
import torch

import oracle


def _all16():
    return np.arange(65536, dtype=np.uint32).astype(np.uint16)


def _pattern_family():
    """fp32 patterns: every upper half combined with the lower halves that decide rounding,
    plus seeded random patterns."""
    hi = np.arange(65536, dtype=np.uint32) << 16
    lows = [0x0000, 0x0001, 0x0FFF, 0x1000, 0x1001, 0x1FFF, 0x2000, 0x3000, 0x7FFF, 0x8000,
            0x8001, 0xFFFF]
    fam = np.concatenate([hi | lo for lo in lows])
    rng = np.random.default_rng(1234)
    rnd = rng.integers(0, 1 << 32, size=2_000_000, dtype=np.uint64).astype(np.uint32)
    return np.concatenate([fam, rnd])


def _golden(golden_dir, fmt):
    rows = []
    with open(golden_dir + "/rne_ties.txt") as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            a = line.split()
            if a[0] == fmt:
                rows.append((int(a[1], 16), int(a[2], 16), " ".join(a[3:])))
    assert len(rows) >= 20
    return rows


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_hand_worked_ties(golden_dir, fmt):
    fn = oracle.round_bf16 if fmt == "bf16" else oracle.round_f16
    for src, want, remark in _golden(golden_dir, fmt):
        x = np.array([src], np.uint32).view(np.float32)
        got = int(fn(x)[0])
        assert got == want, "%s %#010x: got %#06x want %#06x (%s)" % (fmt, src, got, want, remark)


def test_widen_bf16_all_patterns_vs_torch():
    b = _all16()
    got = oracle.widen_bf16(b).view(np.uint32)
    ref = torch.from_numpy(b.view(np.int16)).view(torch.bfloat16).to(torch.float32)
    ref = ref.numpy().view(np.uint32)
    assert np.array_equal(got, ref)  # including NaN payloads: widening is a pure shift


def test_widen_f16_all_patterns_vs_numpy():
    b = _all16()
    got = oracle.widen_f16(b)
    ref = b.view(np.float16).astype(np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got.view(np.uint32)[~nan], ref.view(np.uint32)[~nan])
    # closed form of one subnormal and one normal, by hand: 0x0001 = 2^-24, 0x3555 ~ 1/3
    assert oracle.widen_f16(np.array([0x0001], np.uint16))[0] == np.float32(2.0 ** -24)
    assert oracle.widen_f16(np.array([0x3555], np.uint16))[0] == np.float32(1365.0 / 4096.0)
    assert oracle.widen_f16(np.array([0xC000], np.uint16))[0] == np.float32(-2.0)


def test_round_bf16_vs_integer_rule_and_torch():
    bits = _pattern_family()
    x = bits.view(np.float32)
    got = oracle.round_bf16(x)
    nan = np.isnan(x)
    # add-and-shift rule on the raw pattern (a different mechanism from the oracle's)
    b64 = bits.astype(np.uint64)
    rule = ((b64 + 0x7FFF + ((b64 >> 16) & 1)) >> 16).astype(np.uint16)
    assert np.array_equal(got[~nan], rule[~nan])
    # library converter
    ref = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got[~nan], ref[~nan])
    # NaN stays NaN (exponent all ones, non-zero fraction), sign kept, quiet bit set
    g = got[nan]
    assert np.all((g & 0x7F80) == 0x7F80) and np.all((g & 0x007F) != 0)
    assert np.all((g & 0x0040) != 0)
    assert np.array_equal(g >> 15, (bits[nan] >> 31).astype(np.uint16))


def test_round_f16_vs_numpy():
    bits = _pattern_family()
    x = bits.view(np.float32)
    got = oracle.round_f16(x)
    nan = np.isnan(x)
    with np.errstate(over="ignore", invalid="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(got[~nan], ref[~nan])
    g = got[nan]
    assert np.all((g & 0x7C00) == 0x7C00) and np.all((g & 0x0200) != 0)
    assert np.array_equal(g >> 15, (bits[nan] >> 31).astype(np.uint16))


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_round_trip_is_identity(fmt):
    b = _all16()
    widen = oracle.widen_bf16 if fmt == "bf16" else oracle.widen_f16
    rnd = oracle.round_bf16 if fmt == "bf16" else oracle.round_f16
    quiet = 0x0040 if fmt == "bf16" else 0x0200
    x = widen(b)
    back = rnd(x)
    nan = np.isnan(x)
    assert np.array_equal(back[~nan], b[~nan])
    assert np.array_equal(back[nan], b[nan] | quiet)


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_rounding_is_nearest_and_monotone(fmt):
    """Property form of the definition: the result is never farther from x than either
    neighbouring representable value, and rounding preserves order."""
    widen = oracle.widen_bf16 if fmt == "bf16" else oracle.widen_f16
    rnd = oracle.round_bf16 if fmt == "bf16" else oracle.round_f16
    rng = np.random.default_rng(7)
    if fmt == "bf16":
        x = (rng.standard_normal(200_000) * 10.0 ** rng.uniform(-30, 30, 200_000)).astype(np.float32)
    else:
        x = (rng.standard_normal(200_000) * 10.0 ** rng.uniform(-9, 4, 200_000)).astype(np.float32)
    x = x[np.isfinite(x)]
    r = rnd(x)
    y = widen(r).astype(np.float64)
    fin = np.isfinite(y)
    up = widen((r[fin] + 1).astype(np.uint16)).astype(np.float64)    # next pattern, same sign
    dn_bits = np.where((r[fin] & 0x7FFF) == 0, r[fin] ^ 0x8000 | 1, r[fin] - 1).astype(np.uint16)
    dn = widen(dn_bits).astype(np.float64)
    xd = x[fin].astype(np.float64)
    err = np.abs(y[fin] - xd)
    ok_up = ~np.isfinite(up) | (err <= np.abs(up - xd))
    assert np.all(ok_up)
    assert np.all(err <= np.abs(dn - xd))
    order = np.argsort(x, kind="stable")
    ys = widen(rnd(x[order])).astype(np.float64)
    assert np.all(np.diff(ys) >= 0)
