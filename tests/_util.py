"""Helpers shared by the GPU parity tests: host copies, ulp distance, oracle drivers."""
import numpy as np
import torch

import oracle
from paper_2505_23254_amd import synth

GDT_NAME = {torch.bfloat16: "bf16", torch.float16: "f16", torch.float32: "f32"}

# tolerances of the parity bar
MAX_ULP = 2          # p / m / v against the oracle, in fp32 units in the last place
SUMSQ_RTOL = 1e-5    # relative, sum of squares


def host_f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().numpy().copy()


def host_grad(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.float32:
        return host_f32(t)
    return synth.bits16(t)


def ulp_distance(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Distance in representable fp32 values between a and b (NaN vs NaN counts as 0)."""
    ia = a.view(np.int32).astype(np.int64)
    ib = b.view(np.int32).astype(np.int64)
    ia = np.where(ia < 0, -(ia & 0x7FFFFFFF), ia)
    ib = np.where(ib < 0, -(ib & 0x7FFFFFFF), ib)
    d = np.abs(ia - ib)
    both_nan = np.isnan(a) & np.isnan(b)
    return np.where(both_nan, 0, d)


def oracle_hyper(cfg):
    return oracle.hyper(cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, cfg.weight_decay, 1)


def round_lp(p: np.ndarray, pdt: str) -> np.ndarray:
    return oracle.round_bf16(p) if pdt == "bf16" else oracle.round_f16(p)


def assert_state_close(gpu, ref, what=""):
    """gpu / ref: dicts with fp32 arrays p, m, v and the uint16 array lp plus pdt."""
    for k in ("p", "m", "v"):
        d = ulp_distance(gpu[k], ref[k])
        worst = int(d.max()) if d.size else 0
        assert worst <= MAX_ULP, "%s %s: %d ulp at index %d" % (what, k, worst, int(d.argmax()))
    # the low-precision copy is the rounded fp32 parameter, bit for bit
    assert np.array_equal(gpu["lp"], round_lp(gpu["p"], ref["pdt"])), "%s p_lp != RNE(p)" % what
    same = gpu["p"].view(np.uint32) == ref["p"].view(np.uint32)
    assert np.array_equal(gpu["lp"][same], ref["lp"][same]), "%s p_lp differs from oracle" % what
