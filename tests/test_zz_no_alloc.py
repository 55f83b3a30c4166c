"""The scan entry point that allocates nothing (ma_overflow_norm_static): called through the C ABI,
compared with ma_overflow_norm on the same inputs, twice in a row, the second time on a smaller
input whose result differs (the library's scratch keeps the first call's contents)."""
import gc
import struct

import pytest
import torch

from paper_2505_23254_amd import synth

pytestmark = pytest.mark.gpu


def _raw(res, index=0):
    """The 16 bytes of one result slot: (overflow, reserved, bits of sumsq)."""
    b = res[2 * index:2 * index + 2].cpu().numpy().tobytes()
    ov, rsv = struct.unpack("<ii", b[:8])
    return ov, rsv, b[8:]


@pytest.mark.parametrize("dtype,scale", [(torch.bfloat16, 1.0), (torch.float16, 1024.0), (torch.float32, 8.0)])
def test_static_scratch_scan_matches_workspace_scan(dtype, scale):
    from paper_2505_23254_amd import binding as ma
    assert torch.cuda.is_available()
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1234)
    big = torch.empty(40_000_003, dtype=dtype, device="cuda")         # > 1024 work items: the full grid, ragged tail
    synth._fill_grad(big, 1e-3, scale, gen)
    small = big[5:5 + 300_001]                                        # a few work items, misaligned start
    raw = big.view(torch.int32 if dtype == torch.float32 else torch.int16)
    raw[39_999_999] = {torch.bfloat16: 0x7F80, torch.float16: 0x7C00, torch.float32: 0x7F800000}[dtype]   # +inf
    ws = ma.workspace()
    want, got = ma.new_result(2), ma.new_result(2)
    ma.overflow_norm(big, scale, want, ws, index=0)
    ma.overflow_norm(small, scale, want, ws, index=1)
    gc.collect()                                                      # tensors of earlier tests go now, not in between
    before = torch.cuda.memory_allocated()
    ma.overflow_norm_static(big, scale, got, index=0)                 # first call: overflow, all slots written
    ma.overflow_norm_static(small, scale, got, index=1)               # second call, smaller, clean
    assert torch.cuda.memory_allocated() <= before                    # nothing was allocated through torch either
    torch.cuda.synchronize()
    assert _raw(want, 0)[0] == 1 and _raw(want, 1)[0] == 0
    # flag exact; the sum comes from the same kernels in the same order: the same bits
    assert _raw(got, 0)[:2] == _raw(want, 0)[:2]
    assert _raw(got, 1) == _raw(want, 1)
    ss_w, ss_g = ma.read_result(want, 1)[1], ma.read_result(got, 1)[1]
    assert ss_w > 0 and abs(ss_g - ss_w) <= 1e-5 * ss_w
    # n == 0 writes {0, 0.0}; a size beyond the stated maximum is refused before any launch
    ma.overflow_norm_static(big, scale, got, index=0, n=0)
    assert ma.read_result(got, 0) == (False, 0.0)
    with pytest.raises(ma.MaError) as e:
        ma.overflow_norm_static(big, scale, got, index=0, n=(1 << 38) + 1)
    assert e.value.code == ma.MA_ERR_ARG and "maximum" in str(e.value)
