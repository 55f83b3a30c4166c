"""Host side of the offloading system (no GPU): the parameter-buffer-pool sizes of Sec. III-A / IV-B
and the pinned-allocation sizes of Sec. III-B / IV-C.  The plain oracle (oracle/pool.py) is pinned to
the numbers the paper prints; the library's layout is then compared with the oracle, and the pool
manager is checked by invariants over random acquire / release sequences."""
import ctypes
import random
from fractions import Fraction

import pytest

from oracle import pool as ref
from paper_2505_23254_amd import binding as ma

GIB = 1 << 30


def _golden(golden_dir):
    models, extra = {}, {}
    for line in open(golden_dir + "/buffer_pool_sizes.txt"):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if "|" in line:
            left, vals, _ = [x.strip() for x in line.split("|", 2)]
            name, *dims = left.split()
            models[name] = (tuple(int(d) for d in dims), [None if v == "-" else float(v) for v in vals.split()])
        else:
            k, *v = line.split()
            extra[k] = [float(x) for x in v]
    return models, extra


def test_oracle_reproduces_the_printed_pool_sizes(golden_dir):
    models, extra = _golden(golden_dir)
    assert len(models) == 4
    reductions = []
    for name, (dims, (uni, ada, red)) in models.items():
        u, a = ref.uniform_pool_bytes(dims), ref.adaptive_pool_bytes(dims)
        if uni is not None:
            assert round(u / GIB, 2) == uni, name
        if ada is not None:
            assert round(a / GIB, 2) == ada, name
        if red is not None:
            got = 100 * float(ref.fragmentation(dims))
            assert round(got, 2) == red or round(got) == red, (name, got)
        reductions.append(100 * ref.fragmentation(dims))
    avg = float(sum(reductions) / len(reductions))
    assert abs(avg - extra["average_reduction_percent"][0]) <= 0.01
    # the remark of the evaluation: same uniform pool for the 14B and 32B shapes, adaptive pool larger for 32B
    assert ref.uniform_pool_bytes(models["qwen2.5-14b"][0]) == ref.uniform_pool_bytes(models["qwen2.5-32b"][0])
    assert ref.adaptive_pool_bytes(models["qwen2.5-14b"][0]) < ref.adaptive_pool_bytes(models["qwen2.5-32b"][0])
    # fp32 flat gradient buffer of the 7B model
    gib, params = extra["flat_buffer_qwen2.5-7b_GiB"]
    assert round(params * 4 / GIB, 2) == gib
    # power-of-two rounding example
    req, got = extra["pow2_example_GiB"]
    assert ref.pow2_bytes(int(req * GIB)) == int(got * GIB)


def test_oracle_pool_closed_forms():
    dims = (1000, 64, 256, 16, 64)
    for n in (1, 2, 5):
        # 2 + 7N buffers, N blocks of 3 + 2 + 2 tensors
        assert ref.uniform_pool_bytes(dims, n) == (2 + 7 * n) * 1000 * 64 * 2
        assert ref.adaptive_pool_bytes(dims, n) == 2 * (2 * 64000 + n * (3 * 16384 + 2 * 1024 + 2 * 4096))
    # all tensors equal: no fragmentation at all
    assert ref.fragmentation((64, 64, 64, 64, 64), 3) == 0
    assert ref.fragmentation(dims, 1, 4) == ref.fragmentation(dims, 1, 2)      # independent of the element size
    assert [ref.pow2_bytes(x) for x in (0, 1, 2, 3, 4, 5, 1023, 1024, 1025)] == [0, 1, 2, 4, 4, 8, 1024, 1024, 2048]


def test_library_layout_equals_oracle(golden_dir):
    models, _ = _golden(golden_dir)
    for name, (dims, _) in models.items():
        for n in (1, 2, 4):
            for eb in (1, 2, 4):
                L = ma.pool_layout(*dims, blocks_in_flight=n, elem_bytes=eb)
                assert L.total_bytes == ref.adaptive_pool_bytes(dims, n, eb)
                assert L.uniform_bytes == ref.uniform_pool_bytes(dims, n, eb)
                assert list(L.count) == [2, 3 * n, 2 * n, 2 * n] and L.uniform_count == 2 + 7 * n
                t = ref.tensors(*dims)
                assert list(L.buffer_bytes) == [t[k] * eb for k in ("embed", "ffn", "kv", "qo")]
                off = 0
                for k in range(4):
                    assert L.offset[k] == off
                    off += L.count[k] * L.buffer_bytes[k]
    # sharding over data-parallel processes and page alignment
    dims = models["qwen2.5-7b"][0]
    full = ma.pool_layout(*dims)
    for parts in (2, 3, 8):
        L = ma.pool_layout(*dims, partitions=parts, align=4096)
        for k in range(4):
            exact = -(-full.buffer_bytes[k] // 2 // parts) * 2
            assert L.buffer_bytes[k] == -(-exact // 4096) * 4096
        assert L.total_bytes < full.total_bytes / parts * 1.01 + 9 * 4096


def test_layout_argument_errors():
    d = ma.ModelDims(100, 10, 20, 5, 10)
    out = ma.PoolLayout()
    f = ma.lib.ma_pool_layout_compute
    assert f(None, 1, 2, 1, 1, ctypes.byref(out)) == ma.MA_ERR_NULL
    assert f(ctypes.byref(d), 0, 2, 1, 1, ctypes.byref(out)) == ma.MA_ERR_ARG
    assert f(ctypes.byref(d), 1, 3, 1, 1, ctypes.byref(out)) == ma.MA_ERR_ARG
    assert f(ctypes.byref(d), 1, 2, 0, 1, ctypes.byref(out)) == ma.MA_ERR_ARG
    assert f(ctypes.byref(d), 1, 2, 1, 3, ctypes.byref(out)) == ma.MA_ERR_ARG
    z = ma.ModelDims(100, 0, 20, 5, 10)
    assert f(ctypes.byref(z), 1, 2, 1, 1, ctypes.byref(out)) == ma.MA_ERR_ARG
    huge = ma.ModelDims(1 << 30, 1 << 30, 20, 5, 10)
    assert f(ctypes.byref(huge), 1, 2, 1, 1, ctypes.byref(out)) == ma.MA_ERR_ARG
    bad = ma.PoolLayout()
    h = ctypes.c_void_p()
    assert ma.lib.ma_pool_create(ctypes.byref(bad), ctypes.byref(h)) == ma.MA_ERR_ARG


def test_pool_manager_invariants():
    """Random acquire / release traffic: live buffers never overlap, lie inside their sub-pool, have
    the sub-pool's exact size; a sub-pool never hands out more than its count; keys are unique."""
    L = ma.pool_layout(5000, 64, 300, 16, 64, blocks_in_flight=3, align=64)
    pool = ma.BufferPool(L)
    rng = random.Random(7)
    live = {}
    for step in range(5000):
        kind = rng.randrange(4)
        if live and (rng.random() < 0.45 or pool.in_use(kind) == L.count[kind]):
            key = rng.choice(list(live))
            assert pool.lookup(key) == live[key][1:]
            pool.release(key)
            del live[key]
            with pytest.raises(ma.MaError):
                pool.lookup(key)
            continue
        key = rng.getrandbits(48)
        if key in live:
            continue
        off, nb = pool.acquire(key, kind)
        assert nb == L.buffer_bytes[kind]
        assert L.offset[kind] <= off and off + nb <= L.offset[kind] + L.count[kind] * L.buffer_bytes[kind]
        assert (off - L.offset[kind]) % nb == 0
        for o2, n2 in (v[1:] for v in live.values()):
            assert off + nb <= o2 or o2 + n2 <= off
        live[key] = (kind, off, nb)
        with pytest.raises(ma.MaError) as e:
            pool.acquire(key, kind)
        assert e.value.code == ma.MA_ERR_ARG
        for k in range(4):
            assert pool.in_use(k) == sum(1 for v in live.values() if v[0] == k) <= L.count[k]
    # exhaustion is reported, and a released buffer can be taken again
    for key in list(live):
        pool.release(key)
    taken = [pool.acquire(10_000 + i, ma.MA_POOL_EMBED)[0] for i in range(2)]
    assert sorted(taken) == [0, L.buffer_bytes[0]]
    with pytest.raises(ma.MaError) as e:
        pool.acquire(99, ma.MA_POOL_EMBED)
    assert e.value.code == ma.MA_ERR_FULL
    pool.release(10_000)
    assert pool.acquire(99, ma.MA_POOL_EMBED)[0] == taken[0]
    with pytest.raises(ma.MaError):
        pool.release(123456)
    with pytest.raises(ma.MaError):
        pool.acquire(5, 4)
    pool.close()


def test_pinned_size_policies():
    for req in (0, 1, 4095, 4096, 4097, 10 ** 6, 3 * GIB + 5, int(2.1 * GIB)):
        assert ma.pinned_bytes(req, ma.MA_PINNED_PAGE) == -(-req // 4096) * 4096
        assert ma.pinned_bytes(req, ma.MA_PINNED_POW2) == ref.pow2_bytes(req)
    # Sec. III-B: a 2.1 GiB request rounded to 4 GiB wastes almost 2 GiB; page rounding wastes < 4 KiB
    req = int(2.1 * GIB)
    assert ma.pinned_bytes(req, ma.MA_PINNED_POW2) - req > 1.89 * GIB
    assert ma.pinned_bytes(req, ma.MA_PINNED_PAGE) - req < 4096


@pytest.mark.gpu
def test_pinned_allocation_is_usable_for_dma():
    import numpy as np
    import torch
    n = 3 * (1 << 20) + 123
    ptr = ma.pinned_alloc(n)
    try:
        assert ptr % 4096 == 0
        host = np.ctypeslib.as_array((ctypes.c_uint8 * n).from_address(ptr))
        host[:] = np.arange(n, dtype=np.uint64).astype(np.uint8)
        t = torch.from_numpy(host)
        dev = t.to("cuda", non_blocking=True)
        torch.cuda.synchronize()
        back = dev.cpu().numpy()
        assert np.array_equal(back, host)
        del t, host
    finally:
        ma.pinned_free(ptr)
