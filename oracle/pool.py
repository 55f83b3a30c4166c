"""Plain statement of the parameter-buffer-pool sizes (TEST INFRASTRUCTURE, like the rest of oracle/).

Sec. III-A: the original pool of an SSD-offloading system holds uniform buffers, each as large as the
largest weight tensor; its size is buffer size x buffers per block x blocks in flight.  Sec. IV-B: the
adaptive pool keeps four sub-pools of exactly sized buffers -- embedding / LM head (vocab x hidden),
feed-forward projections (intermediate x hidden), K / V projections, Q / O projections -- with 2, 3N,
2N and 2N buffers for N transformer blocks in flight.

Pinned by the sizes the paper prints (tests/golden/buffer_pool_sizes.txt).
"""
from fractions import Fraction


def tensors(vocab, hidden, intermediate, kv_dim, q_dim):
    """Element counts of one tensor of each of the four kinds."""
    return {"embed": vocab * hidden, "ffn": intermediate * hidden, "kv": kv_dim * hidden,
            "qo": q_dim * hidden}


def buffers_per_kind(n_blocks):
    return {"embed": 2, "ffn": 3 * n_blocks, "kv": 2 * n_blocks, "qo": 2 * n_blocks}


def adaptive_pool_bytes(dims, n_blocks=1, elem_bytes=2):
    t, c = tensors(*dims), buffers_per_kind(n_blocks)
    return sum(c[k] * t[k] * elem_bytes for k in t)


def uniform_pool_bytes(dims, n_blocks=1, elem_bytes=2):
    t, c = tensors(*dims), buffers_per_kind(n_blocks)
    return sum(c.values()) * max(t.values()) * elem_bytes


def fragmentation(dims, n_blocks=1, elem_bytes=2):
    """Share of the uniform pool that the tensors in flight do not need (exact rational)."""
    return 1 - Fraction(adaptive_pool_bytes(dims, n_blocks, elem_bytes),
                        uniform_pool_bytes(dims, n_blocks, elem_bytes))


def pow2_bytes(request):
    """Size a power-of-two rounding allocator gives a request (Sec. III-B)."""
    p = 1
    while p < request:
        p *= 2
    return p if request else 0
