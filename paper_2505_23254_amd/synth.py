"""Seeded synthetic workloads shaped like the optimizer step of LLM fine-tuning.

Only input generation lives here: shapes, value distributions, seeds and the places where
inf/NaN patterns are planted.  None of the step's arithmetic (no scan, no update, no
rounding rule of the method) is in this module; the only casts are the library casts that
produce the low-precision *inputs*.  Both the GPU tests and the CPU oracle tests draw their
inputs from here, so that the two sides see the same arrays.

The step is element-wise, so only element counts, tensor boundaries and value scales
matter; the shapes below stand in for the models the paper fine-tunes (Sec. VI-A lists
Llama3.1-8B and Qwen2.5-7B/14B/32B).
"""
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import torch

_TORCH_LP = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}
_BYTES = {"bf16": 2, "f16": 2, "f32": 4}

# 16-bit non-finite patterns planted by the overflow variants: +inf, -inf, quiet NaN,
# signalling-NaN pattern, negative NaN.
NONFINITE_BITS = {
    "f16": (0x7C00, 0xFC00, 0x7E00, 0x7D01, 0xFE00),
    "bf16": (0x7F80, 0xFF80, 0x7FC0, 0x7FA1, 0xFFC0),
}


@dataclass
class FlatConfig:
    """One flat sub-group."""
    name: str
    n: int
    seed: int = 0
    p_std: float = 0.02
    m_std: float = 0.0        # 0 -> zeros
    v_std: float = 0.0        # 0 -> zeros, else |N(0, v_std)|
    g_std: float = 1e-3
    gdt: str = "bf16"
    pdt: str = "bf16"
    loss_scale: float = 1.0
    step: int = 1
    max_norm: float = 0.0     # <= 0: no clipping
    n_inject: int = 0         # number of planted inf/NaN entries
    lr: float = 1e-5
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.01


def config(name: str) -> FlatConfig:
    """The flat configurations of the benchmark definition."""
    table = {
        "c1": FlatConfig("c1", 1 << 20, seed=0),
        "c2": FlatConfig("c2", 100_000_000, seed=1, m_std=1e-4, v_std=1e-8, step=100,
                         max_norm=1.0),
        "c3a": FlatConfig("c3a", 50_000_000, seed=2, m_std=1e-4, v_std=1e-8, step=100,
                          gdt="f16", loss_scale=65536.0, max_norm=1.0),
        "c3b": FlatConfig("c3b", 50_000_000, seed=2, m_std=1e-4, v_std=1e-8, step=100,
                          gdt="f16", loss_scale=65536.0, max_norm=1.0, n_inject=17),
    }
    return table[name]


@dataclass
class FlatState:
    p: torch.Tensor
    m: torch.Tensor
    v: torch.Tensor
    g: torch.Tensor           # low-precision gradient, already multiplied by loss_scale
    p_lp: torch.Tensor
    inject_idx: List[int] = field(default_factory=list)
    arena: Optional[torch.Tensor] = None      # the allocation the five views are cut from


def _fill_normal(buf: torch.Tensor, std: float, gen: torch.Generator, piece: int = 1 << 27):
    """In-place N(0, std) in bounded pieces (no full-size temporaries)."""
    n = buf.numel()
    for a in range(0, n, piece):
        buf[a:min(n, a + piece)].normal_(0.0, std, generator=gen)


def _fill_grad(g: torch.Tensor, std: float, scale: float, gen: torch.Generator,
               piece: int = 1 << 27):
    n = g.numel()
    for a in range(0, n, piece):
        b = min(n, a + piece)
        tmp = torch.empty(b - a, dtype=torch.float32, device=g.device)
        tmp.normal_(0.0, std, generator=gen)
        if scale != 1.0:
            tmp.mul_(scale)
        g[a:b].copy_(tmp)      # library cast to the gradient's storage type
        del tmp


def plant_nonfinite(g: torch.Tensor, gdt: str, count: int, seed: int) -> List[int]:
    """Overwrite `count` seeded random entries of g with a seeded mix of inf/NaN patterns."""
    cpu_gen = torch.Generator(device="cpu")
    cpu_gen.manual_seed(seed + 7919)
    seen, idx = set(), []
    while len(idx) < count:
        for i in torch.randint(0, g.numel(), (count,), generator=cpu_gen).tolist():
            if i not in seen and len(idx) < count:
                seen.add(i)
                idx.append(i)
    pats = NONFINITE_BITS[gdt]
    which = torch.randint(0, len(pats), (count,), generator=cpu_gen)
    raw = g.view(torch.int16)
    for k in range(count):
        bits = pats[int(which[k])]
        raw[int(idx[k])] = bits - 0x10000 if bits >= 0x8000 else bits
    return idx


ARENA_ALIGN = 2 << 20   # every buffer of a state starts on a 2 MiB boundary of the arena


def _flat_layout(n: int, gdt: str = "bf16"):
    sizes = [4 * n, 4 * n, 4 * n, _BYTES[gdt] * n, 2 * n]
    offs, total = [], 0
    for sz in sizes:
        offs.append(total)
        total += (sz + ARENA_ALIGN - 1) // ARENA_ALIGN * ARENA_ALIGN
    return offs, sizes, max(total, 1)


def flat_state_bytes(n: int, gdt: str = "bf16") -> int:
    """Bytes carve_state needs for n elements (gradient dtype gdt: "bf16", "f16" or "f32")."""
    return _flat_layout(n, gdt)[2]


def flat_traffic(n: int, gdt: str = "bf16"):
    """(bytes, bytes moved per byte stored) of the five pieces in address order: p, m, v are read
    and written by the update, the gradient is only read, the parameter copy only written."""
    offs, _, total = _flat_layout(n, gdt)
    ends = offs[1:] + [total]
    return [(e - o, w) for o, e, w in zip(offs, ends, (2.0, 2.0, 2.0, 1.0, 1.0))]


def flat_state_parts(n: int, gdt: str = "bf16"):
    """(bytes of p | m | v | g, bytes of p_lp) for a state whose parameter copy is placed apart."""
    offs, sizes, _ = _flat_layout(n, gdt)
    return max(offs[4], 1), max(sizes[4], 1)


def carve_state(n: int, gdt: str, pdt: str, device: str, arena=None):
    """One allocation for a whole optimizer state, cut into p | m | v | g | p_lp in that order.

    A single arena keeps the five streams of the update kernel at fixed, known distances from
    each other (the kernel's speed depends on where the streams lie in HBM, and one allocation
    makes that reproducible from process to process).  `arena`: an existing uint8 device buffer
    of at least flat_state_bytes(n) bytes to cut from, instead of a new allocation; or a pair of
    such buffers (flat_state_parts(n) bytes): p | m | v | g from the first, p_lp from the second.
    """
    offs, sizes, total = _flat_layout(n, gdt)
    dts = [torch.float32, torch.float32, torch.float32, _TORCH_LP[gdt], _TORCH_LP[pdt]]
    if isinstance(arena, (tuple, list)):
        main, side = arena
        if main.dtype != torch.uint8 or side.dtype != torch.uint8 or main.numel() < offs[4] or side.numel() < sizes[4]:
            raise ValueError("arena pair must be uint8 buffers of at least %d and %d bytes" % (offs[4], sizes[4]))
        views = [main[o:o + sz].view(dt) for o, sz, dt in zip(offs[:4], sizes[:4], dts[:4])]
        views.append(side[:sizes[4]].view(dts[4]))
        return main, views
    if arena is None:
        arena = torch.empty(total, dtype=torch.uint8, device=device)
    elif arena.dtype != torch.uint8 or arena.numel() < total:
        raise ValueError("arena must be a uint8 buffer of at least %d bytes" % total)
    views = [arena[o:o + sz].view(dt) for o, sz, dt in zip(offs, sizes, dts)]
    return arena, views


def make_flat(cfg: FlatConfig, device: str = "cpu", n: Optional[int] = None,
              arena: Optional[torch.Tensor] = None) -> FlatState:
    """Allocate (or cut from `arena`) and fill one flat sub-group on `device` (n overrides cfg.n
    for small cases)."""
    n = cfg.n if n is None else n
    if arena is not None:
        device = arena[0].device if isinstance(arena, (tuple, list)) else arena.device
    gen = torch.Generator(device=device)
    gen.manual_seed(cfg.seed)
    arena, (p, m, v, g, p_lp) = carve_state(n, cfg.gdt, cfg.pdt, device, arena)
    _fill_normal(p, cfg.p_std, gen)
    m.zero_()
    if cfg.m_std > 0:
        _fill_normal(m, cfg.m_std, gen)
    v.zero_()
    if cfg.v_std > 0:
        _fill_normal(v, cfg.v_std, gen)
        v.abs_()
    _fill_grad(g, cfg.g_std, cfg.loss_scale, gen)
    piece = 1 << 27
    for a in range(0, n, piece):
        p_lp[a:a + piece].copy_(p[a:a + piece])       # library cast: the copy starts in sync with p
    st = FlatState(p, m, v, g, p_lp)
    st.arena = arena
    if cfg.n_inject > 0 and n > 0:
        st.inject_idx = plant_nonfinite(g, cfg.gdt, min(cfg.n_inject, n), cfg.seed)
    return st


# ----------------------------------------------------------------------------------------
# Tensor lists shaped like decoder-only LLMs (element counts only).
# ----------------------------------------------------------------------------------------
def decoder_shapes(hidden: int, intermediate: int, layers: int, kv_heads: int, head_dim: int,
                   vocab: int) -> List[Tuple[str, int]]:
    """(name, numel) for embedding, per-layer q/k/v/o, gate/up/down, two norm vectors, LM head."""
    kv = kv_heads * head_dim
    out = [("embed", vocab * hidden)]
    for i in range(layers):
        out += [
            ("l%d.q" % i, hidden * hidden), ("l%d.k" % i, kv * hidden),
            ("l%d.v" % i, kv * hidden), ("l%d.o" % i, hidden * hidden),
            ("l%d.gate" % i, intermediate * hidden), ("l%d.up" % i, intermediate * hidden),
            ("l%d.down" % i, hidden * intermediate),
            ("l%d.norm1" % i, hidden), ("l%d.norm2" % i, hidden),
        ]
    out.append(("lm_head", vocab * hidden))
    return out


def llama3_8b_shapes() -> List[Tuple[str, int]]:
    """290 tensors, 8,030,257,152 elements (hidden 4096, FFN 14336, 32 layers, 8 KV heads)."""
    return decoder_shapes(4096, 14336, 32, 8, 128, 128256)


def qwen14b_class_shapes() -> List[Tuple[str, int]]:
    """362 tensors, 12,567,592,960 elements (hidden 5120, FFN 13824, 40 layers, 8 KV heads)."""
    return decoder_shapes(5120, 13824, 40, 8, 128, 152064)


def scaled_shapes(shapes: List[Tuple[str, int]], divisor: int, ragged: bool = True):
    """A miniature of a tensor list: every numel divided by `divisor` (at least 1), optionally
    nudged so that sizes are not multiples of the vector width (exercises ragged tails)."""
    out = []
    for k, (name, numel) in enumerate(shapes):
        m = max(1, numel // divisor)
        if ragged:
            m += k % 7
        out.append((name, m))
    return out


@dataclass
class ListState:
    names: List[str]
    p: List[torch.Tensor]
    m: List[torch.Tensor]
    v: List[torch.Tensor]
    g: List[torch.Tensor]
    p_lp: List[torch.Tensor]
    flat: Optional[FlatState] = None     # layout "streams": the flat buffers the views are cut from
    arena: Optional[torch.Tensor] = None  # layout "tensor": the one allocation behind all views

    @property
    def total(self) -> int:
        return sum(t.numel() for t in self.p)


def _round_up(x: int, a: int) -> int:
    return (x + a - 1) // a * a


def _list_offsets(shapes, align_elems: int):
    offs, total = [], 0
    for _, numel in shapes:
        total = _round_up(total, align_elems)
        offs.append(total)
        total += numel
    return offs, total


def _tensor_places(shapes, gdt: str = "bf16"):
    elem = (4, 4, 4, _BYTES[gdt], 2)
    places, total = [], 0
    for _, numel in shapes:
        row = []
        for eb in elem:
            nbytes = eb * numel
            total = _round_up(total, ARENA_ALIGN if nbytes >= ARENA_ALIGN else 4096)
            row.append((total, nbytes))
            total += nbytes
        places.append(row)
    return places, max(total, 1)


def list_state_parts(shapes: List[Tuple[str, int]], align_elems: int = 64, gdt: str = "bf16"):
    """flat_state_parts for a list in layout "streams"."""
    return flat_state_parts(_list_offsets(shapes, align_elems)[1], gdt)


def list_state_bytes(shapes: List[Tuple[str, int]], layout: str = "streams", align_elems: int = 64,
                     gdt: str = "bf16") -> int:
    """Bytes make_list needs for this list, layout and gradient dtype."""
    if layout == "streams":
        return flat_state_bytes(_list_offsets(shapes, align_elems)[1], gdt)
    return _tensor_places(shapes, gdt)[1]


def list_traffic(shapes: List[Tuple[str, int]], layout: str = "streams", align_elems: int = 64,
                 gdt: str = "bf16"):
    """Traffic weights of the list's pieces in address order (None: uniform)."""
    if layout == "streams":
        return flat_traffic(_list_offsets(shapes, align_elems)[1], gdt)
    return None


def make_list(shapes: List[Tuple[str, int]], cfg: FlatConfig, device: str = "cpu",
              align_elems: int = 64, layout: str = "streams",
              arena: Optional[torch.Tensor] = None) -> ListState:
    """A tensor list in one allocation (a new one, or the front of the uint8 buffer `arena`).

    layout "streams": five flat buffers p | m | v | g | p_lp, each tensor a view at its running
    offset.  Each tensor starts at a multiple of `align_elems` elements; align_elems=1 packs them
    back to back, which misaligns most tensors when their sizes are ragged.

    layout "tensor": the five buffers of ONE tensor lie next to each other, tensor after tensor
    (p_k | m_k | v_k | g_k | p_lp_k), as when a framework allocates a parameter together with its
    gradient and optimizer states.  Buffers of 2 MiB or more start on a 2 MiB boundary, smaller
    ones on a 4 KiB boundary.
    """
    if layout == "streams":
        offs, total = _list_offsets(shapes, align_elems)
        flat = make_flat(cfg, device=device, n=total, arena=arena)
        cut = lambda buf: [buf[o:o + numel] for o, (_, numel) in zip(offs, shapes)]
        return ListState([s[0] for s in shapes], cut(flat.p), cut(flat.m), cut(flat.v), cut(flat.g),
                         cut(flat.p_lp), flat, flat.arena)
    if layout != "tensor":
        raise ValueError("layout must be 'streams' or 'tensor'")
    dts = (torch.float32, torch.float32, torch.float32, _TORCH_LP[cfg.gdt], _TORCH_LP[cfg.pdt])
    places, total = _tensor_places(shapes, cfg.gdt)
    if arena is None:
        arena = torch.empty(total, dtype=torch.uint8, device=device)
    elif arena.dtype != torch.uint8 or arena.numel() < total:
        raise ValueError("arena must be a uint8 buffer of at least %d bytes" % total)
    device = arena.device
    gen = torch.Generator(device=device)
    gen.manual_seed(cfg.seed)
    out = ListState([s[0] for s in shapes], [], [], [], [], [], None, arena)
    for row in places:
        p, m, v, g, p_lp = (arena[o:o + nb].view(dt) for (o, nb), dt in zip(row, dts))
        _fill_normal(p, cfg.p_std, gen)
        m.zero_()
        if cfg.m_std > 0:
            _fill_normal(m, cfg.m_std, gen)
        v.zero_()
        if cfg.v_std > 0:
            _fill_normal(v, cfg.v_std, gen)
            v.abs_()
        _fill_grad(g, cfg.g_std, cfg.loss_scale, gen)
        piece = 1 << 27
        for a in range(0, p.numel(), piece):
            p_lp[a:a + piece].copy_(p[a:a + piece])
        for lst, t in zip((out.p, out.m, out.v, out.g, out.p_lp), (p, m, v, g, p_lp)):
            lst.append(t)
    return out


def bits16(t: torch.Tensor):
    """Raw 16-bit patterns of a bf16/fp16 tensor as a numpy uint16 array (host copy); an fp32 tensor
    comes back as a float32 array."""
    import numpy as np
    if t.dtype == torch.float32:
        return t.detach().cpu().contiguous().numpy().copy()
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16).copy()


# ----------------------------------------------------------------------------------------
# Inputs at the edges of the fp32 range (for the oracle's exact-arithmetic pin and the GPU parity
# tests alike; generation and library casts only).
# ----------------------------------------------------------------------------------------
import numpy as _np  # noqa: E402

EXTREME_CASES = ("training", "subnormal", "subnormal_eps", "f16_subnormal_grads")


def _log_uniform(rng, n, lo, hi, signed=True):
    mag = _np.exp2(rng.uniform(lo, hi, n))
    return (mag * (rng.choice([-1.0, 1.0], n) if signed else 1.0)).astype(_np.float32)


def extreme_case(case: str, n: int, seed: int = 0):
    """(p, m, v, grad bits, gdt, loss_scale, clip, eps) with magnitudes drawn log-uniformly:
    "training": ordinary ranges; "subnormal": p, m, v and the unscaled gradient below 2^-126, so that
    every intermediate of the step is subnormal or zero; "subnormal_eps": v = 0 and tiny gradients with
    a subnormal eps, so that the denominator is subnormal and the quotient divides two subnormals;
    "f16_subnormal_grads": fp16 gradients below 2^-14 at loss scale 1, subnormal second moments."""
    rng = _np.random.default_rng(EXTREME_CASES.index(case) + 1 + 1000 * seed)
    gdt, scale, clip, eps = "bf16", 1.0, 1.0, 1e-8
    if case == "training":
        p, m, v = _log_uniform(rng, n, -12, -2), _log_uniform(rng, n, -20, -8), _log_uniform(rng, n, -40, -16, False)
        gf, scale, clip = _log_uniform(rng, n, -6, 8), 1024.0, 0.37
    elif case == "subnormal":
        p, m, v = (_log_uniform(rng, n, -149, -124), _log_uniform(rng, n, -149, -126),
                   _log_uniform(rng, n, -149, -127, False))
        gf, scale = _log_uniform(rng, n, -133, -110), 4.0
    elif case == "subnormal_eps":
        p, m, v = _log_uniform(rng, n, -30, -2), _log_uniform(rng, n, -149, -120), _np.zeros(n, _np.float32)
        gf, eps = _log_uniform(rng, n, -133, -120), 1e-42
        gf[::3] = 0.0
    elif case == "f16_subnormal_grads":
        p, m, v = _log_uniform(rng, n, -12, -2), _log_uniform(rng, n, -30, -14), _log_uniform(rng, n, -149, -120, False)
        gf, gdt = _log_uniform(rng, n, -24, -14), "f16"
    else:
        raise KeyError(case)
    g = bits16(torch.from_numpy(gf).to(torch.bfloat16 if gdt == "bf16" else torch.float16))
    return p, m, v, g, gdt, scale, clip, eps
