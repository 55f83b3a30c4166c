// Unscale + clip + AdamW + low-precision copy in one read/write pass (Sec. II-A names the
// ingredients: fp32 master states, bias correction, decoupled weight decay, fp16/bf16
// parameters).
//
// HBM-bound: per element the kernel reads p, m, v (fp32) and the gradient (16-bit), and writes
// p, m, v and the 16-bit parameter copy: 14 + 14 = 28 bytes, about 40 ALU instructions.  Each
// lane owns groups of four consecutive elements, so p/m/v move as 128-bit packets and the
// 16-bit operands as 64-bit packets; a wave covers 1 KiB (512 B) of contiguous memory per
// instruction.  All loads of a work item are issued before the first use, the arithmetic runs
// in registers, and the stores carry the non-temporal hint since nothing is read again.
// Work items are handed to a persistent, fully resident grid sized to the CU count (WorkIter).

#include "ma_internal.h"

namespace ma {

template <int GDT>
struct GradGroup {  // four consecutive gradient elements as loaded
  using Packet = typename std::conditional<GDT == kF32, f32x4, u32x2>::type;
  Packet raw;
  __device__ __forceinline__ float get(int k) const {
    if constexpr (GDT == kF32) {
      return raw[k];
    } else {
      const uint32_t w = raw[k >> 1];
      return widen16<GDT>((k & 1) ? (w >> 16) : (w & 0xFFFFu));
    }
  }
};

template <int GDT>
__device__ __forceinline__ float load_grad_scalar(MA_GLOBAL const char* g, uint64_t i) {
  if constexpr (GDT == kF32) {
    return reinterpret_cast<MA_GLOBAL const float*>(g)[i];
  } else {
    return widen16<GDT>(reinterpret_cast<MA_GLOBAL const uint16_t*>(g)[i]);
  }
}

template <int PDT>
__device__ __forceinline__ void store_lp_scalar(MA_GLOBAL char* lp, uint64_t i, float x) {
  if constexpr (PDT != kNoLp) {
    reinterpret_cast<MA_GLOBAL uint16_t*>(lp)[i] = static_cast<uint16_t>(narrow16<PDT>(x));
  }
}

template <int GDT, int PDT>
__device__ __forceinline__ void step_scalar_element(const StepScalars& s, MA_GLOBAL float* p,
                                                    MA_GLOBAL float* m, MA_GLOBAL float* v,
                                                    MA_GLOBAL const char* g, MA_GLOBAL char* lp,
                                                    uint64_t i) {
  float pi = p[i], mi = m[i], vi = v[i];
  adamw_element(s, load_grad_scalar<GDT>(g, i), pi, mi, vi);
  p[i] = pi;
  m[i] = mi;
  v[i] = vi;
  store_lp_scalar<PDT>(lp, i, pi);
}

template <int GDT, int PDT>
__device__ __forceinline__ void step_group(const StepScalars& s, f32x4& P, f32x4& M, f32x4& V,
                                           const GradGroup<GDT>& G, u32x2& L) {
  float lpv[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    float pk = P[k], mk = M[k], vk = V[k];
    adamw_element(s, G.get(k), pk, mk, vk);
    P[k] = pk;
    M[k] = mk;
    V[k] = vk;
    lpv[k] = pk;
  }
  if constexpr (PDT != kNoLp) {
    L.x = narrow16<PDT>(lpv[0]) | (narrow16<PDT>(lpv[1]) << 16);
    L.y = narrow16<PDT>(lpv[2]) | (narrow16<PDT>(lpv[3]) << 16);
  }
}

// One work item of a row: kStepChunkElems elements of the group-aligned body; item 0 also takes
// the head elements, the last item the ragged tail.  Rows whose buffers cannot be brought to a
// common group alignment run the scalar loop.
template <int GDT, int PDT>
__device__ __forceinline__ void step_chunk(const StepScalars& s, float* p_, float* m_, float* v_,
                                           const void* g_, void* lp_, uint64_t n, uint32_t head,
                                           uint32_t vec, uint64_t lc) {
  using GPacket = typename GradGroup<GDT>::Packet;
  const uint32_t tid = threadIdx.x;
  MA_GLOBAL float* p = to_global(p_);
  MA_GLOBAL float* m = to_global(m_);
  MA_GLOBAL float* v = to_global(v_);
  MA_GLOBAL const char* g = to_global(static_cast<const char*>(g_));
  MA_GLOBAL char* lp = to_global(static_cast<char*>(lp_));

  if (!vec) {
    const uint64_t e0 = lc * kStepChunkElems;
    const uint64_t e1 = (n - e0 < kStepChunkElems) ? n : e0 + kStepChunkElems;
    for (uint64_t i = e0 + tid; i < e1; i += kBlock) step_scalar_element<GDT, PDT>(s, p, m, v, g, lp, i);
    return;
  }

  if (lc == 0 && tid < head && tid < n) step_scalar_element<GDT, PDT>(s, p, m, v, g, lp, tid);
  if (n <= head) return;

  constexpr uint64_t kChunkGroups = uint64_t(kBlock) * kStepUnroll;
  const uint64_t body = n - head;
  const uint64_t ngroups = body / 4;
  const uint64_t g0 = lc * kChunkGroups;

  MA_GLOBAL f32x4* pb = reinterpret_cast<MA_GLOBAL f32x4*>(p + head);
  MA_GLOBAL f32x4* mb = reinterpret_cast<MA_GLOBAL f32x4*>(m + head);
  MA_GLOBAL f32x4* vb = reinterpret_cast<MA_GLOBAL f32x4*>(v + head);
  MA_GLOBAL const GPacket* gb =
      reinterpret_cast<MA_GLOBAL const GPacket*>(g + uint64_t(head) * (GDT == kF32 ? 4 : 2));
  MA_GLOBAL u32x2* lb = reinterpret_cast<MA_GLOBAL u32x2*>(lp + uint64_t(head) * 2);

  if (g0 + kChunkGroups <= ngroups) {
    f32x4 P[kStepUnroll], M[kStepUnroll], V[kStepUnroll];
    GradGroup<GDT> G[kStepUnroll];
    u32x2 L[kStepUnroll];
#pragma unroll
    for (int u = 0; u < kStepUnroll; ++u) {
      const uint64_t gi = g0 + tid + uint64_t(u) * kBlock;
      G[u].raw = ld_stream(gb + gi);
      P[u] = ld_stream(pb + gi);
      M[u] = ld_stream(mb + gi);
      V[u] = ld_stream(vb + gi);
    }
#pragma unroll
    for (int u = 0; u < kStepUnroll; ++u) step_group<GDT, PDT>(s, P[u], M[u], V[u], G[u], L[u]);
#pragma unroll
    for (int u = 0; u < kStepUnroll; ++u) {
      const uint64_t gi = g0 + tid + uint64_t(u) * kBlock;
      st_stream(pb + gi, P[u]);
      st_stream(mb + gi, M[u]);
      st_stream(vb + gi, V[u]);
      if constexpr (PDT != kNoLp) st_stream(lb + gi, L[u]);
    }
  } else {
#pragma unroll
    for (int u = 0; u < kStepUnroll; ++u) {
      const uint64_t gi = g0 + tid + uint64_t(u) * kBlock;
      if (gi < ngroups) {
        f32x4 P = ld_stream(pb + gi), M = ld_stream(mb + gi), V = ld_stream(vb + gi);
        GradGroup<GDT> G;
        G.raw = ld_stream(gb + gi);
        u32x2 L;
        step_group<GDT, PDT>(s, P, M, V, G, L);
        st_stream(pb + gi, P);
        st_stream(mb + gi, M);
        st_stream(vb + gi, V);
        if constexpr (PDT != kNoLp) st_stream(lb + gi, L);
      }
    }
    // last item of the row: fewer than four elements remain after the last group
    const uint64_t t0 = uint64_t(head) + ngroups * 4;
    if (t0 + tid < n) step_scalar_element<GDT, PDT>(s, p, m, v, g, lp, t0 + tid);
  }
}

// ---- software pipeline over work items ------------------------------------------------------------
// The memory system rewards a small moving window: with few resident waves all writing and
// reading close together, DRAM pages stay open and read/write turnarounds are fewer.  Few waves
// cannot hide latency by occupancy, so each wave hides it itself: the loads of its next work item
// are in flight while it computes and stores the current one (two register tiles, ping-pong).

// A located work item: its row's buffers and its index inside the row.
struct Item {
  float* p;
  float* m;
  float* v;
  const void* g;
  void* lp;
  uint64_t n;
  uint32_t head, vec;
  uint64_t lc;
};

// Whole, aligned work items take the tile path; a row's first item when it has head elements,
// its ragged last item, and every item of a misaligned row go through step_chunk.
__device__ __forceinline__ bool item_is_tile(const Item& it) {
  constexpr uint64_t kChunkGroups = uint64_t(kBlock) * kStepUnroll;
  if (!it.vec || it.n <= it.head) return false;
  if (it.lc == 0 && it.head != 0) return false;
  return (it.lc + 1) * kChunkGroups <= (it.n - it.head) / 4;
}

template <int GDT>
struct Tile {
  f32x4 P[kStepUnroll], M[kStepUnroll], V[kStepUnroll];
  GradGroup<GDT> G[kStepUnroll];
};

template <int GDT>
__device__ __forceinline__ void tile_load(Tile<GDT>& t, const Item& it) {
  using GPacket = typename GradGroup<GDT>::Packet;
  constexpr uint64_t kChunkGroups = uint64_t(kBlock) * kStepUnroll;
  const uint64_t g0 = it.lc * kChunkGroups + threadIdx.x;
  MA_GLOBAL const f32x4* pb = reinterpret_cast<MA_GLOBAL const f32x4*>(to_global(it.p) + it.head);
  MA_GLOBAL const f32x4* mb = reinterpret_cast<MA_GLOBAL const f32x4*>(to_global(it.m) + it.head);
  MA_GLOBAL const f32x4* vb = reinterpret_cast<MA_GLOBAL const f32x4*>(to_global(it.v) + it.head);
  MA_GLOBAL const GPacket* gb = reinterpret_cast<MA_GLOBAL const GPacket*>(
      to_global(static_cast<const char*>(it.g)) + uint64_t(it.head) * (GDT == kF32 ? 4 : 2));
#pragma unroll
  for (int u = 0; u < kStepUnroll; ++u) {
    const uint64_t gi = g0 + uint64_t(u) * kBlock;
    t.G[u].raw = ld_stream(gb + gi);
    t.P[u] = ld_stream(pb + gi);
    t.M[u] = ld_stream(mb + gi);
    t.V[u] = ld_stream(vb + gi);
  }
}

template <int GDT, int PDT>
__device__ __forceinline__ void tile_finish(Tile<GDT>& t, const Item& it, const StepScalars& s) {
  constexpr uint64_t kChunkGroups = uint64_t(kBlock) * kStepUnroll;
  const uint64_t g0 = it.lc * kChunkGroups + threadIdx.x;
  MA_GLOBAL f32x4* pb = reinterpret_cast<MA_GLOBAL f32x4*>(to_global(it.p) + it.head);
  MA_GLOBAL f32x4* mb = reinterpret_cast<MA_GLOBAL f32x4*>(to_global(it.m) + it.head);
  MA_GLOBAL f32x4* vb = reinterpret_cast<MA_GLOBAL f32x4*>(to_global(it.v) + it.head);
  MA_GLOBAL u32x2* lb =
      reinterpret_cast<MA_GLOBAL u32x2*>(to_global(static_cast<char*>(it.lp)) + uint64_t(it.head) * 2);
  u32x2 L[kStepUnroll];
#pragma unroll
  for (int u = 0; u < kStepUnroll; ++u) step_group<GDT, PDT>(s, t.P[u], t.M[u], t.V[u], t.G[u], L[u]);
#pragma unroll
  for (int u = 0; u < kStepUnroll; ++u) {
    const uint64_t gi = g0 + uint64_t(u) * kBlock;
    st_stream(pb + gi, t.P[u]);
    st_stream(mb + gi, t.M[u]);
    st_stream(vb + gi, t.V[u]);
    if constexpr (PDT != kNoLp) st_stream(lb + gi, L[u]);
  }
}

template <int GDT, int PDT>
__device__ __forceinline__ void item_finish(bool tile, Tile<GDT>& t, const Item& it,
                                            const StepScalars& s) {
  if (tile) {
    tile_finish<GDT, PDT>(t, it, s);
  } else {
    step_chunk<GDT, PDT>(s, it.p, it.m, it.v, it.g, it.lp, it.n, it.head, it.vec, it.lc);
  }
}

// locate(c, item) fills `item` for global work item c (c is uniform across the block).
template <int GDT, int PDT, class Locate>
__device__ __forceinline__ void step_pipeline(const StepScalars& s, uint64_t chunks, Locate locate) {
  WorkIter<MA_STEP_MAP> w(chunks);
  if (w.c >= w.end) return;
  Item ia, ib;
  Tile<GDT> ta, tb;
  locate(w.c, ia);
  bool fa = item_is_tile(ia), fb = false;
  if (fa) tile_load<GDT>(ta, ia);
  for (;;) {
    // A is current; start B
    uint64_t next = w.c + w.stride;
    bool more = next < w.end;
    if (more) {
      locate(next, ib);
      fb = item_is_tile(ib);
      if (fb) tile_load<GDT>(tb, ib);
    }
    item_finish<GDT, PDT>(fa, ta, ia, s);
    if (!more) break;
    w.c = next;
    // B is current; start A
    next = w.c + w.stride;
    more = next < w.end;
    if (more) {
      locate(next, ia);
      fa = item_is_tile(ia);
      if (fa) tile_load<GDT>(ta, ia);
    }
    item_finish<GDT, PDT>(fb, tb, ib, s);
    if (!more) break;
    w.c = next;
  }
}

// Device-side gate (Sec. III-C): returns false when the scan saw an overflow, in which case the
// kernel must not touch any buffer.  Otherwise fills in the unscale-and-clip factor from the
// scanned sum of squares, with the same two roundings as the host path: the clip coefficient is
// rounded to fp32, then divided by the loss scale in fp64 and rounded to fp32 again.
__device__ __forceinline__ bool apply_gate(const NormResult* gate, float max_norm, float loss_scale,
                                           StepScalars& s) {
  if (gate == nullptr) return true;
  if (gate->overflow != 0) return false;
  double c = 1.0;
  if (max_norm > 0.0f) {
    c = static_cast<double>(max_norm) / (__builtin_sqrt(gate->sumsq) + 1e-6);
    c = (c < 1.0) ? c : 1.0;
  }
  const float cf = static_cast<float>(c);
  s.gscale = static_cast<float>(static_cast<double>(cf) / static_cast<double>(loss_scale));
  return true;
}

template <int GDT, int PDT>
__global__ __launch_bounds__(kBlock) void step_flat_kernel(Desc row, uint64_t chunks, StepScalars s,
                                                          const NormResult* gate, float max_norm,
                                                          float loss_scale) {
  if (!apply_gate(gate, max_norm, loss_scale, s)) return;
  step_pipeline<GDT, PDT>(s, chunks, [&](uint64_t c, Item& it) {
    it.p = row.p;
    it.m = row.m;
    it.v = row.v;
    it.g = row.g;
    it.lp = row.lp;
    it.n = row.n;
    it.head = row.step_head;
    it.vec = row.step_vec;
    it.lc = c;
  });
}

template <int GDT, int PDT>
__global__ __launch_bounds__(kBlock) void step_multi_kernel(const Desc* __restrict__ table,
                                                           uint32_t rows, uint64_t chunks,
                                                           StepScalars s, const NormResult* gate,
                                                           float max_norm, float loss_scale) {
  if (!apply_gate(gate, max_norm, loss_scale, s)) return;
  uint32_t r = 0;  // rows are visited in increasing order: the last hit bounds the next search
  step_pipeline<GDT, PDT>(s, chunks, [&](uint64_t c, Item& it) {
    // largest row whose first work item is <= c (uniform => scalar unit)
    uint32_t lo = r, hi = rows;
    while (hi - lo > 1) {
      const uint32_t mid = lo + (hi - lo) / 2;
      if (table[mid].step_chunk0 <= c) {
        lo = mid;
      } else {
        hi = mid;
      }
    }
    r = lo;
    const Desc* d = table + r;
    it.p = d->p;
    it.m = d->m;
    it.v = d->v;
    it.g = d->g;
    it.lp = d->lp;
    it.n = d->n;
    it.head = d->step_head;
    it.vec = d->step_vec;
    it.lc = c - d->step_chunk0;
  });
}

// ---- launcher ---------------------------------------------------------------------------------------

// Blocks of one kernel that fit on a compute unit at once (queried once per instantiation).
template <class K>
static int resident_blocks_per_cu(K kernel) {
  int nb = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kernel, kBlock, 0) != hipSuccess || nb < 1) {
    (void)hipGetLastError();
    nb = 1;
  }
  return nb;
}

template <int GDT, int PDT>
static hipError_t launch_step_typed(const Desc* row_host, const Desc* table_dev, uint32_t rows,
                                    uint64_t chunks, const StepScalars& s, const NormResult* gate,
                                    float max_norm, float loss_scale, int device_cus,
                                    hipStream_t stream) {
  // A persistent grid must be fully resident: blocks that wait for a slot would run alone at the
  // end.  So: no more blocks per compute unit than the kernel's occupancy allows.
  static const int occ_flat = resident_blocks_per_cu(step_flat_kernel<GDT, PDT>);
  static const int occ_multi = resident_blocks_per_cu(step_multi_kernel<GDT, PDT>);
  const int occ = row_host ? occ_flat : occ_multi;
  const uint64_t want = uint64_t(device_cus) * (occ < MA_STEP_BLOCKS_PER_CU ? occ : MA_STEP_BLOCKS_PER_CU);
  const uint32_t grid = static_cast<uint32_t>(chunks < want ? chunks : want);
  if (row_host) {
    step_flat_kernel<GDT, PDT><<<grid, kBlock, 0, stream>>>(*row_host, chunks, s, gate, max_norm, loss_scale);
  } else {
    step_multi_kernel<GDT, PDT><<<grid, kBlock, 0, stream>>>(table_dev, rows, chunks, s, gate, max_norm,
                                                            loss_scale);
  }
  return hipGetLastError();
}

template <int GDT>
static hipError_t launch_step_g(int pdt, const Desc* row_host, const Desc* table_dev, uint32_t rows,
                                uint64_t chunks, const StepScalars& s, const NormResult* gate,
                                float max_norm, float loss_scale, int device_cus, hipStream_t stream) {
  switch (pdt) {
    case kBF16: return launch_step_typed<GDT, kBF16>(row_host, table_dev, rows, chunks, s, gate, max_norm, loss_scale, device_cus, stream);
    case kF16: return launch_step_typed<GDT, kF16>(row_host, table_dev, rows, chunks, s, gate, max_norm, loss_scale, device_cus, stream);
    default: return launch_step_typed<GDT, kNoLp>(row_host, table_dev, rows, chunks, s, gate, max_norm, loss_scale, device_cus, stream);
  }
}

hipError_t launch_step(const Desc* row_host, const Desc* table_dev, uint32_t rows, uint64_t chunks,
                       int gdt, int pdt, const StepScalars& s, const NormResult* gate, float max_norm,
                       float loss_scale, int device_cus, hipStream_t stream) {
  if (chunks == 0) return hipSuccess;
  switch (gdt) {
    case kBF16: return launch_step_g<kBF16>(pdt, row_host, table_dev, rows, chunks, s, gate, max_norm, loss_scale, device_cus, stream);
    case kF16: return launch_step_g<kF16>(pdt, row_host, table_dev, rows, chunks, s, gate, max_norm, loss_scale, device_cus, stream);
    default: return launch_step_g<kF32>(pdt, row_host, table_dev, rows, chunks, s, gate, max_norm, loss_scale, device_cus, stream);
  }
}

}  // namespace ma
