// Gradient scan: overflow flag (Sec. IV-D, Algorithm 1) fused with the sum of squares.
//
// One pass, HBM-bound at 2 bytes per element for 16-bit gradients.  Per lane:
//   * flag: the running maximum of the sign-stripped bit patterns.  A pattern has an all-ones
//     exponent exactly when, with the sign removed, it is >= the pattern of infinity
//     (0x7F80 / 0x7C00 / 0x7F800000), so one AND and one (packed 16-bit) unsigned MAX per
//     32-bit word replace Algorithm 1's compare-and-branch, and the single comparison happens
//     once, in the finalize kernel.  There is no early exit: the sum needs the whole pass.
//   * sum: each element is widened exactly to fp32, then squared and accumulated in fp64
//     (two accumulators per lane).  fp64 keeps the result independent of gradient magnitude
//     (no overflow of g^2 for large bf16 values, no underflow for tiny ones) and makes the
//     clip coefficient derived from it reproducible to fp32 rounding.
// Per block: xor-shuffle tree inside each wave, four wave results through LDS, one partial
// per block in the caller's workspace.  A one-block finalize kernel adds the partials in index
// order.  No floating-point atomics anywhere: the result is bit-identical from run to run.
//
// The update kernel reads the same gradient again right after this pass.  Measured on MI355X, a
// line loaded WITHOUT the non-temporal hint stays in the 256 MB memory-side cache, the update
// kernel's own non-temporal traffic does not push it out, and the update then runs 6 % faster when
// the whole gradient was kept (n = 1e8: 0.448 -> 0.423 ms; n = 5e7: 0.229 -> 0.217 ms; scan + update
// 204 -> 214 and 196 -> 203 Gparam/s).  Keeping costs the scan about 10 % on the bytes it keeps, so
// the scan keeps only about what the cache can hold: `keep_of_64` of every 64 work items, chosen on
// the host (all of them for gradients up to MA_NORM_KEEP_MIB, a proportional share above, none once
// the share drops below one in eight: 8.03e9 elements gain nothing and a scan with 1/64 kept was
// 9 % slower there).  The kept items are spread evenly over the gradient, so every part of the update
// launch gains alike, and evenly over the blocks of this launch, so that none of them lags
// (n = 2e8: scan + update 0.954 -> 0.923 ms; 4e8: 1.888 -> 1.849; 1e9: 4.685 -> 4.665).

#include "ma_internal.h"

namespace ma {

// One work item: kNormChunkBytes of the row's 16-byte-aligned body; item 0 also takes the
// unaligned head elements, the last item the ragged tail.
template <int GDT, bool KEEP>
__device__ __forceinline__ void norm_chunk(NormAcc<GDT>& acc, const void* g_, uint64_t n,
                                           uint32_t head, uint64_t lc) {
  MA_GLOBAL const char* g = to_global(static_cast<const char*>(g_));
  constexpr uint64_t kElemBytes = (GDT == kF32) ? 4 : 2;
  constexpr uint64_t kPerVec = 16 / kElemBytes;
  constexpr uint64_t kChunkVecs = uint64_t(kBlock) * kNormUnroll;
  const uint32_t tid = threadIdx.x;

  if (lc == 0 && tid < head && tid < n) acc.element(g, tid);
  if (n <= head) return;

  const uint64_t body = n - head;
  const uint64_t nvec = body / kPerVec;
  MA_GLOBAL const u32x4* base =
      reinterpret_cast<MA_GLOBAL const u32x4*>(g + uint64_t(head) * kElemBytes);
  const uint64_t v0 = lc * kChunkVecs;

  if (v0 + kChunkVecs <= nvec) {
    u32x4 w[kNormUnroll];
#pragma unroll
    for (int u = 0; u < kNormUnroll; ++u) w[u] = ld_scan<KEEP>(base + v0 + tid + uint64_t(u) * kBlock);
#pragma unroll
    for (int u = 0; u < kNormUnroll; ++u) acc.vec(w[u]);
  } else {
#pragma unroll
    for (int u = 0; u < kNormUnroll; ++u) {
      const uint64_t vi = v0 + tid + uint64_t(u) * kBlock;
      if (vi < nvec) acc.vec(ld_scan<KEEP>(base + vi));
    }
    // this is the row's last item: fewer than kPerVec elements remain after the last vector
    const uint64_t t0 = uint64_t(head) + nvec * kPerVec;
    if (t0 + tid < n) acc.element(g, t0 + tid);
  }
}

// c is uniform across the block, so this is a scalar branch between two copies of the loop body.
template <int GDT>
__device__ __forceinline__ void norm_item(NormAcc<GDT>& acc, const void* g, uint64_t n, uint32_t head,
                                          uint64_t lc, uint64_t c, uint32_t keep_of_64) {
  // block b sees items b, b + G, b + 2G, ... (G a multiple of 64 on every device of interest): adding
  // the round number makes every block walk through all 64 residues
  if (((c + c / gridDim.x) & 63u) < keep_of_64) {
    norm_chunk<GDT, true>(acc, g, n, head, lc);
  } else {
    norm_chunk<GDT, false>(acc, g, n, head, lc);
  }
}

// Flat sub-group: the row travels in the kernel arguments.
template <int GDT>
__global__ __launch_bounds__(kBlock) void norm_flat_kernel(Desc row, uint64_t chunks, uint32_t keep_of_64,
                                                          NormPartial* partials) {
  NormAcc<GDT> acc;
  for (WorkIter<MA_NORM_MAP> w(chunks); w.c < w.end; w.c += w.stride) {
    norm_item<GDT>(acc, row.g, row.n, row.norm_head, w.c, w.c, keep_of_64);
  }
  norm_block_finish<GDT>(acc, partials);
}

// Largest row index in [lo, rows) whose first scan work item is <= c.  All operands are uniform
// across the block, so this runs on the scalar unit.
__device__ __forceinline__ uint32_t find_row(const Desc* table, uint32_t lo, uint32_t rows,
                                             uint64_t c) {
  uint32_t hi = rows;
  while (hi - lo > 1) {
    const uint32_t mid = lo + (hi - lo) / 2;
    if (table[mid].norm_chunk0 <= c) {
      lo = mid;
    } else {
      hi = mid;
    }
  }
  return lo;
}

// Tensor list: rows live in device memory; work items are numbered across all rows.
template <int GDT>
__global__ __launch_bounds__(kBlock) void norm_multi_kernel(const Desc* __restrict__ table,
                                                           uint32_t rows, uint64_t chunks,
                                                           uint32_t keep_of_64, NormPartial* partials) {
  NormAcc<GDT> acc;
  uint32_t r = 0;
  for (WorkIter<MA_NORM_MAP> w(chunks); w.c < w.end; w.c += w.stride) {
    const uint64_t c = w.c;
    r = find_row(table, r, rows, c);
    const Desc* d = table + r;
    norm_item<GDT>(acc, d->g, d->n, d->norm_head, c - d->norm_chunk0, c, keep_of_64);
  }
  norm_block_finish<GDT>(acc, partials);
}

// Second level as a launch of its own: one block adds the partials (fold_partials) and writes the result.
// `threshold` is the sign-stripped pattern of infinity for the gradient format.
__global__ __launch_bounds__(kBlock) void norm_finalize_kernel(const NormPartial* __restrict__ partials,
                                                              uint32_t count, double inv_scale_sq,
                                                              const ScalerState* scaler,
                                                              uint32_t threshold, int packed16,
                                                              NormResult* out) {
  const NormResult r = fold_partials(partials, count, inv_scale_sq, scaler, threshold, packed16);
  if (threadIdx.x == 0) *out = r;
}

// Adds scan results of several sub-groups in index order (single thread: count is tiny).
__global__ void norm_combine_kernel(const NormResult* __restrict__ parts, uint32_t count,
                                    NormResult* out) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  int ov = 0;
  double s = 0.0;
  for (uint32_t i = 0; i < count; ++i) {
    ov |= (parts[i].overflow != 0);
    s += parts[i].sumsq;
  }
  NormResult r;
  r.overflow = ov;
  r.reserved = 0;
  r.sumsq = s;
  *out = r;
}

// ---- launchers ------------------------------------------------------------------------------------

static uint32_t threshold_of(int gdt) {
  return gdt == kBF16 ? 0x7F80u : gdt == kF16 ? 0x7C00u : 0x7F800000u;
}

uint32_t norm_threshold(int gdt) { return threshold_of(gdt); }

hipError_t launch_norm(const Desc* row_host, const Desc* table_dev, uint32_t rows, uint64_t chunks,
                       int gdt, double inv_scale_sq, const ScalerState* scaler, NormPartial* partials,
                       NormResult* out, int device_cus, hipStream_t stream, uint32_t* grid_out) {
  uint64_t want = uint64_t(device_cus) * MA_NORM_BLOCKS_PER_CU;
  if (want > kMaxNormBlocks) want = kMaxNormBlocks;
  const uint32_t grid = static_cast<uint32_t>(chunks < want ? (chunks ? chunks : 1) : want);
  // how many of every 64 work items keep their lines in the memory-side cache for the update kernel
  const uint64_t bytes = chunks * kNormChunkBytes, cap = uint64_t(MA_NORM_KEEP_MIB) << 20;
  uint32_t keep = bytes <= cap ? 64u : static_cast<uint32_t>(cap * 64 / bytes);
  if (keep < 8) keep = 0;
  if (row_host) {
    switch (gdt) {
      case kBF16: norm_flat_kernel<kBF16><<<grid, kBlock, 0, stream>>>(*row_host, chunks, keep, partials); break;
      case kF16: norm_flat_kernel<kF16><<<grid, kBlock, 0, stream>>>(*row_host, chunks, keep, partials); break;
      default: norm_flat_kernel<kF32><<<grid, kBlock, 0, stream>>>(*row_host, chunks, keep, partials); break;
    }
  } else {
    switch (gdt) {
      case kBF16: norm_multi_kernel<kBF16><<<grid, kBlock, 0, stream>>>(table_dev, rows, chunks, keep, partials); break;
      case kF16: norm_multi_kernel<kF16><<<grid, kBlock, 0, stream>>>(table_dev, rows, chunks, keep, partials); break;
      default: norm_multi_kernel<kF32><<<grid, kBlock, 0, stream>>>(table_dev, rows, chunks, keep, partials); break;
    }
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (grid_out != nullptr) {  // the caller's next launch adds up the partials itself
    *grid_out = grid;
    return hipSuccess;
  }
  return launch_norm_finalize(partials, grid, gdt, inv_scale_sq, scaler, out, stream);
}

hipError_t launch_norm_finalize(const NormPartial* partials, uint32_t count, int gdt, double inv_scale_sq,
                                const ScalerState* scaler, NormResult* out, hipStream_t stream) {
  norm_finalize_kernel<<<1, kBlock, 0, stream>>>(partials, count, inv_scale_sq, scaler,
                                                 threshold_of(gdt), gdt != kF32, out);
  return hipGetLastError();
}

// ---- dynamic loss scale (Sec. III-C: on overflow the scale factor is reduced) ---------------------
// One thread; reads the gate, rewrites the 24-byte state.  On overflow: scale *= backoff (not below
// min_scale), clean-step count restarts, the iteration counts as skipped.  Otherwise the update
// counts as applied, and after `window` clean steps in a row scale *= growth (not above max_scale).
__global__ void scaler_update_kernel(ScalerState* state, const NormResult* gate, ScalerConfig cfg) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  ScalerState st = *state;
  if (gate->overflow != 0) {
    const float s = st.scale * cfg.backoff;
    st.scale = s < cfg.min_scale ? cfg.min_scale : s;
    st.good_steps = 0;
    st.skipped += 1;
  } else {
    st.step += 1;
    st.good_steps += 1;
    if (st.good_steps >= cfg.window) {
      const float s = st.scale * cfg.growth;
      st.scale = s > cfg.max_scale ? cfg.max_scale : s;
      st.good_steps = 0;
    }
  }
  *state = st;
}

__global__ void scaler_init_kernel(ScalerState* state, float scale, int64_t step) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  ScalerState st;
  st.scale = scale;
  st.good_steps = 0;
  st.step = step;
  st.skipped = 0;
  *state = st;
}

hipError_t launch_scaler_init(ScalerState* state, float scale, int64_t step, hipStream_t stream) {
  scaler_init_kernel<<<1, kWave, 0, stream>>>(state, scale, step);
  return hipGetLastError();
}

hipError_t launch_scaler_update(ScalerState* state, const NormResult* gate, const ScalerConfig& cfg,
                                hipStream_t stream) {
  scaler_update_kernel<<<1, kWave, 0, stream>>>(state, gate, cfg);
  return hipGetLastError();
}

hipError_t launch_norm_combine(const NormResult* parts, uint32_t count, NormResult* out,
                               hipStream_t stream) {
  norm_combine_kernel<<<1, kWave, 0, stream>>>(parts, count, out);
  return hipGetLastError();
}

}  // namespace ma
