// Gradient accumulation into the fp32 flat buffer (Sec. III-C: the partition's flat gradient
// buffer is kept in fp32 so that low-precision micro-batch gradients can be accumulated into it).
//
// acc[i] = first ? widen(g[i]) : acc[i] + widen(g[i])  -- one fp32 addition per element.
// HBM-bound: 2 B read + 4 B written per element for the first micro-batch of an iteration,
// 2 + 4 read and 4 written afterwards (16-bit gradients).  Same packets and hints as the update
// kernel; a persistent grid of one block per CU with the XCD-contiguous work assignment, which
// keeps the eight XCDs at eight different places of the two buffers (with all blocks sweeping one
// moving window the kernel was 25 % slower whenever both buffers lay in the same region of HBM).
// Measured best depth: eight groups per lane in flight for the overwrite, four for the add; fused
// with the scan, whose fp64 arithmetic then overlaps more loads, twelve and eight (8B elements:
// overwrite + scan 8.96 / 8.20 / 7.50 / 7.58 ms with 6 / 8 / 12 / 16 groups against 7.46 ms for the
// plain overwrite; add + scan 12.93 / 12.64 / 12.555 / 12.76 ms with 4 / 6 / 8 / 10 against 12.55).
//
// The memory-side cache does not help here as it helps the update after a scan: writing the buffer
// without the non-temporal hint, with or without also loading the old contents that way, leaves
// the update kernel that reads it next where it was (n = 5e7: 0.233-0.240 ms either way).
//
// The SCAN variant also runs the overflow check of Sec. IV-D / Algorithm 1 (with its fp32 mask)
// and the sum of squares over the values it has just written: after the last micro-batch of an
// iteration (Sec. IV-A: the check validates the accumulated gradients before the optimizer step)
// the flat buffer need not be read again for the check.  Per-block partials and the finalize
// kernel are those of the stand-alone scan.

#include "ma_internal.h"

#ifndef MA_ACCUM_UNROLL_FIRST
#define MA_ACCUM_UNROLL_FIRST 8  // 4-element groups per lane and work item, overwrite
#endif
#ifndef MA_ACCUM_UNROLL_ADD
#define MA_ACCUM_UNROLL_ADD 4  // the same, add
#endif
#ifndef MA_ACCUM_UNROLL_ADD_SCAN
#define MA_ACCUM_UNROLL_ADD_SCAN 8  // the same, add fused with the scan
#endif
#ifndef MA_ACCUM_UNROLL_FIRST_SCAN
#define MA_ACCUM_UNROLL_FIRST_SCAN 12  // the same, overwrite fused with the scan
#endif
#ifndef MA_ACCUM_BLOCKS_PER_CU
#define MA_ACCUM_BLOCKS_PER_CU 1
#endif
#ifndef MA_ACCUM_MAP
#define MA_ACCUM_MAP 2  // work-item assignment (see WorkIter)
#endif

namespace ma {

template <bool FIRST, bool SCAN>
constexpr int accum_unroll() {
  return FIRST ? (SCAN ? MA_ACCUM_UNROLL_FIRST_SCAN : MA_ACCUM_UNROLL_FIRST)
               : (SCAN ? MA_ACCUM_UNROLL_ADD_SCAN : MA_ACCUM_UNROLL_ADD);
}

template <int GDT>
__device__ __forceinline__ float accum_grad1(MA_GLOBAL const char* g, uint64_t i) {
  if constexpr (GDT == kF32) {
    return reinterpret_cast<MA_GLOBAL const float*>(g)[i];
  } else {
    return widen16<GDT>(reinterpret_cast<MA_GLOBAL const uint16_t*>(g)[i]);
  }
}

// What the SCAN variant keeps per lane; empty otherwise.
template <bool SCAN>
struct AccumScan {
  __device__ __forceinline__ void value(float) {}
  __device__ __forceinline__ void packet(f32x4) {}
};
template <>
struct AccumScan<true> {
  NormAcc<kF32> acc;
  __device__ __forceinline__ void value(float x) { acc.word(f32_to_bits(x)); }
  __device__ __forceinline__ void packet(f32x4 x) { acc.vec(__builtin_bit_cast(u32x4, x)); }
};

template <int GDT, bool FIRST, bool SCAN>
__device__ __forceinline__ void accum1(MA_GLOBAL float* acc, MA_GLOBAL const char* g, uint64_t i,
                                       AccumScan<SCAN>& sc) {
  const float x = accum_grad1<GDT>(g, i);
  const float y = FIRST ? x : acc[i] + x;
  acc[i] = y;
  sc.value(y);
}

template <int GDT>
__device__ __forceinline__ f32x4 widen_packet(typename std::conditional<GDT == kF32, f32x4, u32x2>::type r) {
  if constexpr (GDT == kF32) {
    return r;
  } else {
    f32x4 x;
    x[0] = widen16<GDT>(r.x & 0xFFFFu);
    x[1] = widen16<GDT>(r.x >> 16);
    x[2] = widen16<GDT>(r.y & 0xFFFFu);
    x[3] = widen16<GDT>(r.y >> 16);
    return x;
  }
}

template <int GDT, bool FIRST, bool SCAN>
__global__ __launch_bounds__(kBlock) void accumulate_kernel(float* acc_, const void* g_, uint64_t n,
                                                           uint32_t head, uint32_t vec,
                                                           uint64_t chunks, NormPartial* partials) {
  using GPacket = typename std::conditional<GDT == kF32, f32x4, u32x2>::type;
  constexpr int kAccumUnroll = accum_unroll<FIRST, SCAN>();
  constexpr uint64_t kChunkGroups = uint64_t(kBlock) * kAccumUnroll;
  MA_GLOBAL float* acc = to_global(acc_);
  MA_GLOBAL const char* g = to_global(static_cast<const char*>(g_));
  const uint32_t tid = threadIdx.x;
  AccumScan<SCAN> sc;

  if (!vec) {
    for (uint64_t i = uint64_t(blockIdx.x) * kBlock + tid; i < n; i += uint64_t(gridDim.x) * kBlock) {
      accum1<GDT, FIRST, SCAN>(acc, g, i, sc);
    }
  } else {
    const uint64_t ngroups = (n > head) ? (n - head) / 4 : 0;
    MA_GLOBAL f32x4* ab = reinterpret_cast<MA_GLOBAL f32x4*>(acc + head);
    MA_GLOBAL const GPacket* gb =
        reinterpret_cast<MA_GLOBAL const GPacket*>(g + uint64_t(head) * (GDT == kF32 ? 4 : 2));
    if (blockIdx.x == 0) {
      if (tid < head && tid < n) accum1<GDT, FIRST, SCAN>(acc, g, tid, sc);
      const uint64_t t0 = uint64_t(head) + ngroups * 4;
      if (n > head && t0 + tid < n) accum1<GDT, FIRST, SCAN>(acc, g, t0 + tid, sc);
    }
    for (WorkIter<MA_ACCUM_MAP> w(chunks); w.c < w.end; w.c += w.stride) {
      const uint64_t g0 = w.c * kChunkGroups + tid;
      if ((w.c + 1) * kChunkGroups <= ngroups) {
        GPacket G[kAccumUnroll];
        f32x4 A[kAccumUnroll];
#pragma unroll
        for (int u = 0; u < kAccumUnroll; ++u) {
          G[u] = ld_stream(gb + g0 + uint64_t(u) * kBlock);
          if constexpr (!FIRST) A[u] = ld_stream(ab + g0 + uint64_t(u) * kBlock);
        }
#pragma unroll
        for (int u = 0; u < kAccumUnroll; ++u) {
          const f32x4 x = widen_packet<GDT>(G[u]);
          f32x4 y = x;
          if constexpr (!FIRST) y = A[u] + x;
          st_stream(ab + g0 + uint64_t(u) * kBlock, y);
          sc.packet(y);
        }
      } else {
#pragma unroll
        for (int u = 0; u < kAccumUnroll; ++u) {
          const uint64_t gi = g0 + uint64_t(u) * kBlock;
          if (gi < ngroups) {
            const f32x4 x = widen_packet<GDT>(ld_stream(gb + gi));
            f32x4 y = x;
            if constexpr (!FIRST) y = ld_stream(ab + gi) + x;
            st_stream(ab + gi, y);
            sc.packet(y);
          }
        }
      }
    }
  }
  if constexpr (SCAN) norm_block_finish<kF32>(sc.acc, partials);
}

template <int GDT, bool SCAN>
static hipError_t launch_accumulate_g(float* acc, const void* g, uint64_t n, uint32_t head,
                                      uint32_t vec, int first, uint32_t grid, uint64_t chunks,
                                      NormPartial* partials, hipStream_t stream) {
  if (first) {
    accumulate_kernel<GDT, true, SCAN><<<grid, kBlock, 0, stream>>>(acc, g, n, head, vec, chunks, partials);
  } else {
    accumulate_kernel<GDT, false, SCAN><<<grid, kBlock, 0, stream>>>(acc, g, n, head, vec, chunks, partials);
  }
  return hipGetLastError();
}

template <bool SCAN>
static hipError_t launch_accumulate_s(int gdt, float* acc, const void* g, uint64_t n, uint32_t head,
                                      uint32_t vec, int first, uint32_t grid, uint64_t chunks,
                                      NormPartial* partials, hipStream_t stream) {
  switch (gdt) {
    case kBF16: return launch_accumulate_g<kBF16, SCAN>(acc, g, n, head, vec, first, grid, chunks, partials, stream);
    case kF16: return launch_accumulate_g<kF16, SCAN>(acc, g, n, head, vec, first, grid, chunks, partials, stream);
    default: return launch_accumulate_g<kF32, SCAN>(acc, g, n, head, vec, first, grid, chunks, partials, stream);
  }
}

hipError_t launch_accumulate(float* acc, const void* g, int gdt, uint64_t n, uint32_t head,
                             uint32_t vec, int first, NormPartial* partials, double inv_scale_sq,
                             const ScalerState* scaler, NormResult* out, int device_cus,
                             hipStream_t stream) {
  const bool scan = partials != nullptr;
  if (n == 0 && !scan) return hipSuccess;
  const int unroll = first ? (scan ? accum_unroll<true, true>() : accum_unroll<true, false>())
                           : (scan ? accum_unroll<false, true>() : accum_unroll<false, false>());
  const uint64_t kChunkElems = uint64_t(kBlock) * 4 * unroll;
  const uint64_t body = (vec && n > head) ? n - head : 0;
  const uint64_t chunks = vec ? (body + kChunkElems - 1) / kChunkElems : 0;
  uint64_t want = uint64_t(device_cus) * MA_ACCUM_BLOCKS_PER_CU;
  if (want > kMaxNormBlocks) want = kMaxNormBlocks;  // one partial per block must fit the workspace
  const uint64_t items = vec ? chunks : (n + kBlock - 1) / kBlock;
  uint64_t blocks = items < want ? items : want;
  if (blocks == 0) blocks = 1;  // empty, head-only or tail-only input: block 0 handles it
  const uint32_t grid = static_cast<uint32_t>(blocks);
  if (!scan) return launch_accumulate_s<false>(gdt, acc, g, n, head, vec, first, grid, chunks, nullptr, stream);
  hipError_t e = launch_accumulate_s<true>(gdt, acc, g, n, head, vec, first, grid, chunks, partials, stream);
  if (e != hipSuccess) return e;
  return launch_norm_finalize(partials, grid, kF32, inv_scale_sq, scaler, out, stream);
}

}  // namespace ma
