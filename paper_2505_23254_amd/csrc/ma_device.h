// Device-side building blocks shared by the scan and update kernels (gfx950, wave64).
//
// Everything here is written for streaming: each lane moves 128-bit (or 64-bit for 16-bit
// operands of a 4-wide group) packets with non-temporal hints, one wave covers 1 KiB of
// contiguous memory per load instruction, and nothing is re-read.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ma {

#ifndef MA_BLOCK
#define MA_BLOCK 256  // threads per block (a multiple of 64)
#endif
constexpr int kBlock = MA_BLOCK;
constexpr int kWave = 64;

// dtype codes, numerically equal to ma_dtype in the public header
constexpr int kF32 = 0;
constexpr int kBF16 = 1;
constexpr int kF16 = 2;
constexpr int kNoLp = 3;  // update kernel variant that writes no low-precision copy

// Launch shape, chosen by measurement on MI355X (256 CUs, 8 XCDs).  The update kernel moves a 1:1
// read/write mix and is fastest with FEW resident waves that each keep a deep tile in flight (one
// block per CU, four 4-element groups per lane, next tile prefetched) and that pause briefly
// before each tile's stores: more requests in flight than that lower the rate the memory system
// sustains on this mix.  The read-only scan kernel prefers more waves.
#ifndef MA_NORM_UNROLL
#define MA_NORM_UNROLL 8  // 16-byte loads in flight per lane in the scan kernel
#endif
#ifndef MA_STEP_UNROLL
#define MA_STEP_UNROLL 4  // 4-element groups per lane and tile in the update kernel
#endif
#ifndef MA_NORM_MAP
#define MA_NORM_MAP 0  // work-item assignment of the scan kernel (see WorkIter)
#endif
#ifndef MA_NORM_KEEP_MIB
#define MA_NORM_KEEP_MIB 320  // gradient bytes (MiB) the scan leaves in the memory-side cache for the update kernel
#endif
#ifndef MA_STEP_UNROLL_BF16
#define MA_STEP_UNROLL_BF16 8  // 8-element groups per lane and tile when p, m, v are held in bf16
#endif
#ifndef MA_STEP_PACE_MULTI
#define MA_STEP_PACE_MULTI 32  // s_sleep units (64 clocks each) before a tile's stores: multi-tensor kernel, fp32 states
#endif
#ifndef MA_STEP_PACE_FLAT
#define MA_STEP_PACE_FLAT 28  // the same for the flat kernel
#endif
#ifndef MA_STEP_PACE_BF16
#define MA_STEP_PACE_BF16 0  // the same for states held in bf16 (either kernel)
#endif
#ifndef MA_STEP_POOL_SHIFT
#define MA_STEP_POOL_SHIFT 5  // tensor lists: the last 1/2^k of every XCD's share is handed out on demand
#endif
#ifndef MA_STEP_DRAW
#define MA_STEP_DRAW 8  // work items a block takes from a pool at a time
#endif
#ifndef MA_STEP_MAP
#define MA_STEP_MAP 2  // work-item assignment of the update kernel (see WorkIter)
#endif

constexpr int kNormUnroll = MA_NORM_UNROLL;
constexpr int kStepUnroll = MA_STEP_UNROLL;
constexpr uint64_t kNormChunkBytes = uint64_t(kBlock) * 16 * kNormUnroll;  // per work item

// The update kernel moves p, m, v as 16-byte packets: a group is 4 consecutive elements for
// fp32 states and 8 for bf16 states.  sdt: kF32 or kBF16.
__host__ __device__ constexpr int step_group_elems(int sdt) { return sdt == kF32 ? 4 : 8; }
__host__ __device__ constexpr int step_unroll(int sdt) {
  return sdt == kF32 ? MA_STEP_UNROLL : MA_STEP_UNROLL_BF16;
}
__host__ __device__ constexpr int step_pace(int sdt, bool multi) {
  return sdt != kF32 ? MA_STEP_PACE_BF16 : multi ? MA_STEP_PACE_MULTI : MA_STEP_PACE_FLAT;
}
// elements per work item of the update kernel
__host__ __device__ constexpr uint64_t step_chunk_elems(int sdt) {
  return uint64_t(kBlock) * step_group_elems(sdt) * step_unroll(sdt);
}
constexpr uint64_t kStepChunkElems = step_chunk_elems(kF32);

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

// One row of the work table: a tensor (or flat sub-group) and where its work items start.
struct Desc {
  float* p;
  float* m;
  float* v;
  const void* g;
  void* lp;
  uint64_t n;
  uint64_t norm_chunk0;  // index of this row's first scan work item
  uint64_t step_chunk0;  // index of this row's first update work item
  uint32_t norm_head;    // elements before the gradient's first 16-byte boundary
  uint32_t step_head;    // elements before the group boundary common to all buffers
  uint32_t step_vec;     // 1: the packet path is usable after step_head elements
  uint32_t pad;
};
static_assert(sizeof(Desc) == 80, "table row layout");

// Head of a tensor list's device table: shared counters of the list's update launches.  next[y]
// counts the late work items of XCD y's share that have been handed out, done the blocks that have
// finished.  All zero between launches (the last block of a launch clears them).
struct StepQueue {
  uint32_t next[8];
  uint32_t done;
  uint32_t pad[7];
};
static_assert(sizeof(StepQueue) == 64, "table head layout");

// Scalars of one AdamW step, each rounded to fp32 once on the host (or in the gated prologue).
struct StepScalars {
  float beta1, beta2, omb1, omb2, eps, step_size, inv_sqrt_bc2, decay, gscale;
};

// Partial result of one block of the scan kernel.
struct NormPartial {
  double sum;
  uint32_t maxabs;  // running maximum of the sign-stripped patterns (two 16-bit lanes, or one
                    // 32-bit value for fp32 gradients)
  uint32_t pad;
};

struct NormResult {  // same layout as ma_norm_result
  int32_t overflow;
  int32_t reserved;
  double sumsq;
};

// Dynamic loss-scale state in device memory; same layout as ma_scaler_state.
struct ScalerState {
  float scale;
  int32_t good_steps;  // clean steps since the scale last changed
  int64_t step;        // updates applied so far
  int64_t skipped;     // iterations skipped because of an overflow
};

struct ScalerConfig {  // same layout as ma_scaler_config
  float backoff, growth, min_scale, max_scale;
  int32_t window;
};

// What the update kernel reads or derives on the device (every pointer may be null).
struct StepControl {
  const NormResult* gate;     // null: the host-side unscale-and-clip factor is final
  const ScalerState* scaler;  // null: loss scale and update number come from the host
  float max_norm;
  float loss_scale;
  float lr;
  int32_t bias_correction;
  // whole-step calls: the scan's per-block partials take the place of `gate`
  const NormPartial* partials;  // null: not a whole-step call
  NormResult* result_out;       // where block 0 publishes the folded scan result
  double inv_scale_sq;
  uint32_t partial_count;
  uint32_t threshold;  // sign-stripped pattern of infinity in the gradient's format
  int32_t packed16;    // partial maxima hold two 16-bit lanes
};

// ---- beta^t for the bias corrections -----------------------------------------------------------
// One routine for host and device, so that the scalars the device derives (update number read from
// device memory) are bit-identical to those the host passes in kernel arguments.  Square-and-
// multiply over the bits of t in double-double arithmetic (error-free products through fma): the
// value is accurate to ~2^-95 before its one rounding to fp64, i.e. it is the correctly rounded
// power except in astronomically rare near-tie cases, and it needs nothing but IEEE fp64
// multiply, add and fma, which round the same way on both sides.
struct DoubleDouble {
  double hi, lo;
};
__host__ __device__ inline DoubleDouble dd_mul(DoubleDouble a, DoubleDouble b) {
  const double p = a.hi * b.hi;
  double e = __builtin_fma(a.hi, b.hi, -p);  // exact low part of the leading product
  e = __builtin_fma(a.hi, b.lo, e);
  e = __builtin_fma(a.lo, b.hi, e);
  DoubleDouble r;
  r.hi = p + e;
  r.lo = e - (r.hi - p);
  return r;
}
__host__ __device__ inline double pow_int(double base, uint64_t t) {
  DoubleDouble r{1.0, 0.0}, b{base, 0.0};
  while (t != 0) {
    if (t & 1u) r = dd_mul(r, b);
    t >>= 1;
    if (t != 0) b = dd_mul(b, b);
  }
  return r.hi;
}

// ---- memory ------------------------------------------------------------------------------
// Pointers read from a table in memory carry no address-space information, and the compiler
// would fall back to flat addressing for them.  Every buffer of this library is global device
// memory, so the kernels say so once and get global_load / global_store throughout.
#define MA_GLOBAL __attribute__((address_space(1)))

template <class T>
__device__ __forceinline__ MA_GLOBAL T* to_global(T* p) {
  return (MA_GLOBAL T*)p;
}
#ifndef MA_LOAD_NT
#define MA_LOAD_NT 1  // non-temporal hint on streaming loads
#endif
#ifndef MA_STORE_NT
#define MA_STORE_NT 1  // non-temporal hint on streaming stores
#endif
template <class T>
__device__ __forceinline__ T ld_stream(MA_GLOBAL const T* p) {
#if MA_LOAD_NT
  return __builtin_nontemporal_load(p);
#else
  return *p;
#endif
}
// A load whose line may stay in the caches: for data that a later kernel reads again.
template <class T>
__device__ __forceinline__ T ld_keep(MA_GLOBAL const T* p) {
  return *p;
}
template <bool KEEP, class T>
__device__ __forceinline__ T ld_scan(MA_GLOBAL const T* p) {
  if constexpr (KEEP) {
    return ld_keep(p);
  } else {
    return ld_stream(p);
  }
}
template <class T>
__device__ __forceinline__ void st_stream(MA_GLOBAL T* p, T x) {
#if MA_STORE_NT
  __builtin_nontemporal_store(x, p);
#else
  *p = x;
#endif
}

// ---- format conversion ----------------------------------------------------------------------
__device__ __forceinline__ float bits_to_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t f32_to_bits(float x) { return __builtin_bit_cast(uint32_t, x); }

// Widen one 16-bit gradient pattern (in the low half of `h`) to fp32; exact for both formats.
template <int DT>
__device__ __forceinline__ float widen16(uint32_t h) {
  if constexpr (DT == kBF16) {
    return bits_to_f32(h << 16);
  } else {
    return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<unsigned short>(h)));
  }
}

// Round fp32 to a 16-bit pattern, nearest-even.  NaN becomes a quiet NaN keeping the sign and
// the top payload bits.
template <int DT>
__device__ __forceinline__ uint32_t narrow16(float x) {
  const uint32_t b = f32_to_bits(x);
  if constexpr (DT == kBF16) {
    // add half an ulp of the kept part, plus the parity of the kept lsb minus one: ties land
    // on the even neighbour and a carry may run into the exponent (up to infinity)
    uint32_t r = (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) r = (b >> 16) | 0x0040u;
    return r;
  } else {
    // The empty asm pins x as an fp32 value in a register.  Without it the compiler merges the
    // fma that produced x with this conversion into one mixed-precision fma that rounds the
    // exact result straight to fp16, which differs from RNE(fp32 value) on halfway cases.
    float y = x;
    asm("" : "+v"(y));
    uint32_t r = __builtin_bit_cast(unsigned short, static_cast<_Float16>(y));
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) {
      r = ((b >> 16) & 0x8000u) | 0x7E00u | ((b >> 13) & 0x01FFu);
    }
    return r;
  }
}

// ---- the update of one element ------------------------------------------------------------------
// fp32 throughout; products, the quotient and the square root each round once, and every
// addition is the tail of an fma (the translation unit is built with contraction off, so the
// compiler adds no fusion of its own).
__device__ __forceinline__ void adamw_element(const StepScalars& s, float g_raw, float& p, float& m,
                                              float& v) {
  const float g = g_raw * s.gscale;
  const float m1 = __builtin_fmaf(s.beta1, m, s.omb1 * g);
  const float v1 = __builtin_fmaf(s.beta2, v, s.omb2 * (g * g));
  const float d = __builtin_fmaf(__builtin_sqrtf(v1), s.inv_sqrt_bc2, s.eps);
  const float u = m1 / d;
  const float q = __builtin_fmaf(-s.decay, p, p);
  p = __builtin_fmaf(-s.step_size, u, q);
  m = m1;
  v = v1;
}

// ---- assignment of work items to the persistent grid ----------------------------------------------
// MAP 0: round-robin, block b takes items b, b+G, b+2G, ...  (all blocks sweep one moving window)
// MAP 1: one contiguous slab of items per block
// MAP 2: XCD-contiguous: consecutive block indices are dispatched round-robin over the 8 XCDs, so
//        block b runs on XCD b%8; each XCD owns one contiguous eighth of the items and its
//        blocks sweep it round-robin.  Falls back to MAP 0 when the grid is not a multiple of 8.
template <int MAP>
struct WorkIter {
  uint64_t c, end, stride;
  __device__ __forceinline__ explicit WorkIter(uint64_t items) {
    const uint64_t b = blockIdx.x, grid = gridDim.x;
    if (MAP == 1) {
      const uint64_t per = (items + grid - 1) / grid;
      c = b * per;
      end = (c + per < items) ? c + per : items;
      stride = 1;
    } else if (MAP == 2 && (grid & 7) == 0) {
      const uint64_t per_xcd = (items + 7) / 8;
      const uint64_t x = b & 7;
      c = x * per_xcd + (b >> 3);
      end = ((x + 1) * per_xcd < items) ? (x + 1) * per_xcd : items;
      stride = grid >> 3;
    } else {
      c = b;
      end = items;
      stride = grid;
    }
  }
};

// ---- wave / block reductions (fixed order => deterministic) ---------------------------------------
__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) x += __shfl_xor(x, off, kWave);
  return x;
}

template <bool PACKED16>
__device__ __forceinline__ uint32_t max_pattern(uint32_t a, uint32_t b) {
  if constexpr (PACKED16) {
    return __builtin_bit_cast(
        uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b)));
  } else {
    return a > b ? a : b;
  }
}

template <bool PACKED16>
__device__ __forceinline__ uint32_t wave_max_pattern(uint32_t x) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) {
    x = max_pattern<PACKED16>(x, static_cast<uint32_t>(__shfl_xor(static_cast<int>(x), off, kWave)));
  }
  return x;
}

// ---- per-lane state of the gradient scan and its block-level fold -----------------------------------
// Flag: the running maximum of the sign-stripped bit patterns (a pattern has an all-ones exponent
// exactly when, with the sign removed, it is >= the pattern of infinity).  Sum: each element is
// widened exactly, squared and accumulated in fp64.
template <int GDT>
struct NormAcc {
  double a0 = 0.0, a1 = 0.0;
  uint32_t mx = 0;

  __device__ __forceinline__ void word(uint32_t w) {
    if constexpr (GDT == kF32) {
      mx = max_pattern<false>(mx, w & 0x7FFFFFFFu);
      const double x = static_cast<double>(bits_to_f32(w));
      a0 = __builtin_fma(x, x, a0);
    } else {
      mx = max_pattern<true>(mx, w & 0x7FFF7FFFu);
      const double lo = static_cast<double>(widen16<GDT>(w & 0xFFFFu));
      const double hi = static_cast<double>(widen16<GDT>(w >> 16));
      a0 = __builtin_fma(lo, lo, a0);
      a1 = __builtin_fma(hi, hi, a1);
    }
  }
  __device__ __forceinline__ void vec(u32x4 w) {
    word(w.x);
    word(w.y);
    word(w.z);
    word(w.w);
  }
  // one element given by index into the raw gradient buffer
  __device__ __forceinline__ void element(MA_GLOBAL const char* g, uint64_t i) {
    if constexpr (GDT == kF32) {
      word(reinterpret_cast<MA_GLOBAL const uint32_t*>(g)[i]);
    } else {
      const uint32_t h = reinterpret_cast<MA_GLOBAL const uint16_t*>(g)[i];
      mx = max_pattern<true>(mx, h & 0x7FFFu);
      const double x = static_cast<double>(widen16<GDT>(h));
      a0 = __builtin_fma(x, x, a0);
    }
  }
};

// Block-level fold of the per-lane accumulators; thread 0 writes the block's partial.
template <int GDT>
__device__ __forceinline__ void norm_block_finish(NormAcc<GDT>& acc, NormPartial* partials) {
  __shared__ double s_sum[kBlock / kWave];
  __shared__ uint32_t s_max[kBlock / kWave];
  const double ws = wave_sum(acc.a0 + acc.a1);
  const uint32_t wm = wave_max_pattern<GDT != kF32>(acc.mx);
  const int wave = threadIdx.x / kWave;
  if ((threadIdx.x & (kWave - 1)) == 0) {
    s_sum[wave] = ws;
    s_max[wave] = wm;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = s_sum[0];
    uint32_t mx = s_max[0];
#pragma unroll
    for (int k = 1; k < kBlock / kWave; ++k) {
      t += s_sum[k];
      mx = max_pattern<GDT != kF32>(mx, s_max[k]);
    }
    NormPartial out;
    out.sum = t;
    out.maxabs = mx;
    out.pad = 0;
    partials[blockIdx.x] = out;
  }
}

// Second level of the scan: the whole block adds `count` per-block partials.  Thread t takes partials
// t, t + 256, ... in increasing order, then the same wave / LDS fold as above; the order is a function
// of `count` alone, so whoever calls this (the finalize kernel, or every block of an update launch)
// gets the same bits.  Every thread of the block must call it; every thread receives the result.
__device__ __forceinline__ NormResult fold_partials(const NormPartial* __restrict__ partials, uint32_t count,
                                                    double inv_scale_sq, const ScalerState* scaler,
                                                    uint32_t threshold, int packed16) {
  __shared__ double f_sum[kBlock / kWave];
  __shared__ uint32_t f_max[kBlock / kWave];
  __shared__ NormResult f_result;
  double t = 0.0;
  uint32_t mx = 0;
  for (uint32_t i = threadIdx.x; i < count; i += kBlock) {
    t += partials[i].sum;
    const uint32_t w = partials[i].maxabs;
    // fold the two 16-bit lanes into one value; fp32 patterns pass through
    const uint32_t f = packed16 ? ((w & 0xFFFFu) > (w >> 16) ? (w & 0xFFFFu) : (w >> 16)) : w;
    mx = f > mx ? f : mx;
  }
  t = wave_sum(t);
  mx = wave_max_pattern<false>(mx);
  const int wave = threadIdx.x / kWave;
  if ((threadIdx.x & (kWave - 1)) == 0) {
    f_sum[wave] = t;
    f_max[wave] = mx;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double tot = f_sum[0];
    uint32_t m = f_max[0];
#pragma unroll
    for (int k = 1; k < kBlock / kWave; ++k) {
      tot += f_sum[k];
      m = f_max[k] > m ? f_max[k] : m;
    }
    NormResult r;
    r.overflow = (m >= threshold) ? 1 : 0;
    r.reserved = 0;
    if (scaler != nullptr) {
      const double sc = static_cast<double>(scaler->scale);
      inv_scale_sq = 1.0 / (sc * sc);
    }
    r.sumsq = tot * inv_scale_sq;
    f_result = r;
  }
  __syncthreads();
  return f_result;
}

}  // namespace ma
