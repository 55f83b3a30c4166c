// Unscale + clip + AdamW + low-precision copy in one read/write pass (Sec. II-A names the
// ingredients: fp32 master states, bias correction, decoupled weight decay, fp16/bf16
// parameters).
//
// HBM-bound: per element the kernel reads p, m, v (fp32) and the gradient (16-bit), and writes
// p, m, v and the 16-bit parameter copy: 14 + 14 = 28 bytes, about 55 ALU instructions.  Each
// lane owns groups of consecutive elements sized so that p, m, v move as 128-bit packets (four
// fp32 elements; the 16-bit operands of such a group are 64-bit packets).  The arithmetic runs in
// registers and every packet carries the non-temporal hint since nothing is read again.  Work
// items are handed to a persistent, fully resident grid sized to the CU count (WorkIter), and
// each wave keeps the loads of its next work item in flight while it finishes the current one.
//
// The same code also serves optimizer states held in bf16 and stored by truncation (Extended
// Experiments, bf16 half-precision optimizer): a group is then eight elements, again one 128-bit
// packet per state stream, widened by a shift and stored back by dropping the low half.

#include "ma_internal.h"

namespace ma {

// ---- operand packets: one group of consecutive elements of one stream -------------------------------

// Gradient of a group of GROUP elements: one packet of 16-bit values, or GROUP/4 fp32 packets.
template <int GDT, int GROUP>
struct GradGroup {
  static constexpr int kPackets = (GDT == kF32) ? GROUP / 4 : 1;
  using Packet = typename std::conditional<
      GDT == kF32, f32x4, typename std::conditional<GROUP == 4, u32x2, u32x4>::type>::type;
  Packet raw[kPackets];
  __device__ __forceinline__ float get(int k) const {
    if constexpr (GDT == kF32) {
      return raw[k >> 2][k & 3];
    } else {
      const uint32_t w = raw[0][k >> 1];
      return widen16<GDT>((k & 1) ? (w >> 16) : (w & 0xFFFFu));
    }
  }
  // base points at the row's first whole group
  __device__ __forceinline__ void load(MA_GLOBAL const Packet* base, uint64_t gi) {
#pragma unroll
    for (int j = 0; j < kPackets; ++j) raw[j] = ld_stream(base + gi * kPackets + j);
  }
};

// fp32 -> bf16 by dropping the low half (Extended Experiments: direct truncation).  A NaN whose
// payload sits only in the dropped bits is kept a NaN by setting the quiet bit.
__device__ __forceinline__ uint32_t truncate_bf16(float x) {
  const uint32_t b = f32_to_bits(x);
  uint32_t h = b >> 16;
  if ((b & 0x7FFFFFFFu) > 0x7F800000u) h |= 0x0040u;
  return h;
}

#ifndef MA_TRUNCATE_GUARD
#define MA_TRUNCATE_GUARD 0  // 1: re-check every value of a packet for a NaN that truncation would turn into infinity
#endif

// State streams (p, m, v): fp32, or bf16 widened on load and truncated on store.  One packet is
// 16 bytes = one group.
template <int SDT>
struct StateIO {
  static constexpr int kGroup = step_group_elems(SDT);
  static constexpr int kUnroll = step_unroll(SDT);
  static constexpr uint64_t kBytes = (SDT == kF32) ? 4 : 2;
  using Packet = typename std::conditional<SDT == kF32, f32x4, u32x4>::type;

  static __device__ __forceinline__ void unpack(Packet r, float (&x)[kGroup]) {
    if constexpr (SDT == kF32) {
#pragma unroll
      for (int k = 0; k < 4; ++k) x[k] = r[k];
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        x[2 * k] = bits_to_f32(r[k] << 16);
        x[2 * k + 1] = bits_to_f32(r[k] & 0xFFFF0000u);
      }
    }
  }
  static __device__ __forceinline__ Packet pack(const float (&x)[kGroup]) {
    Packet r;
    if constexpr (SDT == kF32) {
#pragma unroll
      for (int k = 0; k < 4; ++k) r[k] = x[k];
    } else {
      // Two upper halves per word.  No NaN fix-up here: every value that reaches a packet store is the
      // result of an fma, and an fma returns a QUIET NaN whenever it returns a NaN, so the kept half
      // (which holds the quiet bit) is a NaN pattern already.  Measured: the fix-up was 11 of the 60
      // vector instructions per element of this variant, whose vector unit is busy 77 % of the time.
#pragma unroll
      for (int k = 0; k < 4; ++k) {
#if MA_TRUNCATE_GUARD
        r[k] = truncate_bf16(x[2 * k]) | (truncate_bf16(x[2 * k + 1]) << 16);
#else
        r[k] = (f32_to_bits(x[2 * k]) >> 16) | (f32_to_bits(x[2 * k + 1]) & 0xFFFF0000u);
#endif
      }
    }
    return r;
  }
  static __device__ __forceinline__ float load1(MA_GLOBAL const char* base, uint64_t i) {
    if constexpr (SDT == kF32) {
      return reinterpret_cast<MA_GLOBAL const float*>(base)[i];
    } else {
      return bits_to_f32(uint32_t(reinterpret_cast<MA_GLOBAL const uint16_t*>(base)[i]) << 16);
    }
  }
  static __device__ __forceinline__ void store1(MA_GLOBAL char* base, uint64_t i, float x) {
    if constexpr (SDT == kF32) {
      reinterpret_cast<MA_GLOBAL float*>(base)[i] = x;
    } else {
      reinterpret_cast<MA_GLOBAL uint16_t*>(base)[i] = static_cast<uint16_t>(truncate_bf16(x));
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

// The buffers of one row, as global byte pointers.
struct RowPtrs {
  MA_GLOBAL char* p;
  MA_GLOBAL char* m;
  MA_GLOBAL char* v;
  MA_GLOBAL const char* g;
  MA_GLOBAL char* lp;
};

template <int SDT, int GDT, int PDT>
__device__ __forceinline__ void step_scalar_element(const StepScalars& s, const RowPtrs& r, uint64_t i) {
  using S = StateIO<SDT>;
  float pi = S::load1(r.p, i), mi = S::load1(r.m, i), vi = S::load1(r.v, i);
  adamw_element(s, load_grad_scalar<GDT>(r.g, i), pi, mi, vi);
  S::store1(r.p, i, pi);
  S::store1(r.m, i, mi);
  S::store1(r.v, i, vi);
  store_lp_scalar<PDT>(r.lp, i, pi);
}

// One group: unpack, update, pack.  L receives the 16-bit parameter copy (fp32 states only, where a
// group is four elements).
template <int SDT, int GDT, int PDT>
__device__ __forceinline__ void step_group(const StepScalars& s, typename StateIO<SDT>::Packet& Pr,
                                           typename StateIO<SDT>::Packet& Mr,
                                           typename StateIO<SDT>::Packet& Vr,
                                           const GradGroup<GDT, StateIO<SDT>::kGroup>& G, u32x2& L) {
  using S = StateIO<SDT>;
  constexpr int N = S::kGroup;
  float P[N], M[N], V[N];
  S::unpack(Pr, P);
  S::unpack(Mr, M);
  S::unpack(Vr, V);
#pragma unroll
  for (int k = 0; k < N; ++k) adamw_element(s, G.get(k), P[k], M[k], V[k]);
  if constexpr (PDT != kNoLp) {
    static_assert(N == 4, "the 16-bit parameter copy exists for fp32 states only");
    L.x = narrow16<PDT>(P[0]) | (narrow16<PDT>(P[1]) << 16);
    L.y = narrow16<PDT>(P[2]) | (narrow16<PDT>(P[3]) << 16);
  }
  Pr = S::pack(P);
  Mr = S::pack(M);
  Vr = S::pack(V);
}

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

__device__ __forceinline__ RowPtrs row_ptrs(const Item& it) {
  RowPtrs r;
  r.p = to_global(reinterpret_cast<char*>(it.p));
  r.m = to_global(reinterpret_cast<char*>(it.m));
  r.v = to_global(reinterpret_cast<char*>(it.v));
  r.g = to_global(static_cast<const char*>(it.g));
  r.lp = to_global(static_cast<char*>(it.lp));
  return r;
}

// Packet pointers of the row's group-aligned body.
template <int SDT, int GDT>
struct BodyPtrs {
  using SPacket = typename StateIO<SDT>::Packet;
  using GPacket = typename GradGroup<GDT, StateIO<SDT>::kGroup>::Packet;
  MA_GLOBAL SPacket* p;
  MA_GLOBAL SPacket* m;
  MA_GLOBAL SPacket* v;
  MA_GLOBAL const GPacket* g;
  MA_GLOBAL u32x2* lp;
  __device__ __forceinline__ BodyPtrs(const RowPtrs& r, uint32_t head) {
    const uint64_t so = uint64_t(head) * StateIO<SDT>::kBytes;
    p = reinterpret_cast<MA_GLOBAL SPacket*>(r.p + so);
    m = reinterpret_cast<MA_GLOBAL SPacket*>(r.m + so);
    v = reinterpret_cast<MA_GLOBAL SPacket*>(r.v + so);
    g = reinterpret_cast<MA_GLOBAL const GPacket*>(r.g + uint64_t(head) * (GDT == kF32 ? 4 : 2));
    lp = reinterpret_cast<MA_GLOBAL u32x2*>(r.lp + uint64_t(head) * 2);
  }
};

// ---- the general work item (ragged, head-carrying or misaligned) --------------------------------------
// step_chunk_elems(SDT) elements of the group-aligned body; item 0 also takes the head elements,
// the last item the ragged tail.  Rows whose buffers cannot be brought to a common group alignment
// run the scalar loop.
template <int SDT, int GDT, int PDT>
__device__ __forceinline__ void step_chunk(const StepScalars& s, const Item& it) {
  using S = StateIO<SDT>;
  constexpr uint64_t kChunkElems = step_chunk_elems(SDT);
  constexpr uint64_t kChunkGroups = uint64_t(kBlock) * S::kUnroll;
  const uint32_t tid = threadIdx.x;
  const RowPtrs r = row_ptrs(it);
  const uint64_t n = it.n, lc = it.lc;
  const uint32_t head = it.head;

  if (!it.vec) {
    const uint64_t e0 = lc * kChunkElems;
    const uint64_t e1 = (n - e0 < kChunkElems) ? n : e0 + kChunkElems;
    for (uint64_t i = e0 + tid; i < e1; i += kBlock) step_scalar_element<SDT, GDT, PDT>(s, r, i);
    return;
  }

  if (lc == 0 && tid < head && tid < n) step_scalar_element<SDT, GDT, PDT>(s, r, tid);
  if (n <= head) return;

  const uint64_t ngroups = (n - head) / S::kGroup;
  const uint64_t g0 = lc * kChunkGroups;
  const BodyPtrs<SDT, GDT> b(r, head);

#pragma unroll
  for (int u = 0; u < S::kUnroll; ++u) {
    const uint64_t gi = g0 + tid + uint64_t(u) * kBlock;
    if (gi < ngroups) {
      typename S::Packet P = ld_stream(b.p + gi), M = ld_stream(b.m + gi), V = ld_stream(b.v + gi);
      GradGroup<GDT, S::kGroup> G;
      G.load(b.g, gi);
      u32x2 L;
      step_group<SDT, GDT, PDT>(s, P, M, V, G, L);
      st_stream(b.p + gi, P);
      st_stream(b.m + gi, M);
      st_stream(b.v + gi, V);
      if constexpr (PDT != kNoLp) st_stream(b.lp + gi, L);
    }
  }
  // fewer than one group's elements remain after the row's last group; they belong to its last item
  const uint64_t t0 = uint64_t(head) + ngroups * S::kGroup;
  if (g0 + kChunkGroups > ngroups && t0 + tid < n) step_scalar_element<SDT, GDT, PDT>(s, r, t0 + tid);
}

// ---- software pipeline over work items ------------------------------------------------------------
// The memory system rewards a small moving window: with few resident waves all writing and
// reading close together, DRAM pages stay open and read/write turnarounds are fewer.  Few waves
// cannot hide latency by occupancy, so each wave hides it itself: the loads of its next work item
// are in flight while it computes and stores the current one (two register tiles, ping-pong).

// Whole, aligned work items take the tile path; a row's first item when it has head elements,
// its ragged last item, and every item of a misaligned row go through step_chunk.
template <int SDT>
__device__ __forceinline__ bool item_is_tile(const Item& it) {
  constexpr uint64_t kChunkGroups = uint64_t(kBlock) * StateIO<SDT>::kUnroll;
  if (!it.vec || it.n <= it.head) return false;
  if (it.lc == 0 && it.head != 0) return false;
  return (it.lc + 1) * kChunkGroups <= (it.n - it.head) / StateIO<SDT>::kGroup;
}

template <int SDT, int GDT>
struct Tile {
  static constexpr int kUnroll = StateIO<SDT>::kUnroll;
  typename StateIO<SDT>::Packet P[kUnroll], M[kUnroll], V[kUnroll];
  GradGroup<GDT, StateIO<SDT>::kGroup> G[kUnroll];
};

template <int SDT, int GDT>
__device__ __forceinline__ void tile_load(Tile<SDT, GDT>& t, const Item& it) {
  constexpr int kUnroll = StateIO<SDT>::kUnroll;
  constexpr uint64_t kChunkGroups = uint64_t(kBlock) * kUnroll;
  const uint64_t g0 = it.lc * kChunkGroups + threadIdx.x;
  const BodyPtrs<SDT, GDT> b(row_ptrs(it), it.head);
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint64_t gi = g0 + uint64_t(u) * kBlock;
    t.G[u].load(b.g, gi);
    t.P[u] = ld_stream(b.p + gi);
    t.M[u] = ld_stream(b.m + gi);
    t.V[u] = ld_stream(b.v + gi);
  }
}

// PACE: a pause (s_sleep units) between the computation of a tile and its stores.  Measured on
// MI355X with one block per CU, the 1:1 read/write mix of fp32 states sustains more when every CU
// holds back a little (about 0.8 us of a 4.6 us tile period): 8B-shaped list 6.25-6.28 TB/s
// without a pause, 6.32 at 24 units, 6.35 at 28, 6.38 at 32, 6.36 at 36, 6.34 at 40; a flat
// 3.7e9-element sub-group 6.27 / 6.37 / 6.41 / 6.40 / 6.38 / 6.36.  The same pause before the
// tile's loads does as well on large inputs and 1-3 % worse on small ones; split over both places,
// or spread between the groups of a tile, it is worse.  bf16 states do not react to it.
template <int SDT, int GDT, int PDT, int PACE>
__device__ __forceinline__ void tile_finish(Tile<SDT, GDT>& t, const Item& it, const StepScalars& s) {
  constexpr int kUnroll = StateIO<SDT>::kUnroll;
  constexpr uint64_t kChunkGroups = uint64_t(kBlock) * kUnroll;
  const uint64_t g0 = it.lc * kChunkGroups + threadIdx.x;
  const BodyPtrs<SDT, GDT> b(row_ptrs(it), it.head);
  u32x2 L[kUnroll];
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) step_group<SDT, GDT, PDT>(s, t.P[u], t.M[u], t.V[u], t.G[u], L[u]);
  if constexpr (PACE > 0) __builtin_amdgcn_s_sleep(PACE);
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint64_t gi = g0 + uint64_t(u) * kBlock;
    st_stream(b.p + gi, t.P[u]);
    st_stream(b.m + gi, t.M[u]);
    st_stream(b.v + gi, t.V[u]);
    if constexpr (PDT != kNoLp) st_stream(b.lp + gi, L[u]);
  }
}

template <int SDT, int GDT, int PDT, int PACE>
__device__ __forceinline__ void item_finish(bool tile, Tile<SDT, GDT>& t, const Item& it,
                                            const StepScalars& s) {
  if (tile) {
    tile_finish<SDT, GDT, PDT, PACE>(t, it, s);
  } else {
    step_chunk<SDT, GDT, PDT>(s, it);
  }
}

// ---- which work items a block takes ------------------------------------------------------------------
// Every block first sweeps a fixed share.  A tensor list brings device memory for a few counters
// (StepQueue), and then the last 1/2^MA_STEP_POOL_SHIFT of every XCD's share is not dealt out in
// advance: a block that has finished its fixed share draws items from its own XCD's pool, then
// from the other XCDs' pools, until all are empty.  Measured on MI355X the blocks of a launch do not
// run at one speed (the odd-numbered XCDs end 0.8-1.6 % later than the even ones on equal shares,
// and the blocks of one XCD spread by another 0.3 %); on equal fixed shares the early blocks idle
// until the last one ends.  Each pool index is handed out exactly once (one atomic add per item,
// by one lane, passed on through LDS), so every work item is still processed exactly once, by
// whichever block gets there.  The two phases are separate loops: the fixed-share loop is the one
// whose timing the pause of tile_finish is tuned to, and it stays as it is without pools.

// Pool of XCD y for a launch of `chunks` items: [base, base + pool).
__device__ __forceinline__ void step_pool_of(uint64_t chunks, uint32_t y, uint64_t& base, uint64_t& pool) {
  const uint64_t per_xcd = (chunks + 7) / 8;
  const uint64_t lo = uint64_t(y) * per_xcd;
  const uint64_t hi = (lo + per_xcd < chunks) ? lo + per_xcd : chunks;
  const uint64_t count = hi > lo ? hi - lo : 0;
  pool = count >> MA_STEP_POOL_SHIFT;
  base = hi - pool;
}

// The fixed share.  pools: leave the XCDs' pools out (the grid is then a multiple of 8 blocks).
struct FixedItems {
  uint64_t c, end, stride;
  __device__ __forceinline__ FixedItems(uint64_t chunks, bool pools) {
    const WorkIter<MA_STEP_MAP> w(chunks);
    c = w.c;
    end = w.end;
    stride = w.stride;
    if (pools) {
      uint64_t base, pool;
      step_pool_of(chunks, blockIdx.x & 7, base, pool);
      end = base;
    }
  }
  __device__ __forceinline__ bool next(uint64_t& out) {
    if (c >= end) return false;
    out = c;
    c += stride;
    return true;
  }
};

// Items drawn from the pools, several consecutive ones per draw: a draw costs the block a barrier,
// which lines up its four otherwise free-running waves.  Up to MA_STEP_DRAW items per draw, fewer
// when the pools are small, so that a pool always makes at least four draws per block of its XCD
// (the last draws decide how evenly the launch ends).
struct PoolItems {
  StepQueue* q;
  uint32_t* slot;  // two words of LDS
  uint64_t chunks;
  uint64_t cur = 0;  // next item of the current draw
  uint32_t left = 0;  // items of the current draw not yet handed out
  uint32_t x, visited = 0, parity = 0;
  uint32_t draw;

  __device__ __forceinline__ PoolItems(uint64_t chunks_, StepQueue* q_, uint32_t* slot_)
      : q(q_), slot(slot_), chunks(chunks_), x(blockIdx.x & 7) {
    uint64_t base, pool;
    step_pool_of(chunks, x, base, pool);
    const uint64_t fine = pool / (uint64_t(gridDim.x >> 3) * 4);
    draw = fine < 1 ? 1u : fine > MA_STEP_DRAW ? uint32_t(MA_STEP_DRAW) : uint32_t(fine);
  }

  __device__ __forceinline__ bool next(uint64_t& out) {
    while (left == 0) {
      if (visited >= 8) return false;
      const uint32_t y = (x + visited) & 7;
      uint64_t base, pool;
      step_pool_of(chunks, y, base, pool);
      if (threadIdx.x == 0) slot[parity] = atomicAdd(&q->next[y], draw);
      __syncthreads();
      const uint32_t idx = __builtin_amdgcn_readfirstlane(slot[parity]);
      parity ^= 1u;  // the next draw writes the other word: one barrier per draw is enough
      if (idx < pool) {
        const uint64_t rest = pool - idx;
        left = rest < draw ? uint32_t(rest) : draw;
        cur = base + idx;
      } else {
        ++visited;
      }
    }
    out = cur++;
    --left;
    return true;
  }

  // Called once by every block after its last item: the last block to arrive clears the queue.
  __device__ __forceinline__ void finish() {
    if (threadIdx.x != 0) return;
    __threadfence();
    if (atomicAdd(&q->done, 1u) == gridDim.x - 1) {
#pragma unroll
      for (int y = 0; y < 8; ++y) atomicExch(&q->next[y], 0u);
      atomicExch(&q->done, 0u);
    }
  }
};

// locate(c, item) fills `item` for global work item c (c is uniform across the block).
//
// Two register tiles alternate: the loads of the next item are issued, then the current item is
// computed and stored.  Because "is the next item a whole tile" is a run-time condition, the waits
// the compiler places inside the computation also cover part of the prefetch, so the stores of a
// tile are issued once the next tile has (nearly) arrived.  Measured on MI355X this is the faster
// form: a variant with straight-line runs of tiles, whose stores go out while the prefetch is
// still in flight, was 1 % slower (more reads and writes in flight at once lower the bandwidth the
// memory system sustains), and an explicit drain before the stores changed nothing.
template <int SDT, int GDT, int PDT, int PACE, class Items, class Locate>
__device__ __forceinline__ void step_pipeline(const StepScalars& s, Items& items, Locate locate) {
  Item ia, ib;
  Tile<SDT, GDT> ta, tb;
  uint64_t c = 0;
  bool fa = false, fb = false;
  if (items.next(c)) {
    locate(c, ia);
    fa = item_is_tile<SDT>(ia);
    if (fa) tile_load<SDT, GDT>(ta, ia);
    for (;;) {
      // A is current; start B
      bool more = items.next(c);
      if (more) {
        locate(c, ib);
        fb = item_is_tile<SDT>(ib);
        if (fb) tile_load<SDT, GDT>(tb, ib);
      }
      item_finish<SDT, GDT, PDT, PACE>(fa, ta, ia, s);
      if (!more) break;
      // B is current; start A
      more = items.next(c);
      if (more) {
        locate(c, ia);
        fa = item_is_tile<SDT>(ia);
        if (fa) tile_load<SDT, GDT>(ta, ia);
      }
      item_finish<SDT, GDT, PDT, PACE>(fb, tb, ib, s);
      if (!more) break;
    }
  }
}


// ---- what the kernel decides on the device ---------------------------------------------------------
// Returns false when the step must not touch any buffer (Sec. III-C: the scan saw an overflow).
//   * scaler state present: the loss scale and the update number (applied steps + 1) come from
//     device memory, and the two bias-correction scalars are evaluated here, in fp64, by the same
//     routine the host uses (pow_int, then one rounding to fp32 each): bit-identical scalars;
//   * gate present: the unscale-and-clip factor follows from the scanned sum of squares with the
//     same two roundings as the host path (clip coefficient to fp32, then c/S in fp64 to fp32).
__device__ __forceinline__ bool prepare_step(const StepControl& ctl, StepScalars& s) {
  float loss_scale = ctl.loss_scale;
  // The scan's per-block partials instead of a finished result: every block adds them up itself, in
  // the order of the stand-alone finalize kernel (same function, same bits), which saves that launch;
  // block 0 publishes the result for the caller.
  NormResult folded;
  const bool fold = ctl.partials != nullptr;
  if (fold) {
    folded = fold_partials(ctl.partials, ctl.partial_count, ctl.inv_scale_sq, nullptr, ctl.threshold,
                           ctl.packed16);
    if (blockIdx.x == 0 && threadIdx.x == 0) *ctl.result_out = folded;
  }
  if (ctl.scaler != nullptr) {
    loss_scale = ctl.scaler->scale;
    double bc1 = 1.0, bc2 = 1.0;
    if (ctl.bias_correction) {
      const uint64_t t = static_cast<uint64_t>(ctl.scaler->step + 1);
      bc1 = 1.0 - pow_int(static_cast<double>(s.beta1), t);
      bc2 = 1.0 - pow_int(static_cast<double>(s.beta2), t);
    }
    s.step_size = static_cast<float>(static_cast<double>(ctl.lr) / bc1);
    s.inv_sqrt_bc2 = static_cast<float>(1.0 / __builtin_sqrt(bc2));
  }
  if (ctl.gate != nullptr || fold) {
    const int overflow = fold ? folded.overflow : ctl.gate->overflow;
    const double sumsq = fold ? folded.sumsq : ctl.gate->sumsq;
    if (overflow != 0) return false;
    double c = 1.0;
    if (ctl.max_norm > 0.0f) {
      c = static_cast<double>(ctl.max_norm) / (__builtin_sqrt(sumsq) + 1e-6);
      c = (c < 1.0) ? c : 1.0;
    }
    const float cf = static_cast<float>(c);
    s.gscale = static_cast<float>(static_cast<double>(cf) / static_cast<double>(loss_scale));
  }
  return true;
}

template <int SDT, int GDT, int PDT>
__global__ __launch_bounds__(kBlock) void step_flat_kernel(Desc row, uint64_t chunks, StepScalars s,
                                                          StepControl ctl) {
  if (!prepare_step(ctl, s)) return;
  FixedItems items(chunks, false);
  step_pipeline<SDT, GDT, PDT, step_pace(SDT, false)>(s, items, [&](uint64_t c, Item& it) {
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

template <int SDT, int GDT, int PDT>
__global__ __launch_bounds__(kBlock) void step_multi_kernel(const Desc* __restrict__ table,
                                                           uint32_t rows, uint64_t chunks,
                                                           StepScalars s, StepControl ctl,
                                                           StepQueue* queue) {
  __shared__ uint32_t draw_slot[2];
  if (!prepare_step(ctl, s)) return;
  // A block's work items advance in steps much smaller than a typical tensor, so the row of the
  // previous item is kept (in scalar registers) together with the range of items it covers, and
  // the table is searched only when an item falls outside that range.  While items increase the
  // last hit bounds the search from below.
  uint32_t r = 0;
  uint64_t row_first = 1, row_end = 0;  // empty range: the first item always searches
  Item row{};
  auto locate = [&](uint64_t c, Item& it) {
    if (c < row_first || c >= row_end) {
      // largest row whose first work item is <= c (uniform => scalar unit)
      uint32_t lo = (c >= row_first) ? r : 0, hi = rows;
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
      row.p = d->p;
      row.m = d->m;
      row.v = d->v;
      row.g = d->g;
      row.lp = d->lp;
      row.n = d->n;
      row.head = d->step_head;
      row.vec = d->step_vec;
      row_first = d->step_chunk0;
      row_end = (r + 1 < rows) ? table[r + 1].step_chunk0 : chunks;
    }
    it = row;
    it.lc = c - row_first;
  };
  FixedItems fixed(chunks, queue != nullptr);
  step_pipeline<SDT, GDT, PDT, step_pace(SDT, true)>(s, fixed, locate);
  if (queue != nullptr) {
    PoolItems drawn(chunks, queue, draw_slot);
    step_pipeline<SDT, GDT, PDT, step_pace(SDT, true)>(s, drawn, locate);
    drawn.finish();
  }
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

// Fewest work items of a launch that uses pools.  Measured on 8B-shaped lists scaled down: with
// 30,000 items (1.3e8 elements) pools cost 1.5-2 % (the second loop's start-up and the eight empty
// draws at the end weigh more than the evening-out gains), with 120,000 items they gain 0.5 %, from
// 500,000 items on 0.6-0.8 %.
#ifndef MA_STEP_POOL_MIN_ITEMS
#define MA_STEP_POOL_MIN_ITEMS 65536
#endif
constexpr uint64_t kMinItemsForPools = MA_STEP_POOL_MIN_ITEMS;
static_assert(kMinItemsForPools >= (uint64_t(8) << MA_STEP_POOL_SHIFT), "every XCD's pool must hold an item");

template <int SDT, int GDT, int PDT>
static hipError_t launch_step_typed(const Desc* row_host, const Desc* table_dev, uint32_t rows,
                                    uint64_t chunks, const StepScalars& s, const StepControl& ctl,
                                    StepQueue* queue, int device_cus, hipStream_t stream) {
  // A persistent grid must be fully resident: blocks that wait for a slot would run alone at the
  // end.  So: no more blocks per compute unit than the kernel's occupancy allows.  Queried once per
  // process and instantiation (thread-safe static initialisation), for the device current at that
  // moment: all GPUs of one process are taken to be the same model.
  static const int occ_flat = resident_blocks_per_cu(step_flat_kernel<SDT, GDT, PDT>);
  static const int occ_multi = resident_blocks_per_cu(step_multi_kernel<SDT, GDT, PDT>);
  const int occ = row_host ? occ_flat : occ_multi;
  // One block per CU: the 1:1 read/write mix is fastest with few, deep waves.  bf16 states move
  // half the bytes per element, so arithmetic takes a larger share of a tile's time (hardware
  // counters: the vector unit executes an instruction in 77 % of the wave's cycles, against 31 % for
  // fp32 states) and the tile is deeper (eight groups) to keep enough loads in flight meanwhile.
  // 8.03e9 elements, one machine: 6 / 7 / 8 / 9 / 10 / 12 groups 18.1 / 18.2 / 17.8 / 18.0 / 18.0 /
  // 18.1 ms; two blocks per CU with four-group tiles 18.1 ms (18.4 before the truncating store lost
  // its per-value NaN re-check).
  constexpr int kPerCu = (SDT == kF32) ? MA_STEP_BLOCKS_PER_CU : MA_STEP_BLOCKS_PER_CU_BF16;
  const uint64_t want = uint64_t(device_cus) * (occ < kPerCu ? occ : kPerCu);
  const uint32_t grid = static_cast<uint32_t>(chunks < want ? chunks : want);
  if (row_host) {
    step_flat_kernel<SDT, GDT, PDT><<<grid, kBlock, 0, stream>>>(*row_host, chunks, s, ctl);
  } else {
    // pools of late items need whole XCD groups of blocks and something to put into them
    StepQueue* q = ((grid & 7u) == 0 && chunks >= kMinItemsForPools) ? queue : nullptr;
    step_multi_kernel<SDT, GDT, PDT><<<grid, kBlock, 0, stream>>>(table_dev, rows, chunks, s, ctl, q);
  }
  return hipGetLastError();
}

template <int SDT, int GDT>
static hipError_t launch_step_g(int pdt, const Desc* row_host, const Desc* table_dev, uint32_t rows,
                                uint64_t chunks, const StepScalars& s, const StepControl& ctl,
                                StepQueue* queue, int device_cus, hipStream_t stream) {
  if constexpr (SDT != kF32) {
    // half-precision states: the parameter itself is the 16-bit copy
    return launch_step_typed<SDT, GDT, kNoLp>(row_host, table_dev, rows, chunks, s, ctl, queue, device_cus, stream);
  } else {
    switch (pdt) {
      case kBF16: return launch_step_typed<SDT, GDT, kBF16>(row_host, table_dev, rows, chunks, s, ctl, queue, device_cus, stream);
      case kF16: return launch_step_typed<SDT, GDT, kF16>(row_host, table_dev, rows, chunks, s, ctl, queue, device_cus, stream);
      default: return launch_step_typed<SDT, GDT, kNoLp>(row_host, table_dev, rows, chunks, s, ctl, queue, device_cus, stream);
    }
  }
}

template <int SDT>
static hipError_t launch_step_s(int gdt, int pdt, const Desc* row_host, const Desc* table_dev,
                                uint32_t rows, uint64_t chunks, const StepScalars& s,
                                const StepControl& ctl, StepQueue* queue, int device_cus,
                                hipStream_t stream) {
  switch (gdt) {
    case kBF16: return launch_step_g<SDT, kBF16>(pdt, row_host, table_dev, rows, chunks, s, ctl, queue, device_cus, stream);
    case kF16: return launch_step_g<SDT, kF16>(pdt, row_host, table_dev, rows, chunks, s, ctl, queue, device_cus, stream);
    default: return launch_step_g<SDT, kF32>(pdt, row_host, table_dev, rows, chunks, s, ctl, queue, device_cus, stream);
  }
}

hipError_t launch_step(const Desc* row_host, const Desc* table_dev, uint32_t rows, uint64_t chunks,
                       int sdt, int gdt, int pdt, const StepScalars& s, const StepControl& ctl,
                       StepQueue* queue, int device_cus, hipStream_t stream) {
  if (chunks == 0) return hipSuccess;
  if (sdt == kBF16) return launch_step_s<kBF16>(gdt, pdt, row_host, table_dev, rows, chunks, s, ctl, queue, device_cus, stream);
  return launch_step_s<kF32>(gdt, pdt, row_host, table_dev, rows, chunks, s, ctl, queue, device_cus, stream);
}

}  // namespace ma
