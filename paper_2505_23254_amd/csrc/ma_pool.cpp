// Host side of the offloading system that feeds the optimizer step: the adaptive parameter buffer
// pool (Sec. IV-B) and the sizes of pinned allocations (Sec. III-B, Sec. IV-C).  Plain C++, no
// device code.  See include/ma.h for the contract of every entry point.
//
// Adaptive buffer pool.  While parameters are prefetched, N transformer blocks are in flight, and
// the tensors that travel are, per block, three feed-forward projections (intermediate x hidden),
// the K and V projections (kv_dim x hidden), the Q and O projections (q_dim x hidden), plus the
// embedding and the LM head (vocab x hidden each).  The original pool holds 2 + 7N buffers that all
// have the size of the largest tensor; the adaptive pool keeps four sub-pools of exactly sized
// buffers, 2, 3N, 2N and 2N of them, carved from one monolithic allocation, and a table from a
// caller's key to {sub-pool, slot}.

#include <cstdint>
#include <cstdio>
#include <new>
#include <unordered_map>
#include <vector>

#include "../../include/ma.h"

namespace {

int pool_fail(int code, const char* msg);

struct Held {
  int kind;
  uint32_t slot;
};

}  // namespace

struct ma_pool {
  ma_pool_layout layout;
  std::vector<uint32_t> free_slots[4];  // stack of free slot indices per sub-pool
  std::unordered_map<uint64_t, Held> held;
};

// the library's thread-local error channel (defined beside ma_last_error); not exported
extern "C" __attribute__((visibility("hidden"))) int ma_set_error_message(int code, const char* msg);

namespace {
int pool_fail(int code, const char* msg) { return ma_set_error_message(code, msg); }

uint64_t round_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }
uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }
}  // namespace

extern "C" {

int ma_pool_layout_compute(const ma_model_dims* dims, uint32_t blocks_in_flight, uint32_t elem_bytes,
                           uint32_t partitions, uint32_t align, ma_pool_layout* out_host) {
  if (!dims || !out_host) return pool_fail(MA_ERR_NULL, "dims and out_host must not be NULL");
  if (blocks_in_flight < 1) return pool_fail(MA_ERR_ARG, "blocks_in_flight must be >= 1");
  if (!(elem_bytes == 1 || elem_bytes == 2 || elem_bytes == 4))
    return pool_fail(MA_ERR_ARG, "elem_bytes must be 1, 2 or 4");
  if (partitions < 1) return pool_fail(MA_ERR_ARG, "partitions must be >= 1");
  if (align < 1 || (align & (align - 1)) != 0) return pool_fail(MA_ERR_ARG, "align must be a power of two");
  if (!dims->vocab || !dims->hidden || !dims->intermediate || !dims->kv_dim || !dims->q_dim)
    return pool_fail(MA_ERR_ARG, "all model dimensions must be non-zero");
  const uint64_t limit = uint64_t(1) << 40;  // elements of one tensor; keeps every product in range
  const uint64_t rows[4] = {dims->vocab, dims->intermediate, dims->kv_dim, dims->q_dim};
  for (uint64_t r : rows)
    if (r > limit / dims->hidden) return pool_fail(MA_ERR_ARG, "tensor of more than 2^40 elements");
  const uint64_t n = blocks_in_flight;
  ma_pool_layout L{};
  const uint64_t counts[4] = {2, 3 * n, 2 * n, 2 * n};
  uint64_t off = 0, largest = 0;
  for (int k = 0; k < 4; ++k) {
    // each process holds its own shard of a partitioned tensor
    const uint64_t shard = ceil_div(rows[k] * dims->hidden, partitions);
    L.count[k] = counts[k];
    L.buffer_bytes[k] = round_up(shard * elem_bytes, align);
    L.offset[k] = off;
    off += L.count[k] * L.buffer_bytes[k];
    if (L.buffer_bytes[k] > largest) largest = L.buffer_bytes[k];
  }
  L.total_bytes = off;
  L.uniform_count = 2 + 7 * n;
  L.uniform_buffer_bytes = largest;
  L.uniform_bytes = L.uniform_count * largest;
  *out_host = L;
  return MA_OK;
}

int ma_pool_create(const ma_pool_layout* layout, ma_pool** pool_out) {
  if (!layout || !pool_out) return pool_fail(MA_ERR_NULL, "layout and pool_out must not be NULL");
  uint64_t off = 0;
  for (int k = 0; k < 4; ++k) {
    if (layout->count[k] == 0 || layout->count[k] > (1u << 20) || layout->buffer_bytes[k] == 0 ||
        layout->offset[k] != off)
      return pool_fail(MA_ERR_ARG, "layout was not written by ma_pool_layout_compute");
    off += layout->count[k] * layout->buffer_bytes[k];
  }
  if (off != layout->total_bytes) return pool_fail(MA_ERR_ARG, "layout was not written by ma_pool_layout_compute");
  ma_pool* p = new (std::nothrow) ma_pool;
  if (!p) return pool_fail(MA_ERR_ARG, "out of host memory");
  p->layout = *layout;
  for (int k = 0; k < 4; ++k) {
    // slots are handed out in increasing order
    for (uint32_t s = uint32_t(layout->count[k]); s > 0; --s) p->free_slots[k].push_back(s - 1);
  }
  *pool_out = p;
  return MA_OK;
}

void ma_pool_destroy(ma_pool* pool) { delete pool; }

int ma_pool_acquire(ma_pool* pool, uint64_t key, int kind, uint64_t* offset_out, uint64_t* bytes_out) {
  if (!pool || !offset_out) return pool_fail(MA_ERR_NULL, "pool and offset_out must not be NULL");
  if (kind < 0 || kind > 3) return pool_fail(MA_ERR_ARG, "kind must be one of the four sub-pools");
  if (pool->held.count(key)) return pool_fail(MA_ERR_ARG, "key already holds a buffer");
  std::vector<uint32_t>& fs = pool->free_slots[kind];
  if (fs.empty()) return pool_fail(MA_ERR_FULL, "every buffer of this sub-pool is in use");
  const uint32_t slot = fs.back();
  fs.pop_back();
  pool->held[key] = Held{kind, slot};
  *offset_out = pool->layout.offset[kind] + uint64_t(slot) * pool->layout.buffer_bytes[kind];
  if (bytes_out) *bytes_out = pool->layout.buffer_bytes[kind];
  return MA_OK;
}

int ma_pool_lookup(const ma_pool* pool, uint64_t key, uint64_t* offset_out, uint64_t* bytes_out) {
  if (!pool || !offset_out) return pool_fail(MA_ERR_NULL, "pool and offset_out must not be NULL");
  auto it = pool->held.find(key);
  if (it == pool->held.end()) return pool_fail(MA_ERR_ARG, "key holds no buffer");
  const Held h = it->second;
  *offset_out = pool->layout.offset[h.kind] + uint64_t(h.slot) * pool->layout.buffer_bytes[h.kind];
  if (bytes_out) *bytes_out = pool->layout.buffer_bytes[h.kind];
  return MA_OK;
}

int ma_pool_release(ma_pool* pool, uint64_t key) {
  if (!pool) return pool_fail(MA_ERR_NULL, "pool is NULL");
  auto it = pool->held.find(key);
  if (it == pool->held.end()) return pool_fail(MA_ERR_ARG, "key holds no buffer");
  pool->free_slots[it->second.kind].push_back(it->second.slot);
  pool->held.erase(it);
  return MA_OK;
}

uint64_t ma_pool_in_use(const ma_pool* pool, int kind) {
  if (!pool || kind < 0 || kind > 3) return 0;
  return pool->layout.count[kind] - pool->free_slots[kind].size();
}

uint64_t ma_pinned_bytes(uint64_t request, int policy) {
  if (request == 0) return 0;
  if (policy == MA_PINNED_POW2) {
    uint64_t p = 1;
    while (p < request) {
      if (p > (uint64_t(1) << 62)) return UINT64_MAX;
      p <<= 1;
    }
    return p;
  }
  return round_up(request, 4096);
}

}  // extern "C"
