// C ABI of libma_step.so: argument checking, work-table construction, host scalars, launches.
// See include/ma.h for the contract of every entry point.

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "../../include/ma.h"
#include "ma_internal.h"

static_assert(sizeof(ma_norm_result) == sizeof(ma::NormResult), "result layout");
static_assert(sizeof(ma_norm_result) == 16, "result layout");
static_assert(sizeof(ma_scaler_state) == sizeof(ma::ScalerState) && sizeof(ma_scaler_state) == 24,
              "scaler state layout");
static_assert(sizeof(ma_scaler_config) == sizeof(ma::ScalerConfig), "scaler config layout");
static_assert(int(MA_F32) == ma::kF32 && int(MA_BF16) == ma::kBF16 && int(MA_F16) == ma::kF16,
              "dtype codes");

// Scratch of ma_overflow_norm_static: the per-block partial results of one scan launch, owned by
// the library so that the call needs no workspace from the caller.  Every GPU the library runs on
// holds its own copy at its own address until the process ends.  In host code this name only
// identifies the symbol; the memory is reached through the address scratch_address() returns.
static __device__ __align__(256) unsigned char scratch[ma::kMaxNormBlocks * sizeof(ma::NormPartial)];

namespace {

thread_local char g_error[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  std::vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
  return code;
}

int fail_hip(hipError_t e, const char* what) {
  return fail(MA_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

constexpr uint32_t kPlanMagic = 0x4D415450u;  // "MATP"


bool dtype_ok(int dt) { return dt == MA_F32 || dt == MA_BF16 || dt == MA_F16; }
size_t elem_bytes(int dt) { return dt == MA_F32 ? 4 : 2; }
bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

constexpr int kMaxDevices = 64;

// Compute units of the current device (queried once per device index; threads may race to fill a
// slot, they all store the same value).
int device_cus(int* out) {
  static std::atomic<int> cached[kMaxDevices];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
  const bool slot = dev >= 0 && dev < kMaxDevices;
  if (slot) {
    const int c = cached[dev].load(std::memory_order_relaxed);
    if (c > 0) {
      *out = c;
      return MA_OK;
    }
  }
  int cus = 0;
  e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return fail_hip(e, "hipDeviceGetAttribute");
  if (cus <= 0) return fail(MA_ERR_HIP, "device reports %d compute units", cus);
  if (slot) cached[dev].store(cus, std::memory_order_relaxed);
  *out = cus;
  return MA_OK;
}

// Device address of `scratch` on the current device.  Looked up once per device, with that device
// current (each GPU has its own copy of the array), and kept; the lookup allocates nothing.
int scratch_address(void** out) {
  static std::mutex mu;
  static void* addr[kMaxDevices] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(MA_ERR_ARG, "device index %d is beyond the %d this library keeps scratch for", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(mu);
  if (addr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return fail_hip(e, "hipGetSymbolAddress(scratch)");
    if (p == nullptr) return fail(MA_ERR_HIP, "hipGetSymbolAddress(scratch) returned a null address");
    addr[dev] = p;
  }
  *out = addr[dev];
  return MA_OK;
}

int check_scale(float loss_scale) {
  if (!(loss_scale > 0.0f) || !std::isfinite(loss_scale))
    return fail(MA_ERR_ARG, "loss_scale must be finite and > 0 (got %g)", double(loss_scale));
  return MA_OK;
}

int check_hyper(const ma_hyper* h, int64_t step) {
  if (!h) return fail(MA_ERR_NULL, "hyper is NULL");
  if (step < 1) return fail(MA_ERR_ARG, "step must be >= 1 (got %lld)", (long long)step);
  if (!(h->lr >= 0.0f) || !std::isfinite(h->lr)) return fail(MA_ERR_ARG, "lr must be finite and >= 0");
  if (!(h->beta1 >= 0.0f && h->beta1 < 1.0f)) return fail(MA_ERR_ARG, "beta1 must be in [0, 1)");
  if (!(h->beta2 >= 0.0f && h->beta2 < 1.0f)) return fail(MA_ERR_ARG, "beta2 must be in [0, 1)");
  if (!(h->eps > 0.0f) || !std::isfinite(h->eps)) return fail(MA_ERR_ARG, "eps must be finite and > 0");
  if (!(h->weight_decay >= 0.0f) || !std::isfinite(h->weight_decay))
    return fail(MA_ERR_ARG, "weight_decay must be finite and >= 0");
  return MA_OK;
}

// The fp32 scalars of one step: evaluated in fp64 from the fp32 hyper-parameters, rounded once.
ma::StepScalars host_scalars(const ma_hyper& h, int64_t step, float loss_scale, float clip_coef) {
  ma::StepScalars s;
  const double b1 = h.beta1, b2 = h.beta2;
  double bc1 = 1.0, bc2 = 1.0;
  if (h.bias_correction) {
    bc1 = 1.0 - ma::pow_int(b1, uint64_t(step));
    bc2 = 1.0 - ma::pow_int(b2, uint64_t(step));
  }
  s.beta1 = h.beta1;
  s.beta2 = h.beta2;
  s.omb1 = float(1.0 - b1);
  s.omb2 = float(1.0 - b2);
  s.eps = h.eps;
  s.step_size = float(double(h.lr) / bc1);
  s.inv_sqrt_bc2 = float(1.0 / std::sqrt(bc2));
  s.decay = float(double(h.lr) * double(h.weight_decay));
  s.gscale = float(double(clip_coef) / double(loss_scale));
  return s;
}

uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

// A buffer named in a call, as a byte range.
struct Range {
  uintptr_t lo, hi;
  uint32_t owner;  // index of the tensor it belongs to (lists)
};
Range range_of(const void* p, uint64_t bytes, uint32_t owner = 0) {
  const uintptr_t a = reinterpret_cast<uintptr_t>(p);
  return Range{a, a + bytes, owner};
}
// True when two of the (non-empty) ranges share a byte; a and b receive their positions in `r`.
bool any_overlap(std::vector<Range>& r, const Range** a, const Range** b) {
  std::sort(r.begin(), r.end(), [](const Range& x, const Range& y) { return x.lo < y.lo; });
  for (size_t i = 1; i < r.size(); ++i) {
    if (r[i].lo < r[i - 1].hi) {
      *a = &r[i - 1];
      *b = &r[i];
      return true;
    }
  }
  return false;
}
// The buffers of one row: p, m, v (sb bytes per element), the gradient, the optional 16-bit copy.
void row_ranges(const ma::Desc& d, int gdt, size_t sb, uint32_t owner, std::vector<Range>& out) {
  out.push_back(range_of(d.p, d.n * sb, owner));
  out.push_back(range_of(d.m, d.n * sb, owner));
  out.push_back(range_of(d.v, d.n * sb, owner));
  out.push_back(range_of(d.g, d.n * elem_bytes(gdt), owner));
  if (d.lp) out.push_back(range_of(d.lp, d.n * 2, owner));
}

// Fills the alignment-dependent fields of a row and returns its work-item counts.
// Returns a negative status if a pointer is not aligned to its element size.
int plan_row(ma::Desc& d, int gdt, bool has_lp, uint64_t* norm_chunks, uint64_t* step_chunks,
             size_t sb = 4) {
  const size_t gb = elem_bytes(gdt);
  if (!aligned(d.g, gb)) return fail(MA_ERR_ALIGN, "grad pointer not aligned to its element size");
  // scan: elements before the gradient's first 16-byte boundary
  const uintptr_t ga = reinterpret_cast<uintptr_t>(d.g);
  d.norm_head = uint32_t(((16 - (ga % 16)) % 16) / gb);
  const uint64_t chunk_elems = ma::kNormChunkBytes / gb;
  *norm_chunks = (d.n <= d.norm_head) ? 1 : ceil_div(d.n - d.norm_head, chunk_elems);

  if (step_chunks == nullptr) return MA_OK;  // scan-only row
  if (!aligned(d.p, sb) || !aligned(d.m, sb) || !aligned(d.v, sb))
    return fail(MA_ERR_ALIGN, "p/m/v pointers must be aligned to their element size");
  if (has_lp && !aligned(d.lp, 2)) return fail(MA_ERR_ALIGN, "p_lp pointer must be 2-byte aligned");
  // update: p, m, v move as 16-byte packets (a group: 4 fp32 or 8 bf16 elements).  A head of h
  // elements must bring every buffer to the boundary its packets need: 16 bytes for p, m, v, one
  // group's worth (at most 16 bytes) for the gradient and the parameter copy.
  const int sdt = (sb == 4) ? ma::kF32 : ma::kBF16;
  const size_t group = size_t(ma::step_group_elems(sdt));
  const uint32_t h = uint32_t(((16 - (reinterpret_cast<uintptr_t>(d.p) % 16)) % 16) / sb);
  auto ok = [&](const void* ptr, size_t eb) {
    const size_t need = group * eb < 16 ? group * eb : 16;
    return ((reinterpret_cast<uintptr_t>(ptr) + uint64_t(h) * eb) % need) == 0;
  };
  const bool vec = ok(d.m, sb) && ok(d.v, sb) && ok(d.g, gb) && (!has_lp || ok(d.lp, 2));
  d.step_head = vec ? h : 0;
  d.step_vec = vec ? 1 : 0;
  d.pad = 0;
  const uint64_t chunk = ma::step_chunk_elems(sdt);
  if (vec) {
    *step_chunks = (d.n <= h) ? 1 : ceil_div(d.n - h, chunk);
  } else {
    *step_chunks = ceil_div(d.n, chunk);
  }
  return MA_OK;
}

int check_ws(const void* ws, size_t ws_bytes) {
  if (!ws) return fail(MA_ERR_NULL, "workspace is NULL");
  if (!aligned(ws, 16)) return fail(MA_ERR_ALIGN, "workspace must be 16-byte aligned");
  if (ws_bytes < ma_workspace_bytes())
    return fail(MA_ERR_ARG, "workspace too small: %zu < %zu bytes", ws_bytes, ma_workspace_bytes());
  return MA_OK;
}

int check_plan(const ma_multi_plan* plan) {
  if (!plan) return fail(MA_ERR_NULL, "plan is NULL");
  if (plan->magic != kPlanMagic) return fail(MA_ERR_ARG, "plan was not written by ma_multi_prepare");
  if (plan->entries > 0 && !plan->table_dev) return fail(MA_ERR_NULL, "plan has no device table");
  if (!(plan->sdt == MA_F32 || plan->sdt == MA_BF16)) return fail(MA_ERR_ARG, "plan has an unknown state dtype");
  return MA_OK;
}

struct StepRequest {
  const ma_hyper* hyper = nullptr;
  int64_t step = 1;                      // ignored when scaler != nullptr
  float loss_scale = 1.0f;               // ignored when scaler != nullptr
  float clip_coef = 1.0f;                // used when gate == nullptr
  const ma_norm_result* gate = nullptr;  // device gate (gated / auto variants)
  const void* scaler = nullptr;          // device ma_scaler_state (auto variants)
  float max_norm = 0.0f;
  bool gated = false, automatic = false;
  // whole-step calls: the update launch adds up the scan's partials itself and publishes the result
  const void* partials = nullptr;
  uint32_t partial_count = 0;
  ma_norm_result* result_out = nullptr;
};

int check_request(const StepRequest& q) {
  if (int rc = check_hyper(q.hyper, q.automatic ? 1 : q.step)) return rc;
  if (!q.automatic) {
    if (int rc = check_scale(q.loss_scale)) return rc;
  } else {
    if (!q.scaler) return fail(MA_ERR_NULL, "scaler_dev is NULL");
    if (!aligned(q.scaler, 8)) return fail(MA_ERR_ALIGN, "scaler_dev must be 8-byte aligned");
  }
  if (q.result_out) {
    if (std::isnan(q.max_norm)) return fail(MA_ERR_ARG, "max_norm is NaN");
  } else if (q.gated || q.automatic) {
    if (!q.gate) return fail(MA_ERR_NULL, "gate_dev is NULL");
    if (!aligned(q.gate, 8)) return fail(MA_ERR_ALIGN, "gate_dev must be 8-byte aligned");
    if (std::isnan(q.max_norm)) return fail(MA_ERR_ARG, "max_norm is NaN");
  } else if (!(q.clip_coef > 0.0f && q.clip_coef <= 1.0f)) {
    return fail(MA_ERR_ARG, "clip_coef must be in (0, 1] (got %g)", double(q.clip_coef));
  }
  return MA_OK;
}

// A plan's device table: the update kernel's counters, then the rows.
const ma::Desc* plan_rows(const ma_multi_plan* plan) {
  return reinterpret_cast<const ma::Desc*>(static_cast<const char*>(plan->table_dev) + ma::kTableHeadBytes);
}
ma::StepQueue* plan_queue(const ma_multi_plan* plan) {
  return static_cast<ma::StepQueue*>(const_cast<void*>(plan->table_dev));
}

int step_common(const ma::Desc* row, const ma_multi_plan* plan, uint64_t chunks, int sdt, int gdt,
                int pdt, const StepRequest& q, void* stream) {
  int cus = 0;
  if (int rc = device_cus(&cus)) return rc;
  const bool host_gscale = !(q.gated || q.automatic || q.result_out);
  const ma::StepScalars s = host_scalars(*q.hyper, q.automatic ? 1 : q.step,
                                         q.automatic ? 1.0f : q.loss_scale,
                                         host_gscale ? q.clip_coef : 1.0f);
  ma::StepControl ctl{};
  ctl.gate = reinterpret_cast<const ma::NormResult*>(q.gate);
  ctl.scaler = static_cast<const ma::ScalerState*>(q.scaler);
  ctl.max_norm = q.max_norm;
  ctl.loss_scale = q.loss_scale;
  ctl.lr = q.hyper->lr;
  ctl.bias_correction = q.hyper->bias_correction;
  if (q.result_out) {
    ctl.partials = static_cast<const ma::NormPartial*>(q.partials);
    ctl.partial_count = q.partial_count;
    ctl.result_out = reinterpret_cast<ma::NormResult*>(q.result_out);
    ctl.inv_scale_sq = 1.0 / (double(q.loss_scale) * double(q.loss_scale));
    ctl.threshold = ma::norm_threshold(gdt);
    ctl.packed16 = gdt != MA_F32;
  }
  hipError_t e = ma::launch_step(row, plan ? plan_rows(plan) : nullptr,
                                 plan ? uint32_t(plan->entries) : 1u, chunks, sdt, gdt, pdt, s, ctl,
                                 plan ? plan_queue(plan) : nullptr, cus, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail_hip(e, "update kernel launch");
  return MA_OK;
}

// Every check of a flat update call; fills the row and its number of work items (0 for n == 0).
// sdt: MA_F32 (fp32 master states, optional 16-bit copy) or MA_BF16 (states held in bf16).
int flat_step_check(void* p, void* m, void* v, const void* grad, ma_dtype gdt, void* p_lp, ma_dtype pdt,
                    int sdt, size_t n, const StepRequest& q, ma::Desc& d, uint64_t& sc) {
  sc = 0;
  if (int rc = check_request(q)) return rc;
  if (!dtype_ok(gdt)) return fail(MA_ERR_DTYPE, "unsupported gradient dtype %d", int(gdt));
  if (p_lp && !(pdt == MA_BF16 || pdt == MA_F16))
    return fail(MA_ERR_DTYPE, "low-precision parameter dtype must be MA_BF16 or MA_F16");
  if (n == 0) return MA_OK;
  if (!p || !m || !v || !grad) return fail(MA_ERR_NULL, "p, m, v and grad must not be NULL");
  d = ma::Desc{};
  d.p = static_cast<float*>(p);
  d.m = static_cast<float*>(m);
  d.v = static_cast<float*>(v);
  d.g = grad;
  d.lp = p_lp;
  d.n = n;
  uint64_t nc = 0;
  if (int rc = plan_row(d, gdt, p_lp != nullptr, &nc, &sc, sdt == MA_F32 ? 4 : 2)) return rc;
  std::vector<Range> r;
  row_ranges(d, gdt, sdt == MA_F32 ? 4 : 2, 0, r);
  const Range *a = nullptr, *b = nullptr;
  if (any_overlap(r, &a, &b))
    return fail(MA_ERR_ARG, "buffers overlap: [%p, %p) and [%p, %p)", (void*)a->lo, (void*)a->hi, (void*)b->lo, (void*)b->hi);
  return MA_OK;
}

int flat_step(void* p, void* m, void* v, const void* grad, ma_dtype gdt, void* p_lp, ma_dtype pdt,
              int sdt, size_t n, const StepRequest& q, void* stream) {
  ma::Desc d{};
  uint64_t sc = 0;
  if (int rc = flat_step_check(p, m, v, grad, gdt, p_lp, pdt, sdt, n, q, d, sc)) return rc;
  if (n == 0) return MA_OK;
  return step_common(&d, nullptr, sc, sdt, gdt, p_lp ? int(pdt) : ma::kNoLp, q, stream);
}

int multi_step(const ma_multi_plan* plan, const StepRequest& q, void* stream) {
  if (int rc = check_plan(plan)) return rc;
  if (int rc = check_request(q)) return rc;
  if (plan->entries == 0) return MA_OK;
  return step_common(nullptr, plan, plan->step_chunks, int(plan->sdt), plan->gdt, plan->pdt, q, stream);
}

// Passed as `ws` by the entry point that brings no workspace: never dereferenced.
void* const kLibraryScratch = reinterpret_cast<void*>(uintptr_t(1));

int norm_common(const ma::Desc* row, const ma_multi_plan* plan, uint64_t chunks, int gdt,
                float loss_scale, const void* scaler, ma_norm_result* out_dev, void* ws,
                size_t ws_bytes, void* stream, uint32_t* grid_out = nullptr) {
  if (scaler) {
    if (!aligned(scaler, 8)) return fail(MA_ERR_ALIGN, "scaler_dev must be 8-byte aligned");
  } else if (int rc = check_scale(loss_scale)) {
    return rc;
  }
  if (!out_dev) return fail(MA_ERR_NULL, "out_dev is NULL");
  if (!aligned(out_dev, 8)) return fail(MA_ERR_ALIGN, "out_dev must be 8-byte aligned");
  if (ws == kLibraryScratch) {
    // every argument has been checked; now the partials go to the library's own array
    if (int rc = scratch_address(&ws)) return rc;
  } else if (int rc = check_ws(ws, ws_bytes)) {
    return rc;
  }
  int cus = 0;
  if (int rc = device_cus(&cus)) return rc;
  const double inv = scaler ? 1.0 : 1.0 / (double(loss_scale) * double(loss_scale));
  hipError_t e = ma::launch_norm(row, plan ? plan_rows(plan) : nullptr,
                                 plan ? uint32_t(plan->entries) : 1u, chunks, gdt, inv,
                                 static_cast<const ma::ScalerState*>(scaler),
                                 static_cast<ma::NormPartial*>(ws),
                                 reinterpret_cast<ma::NormResult*>(out_dev), cus,
                                 static_cast<hipStream_t>(stream), grid_out);
  if (e != hipSuccess) return fail_hip(e, "scan kernel launch");
  return MA_OK;
}

int flat_norm(const void* grad, ma_dtype gdt, size_t n, float loss_scale, const void* scaler,
              bool automatic, ma_norm_result* out_dev, void* ws, size_t ws_bytes, void* stream,
              uint32_t* grid_out = nullptr) {
  if (!dtype_ok(gdt)) return fail(MA_ERR_DTYPE, "unsupported gradient dtype %d", int(gdt));
  if (automatic && !scaler) return fail(MA_ERR_NULL, "scaler_dev is NULL");
  if (n > 0 && !grad) return fail(MA_ERR_NULL, "grad is NULL");
  ma::Desc d{};
  d.g = grad;
  d.n = n;
  uint64_t chunks = 0;
  if (n > 0) {
    if (int rc = plan_row(d, gdt, false, &chunks, nullptr)) return rc;
  }
  return norm_common(&d, nullptr, chunks, gdt, loss_scale, scaler, out_dev, ws, ws_bytes, stream, grid_out);
}

// Shared by the two prepare calls: `row(i, d)` fills the pointers and n of tensor i and returns
// whether it carries a low-precision copy.
template <class Row>
int prepare_common(size_t count, ma_dtype gdt, int pdt, int sdt, void* table_dev, size_t table_bytes,
                   void* stream, ma_multi_plan* plan_out, Row row) {
  if (!plan_out) return fail(MA_ERR_NULL, "plan_out is NULL");
  if (count < 1 || count > (1u << 24)) return fail(MA_ERR_ARG, "count must be in [1, 2^24]");
  if (!dtype_ok(gdt)) return fail(MA_ERR_DTYPE, "unsupported gradient dtype %d", int(gdt));
  if (!table_dev) return fail(MA_ERR_NULL, "table_dev is NULL");
  if (!aligned(table_dev, 16)) return fail(MA_ERR_ALIGN, "table_dev must be 16-byte aligned");
  if (table_bytes < ma_multi_table_bytes(count))
    return fail(MA_ERR_ARG, "table too small: %zu < %zu bytes", table_bytes, ma_multi_table_bytes(count));

  std::vector<ma::Desc> rows;
  rows.reserve(count);
  std::vector<Range> ranges;
  ranges.reserve(5 * count);
  uint64_t norm_total = 0, step_total = 0, elems = 0;
  int has_lp = -1;
  for (size_t i = 0; i < count; ++i) {
    ma::Desc d{};
    const int lp = row(i, d) ? 1 : 0;
    if (d.n == 0) continue;
    if (!d.p || !d.m || !d.v || !d.g)
      return fail(MA_ERR_NULL, "tensor %zu: p, m, v and grad must not be NULL", i);
    if (has_lp < 0) has_lp = lp;
    if (lp != has_lp)
      return fail(MA_ERR_ARG, "tensor %zu: p_lp must be set for all tensors of a list or for none", i);
    uint64_t nc = 0, sc = 0;
    if (int rc = plan_row(d, gdt, lp != 0, &nc, &sc, sdt == MA_F32 ? 4 : 2)) {
      char msg[400];
      std::snprintf(msg, sizeof(msg), "%s", g_error);
      return fail(rc, "tensor %zu: %s", i, msg);
    }
    row_ranges(d, gdt, sdt == MA_F32 ? 4 : 2, uint32_t(i), ranges);
    d.norm_chunk0 = norm_total;
    d.step_chunk0 = step_total;
    norm_total += nc;
    step_total += sc;
    elems += d.n;
    rows.push_back(d);
  }
  {
    const Range *a = nullptr, *b = nullptr;
    if (any_overlap(ranges, &a, &b))
      return fail(MA_ERR_ARG, "buffers overlap: tensor %u [%p, %p) and tensor %u [%p, %p)", a->owner, (void*)a->lo,
                  (void*)a->hi, b->owner, (void*)b->lo, (void*)b->hi);
  }
  {
    // the counters (all zero), then the rows, in one copy
    std::vector<char> image(ma::kTableHeadBytes + rows.size() * sizeof(ma::Desc), 0);
    if (!rows.empty()) std::memcpy(image.data() + ma::kTableHeadBytes, rows.data(), rows.size() * sizeof(ma::Desc));
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = hipMemcpyAsync(table_dev, image.data(), image.size(), hipMemcpyHostToDevice, s);
    if (e != hipSuccess) return fail_hip(e, "table upload");
    e = hipStreamSynchronize(s);
    if (e != hipSuccess) return fail_hip(e, "table upload (sync)");
  }
  ma_multi_plan plan{};
  plan.table_dev = table_dev;
  plan.entries = rows.size();
  plan.total_elems = elems;
  plan.norm_chunks = norm_total;
  plan.step_chunks = step_total;
  plan.gdt = gdt;
  plan.pdt = (has_lp <= 0) ? ma::kNoLp : pdt;
  plan.magic = kPlanMagic;
  plan.sdt = uint32_t(sdt);
  *plan_out = plan;
  return MA_OK;
}

}  // namespace

extern "C" {

int ma_version(void) { return 100; }

const char* ma_last_error(void) { return g_error; }

// error channel for the host-only translation unit; not exported
__attribute__((visibility("hidden"))) int ma_set_error_message(int code, const char* msg) {
  return fail(code, "%s", msg);
}

int ma_pinned_alloc(size_t bytes, void** host_ptr_out) {
  if (!host_ptr_out) return fail(MA_ERR_NULL, "host_ptr_out is NULL");
  if (bytes == 0) return fail(MA_ERR_ARG, "bytes must be > 0");
  void* p = nullptr;
  hipError_t e = hipHostMalloc(&p, ma_pinned_bytes(bytes, MA_PINNED_PAGE), hipHostMallocPortable);
  if (e != hipSuccess) return fail_hip(e, "hipHostMalloc");
  *host_ptr_out = p;
  return MA_OK;
}

int ma_pinned_free(void* host_ptr) {
  if (!host_ptr) return fail(MA_ERR_NULL, "host_ptr is NULL");
  hipError_t e = hipHostFree(host_ptr);
  if (e != hipSuccess) return fail_hip(e, "hipHostFree");
  return MA_OK;
}

size_t ma_workspace_bytes(void) { return size_t(ma::kMaxNormBlocks) * sizeof(ma::NormPartial); }

float ma_clip_coef(double sumsq, float max_norm) {
  if (!(max_norm > 0.0f)) return 1.0f;
  const double c = double(max_norm) / (std::sqrt(sumsq) + 1e-6);
  return float(c < 1.0 ? c : 1.0);
}

int ma_step_scalars(const ma_hyper* hyper, int64_t step, float loss_scale, float clip_coef,
                    float out_host[9]) {
  if (int rc = check_hyper(hyper, step)) return rc;
  if (int rc = check_scale(loss_scale)) return rc;
  if (!(clip_coef > 0.0f && clip_coef <= 1.0f))
    return fail(MA_ERR_ARG, "clip_coef must be in (0, 1] (got %g)", double(clip_coef));
  if (!out_host) return fail(MA_ERR_NULL, "out_host is NULL");
  const ma::StepScalars s = host_scalars(*hyper, step, loss_scale, clip_coef);
  const float a[9] = {s.beta1, s.beta2, s.omb1, s.omb2, s.eps,
                      s.step_size, s.inv_sqrt_bc2, s.decay, s.gscale};
  std::memcpy(out_host, a, sizeof(a));
  return MA_OK;
}

int ma_plan_tensor(const ma_tensor* t, ma_dtype gdt, uint64_t* norm_items, uint64_t* step_items,
                   uint32_t* norm_head, uint32_t* step_head, uint32_t* step_vec) {
  if (!t) return fail(MA_ERR_NULL, "tensor_host is NULL");
  if (!dtype_ok(gdt)) return fail(MA_ERR_DTYPE, "unsupported gradient dtype %d", int(gdt));
  ma::Desc d{};
  d.p = t->p32;
  d.m = t->m;
  d.v = t->v;
  d.g = t->grad;
  d.lp = t->p_lp;
  d.n = t->n;
  uint64_t nc = 0, sc = 0;
  if (t->n > 0) {
    if (int rc = plan_row(d, gdt, t->p_lp != nullptr, &nc, &sc)) return rc;
  }
  if (norm_items) *norm_items = nc;
  if (step_items) *step_items = sc;
  if (norm_head) *norm_head = d.norm_head;
  if (step_head) *step_head = d.step_head;
  if (step_vec) *step_vec = d.step_vec;
  return MA_OK;
}

int ma_overflow_norm(const void* grad, ma_dtype gdt, size_t n, float loss_scale,
                     ma_norm_result* out_dev, void* ws, size_t ws_bytes, void* stream) {
  return flat_norm(grad, gdt, n, loss_scale, nullptr, false, out_dev, ws, ws_bytes, stream);
}

int ma_overflow_norm_static(const void* grad, ma_dtype gdt, size_t n, float loss_scale,
                            ma_norm_result* out_dev, void* stream) {
  static_assert(sizeof(scratch) == size_t(ma::kMaxNormBlocks) * sizeof(ma::NormPartial) &&
                    sizeof(scratch) == MA_STATIC_SCRATCH_BYTES,
                "one partial per block of the largest scan grid");
  if (n > MA_STATIC_SCAN_MAX_ELEMS)
    return fail(MA_ERR_ARG, "ma_overflow_norm_static: n = %zu exceeds the maximum of %zu elements", n,
                size_t(MA_STATIC_SCAN_MAX_ELEMS));
  return flat_norm(grad, gdt, n, loss_scale, nullptr, false, out_dev, kLibraryScratch, 0, stream);
}

int ma_norm_combine(const ma_norm_result* parts_dev, size_t count, ma_norm_result* out_dev,
                    void* stream) {
  if (!parts_dev || !out_dev) return fail(MA_ERR_NULL, "parts_dev and out_dev must not be NULL");
  if (count < 1 || count > (1u << 20)) return fail(MA_ERR_ARG, "count must be in [1, 2^20]");
  if (!aligned(parts_dev, 8) || !aligned(out_dev, 8))
    return fail(MA_ERR_ALIGN, "results must be 8-byte aligned");
  if (out_dev >= parts_dev && out_dev < parts_dev + count)
    return fail(MA_ERR_ARG, "out_dev must not be an element of parts_dev");
  hipError_t e = ma::launch_norm_combine(reinterpret_cast<const ma::NormResult*>(parts_dev),
                                         uint32_t(count), reinterpret_cast<ma::NormResult*>(out_dev),
                                         static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail_hip(e, "combine kernel launch");
  return MA_OK;
}

int ma_adamw_step(float* p32, float* m, float* v, const void* grad, ma_dtype gdt, void* p_lp,
                  ma_dtype pdt, size_t n, const ma_hyper* hyper, int64_t step, float loss_scale,
                  float clip_coef, void* stream) {
  StepRequest q;
  q.hyper = hyper;
  q.step = step;
  q.loss_scale = loss_scale;
  q.clip_coef = clip_coef;
  return flat_step(p32, m, v, grad, gdt, p_lp, pdt, MA_F32, n, q, stream);
}

int ma_adamw_step_gated(float* p32, float* m, float* v, const void* grad, ma_dtype gdt, void* p_lp,
                        ma_dtype pdt, size_t n, const ma_hyper* hyper, int64_t step,
                        float loss_scale, const ma_norm_result* gate_dev, float max_norm,
                        void* stream) {
  StepRequest q;
  q.hyper = hyper;
  q.step = step;
  q.loss_scale = loss_scale;
  q.gate = gate_dev;
  q.max_norm = max_norm;
  q.gated = true;
  return flat_step(p32, m, v, grad, gdt, p_lp, pdt, MA_F32, n, q, stream);
}

int ma_optimizer_step(float* p32, float* m, float* v, const void* grad, ma_dtype gdt, void* p_lp,
                      ma_dtype pdt, size_t n, const ma_hyper* hyper, int64_t step, float loss_scale,
                      float max_norm, ma_norm_result* out_dev, void* ws, size_t ws_bytes, void* stream) {
  StepRequest q;
  q.hyper = hyper;
  q.step = step;
  q.loss_scale = loss_scale;
  q.max_norm = max_norm;
  q.result_out = out_dev;
  q.partials = ws;
  // every argument of both launches is checked before the first one is enqueued
  if (!out_dev) return fail(MA_ERR_NULL, "out_dev is NULL");
  if (!aligned(out_dev, 8)) return fail(MA_ERR_ALIGN, "out_dev must be 8-byte aligned");
  if (int rc = check_ws(ws, ws_bytes)) return rc;
  ma::Desc d{};
  uint64_t sc = 0;
  if (int rc = flat_step_check(p32, m, v, grad, gdt, p_lp, pdt, MA_F32, n, q, d, sc)) return rc;
  if (n == 0)  // nothing to update: the plain scan writes {0, 0.0}
    return flat_norm(grad, gdt, 0, loss_scale, nullptr, false, out_dev, ws, ws_bytes, stream);
  {
    std::vector<Range> r;
    row_ranges(d, gdt, 4, 0, r);
    r.push_back(range_of(ws, ma_workspace_bytes()));
    r.push_back(range_of(out_dev, sizeof(ma_norm_result)));
    const Range *a = nullptr, *b = nullptr;
    if (any_overlap(r, &a, &b))
      return fail(MA_ERR_ARG, "buffers overlap: [%p, %p) and [%p, %p)", (void*)a->lo, (void*)a->hi, (void*)b->lo, (void*)b->hi);
  }
  if (int rc = flat_norm(grad, gdt, n, loss_scale, nullptr, false, out_dev, ws, ws_bytes, stream, &q.partial_count))
    return rc;
  return step_common(&d, nullptr, sc, MA_F32, gdt, p_lp ? int(pdt) : ma::kNoLp, q, stream);
}

int ma_multi_optimizer_step(const ma_multi_plan* plan, const ma_hyper* hyper, int64_t step, float loss_scale,
                            float max_norm, ma_norm_result* out_dev, void* ws, size_t ws_bytes,
                            void* stream) {
  StepRequest q;
  q.hyper = hyper;
  q.step = step;
  q.loss_scale = loss_scale;
  q.max_norm = max_norm;
  q.result_out = out_dev;
  q.partials = ws;
  if (int rc = check_plan(plan)) return rc;
  if (!out_dev) return fail(MA_ERR_NULL, "out_dev is NULL");
  if (!aligned(out_dev, 8)) return fail(MA_ERR_ALIGN, "out_dev must be 8-byte aligned");
  if (int rc = check_ws(ws, ws_bytes)) return rc;
  if (int rc = check_request(q)) return rc;
  if (plan->entries == 0)
    return norm_common(nullptr, plan, plan->norm_chunks, plan->gdt, loss_scale, nullptr, out_dev, ws, ws_bytes, stream);
  if (int rc = norm_common(nullptr, plan, plan->norm_chunks, plan->gdt, loss_scale, nullptr, out_dev, ws,
                           ws_bytes, stream, &q.partial_count))
    return rc;
  return step_common(nullptr, plan, plan->step_chunks, int(plan->sdt), plan->gdt, plan->pdt, q, stream);
}

int ma_adamw_step_auto(float* p32, float* m, float* v, const void* grad, ma_dtype gdt, void* p_lp,
                       ma_dtype pdt, size_t n, const ma_hyper* hyper,
                       const ma_scaler_state* scaler_dev, const ma_norm_result* gate_dev,
                       float max_norm, void* stream) {
  StepRequest q;
  q.hyper = hyper;
  q.gate = gate_dev;
  q.scaler = scaler_dev;
  q.max_norm = max_norm;
  q.automatic = true;
  return flat_step(p32, m, v, grad, gdt, p_lp, pdt, MA_F32, n, q, stream);
}

int ma_overflow_norm_auto(const void* grad, ma_dtype gdt, size_t n, const ma_scaler_state* scaler_dev,
                          ma_norm_result* out_dev, void* ws, size_t ws_bytes, void* stream) {
  return flat_norm(grad, gdt, n, 1.0f, scaler_dev, true, out_dev, ws, ws_bytes, stream);
}

int ma_adamw_step_bf16(void* p, void* m, void* v, const void* grad, ma_dtype gdt, size_t n,
                       const ma_hyper* hyper, int64_t step, float loss_scale, float clip_coef,
                       void* stream) {
  StepRequest q;
  q.hyper = hyper;
  q.step = step;
  q.loss_scale = loss_scale;
  q.clip_coef = clip_coef;
  return flat_step(p, m, v, grad, gdt, nullptr, MA_BF16, MA_BF16, n, q, stream);
}

int ma_adamw_step_bf16_gated(void* p, void* m, void* v, const void* grad, ma_dtype gdt, size_t n,
                             const ma_hyper* hyper, int64_t step, float loss_scale,
                             const ma_norm_result* gate_dev, float max_norm, void* stream) {
  StepRequest q;
  q.hyper = hyper;
  q.step = step;
  q.loss_scale = loss_scale;
  q.gate = gate_dev;
  q.max_norm = max_norm;
  q.gated = true;
  return flat_step(p, m, v, grad, gdt, nullptr, MA_BF16, MA_BF16, n, q, stream);
}

namespace {

int accumulate_common(float* acc32, const void* grad, ma_dtype gdt, size_t n, int first, bool scan,
                      float loss_scale, const ma_scaler_state* scaler_dev, ma_norm_result* out_dev,
                      void* ws, size_t ws_bytes, void* stream) {
  if (!dtype_ok(gdt)) return fail(MA_ERR_DTYPE, "unsupported gradient dtype %d", int(gdt));
  if (scan) {
    if (scaler_dev) {
      if (!aligned(scaler_dev, 8)) return fail(MA_ERR_ALIGN, "scaler_dev must be 8-byte aligned");
    } else if (int rc = check_scale(loss_scale)) {
      return rc;
    }
    if (!out_dev) return fail(MA_ERR_NULL, "out_dev is NULL");
    if (!aligned(out_dev, 8)) return fail(MA_ERR_ALIGN, "out_dev must be 8-byte aligned");
    if (int rc = check_ws(ws, ws_bytes)) return rc;
  } else if (n == 0) {
    return MA_OK;
  }
  if (n > 0 && (!acc32 || !grad)) return fail(MA_ERR_NULL, "acc32 and grad must not be NULL");
  const size_t gb = elem_bytes(gdt);
  if (!aligned(acc32, 4) || !aligned(grad, gb))
    return fail(MA_ERR_ALIGN, "acc32 / grad not aligned to their element size");
  if (n > 0) {
    std::vector<Range> r{range_of(acc32, uint64_t(n) * 4), range_of(grad, uint64_t(n) * gb)};
    const Range *a = nullptr, *b = nullptr;
    if (any_overlap(r, &a, &b)) return fail(MA_ERR_ARG, "acc32 and grad overlap");
  }
  const uint32_t h = uint32_t(((16 - (reinterpret_cast<uintptr_t>(acc32) % 16)) % 16) / 4);
  const uint32_t vec = ((reinterpret_cast<uintptr_t>(grad) + uint64_t(h) * gb) % (4 * gb)) == 0;
  int cus = 0;
  if (int rc = device_cus(&cus)) return rc;
  const double inv = (scan && !scaler_dev) ? 1.0 / (double(loss_scale) * double(loss_scale)) : 1.0;
  hipError_t e = ma::launch_accumulate(
      acc32, grad, gdt, n, vec ? h : 0, vec, first != 0, scan ? static_cast<ma::NormPartial*>(ws) : nullptr,
      inv, reinterpret_cast<const ma::ScalerState*>(scaler_dev), reinterpret_cast<ma::NormResult*>(out_dev),
      cus, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail_hip(e, "accumulate kernel launch");
  return MA_OK;
}

}  // namespace

int ma_grad_accumulate(float* acc32, const void* grad, ma_dtype gdt, size_t n, int first,
                       void* stream) {
  return accumulate_common(acc32, grad, gdt, n, first, false, 1.0f, nullptr, nullptr, nullptr, 0, stream);
}

int ma_grad_accumulate_scan(float* acc32, const void* grad, ma_dtype gdt, size_t n, int first,
                            float loss_scale, const ma_scaler_state* scaler_dev,
                            ma_norm_result* out_dev, void* ws, size_t ws_bytes, void* stream) {
  return accumulate_common(acc32, grad, gdt, n, first, true, loss_scale, scaler_dev, out_dev, ws,
                           ws_bytes, stream);
}

int ma_scaler_init(ma_scaler_state* scaler_dev, float scale, int64_t applied_steps, void* stream) {
  if (!scaler_dev) return fail(MA_ERR_NULL, "scaler_dev is NULL");
  if (!aligned(scaler_dev, 8)) return fail(MA_ERR_ALIGN, "scaler_dev must be 8-byte aligned");
  if (int rc = check_scale(scale)) return rc;
  if (applied_steps < 0) return fail(MA_ERR_ARG, "applied_steps must be >= 0");
  hipError_t e = ma::launch_scaler_init(reinterpret_cast<ma::ScalerState*>(scaler_dev), scale,
                                        applied_steps, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail_hip(e, "scaler init launch");
  return MA_OK;
}

int ma_scaler_update(ma_scaler_state* scaler_dev, const ma_norm_result* gate_dev,
                     const ma_scaler_config* cfg, void* stream) {
  if (!scaler_dev || !gate_dev || !cfg) return fail(MA_ERR_NULL, "scaler_dev, gate_dev and cfg must not be NULL");
  if (!aligned(scaler_dev, 8) || !aligned(gate_dev, 8))
    return fail(MA_ERR_ALIGN, "scaler_dev and gate_dev must be 8-byte aligned");
  if (!(cfg->backoff > 0.0f && cfg->backoff < 1.0f)) return fail(MA_ERR_ARG, "backoff must be in (0, 1)");
  if (!(cfg->growth >= 1.0f) || !std::isfinite(cfg->growth)) return fail(MA_ERR_ARG, "growth must be finite and >= 1");
  if (!(cfg->min_scale > 0.0f) || !(cfg->max_scale >= cfg->min_scale) || !std::isfinite(cfg->max_scale))
    return fail(MA_ERR_ARG, "need 0 < min_scale <= max_scale < inf");
  if (cfg->window < 1) return fail(MA_ERR_ARG, "window must be >= 1");
  ma::ScalerConfig c;
  c.backoff = cfg->backoff;
  c.growth = cfg->growth;
  c.min_scale = cfg->min_scale;
  c.max_scale = cfg->max_scale;
  c.window = cfg->window;
  hipError_t e = ma::launch_scaler_update(reinterpret_cast<ma::ScalerState*>(scaler_dev),
                                          reinterpret_cast<const ma::NormResult*>(gate_dev), c,
                                          static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail_hip(e, "scaler update launch");
  return MA_OK;
}

size_t ma_multi_table_bytes(size_t count) {
  return ma::kTableHeadBytes + (count ? count : 1) * sizeof(ma::Desc);
}

int ma_multi_prepare(const ma_tensor* list_host, size_t count, ma_dtype gdt, ma_dtype pdt,
                     void* table_dev, size_t table_bytes, void* stream, ma_multi_plan* plan_out) {
  if (!list_host) return fail(MA_ERR_NULL, "list_host is NULL");
  if (!(pdt == MA_BF16 || pdt == MA_F16))
    return fail(MA_ERR_DTYPE, "low-precision parameter dtype must be MA_BF16 or MA_F16");
  return prepare_common(count, gdt, int(pdt), MA_F32, table_dev, table_bytes, stream, plan_out,
                        [&](size_t i, ma::Desc& d) {
                          const ma_tensor& t = list_host[i];
                          d.p = t.p32;
                          d.m = t.m;
                          d.v = t.v;
                          d.g = t.grad;
                          d.lp = t.p_lp;
                          d.n = t.n;
                          return t.p_lp != nullptr;
                        });
}

int ma_multi_prepare_bf16(const ma_tensor_bf16* list_host, size_t count, ma_dtype gdt, void* table_dev,
                          size_t table_bytes, void* stream, ma_multi_plan* plan_out) {
  if (!list_host) return fail(MA_ERR_NULL, "list_host is NULL");
  return prepare_common(count, gdt, ma::kNoLp, MA_BF16, table_dev, table_bytes, stream, plan_out,
                        [&](size_t i, ma::Desc& d) {
                          const ma_tensor_bf16& t = list_host[i];
                          d.p = static_cast<float*>(t.p);
                          d.m = static_cast<float*>(t.m);
                          d.v = static_cast<float*>(t.v);
                          d.g = t.grad;
                          d.lp = nullptr;
                          d.n = t.n;
                          return false;
                        });
}

int ma_multi_overflow_norm(const ma_multi_plan* plan, float loss_scale, ma_norm_result* out_dev,
                           void* ws, size_t ws_bytes, void* stream) {
  if (int rc = check_plan(plan)) return rc;
  return norm_common(nullptr, plan, plan->norm_chunks, plan->gdt, loss_scale, nullptr, out_dev, ws,
                     ws_bytes, stream);
}

int ma_multi_overflow_norm_auto(const ma_multi_plan* plan, const ma_scaler_state* scaler_dev,
                                ma_norm_result* out_dev, void* ws, size_t ws_bytes, void* stream) {
  if (int rc = check_plan(plan)) return rc;
  if (!scaler_dev) return fail(MA_ERR_NULL, "scaler_dev is NULL");
  return norm_common(nullptr, plan, plan->norm_chunks, plan->gdt, 1.0f, scaler_dev, out_dev, ws,
                     ws_bytes, stream);
}

int ma_multi_adamw_step(const ma_multi_plan* plan, const ma_hyper* hyper, int64_t step,
                        float loss_scale, float clip_coef, void* stream) {
  StepRequest q;
  q.hyper = hyper;
  q.step = step;
  q.loss_scale = loss_scale;
  q.clip_coef = clip_coef;
  return multi_step(plan, q, stream);
}

int ma_multi_adamw_step_gated(const ma_multi_plan* plan, const ma_hyper* hyper, int64_t step,
                              float loss_scale, const ma_norm_result* gate_dev, float max_norm,
                              void* stream) {
  StepRequest q;
  q.hyper = hyper;
  q.step = step;
  q.loss_scale = loss_scale;
  q.gate = gate_dev;
  q.max_norm = max_norm;
  q.gated = true;
  return multi_step(plan, q, stream);
}

int ma_multi_adamw_step_auto(const ma_multi_plan* plan, const ma_hyper* hyper,
                             const ma_scaler_state* scaler_dev, const ma_norm_result* gate_dev,
                             float max_norm, void* stream) {
  StepRequest q;
  q.hyper = hyper;
  q.gate = gate_dev;
  q.scaler = scaler_dev;
  q.max_norm = max_norm;
  q.automatic = true;
  return multi_step(plan, q, stream);
}

}  // extern "C"
