// C ABI of libma_step.so: argument checking, work-table construction, host scalars, launches.
// See include/ma.h for the contract of every entry point.

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

#include "../../include/ma.h"
#include "ma_internal.h"

static_assert(sizeof(ma_norm_result) == sizeof(ma::NormResult), "result layout");
static_assert(sizeof(ma_norm_result) == 16, "result layout");
static_assert(int(MA_F32) == ma::kF32 && int(MA_BF16) == ma::kBF16 && int(MA_F16) == ma::kF16,
              "dtype codes");

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

// Compute units of the current device (queried once per device index).
int device_cus(int* out) {
  static int cached[64] = {0};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
  if (dev >= 0 && dev < 64 && cached[dev] > 0) {
    *out = cached[dev];
    return MA_OK;
  }
  int cus = 0;
  e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return fail_hip(e, "hipDeviceGetAttribute");
  if (cus <= 0) return fail(MA_ERR_HIP, "device reports %d compute units", cus);
  if (dev >= 0 && dev < 64) cached[dev] = cus;
  *out = cus;
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
    bc1 = 1.0 - std::pow(b1, double(step));
    bc2 = 1.0 - std::pow(b2, double(step));
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

// Fills the alignment-dependent fields of a row and returns its work-item counts.
// Returns a negative status if a pointer is not aligned to its element size.
int plan_row(ma::Desc& d, int gdt, bool has_lp, uint64_t* norm_chunks, uint64_t* step_chunks) {
  const size_t gb = elem_bytes(gdt);
  if (!aligned(d.g, gb)) return fail(MA_ERR_ALIGN, "grad pointer not aligned to its element size");
  // scan: elements before the gradient's first 16-byte boundary
  const uintptr_t ga = reinterpret_cast<uintptr_t>(d.g);
  d.norm_head = uint32_t(((16 - (ga % 16)) % 16) / gb);
  const uint64_t chunk_elems = ma::kNormChunkBytes / gb;
  *norm_chunks = (d.n <= d.norm_head) ? 1 : ceil_div(d.n - d.norm_head, chunk_elems);

  if (step_chunks == nullptr) return MA_OK;  // scan-only row
  if (!aligned(d.p, 4) || !aligned(d.m, 4) || !aligned(d.v, 4))
    return fail(MA_ERR_ALIGN, "p32/m/v pointers must be 4-byte aligned");
  if (has_lp && !aligned(d.lp, 2)) return fail(MA_ERR_ALIGN, "p_lp pointer must be 2-byte aligned");
  // update: a head of h elements must bring all five buffers to a 4-element-group boundary
  const uint32_t h = uint32_t(((16 - (reinterpret_cast<uintptr_t>(d.p) % 16)) % 16) / 4);
  auto ok = [&](const void* ptr, size_t eb) {
    return ((reinterpret_cast<uintptr_t>(ptr) + uint64_t(h) * eb) % (4 * eb)) == 0;
  };
  const bool vec = ok(d.m, 4) && ok(d.v, 4) && ok(d.g, gb) && (!has_lp || ok(d.lp, 2));
  d.step_head = vec ? h : 0;
  d.step_vec = vec ? 1 : 0;
  d.pad = 0;
  if (vec) {
    *step_chunks = (d.n <= h) ? 1 : ceil_div(d.n - h, ma::kStepChunkElems);
  } else {
    *step_chunks = ceil_div(d.n, ma::kStepChunkElems);
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
  return MA_OK;
}

int step_common(const ma::Desc* row, const ma_multi_plan* plan, uint64_t chunks, int gdt, int pdt,
                const ma_hyper* hyper, int64_t step, float loss_scale, float clip_coef,
                const ma_norm_result* gate, float max_norm, void* stream) {
  int cus = 0;
  if (int rc = device_cus(&cus)) return rc;
  const ma::StepScalars s = host_scalars(*hyper, step, loss_scale, clip_coef);
  hipError_t e = ma::launch_step(
      row, plan ? static_cast<const ma::Desc*>(plan->table_dev) : nullptr,
      plan ? uint32_t(plan->entries) : 1u, chunks, gdt, pdt, s,
      reinterpret_cast<const ma::NormResult*>(gate), max_norm, loss_scale, cus,
      static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail_hip(e, "update kernel launch");
  return MA_OK;
}

int flat_step(float* p32, float* m, float* v, const void* grad, ma_dtype gdt, void* p_lp, ma_dtype pdt,
              size_t n, const ma_hyper* hyper, int64_t step, float loss_scale, float clip_coef,
              const ma_norm_result* gate, float max_norm, bool gated, void* stream) {
  if (int rc = check_hyper(hyper, step)) return rc;
  if (int rc = check_scale(loss_scale)) return rc;
  if (!dtype_ok(gdt)) return fail(MA_ERR_DTYPE, "unsupported gradient dtype %d", int(gdt));
  if (p_lp && !(pdt == MA_BF16 || pdt == MA_F16))
    return fail(MA_ERR_DTYPE, "low-precision parameter dtype must be MA_BF16 or MA_F16");
  if (gated) {
    if (!gate) return fail(MA_ERR_NULL, "gate_dev is NULL");
    if (!aligned(gate, 8)) return fail(MA_ERR_ALIGN, "gate_dev must be 8-byte aligned");
    if (std::isnan(max_norm)) return fail(MA_ERR_ARG, "max_norm is NaN");
  } else if (!(clip_coef > 0.0f && clip_coef <= 1.0f)) {
    return fail(MA_ERR_ARG, "clip_coef must be in (0, 1] (got %g)", double(clip_coef));
  }
  if (n == 0) return MA_OK;
  if (!p32 || !m || !v || !grad) return fail(MA_ERR_NULL, "p32, m, v and grad must not be NULL");
  ma::Desc d{};
  d.p = p32;
  d.m = m;
  d.v = v;
  d.g = grad;
  d.lp = p_lp;
  d.n = n;
  uint64_t nc = 0, sc = 0;
  if (int rc = plan_row(d, gdt, p_lp != nullptr, &nc, &sc)) return rc;
  return step_common(&d, nullptr, sc, gdt, p_lp ? int(pdt) : ma::kNoLp, hyper, step, loss_scale,
                     gated ? 1.0f : clip_coef, gated ? gate : nullptr, max_norm, stream);
}

}  // namespace

extern "C" {

int ma_version(void) { return 100; }

const char* ma_last_error(void) { return g_error; }

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
  if (!dtype_ok(gdt)) return fail(MA_ERR_DTYPE, "unsupported gradient dtype %d", int(gdt));
  if (int rc = check_scale(loss_scale)) return rc;
  if (!out_dev) return fail(MA_ERR_NULL, "out_dev is NULL");
  if (!aligned(out_dev, 8)) return fail(MA_ERR_ALIGN, "out_dev must be 8-byte aligned");
  if (int rc = check_ws(ws, ws_bytes)) return rc;
  if (n > 0 && !grad) return fail(MA_ERR_NULL, "grad is NULL");
  ma::Desc d{};
  d.g = grad;
  d.n = n;
  uint64_t chunks = 0;
  if (n > 0) {
    if (int rc = plan_row(d, gdt, false, &chunks, nullptr)) return rc;
  }
  int cus = 0;
  if (int rc = device_cus(&cus)) return rc;
  const double inv = 1.0 / (double(loss_scale) * double(loss_scale));
  hipError_t e = ma::launch_norm(&d, nullptr, 1, chunks, gdt, inv, static_cast<ma::NormPartial*>(ws),
                                 reinterpret_cast<ma::NormResult*>(out_dev), cus,
                                 static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail_hip(e, "scan kernel launch");
  return MA_OK;
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
  return flat_step(p32, m, v, grad, gdt, p_lp, pdt, n, hyper, step, loss_scale, clip_coef, nullptr,
                   0.0f, false, stream);
}

int ma_adamw_step_gated(float* p32, float* m, float* v, const void* grad, ma_dtype gdt, void* p_lp,
                        ma_dtype pdt, size_t n, const ma_hyper* hyper, int64_t step,
                        float loss_scale, const ma_norm_result* gate_dev, float max_norm,
                        void* stream) {
  return flat_step(p32, m, v, grad, gdt, p_lp, pdt, n, hyper, step, loss_scale, 1.0f, gate_dev,
                   max_norm, true, stream);
}

size_t ma_multi_table_bytes(size_t count) { return (count ? count : 1) * sizeof(ma::Desc); }

int ma_multi_prepare(const ma_tensor* list_host, size_t count, ma_dtype gdt, ma_dtype pdt,
                     void* table_dev, size_t table_bytes, void* stream, ma_multi_plan* plan_out) {
  if (!list_host || !plan_out) return fail(MA_ERR_NULL, "list_host and plan_out must not be NULL");
  if (count < 1 || count > (1u << 24)) return fail(MA_ERR_ARG, "count must be in [1, 2^24]");
  if (!dtype_ok(gdt)) return fail(MA_ERR_DTYPE, "unsupported gradient dtype %d", int(gdt));
  if (!(pdt == MA_BF16 || pdt == MA_F16))
    return fail(MA_ERR_DTYPE, "low-precision parameter dtype must be MA_BF16 or MA_F16");
  if (!table_dev) return fail(MA_ERR_NULL, "table_dev is NULL");
  if (!aligned(table_dev, 16)) return fail(MA_ERR_ALIGN, "table_dev must be 16-byte aligned");
  if (table_bytes < ma_multi_table_bytes(count))
    return fail(MA_ERR_ARG, "table too small: %zu < %zu bytes", table_bytes, ma_multi_table_bytes(count));

  std::vector<ma::Desc> rows;
  rows.reserve(count);
  uint64_t norm_total = 0, step_total = 0, elems = 0;
  int has_lp = -1;
  for (size_t i = 0; i < count; ++i) {
    const ma_tensor& t = list_host[i];
    if (t.n == 0) continue;
    if (!t.p32 || !t.m || !t.v || !t.grad)
      return fail(MA_ERR_NULL, "tensor %zu: p32, m, v and grad must not be NULL", i);
    const int lp = t.p_lp != nullptr;
    if (has_lp < 0) has_lp = lp;
    if (lp != has_lp)
      return fail(MA_ERR_ARG, "tensor %zu: p_lp must be set for all tensors of a list or for none", i);
    ma::Desc d{};
    d.p = t.p32;
    d.m = t.m;
    d.v = t.v;
    d.g = t.grad;
    d.lp = t.p_lp;
    d.n = t.n;
    uint64_t nc = 0, sc = 0;
    if (int rc = plan_row(d, gdt, lp != 0, &nc, &sc)) {
      char msg[400];
      std::snprintf(msg, sizeof(msg), "%s", g_error);
      return fail(rc, "tensor %zu: %s", i, msg);
    }
    d.norm_chunk0 = norm_total;
    d.step_chunk0 = step_total;
    norm_total += nc;
    step_total += sc;
    elems += t.n;
    rows.push_back(d);
  }
  if (!rows.empty()) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = hipMemcpyAsync(table_dev, rows.data(), rows.size() * sizeof(ma::Desc),
                                  hipMemcpyHostToDevice, s);
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
  plan.pdt = (has_lp == 0) ? ma::kNoLp : int(pdt);
  plan.magic = kPlanMagic;
  *plan_out = plan;
  return MA_OK;
}

int ma_multi_overflow_norm(const ma_multi_plan* plan, float loss_scale, ma_norm_result* out_dev,
                           void* ws, size_t ws_bytes, void* stream) {
  if (int rc = check_plan(plan)) return rc;
  if (int rc = check_scale(loss_scale)) return rc;
  if (!out_dev) return fail(MA_ERR_NULL, "out_dev is NULL");
  if (!aligned(out_dev, 8)) return fail(MA_ERR_ALIGN, "out_dev must be 8-byte aligned");
  if (int rc = check_ws(ws, ws_bytes)) return rc;
  int cus = 0;
  if (int rc = device_cus(&cus)) return rc;
  const double inv = 1.0 / (double(loss_scale) * double(loss_scale));
  hipError_t e = ma::launch_norm(nullptr, static_cast<const ma::Desc*>(plan->table_dev),
                                 uint32_t(plan->entries), plan->norm_chunks, plan->gdt, inv,
                                 static_cast<ma::NormPartial*>(ws),
                                 reinterpret_cast<ma::NormResult*>(out_dev), cus,
                                 static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail_hip(e, "scan kernel launch");
  return MA_OK;
}

int ma_multi_adamw_step(const ma_multi_plan* plan, const ma_hyper* hyper, int64_t step,
                        float loss_scale, float clip_coef, void* stream) {
  if (int rc = check_plan(plan)) return rc;
  if (int rc = check_hyper(hyper, step)) return rc;
  if (int rc = check_scale(loss_scale)) return rc;
  if (!(clip_coef > 0.0f && clip_coef <= 1.0f))
    return fail(MA_ERR_ARG, "clip_coef must be in (0, 1] (got %g)", double(clip_coef));
  if (plan->entries == 0) return MA_OK;
  return step_common(nullptr, plan, plan->step_chunks, plan->gdt, plan->pdt, hyper, step, loss_scale,
                     clip_coef, nullptr, 0.0f, stream);
}

int ma_multi_adamw_step_gated(const ma_multi_plan* plan, const ma_hyper* hyper, int64_t step,
                              float loss_scale, const ma_norm_result* gate_dev, float max_norm,
                              void* stream) {
  if (int rc = check_plan(plan)) return rc;
  if (int rc = check_hyper(hyper, step)) return rc;
  if (int rc = check_scale(loss_scale)) return rc;
  if (!gate_dev) return fail(MA_ERR_NULL, "gate_dev is NULL");
  if (!aligned(gate_dev, 8)) return fail(MA_ERR_ALIGN, "gate_dev must be 8-byte aligned");
  if (std::isnan(max_norm)) return fail(MA_ERR_ARG, "max_norm is NaN");
  if (plan->entries == 0) return MA_OK;
  return step_common(nullptr, plan, plan->step_chunks, plan->gdt, plan->pdt, hyper, step, loss_scale,
                     1.0f, gate_dev, max_norm, stream);
}

}  // extern "C"
