// CPU oracle for the per-sub-group optimizer step of SSD-offloaded mixed-precision
// fine-tuning (MemAscend, arXiv 2505.23254).
//
// THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, scalar statement of what the step
// computes, used only to check the GPU library and to report a host baseline.  It shares
// no code, header, table or constant generator with the HIP path, and nothing in the
// product path may call it.
//
// What it follows:
//   * Overflow flag  -- Sec. III-C (the three conditions a value is examined for) and
//     Sec. IV-D / Algorithm 1: an element overflows when it is +inf, -inf or NaN.  Written
//     here as the plain definition (classify the widened value), not as the exponent-mask
//     test.
//   * Skip on overflow -- Sec. III-C: when any value overflows the update is not applied
//     and the caller lowers the scale factor.
//   * AdamW           -- Sec. II-A names the ingredients of the host optimizer (bias
//     correction, decoupled weight decay, fp32 master states paired with fp16/bf16
//     parameters); the formula is the Adam / AdamW update the paper cites.  The paper
//     prints no formula, so the operation order below is a stated reading (see
//     ora_adamw_step).
//   * Low-precision parameter copy -- Sec. III-D lists low-precision compute weights stored
//     beside the fp32 masters; the cast is round-to-nearest-even, written from the IEEE
//     definition (nearest representable value, ties to the even significand).
//   * Sum of squares / clipping -- not in the paper; global-L2-norm clipping as commonly
//     paired with this step.  sumsq = sum_i (g_i / S)^2 in fp64, index order.
//   * Gradient accumulation into the fp32 flat buffer -- Sec. III-C.
//   * bf16 optimizer states stored by truncation -- Extended Experiments.
//   * Dynamic loss scale -- Sec. III-C gives the reaction to an overflow, not a policy; the
//     policy below is a stated reading.
//
// Parity pins (tests/test_oracle_*.py): casts vs. two independent library converters and
// hand-worked ties; flag vs. the exponent-mask rule of Algorithm 1 on every 16-bit pattern;
// sumsq vs. closed forms and exact rational arithmetic; AdamW vs. the first-step closed form,
// an fp64 evaluation of the textbook formula, and a library AdamW run in fp64; accumulation vs.
// IEEE fp32 addition in a library; the bf16-state step vs. widen / fp32 step / shift; the loss
// scale vs. hand-worked sequences (tests/golden/loss_scale_sequence.txt).
//
// Build: g++ -O2 -ffp-contract=off -std=c++17 -shared -fPIC (see oracle/build.py).
// -ffp-contract=off matters: every fp32 operation below rounds once, and additions happen
// only inside explicit fmaf calls.

#include <cmath>
#include <cstddef>
#include <cstdint>
#include <cstring>
#include <thread>
#include <vector>

namespace {

enum : int { DT_F32 = 0, DT_BF16 = 1, DT_F16 = 2 };

inline uint32_t bits_of(float x) {
  uint32_t u;
  std::memcpy(&u, &x, 4);
  return u;
}
inline float float_of(uint32_t u) {
  float x;
  std::memcpy(&x, &u, 4);
  return x;
}

// ---------------------------------------------------------------------------------------
// Widening.  bf16 is by definition the upper half of the fp32 encoding.  fp16 is decoded
// arithmetically from its sign / exponent / fraction fields (IEEE 754 binary16).
// ---------------------------------------------------------------------------------------
inline float widen_bf16(uint16_t h) { return float_of(static_cast<uint32_t>(h) << 16); }

inline float widen_f16(uint16_t h) {
  const int sign = h >> 15;
  const int e = (h >> 10) & 0x1F;
  const int f = h & 0x3FF;
  float mag;
  if (e == 0) {
    mag = std::ldexp(static_cast<float>(f), -24);  // zero and subnormals: f * 2^-24
  } else if (e == 31) {
    if (f == 0) {
      mag = INFINITY;
    } else {
      // NaN: keep the payload in the top fraction bits so the class survives widening.
      return float_of((static_cast<uint32_t>(sign) << 31) | 0x7F800000u |
                      (static_cast<uint32_t>(f) << 13));
    }
  } else {
    mag = std::ldexp(static_cast<float>(1024 + f), e - 25);  // (1 + f/1024) * 2^(e-15)
  }
  return sign ? -mag : mag;
}

inline float widen(const void* g, int dt, size_t i) {
  switch (dt) {
    case DT_BF16: return widen_bf16(static_cast<const uint16_t*>(g)[i]);
    case DT_F16: return widen_f16(static_cast<const uint16_t*>(g)[i]);
    default: return static_cast<const float*>(g)[i];
  }
}

// ---------------------------------------------------------------------------------------
// Round-to-nearest-even narrowing from the definition: pick the representable value of the
// target format nearest to x; on a tie pick the one with an even significand; values that
// round to 2^(emax+1) or beyond become infinity.
//   P    = significand bits including the hidden one (bf16: 8, fp16: 11)
//   EMIN = exponent of the smallest normal (bf16: -126, fp16: -14)
//   EMAX = exponent of the largest finite binade (bf16: 127, fp16: 15)
//   EB   = exponent field width (bf16: 8, fp16: 5)
// NaN maps to a quiet NaN that keeps the sign and the top payload bits.
// ---------------------------------------------------------------------------------------
template <int P, int EMIN, int EMAX, int EB>
inline uint16_t round_nearest_even(float x) {
  constexpr int FB = P - 1;  // stored fraction bits
  constexpr int BIAS = EMAX;
  const uint32_t xb = bits_of(x);
  const uint16_t sign = static_cast<uint16_t>((xb >> 31) << (EB + FB));
  const uint16_t exp_all_ones = static_cast<uint16_t>(((1u << EB) - 1u) << FB);
  if (std::isnan(x)) {
    const uint32_t payload = (xb & 0x007FFFFFu) >> (23 - FB);
    return static_cast<uint16_t>(sign | exp_all_ones | (1u << (FB - 1)) | payload);
  }
  if (std::isinf(x)) return static_cast<uint16_t>(sign | exp_all_ones);
  const double a = std::fabs(static_cast<double>(x));
  if (a == 0.0) return sign;

  int e2;
  std::frexp(a, &e2);     // a = f * 2^e2, f in [0.5, 1)  =>  leading bit has weight 2^(e2-1)
  int E = e2 - 1;
  if (E < EMIN) E = EMIN;  // below the smallest normal the spacing stays that of EMIN
  const double quantum = std::ldexp(1.0, E - FB);
  const double t = a / quantum;  // exact: division by a power of two
  double r = std::floor(t);
  const double frac = t - r;     // exact: t has at most 24 significant bits
  if (frac > 0.5) {
    r += 1.0;
  } else if (frac == 0.5) {
    if (std::fmod(r, 2.0) != 0.0) r += 1.0;  // tie: go to the even neighbour
  }
  const double val = r * quantum;  // the rounded magnitude, exact
  if (val >= std::ldexp(1.0, EMAX + 1)) return static_cast<uint16_t>(sign | exp_all_ones);
  if (val < std::ldexp(1.0, EMIN)) {
    // zero or subnormal result: exponent field 0, fraction = r (quantum is 2^(EMIN-FB))
    return static_cast<uint16_t>(sign | static_cast<uint16_t>(r));
  }
  int e3;
  std::frexp(val, &e3);
  const int E2 = e3 - 1;  // may be E+1 if rounding carried into the next binade
  const double sig = val / std::ldexp(1.0, E2 - FB);  // in [2^FB, 2^(FB+1))
  const uint32_t frac_field = static_cast<uint32_t>(sig) - (1u << FB);
  const uint32_t exp_field = static_cast<uint32_t>(E2 + BIAS);
  return static_cast<uint16_t>(sign | (exp_field << FB) | frac_field);
}

inline uint16_t round_bf16(float x) { return round_nearest_even<8, -126, 127, 8>(x); }
inline uint16_t round_f16(float x) { return round_nearest_even<11, -14, 15, 5>(x); }

inline void store_lp(void* out, int dt, size_t i, float x) {
  if (out == nullptr) return;
  switch (dt) {
    case DT_BF16: static_cast<uint16_t*>(out)[i] = round_bf16(x); break;
    case DT_F16: static_cast<uint16_t*>(out)[i] = round_f16(x); break;
    default: static_cast<float*>(out)[i] = x; break;
  }
}

// ---------------------------------------------------------------------------------------
// Host scalars of one AdamW step, each evaluated in fp64 from the fp32 hyper-parameters and
// rounded to fp32 exactly once.
// ---------------------------------------------------------------------------------------
struct Hyper {
  float lr, beta1, beta2, eps, weight_decay;
  int32_t bias_correction;
};

struct StepScalars {
  float beta1, beta2, omb1, omb2, eps, step_size, inv_sqrt_bc2, decay, gscale;
};

inline StepScalars make_scalars(const Hyper& h, int64_t step, float loss_scale, float clip_coef) {
  StepScalars s;
  const double b1 = h.beta1, b2 = h.beta2, lr = h.lr, wd = h.weight_decay;
  double bc1 = 1.0, bc2 = 1.0;
  if (h.bias_correction) {
    bc1 = 1.0 - std::pow(b1, static_cast<double>(step));
    bc2 = 1.0 - std::pow(b2, static_cast<double>(step));
  }
  s.beta1 = h.beta1;
  s.beta2 = h.beta2;
  s.omb1 = static_cast<float>(1.0 - b1);
  s.omb2 = static_cast<float>(1.0 - b2);
  s.eps = h.eps;
  s.step_size = static_cast<float>(lr / bc1);
  s.inv_sqrt_bc2 = static_cast<float>(1.0 / std::sqrt(bc2));
  s.decay = static_cast<float>(lr * wd);
  s.gscale = static_cast<float>(static_cast<double>(clip_coef) / static_cast<double>(loss_scale));
  return s;
}

// One element of the step in fp32.  Reading of the silent points (Sec. II-A says only that the
// host optimizer applies bias correction and a decoupled weight decay):
//   g   = widen(grad) * (clip / S)                       unscale and clip in one multiply
//   m'  = beta1 * m + (1 - beta1) * g
//   v'  = beta2 * v + (1 - beta2) * g^2
//   d   = sqrt(v') / sqrt(1 - beta2^t) + eps             eps added after the bias correction
//   p'  = (p - lr*wd*p) - (lr / (1 - beta1^t)) * m' / d  decay acts on the old p, scaled by lr
// Every product, quotient and square root rounds to fp32 on its own; each addition is the
// final step of an fmaf.
inline void adamw_element(const StepScalars& s, float g_raw, float& p, float& m, float& v) {
  const float g = g_raw * s.gscale;
  const float m1 = std::fmaf(s.beta1, m, s.omb1 * g);
  const float v1 = std::fmaf(s.beta2, v, s.omb2 * (g * g));
  const float d = std::fmaf(std::sqrt(v1), s.inv_sqrt_bc2, s.eps);
  const float u = m1 / d;
  const float q = std::fmaf(-s.decay, p, p);
  const float p1 = std::fmaf(-s.step_size, u, q);
  p = p1;
  m = m1;
  v = v1;
}

void adamw_range(float* p, float* m, float* v, const void* g, int gdt, void* p_lp, int pdt,
                 size_t lo, size_t hi, const StepScalars& s) {
  for (size_t i = lo; i < hi; ++i) {
    adamw_element(s, widen(g, gdt, i), p[i], m[i], v[i]);
    store_lp(p_lp, pdt, i, p[i]);
  }
}

void norm_range(const void* g, int gdt, size_t lo, size_t hi, double scale, int* overflow,
                double* sumsq) {
  int ov = 0;
  double acc = 0.0;
  for (size_t i = lo; i < hi; ++i) {
    const float x = widen(g, gdt, i);
    if (std::isinf(x) || std::isnan(x)) ov = 1;
    const double y = static_cast<double>(x) / scale;
    acc += y * y;
  }
  *overflow = ov;
  *sumsq = acc;
}

// Run fn(lo, hi, k) over nthreads disjoint contiguous ranges of [0, n).
template <class F>
void over_ranges(size_t n, int nthreads, F fn) {
  if (nthreads < 1) nthreads = 1;
  std::vector<std::thread> pool;
  const size_t per = (n + static_cast<size_t>(nthreads) - 1) / static_cast<size_t>(nthreads);
  for (int k = 0; k < nthreads; ++k) {
    const size_t lo = std::min(n, per * static_cast<size_t>(k));
    const size_t hi = std::min(n, lo + per);
    pool.emplace_back(fn, lo, hi, k);
  }
  for (auto& t : pool) t.join();
}

}  // namespace

extern "C" {

// ---- element-wise converters (array forms, for the pins) --------------------------------
void ora_widen_bf16(const uint16_t* in, float* out, size_t n) {
  for (size_t i = 0; i < n; ++i) out[i] = widen_bf16(in[i]);
}
void ora_widen_f16(const uint16_t* in, float* out, size_t n) {
  for (size_t i = 0; i < n; ++i) out[i] = widen_f16(in[i]);
}
void ora_round_bf16(const float* in, uint16_t* out, size_t n) {
  for (size_t i = 0; i < n; ++i) out[i] = round_bf16(in[i]);
}
void ora_round_f16(const float* in, uint16_t* out, size_t n) {
  for (size_t i = 0; i < n; ++i) out[i] = round_f16(in[i]);
}

// ---- overflow flag and sum of squares -----------------------------------------------------
// overflow = 1 iff some element is +inf, -inf or NaN (Sec. III-C).  sumsq = sum (g_i/S)^2 in
// fp64, accumulated in index order.  With nthreads > 1 the same loop runs over contiguous
// ranges and the partial sums are added in range order.
void ora_overflow_norm(const void* grad, int gdt, size_t n, float loss_scale, int nthreads,
                       int32_t* overflow, double* sumsq) {
  const double S = static_cast<double>(loss_scale);
  if (nthreads <= 1) {
    int ov;
    double ss;
    norm_range(grad, gdt, 0, n, S, &ov, &ss);
    *overflow = ov;
    *sumsq = ss;
    return;
  }
  std::vector<int> ovs(nthreads, 0);
  std::vector<double> sums(nthreads, 0.0);
  over_ranges(n, nthreads, [&](size_t lo, size_t hi, int k) {
    norm_range(grad, gdt, lo, hi, S, &ovs[k], &sums[k]);
  });
  int ov = 0;
  double ss = 0.0;
  for (int k = 0; k < nthreads; ++k) {
    ov |= ovs[k];
    ss += sums[k];
  }
  *overflow = ov;
  *sumsq = ss;
}

// ---- clip coefficient ---------------------------------------------------------------------
// Global-norm clipping: c = min(1, max_norm / (sqrt(sumsq) + 1e-6)), evaluated in fp64 and
// rounded once to fp32.  max_norm <= 0 disables clipping.
float ora_clip_coef(double sumsq, double max_norm) {
  if (!(max_norm > 0.0)) return 1.0f;
  const double c = max_norm / (std::sqrt(sumsq) + 1e-6);
  return static_cast<float>(c < 1.0 ? c : 1.0);
}

// ---- AdamW step, fp32 states ----------------------------------------------------------------
// p, m, v updated in place; p_lp (may be null) receives the rounded low-precision copy of the
// new p.  hyper = {lr, beta1, beta2, eps, weight_decay, bias_correction}.
void ora_adamw_step(float* p, float* m, float* v, const void* grad, int gdt, void* p_lp, int pdt,
                    size_t n, const void* hyper, int64_t step, float loss_scale, float clip_coef,
                    int nthreads) {
  Hyper h;
  std::memcpy(&h, hyper, sizeof(Hyper));
  const StepScalars s = make_scalars(h, step, loss_scale, clip_coef);
  if (nthreads <= 1) {
    adamw_range(p, m, v, grad, gdt, p_lp, pdt, 0, n, s);
  } else {
    over_ranges(n, nthreads, [&](size_t lo, size_t hi, int) {
      adamw_range(p, m, v, grad, gdt, p_lp, pdt, lo, hi, s);
    });
  }
}

// The nine fp32 scalars a step uses, in the order
// {beta1, beta2, 1-beta1, 1-beta2, eps, lr/bc1, 1/sqrt(bc2), lr*wd, clip/S}.
void ora_step_scalars(const void* hyper, int64_t step, float loss_scale, float clip_coef,
                      float* out9) {
  Hyper h;
  std::memcpy(&h, hyper, sizeof(Hyper));
  const StepScalars s = make_scalars(h, step, loss_scale, clip_coef);
  const float a[9] = {s.beta1, s.beta2, s.omb1, s.omb2, s.eps,
                      s.step_size, s.inv_sqrt_bc2, s.decay, s.gscale};
  std::memcpy(out9, a, sizeof(a));
}

// ---- the same step evaluated in fp64 from the textbook formula ------------------------------
// Inputs are the fp32 states and the raw gradient; outputs are doubles.  No operation order is
// pinned here: this is the real-number update evaluated in double, used to bound the rounding
// error of the fp32 version above.
void ora_adamw_step_f64(const float* p, const float* m, const float* v, const void* grad, int gdt,
                        size_t n, const void* hyper, int64_t step, float loss_scale,
                        float clip_coef, double* p_out, double* m_out, double* v_out) {
  Hyper h;
  std::memcpy(&h, hyper, sizeof(Hyper));
  const double b1 = h.beta1, b2 = h.beta2, lr = h.lr, wd = h.weight_decay, eps = h.eps;
  double bc1 = 1.0, bc2 = 1.0;
  if (h.bias_correction) {
    bc1 = 1.0 - std::pow(b1, static_cast<double>(step));
    bc2 = 1.0 - std::pow(b2, static_cast<double>(step));
  }
  const double gs = static_cast<double>(clip_coef) / static_cast<double>(loss_scale);
  for (size_t i = 0; i < n; ++i) {
    const double g = static_cast<double>(widen(grad, gdt, i)) * gs;
    const double m1 = b1 * m[i] + (1.0 - b1) * g;
    const double v1 = b2 * v[i] + (1.0 - b2) * g * g;
    const double mhat = m1 / bc1;
    const double vhat = v1 / bc2;
    const double pi = p[i];
    p_out[i] = pi - lr * (mhat / (std::sqrt(vhat) + eps) + wd * pi);
    m_out[i] = m1;
    v_out[i] = v1;
  }
}

// ---- the whole path: scan, gate, update ------------------------------------------------------
// Scans the gradient; on overflow leaves p, m, v and p_lp untouched (Sec. III-C: the step is
// skipped and the caller reduces the scale).  Otherwise clips by the global norm (max_norm <= 0:
// no clipping) and applies the AdamW step.  Returns the overflow flag.
int32_t ora_optimizer_step(float* p, float* m, float* v, const void* grad, int gdt, void* p_lp,
                           int pdt, size_t n, const void* hyper, int64_t step, float loss_scale,
                           float max_norm, int nthreads, double* sumsq_out, float* clip_out) {
  int32_t ov;
  double ss;
  ora_overflow_norm(grad, gdt, n, loss_scale, nthreads, &ov, &ss);
  if (sumsq_out) *sumsq_out = ss;
  if (ov) {
    if (clip_out) *clip_out = 0.0f;
    return 1;
  }
  const float c = ora_clip_coef(ss, static_cast<double>(max_norm));
  if (clip_out) *clip_out = c;
  ora_adamw_step(p, m, v, grad, gdt, p_lp, pdt, n, hyper, step, loss_scale, c, nthreads);
  return 0;
}

// ---- gradient accumulation into the fp32 flat buffer ------------------------------------------
// Sec. III-C: the partition's flat gradient buffer is kept in fp32 so that low-precision
// micro-batch gradients can be accumulated into it.  One fp32 addition per element; the first
// micro-batch of an iteration overwrites (first != 0), later ones add.
void ora_grad_accumulate(float* acc, const void* grad, int gdt, size_t n, int first) {
  for (size_t i = 0; i < n; ++i) {
    const float g = widen(grad, gdt, i);
    acc[i] = first ? g : acc[i] + g;
  }
}

// ---- half-precision optimizer states -----------------------------------------------------------
// Extended Experiments (bf16 half-precision optimizer): parameters, gradients and both moments
// are held in bf16; the only conversion back from fp32 is a direct truncation (the low 16 bits
// are dropped).  The arithmetic between widening and truncation is the fp32 step above.
// Reading of a silent point: a NaN whose payload lies only in the dropped bits would truncate to
// infinity; it is kept a NaN by setting the quiet bit.
uint16_t ora_truncate_bf16_one(float x) {
  const uint32_t b = bits_of(x);
  uint16_t h = static_cast<uint16_t>(b >> 16);
  if (std::isnan(x)) h |= 0x0040;
  return h;
}

void ora_truncate_bf16(const float* in, uint16_t* out, size_t n) {
  for (size_t i = 0; i < n; ++i) out[i] = ora_truncate_bf16_one(in[i]);
}

void ora_adamw_step_bf16(uint16_t* p, uint16_t* m, uint16_t* v, const void* grad, int gdt, size_t n,
                         const void* hyper, int64_t step, float loss_scale, float clip_coef,
                         int nthreads) {
  Hyper h;
  std::memcpy(&h, hyper, sizeof(Hyper));
  const StepScalars s = make_scalars(h, step, loss_scale, clip_coef);
  auto range = [&](size_t lo, size_t hi, int) {
    for (size_t i = lo; i < hi; ++i) {
      float pf = widen_bf16(p[i]), mf = widen_bf16(m[i]), vf = widen_bf16(v[i]);
      adamw_element(s, widen(grad, gdt, i), pf, mf, vf);
      p[i] = ora_truncate_bf16_one(pf);
      m[i] = ora_truncate_bf16_one(mf);
      v[i] = ora_truncate_bf16_one(vf);
    }
  };
  if (nthreads <= 1) {
    range(0, n, 0);
  } else {
    over_ranges(n, nthreads, range);
  }
}

// ---- dynamic loss scale --------------------------------------------------------------------------
// Sec. III-C: when any value overflows, the scale factor is reduced (and the step is skipped).
// The paper gives no policy; the reading is the usual dynamic scaling: on overflow multiply the
// scale by `backoff` (not below min_scale) and restart the count of clean steps; after `window`
// clean steps in a row multiply it by `growth` (not above max_scale).  `step` counts applied
// updates; a skipped iteration does not advance it.
struct ScalerCfg {
  float backoff, growth, min_scale, max_scale;
  int32_t window;
};
struct ScalerState {
  float scale;
  int32_t good_steps;
  int64_t step;
  int64_t skipped;
};

void ora_scaler_update(void* state, const void* cfg_, int32_t overflow) {
  ScalerState st;
  ScalerCfg cfg;
  std::memcpy(&st, state, sizeof(st));
  std::memcpy(&cfg, cfg_, sizeof(cfg));
  if (overflow) {
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
  std::memcpy(state, &st, sizeof(st));
}

// One whole iteration driven by the scaler state: scan at the current scale; on overflow skip and
// back off; otherwise clip, apply update number step+1, and count the clean step.
int32_t ora_optimizer_step_auto(float* p, float* m, float* v, const void* grad, int gdt, void* p_lp,
                                int pdt, size_t n, const void* hyper, void* state, const void* cfg,
                                float max_norm, int nthreads, double* sumsq_out) {
  ScalerState st;
  std::memcpy(&st, state, sizeof(st));
  const int32_t ov = ora_optimizer_step(p, m, v, grad, gdt, p_lp, pdt, n, hyper, st.step + 1, st.scale,
                                        max_norm, nthreads, sumsq_out, nullptr);
  ora_scaler_update(state, cfg, ov);
  return ov;
}

}  // extern "C"
