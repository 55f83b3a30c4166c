// Drives every entry point of the CPU oracle over ragged sizes with exactly-sized heap buffers,
// for a build with -fsanitize=address,undefined (see tests/test_oracle_sanitized.py).  Checks no
// values: an out-of-bounds access, a misaligned access or undefined arithmetic aborts the run.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

extern "C" {
void ora_widen_bf16(const uint16_t*, float*, size_t);
void ora_widen_f16(const uint16_t*, float*, size_t);
void ora_round_bf16(const float*, uint16_t*, size_t);
void ora_round_f16(const float*, uint16_t*, size_t);
void ora_truncate_bf16(const float*, uint16_t*, size_t);
void ora_overflow_norm(const void*, int, size_t, float, int, int32_t*, double*);
void ora_adamw_step(float*, float*, float*, const void*, int, void*, int, size_t, const void*, int64_t,
                    float, float, int);
void ora_adamw_step_f64(const float*, const float*, const float*, const void*, int, size_t, const void*,
                        int64_t, float, float, double*, double*, double*);
int32_t ora_optimizer_step(float*, float*, float*, const void*, int, void*, int, size_t, const void*,
                           int64_t, float, float, int, double*, float*);
void ora_grad_accumulate(float*, const void*, int, size_t, int);
void ora_adamw_step_bf16(uint16_t*, uint16_t*, uint16_t*, const void*, int, size_t, const void*, int64_t,
                         float, float, int);
void ora_scaler_update(void*, const void*, int32_t);
int32_t ora_optimizer_step_auto(float*, float*, float*, const void*, int, void*, int, size_t, const void*,
                                void*, const void*, float, int, double*);
}

struct Hyper { float lr, b1, b2, eps, wd; int32_t bc; };
struct ScalerCfg { float backoff, growth, min_scale, max_scale; int32_t window; };
struct ScalerState { float scale; int32_t good; int64_t step, skipped; };

static uint32_t rng_state = 12345u;
static uint32_t rnd() { rng_state = rng_state * 1664525u + 1013904223u; return rng_state; }

int main() {
  const Hyper h{1e-3f, 0.9f, 0.999f, 1e-8f, 0.01f, 1};
  const ScalerCfg sc{0.5f, 2.0f, 1.0f, 16777216.0f, 2};
  const size_t sizes[] = {0, 1, 2, 3, 5, 17, 255, 256, 1001, 4099};
  for (size_t n : sizes) {
    for (int gdt = 0; gdt < 3; ++gdt) {
      const size_t gb = gdt == 0 ? 4 : 2;
      std::vector<float> p(n), m(n), v(n), acc(n);
      std::vector<unsigned char> g(n * gb);
      std::vector<uint16_t> lp(n), hp(n), hm(n), hv(n);
      std::vector<double> po(n), mo(n), vo(n);
      for (size_t i = 0; i < n; ++i) {
        // every bit pattern class, inf and NaN included
        uint32_t pb = rnd(), gbits = rnd();
        std::memcpy(&p[i], &pb, 4);
        m[i] = 1e-4f * float(int(rnd() % 2001) - 1000);
        v[i] = 1e-9f * float(rnd() % 1000);
        std::memcpy(&g[i * gb], &gbits, gb);
        hp[i] = uint16_t(rnd()); hm[i] = uint16_t(rnd()); hv[i] = uint16_t(rnd() & 0x7FFF);
      }
      for (int threads : {1, 3}) {
        int32_t ov = 0; double ss = 0; float c = 0;
        ora_overflow_norm(g.data(), gdt, n, 64.0f, threads, &ov, &ss);
        for (int pdt = 1; pdt < 3; ++pdt) {
          ora_adamw_step(p.data(), m.data(), v.data(), g.data(), gdt, lp.data(), pdt, n, &h, 3, 64.0f, 0.5f, threads);
          ora_optimizer_step(p.data(), m.data(), v.data(), g.data(), gdt, lp.data(), pdt, n, &h, 4, 64.0f, 1.0f, threads, &ss, &c);
          ScalerState st{64.0f, 0, 10, 0};
          ora_optimizer_step_auto(p.data(), m.data(), v.data(), g.data(), gdt, lp.data(), pdt, n, &h, &st, &sc, 1.0f, threads, &ss);
        }
        ora_adamw_step(p.data(), m.data(), v.data(), g.data(), gdt, nullptr, 1, n, &h, 5, 1.0f, 1.0f, threads);
        ora_adamw_step_bf16(hp.data(), hm.data(), hv.data(), g.data(), gdt, n, &h, 2, 1.0f, 0.25f, threads);
      }
      ora_adamw_step_f64(p.data(), m.data(), v.data(), g.data(), gdt, n, &h, 7, 2.0f, 1.0f, po.data(), mo.data(), vo.data());
      ora_grad_accumulate(acc.data(), g.data(), gdt, n, 1);
      ora_grad_accumulate(acc.data(), g.data(), gdt, n, 0);
      ora_round_bf16(p.data(), lp.data(), n);
      ora_round_f16(p.data(), lp.data(), n);
      ora_truncate_bf16(p.data(), lp.data(), n);
      ora_widen_bf16(hp.data(), acc.data(), n);
      ora_widen_f16(hp.data(), acc.data(), n);
    }
  }
  ScalerState st{2.0f, 0, 0, 0};
  for (int k = 0; k < 50; ++k) ora_scaler_update(&st, &sc, k % 7 == 3);
  std::puts("sanitized oracle run ok");
  return 0;
}
