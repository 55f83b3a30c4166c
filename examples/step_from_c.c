/* One optimizer step of a flat sub-group through the C ABI, from plain C99: no Python, no C++.
 *
 *   gcc -std=c99 -D__HIP_PLATFORM_AMD__ -I include -I /opt/rocm/include examples/step_from_c.c \
 *       -L paper_2505_23254_amd -lma_step -L /opt/rocm/lib -lamdhip64 -lm -o step_from_c
 *
 * The state lies in a range built by the placement helper (ma_arena_create), the step is the
 * whole-step call (overflow / norm scan, gate, clip, AdamW, bf16 copy).  First update (t = 1,
 * m = v = 0) of p = 1, g = +-0.5: every element must end at the closed form
 *   p' = p - lr*wd*p - lr * c*g / (|c*g| + eps')     (Sec. II-A: bias correction, decoupled decay)
 * which the program evaluates in double and compares with what the device wrote. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "ma.h"

#define CHECK_HIP(x)                                                                  \
  do {                                                                                \
    hipError_t e_ = (x);                                                              \
    if (e_ != hipSuccess) {                                                           \
      fprintf(stderr, "HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); \
      return 2;                                                                       \
    }                                                                                 \
  } while (0)
#define CHECK_MA(x)                                                                   \
  do {                                                                                \
    int rc_ = (x);                                                                    \
    if (rc_ != MA_OK) {                                                               \
      fprintf(stderr, "libma_step error %d: %s (%s:%d)\n", rc_, ma_last_error(), __FILE__, __LINE__); \
      return 3;                                                                       \
    }                                                                                 \
  } while (0)

static uint16_t bf16_of(float x) { /* exact for the values used here */
  uint32_t u;
  memcpy(&u, &x, 4);
  return (uint16_t)(u >> 16);
}

int main(void) {
  const size_t n = 3u * 1000u * 1000u + 7u; /* several work items per block and a ragged tail */
  const size_t MiB = (size_t)1 << 20;
  const size_t block = 64 * MiB;
  /* p | m | v | g in the main part (4 + 4 + 4 + 2 bytes per element), the bf16 copy in the side part */
  const size_t stride = ((4 * n + 2 * MiB - 1) / (2 * MiB)) * (2 * MiB);
  const size_t main_bytes = 3 * stride + 2 * n, side_bytes = 2 * n;
  ma_arena* arena = NULL;
  CHECK_MA(ma_arena_create(main_bytes, main_bytes / 2, side_bytes, block, (size_t)2 << 30, &arena));
  ma_arena_report rep;
  CHECK_MA(ma_arena_get_report(arena, &rep));
  char* base = (char*)ma_arena_main(arena);
  float *p = (float*)base, *m = (float*)(base + stride), *v = (float*)(base + 2 * stride);
  uint16_t *g = (uint16_t*)(base + 3 * stride), *p_lp = (uint16_t*)ma_arena_side(arena);

  float* hp = (float*)malloc(4 * n);
  uint16_t* hg = (uint16_t*)malloc(2 * n);
  if (!hp || !hg) return 1;
  for (size_t i = 0; i < n; ++i) {
    hp[i] = 1.0f;
    hg[i] = bf16_of((i & 1) ? -0.5f : 0.5f);
  }
  CHECK_HIP(hipMemcpy(p, hp, 4 * n, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(g, hg, 2 * n, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemset(m, 0, 4 * n));
  CHECK_HIP(hipMemset(v, 0, 4 * n));

  void* ws = NULL;
  ma_norm_result* out = NULL;
  CHECK_HIP(hipMalloc(&ws, ma_workspace_bytes()));
  CHECK_HIP(hipMalloc((void**)&out, sizeof(ma_norm_result)));
  const ma_hyper h = {1e-3f, 0.9f, 0.999f, 1e-8f, 0.01f, 1};
  const float max_norm = 100.0f; /* the norm is 0.5 * sqrt(n) ~ 866: the step is clipped */
  CHECK_MA(ma_optimizer_step(p, m, v, g, MA_BF16, p_lp, MA_BF16, n, &h, 1, 1.0f, max_norm, out, ws,
                             ma_workspace_bytes(), NULL));
  CHECK_HIP(hipDeviceSynchronize());

  ma_norm_result res;
  uint16_t* hl = (uint16_t*)malloc(2 * n);
  if (!hl) return 1;
  CHECK_HIP(hipMemcpy(&res, out, sizeof(res), hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(hp, p, 4 * n, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(hl, p_lp, 2 * n, hipMemcpyDeviceToHost));

  const double sumsq = 0.25 * (double)n;
  const double c = (double)max_norm / (sqrt(sumsq) + 1e-6);
  /* t = 1: m' = (1-b1) cg, v' = (1-b2) (cg)^2, bias corrections 1-b1 and 1-b2 cancel them:
   * the quotient is cg / (|cg| + eps) */
  const double cg = 0.5 * (double)(float)c;
  const double up = 1.0 - (double)h.lr * (double)h.weight_decay - (double)h.lr * cg / (cg + (double)h.eps);
  const double dn = 1.0 - (double)h.lr * (double)h.weight_decay + (double)h.lr * cg / (cg + (double)h.eps);
  size_t bad = 0;
  for (size_t i = 0; i < n; ++i) {
    const double want = (i & 1) ? dn : up;
    if (fabs((double)hp[i] - want) > 4e-7 || hl[i] != 0x3F80) ++bad; /* 2-3 ulp of 1.0; the copy rounds to 1.0 */
  }
  printf("arena: %u region(s) seen, %llu blocks created; overflow %d, sumsq %.6f (exact %.6f); p' = %.9f / %.9f "
         "(closed form %.9f / %.9f); %zu of %zu elements off\n",
         rep.regions_seen, (unsigned long long)rep.blocks_created, res.overflow, res.sumsq, sumsq, hp[0], hp[1], up,
         dn, bad, n);
  const int ok = res.overflow == 0 && fabs(res.sumsq - sumsq) <= 1e-9 * sumsq && bad == 0;
  CHECK_HIP(hipFree(ws));
  CHECK_HIP(hipFree(out));
  CHECK_MA(ma_arena_destroy(arena));
  free(hp);
  free(hg);
  free(hl);
  puts(ok ? "OK" : "MISMATCH");
  return ok ? 0 : 4;
}
