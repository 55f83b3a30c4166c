// Measurement aids, not steps of the optimizer path: two plain streaming kernels of known traffic
// that a benchmark runs beside the real kernels.
//
//   * probe_update_mix: the update kernel's stream mix with trivial arithmetic.  Per element it reads
//     three fp32 buffers and one 16-bit buffer and writes the three fp32 buffers and another 16-bit
//     buffer: 14 bytes in, 14 bytes out, as 128-bit / 64-bit non-temporal packets, one block per CU,
//     four groups per lane, no software pipeline, no pacing, no table.  What it reaches on a given
//     placement of the buffers is what the memory system sustains for a 1:1 read/write mix there; the
//     update kernel is judged against it as well as against the nominal peak.
//   * probe_two_writes: two write-only streams.  Two streams that lie in the same 96 GiB region of
//     the HBM share a lower ceiling than two streams in different regions, which makes this kernel a
//     quick test of where an allocation's offsets lie physically.

#include "../../include/ma.h"
#include "ma_internal.h"

namespace ma {

__global__ __launch_bounds__(kBlock) void probe_update_mix_kernel(f32x4* a_, f32x4* b_, f32x4* c_,
                                                                 const u32x2* d_, u32x2* e_,
                                                                 uint64_t groups) {
  constexpr int U = 4;
  MA_GLOBAL f32x4* a = to_global(a_);
  MA_GLOBAL f32x4* b = to_global(b_);
  MA_GLOBAL f32x4* c = to_global(c_);
  MA_GLOBAL const u32x2* d = to_global(d_);
  MA_GLOBAL u32x2* e = to_global(e_);
  const uint64_t items = groups / (uint64_t(kBlock) * U);  // the ragged rest is left untouched
  for (WorkIter<2> w(items); w.c < w.end; w.c += w.stride) {
    const uint64_t g0 = w.c * (uint64_t(kBlock) * U) + threadIdx.x;
    f32x4 A[U], B[U], C[U];
    u32x2 D[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint64_t i = g0 + uint64_t(u) * kBlock;
      D[u] = ld_stream(d + i);
      A[u] = ld_stream(a + i);
      B[u] = ld_stream(b + i);
      C[u] = ld_stream(c + i);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint64_t i = g0 + uint64_t(u) * kBlock;
      const float x = bits_to_f32(D[u].x << 16);
      st_stream(a + i, A[u] + x);
      st_stream(b + i, B[u] * 0.5f + x);
      st_stream(c + i, C[u] * 0.5f + x * x);
      u32x2 L;
      L.x = (f32_to_bits(A[u].x) >> 16) | (f32_to_bits(A[u].y) & 0xFFFF0000u);
      L.y = (f32_to_bits(A[u].z) >> 16) | (f32_to_bits(A[u].w) & 0xFFFF0000u);
      st_stream(e + i, L);
    }
  }
}

// The same for states held in 16 bits: reads four 16-bit buffers, writes three (8 bytes in, 6 out per
// element), eight elements per 128-bit packet.
__global__ __launch_bounds__(kBlock) void probe_update_mix16_kernel(u32x4* a_, u32x4* b_, u32x4* c_,
                                                                   const u32x4* d_, uint64_t groups) {
  constexpr int U = 4;
  MA_GLOBAL u32x4* a = to_global(a_);
  MA_GLOBAL u32x4* b = to_global(b_);
  MA_GLOBAL u32x4* c = to_global(c_);
  MA_GLOBAL const u32x4* d = to_global(d_);
  const uint64_t items = groups / (uint64_t(kBlock) * U);
  for (WorkIter<2> w(items); w.c < w.end; w.c += w.stride) {
    const uint64_t g0 = w.c * (uint64_t(kBlock) * U) + threadIdx.x;
    u32x4 A[U], B[U], C[U], D[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint64_t i = g0 + uint64_t(u) * kBlock;
      D[u] = ld_stream(d + i);
      A[u] = ld_stream(a + i);
      B[u] = ld_stream(b + i);
      C[u] = ld_stream(c + i);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint64_t i = g0 + uint64_t(u) * kBlock;
      st_stream(a + i, A[u] + D[u]);
      st_stream(b + i, B[u] ^ D[u]);
      st_stream(c + i, C[u] + (D[u] >> 1));
    }
  }
}

__global__ __launch_bounds__(kBlock) void probe_two_writes_kernel(f32x4* x_, f32x4* y_, uint64_t packets) {
  constexpr int U = 8;
  MA_GLOBAL f32x4* x = to_global(x_);
  MA_GLOBAL f32x4* y = to_global(y_);
  const f32x4 val = {1.0f, 2.0f, 3.0f, 4.0f};
  const uint64_t items = packets / (uint64_t(kBlock) * U);
  for (uint64_t c = blockIdx.x; c < items; c += gridDim.x) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint64_t i = c * (uint64_t(kBlock) * U) + threadIdx.x + uint64_t(u) * kBlock;
      st_stream(x + i, val);
      st_stream(y + i, val);
    }
  }
}

hipError_t launch_probe_two_writes(void* x, void* y, size_t bytes_each, hipStream_t stream) {
  int dev = 0, cus = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return e;
  probe_two_writes_kernel<<<cus * 4, kBlock, 0, stream>>>(static_cast<f32x4*>(x), static_cast<f32x4*>(y), bytes_each / 16);
  return hipGetLastError();
}

}  // namespace ma

// error channel of the library (ma_api.hip)
extern "C" __attribute__((visibility("hidden"))) int ma_set_error_message(int code, const char* msg);

namespace {
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
int probe_grid(int* out) {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
    (void)hipGetLastError();
    return ma_set_error_message(MA_ERR_HIP, "cannot query the device's compute units");
  }
  *out = cus;
  return MA_OK;
}
}  // namespace

extern "C" {

int ma_probe_update_mix(void* a, void* b, void* c, const void* d16, void* e16, size_t n,
                        int state_elem_bytes, void* stream) {
  if (state_elem_bytes != 4 && state_elem_bytes != 2)
    return ma_set_error_message(MA_ERR_ARG, "state_elem_bytes must be 4 or 2");
  const bool wide = state_elem_bytes == 4;
  if (!a || !b || !c || !d16 || (wide && !e16)) return ma_set_error_message(MA_ERR_NULL, "probe buffers must not be NULL");
  if (!aligned16(a) || !aligned16(b) || !aligned16(c) || !aligned16(d16) || (wide && !aligned16(e16)))
    return ma_set_error_message(MA_ERR_ALIGN, "probe buffers must be 16-byte aligned");
  if (n < size_t(ma::kBlock) * 32) return ma_set_error_message(MA_ERR_ARG, "probe needs at least 8192 elements");
  int cus = 0;
  if (int rc = probe_grid(&cus)) return rc;
  if (wide) {
    ma::probe_update_mix_kernel<<<cus, ma::kBlock, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<ma::f32x4*>(a), static_cast<ma::f32x4*>(b), static_cast<ma::f32x4*>(c),
        static_cast<const ma::u32x2*>(d16), static_cast<ma::u32x2*>(e16), n / 4);
  } else {
    ma::probe_update_mix16_kernel<<<cus, ma::kBlock, 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<ma::u32x4*>(a), static_cast<ma::u32x4*>(b), static_cast<ma::u32x4*>(c),
        static_cast<const ma::u32x4*>(d16), n / 8);
  }
  if (hipGetLastError() != hipSuccess) return ma_set_error_message(MA_ERR_HIP, "probe launch failed");
  return MA_OK;
}

int ma_probe_two_writes(void* x, void* y, size_t bytes_each, void* stream) {
  if (!x || !y) return ma_set_error_message(MA_ERR_NULL, "probe buffers must not be NULL");
  if (!aligned16(x) || !aligned16(y)) return ma_set_error_message(MA_ERR_ALIGN, "probe buffers must be 16-byte aligned");
  if (bytes_each < size_t(ma::kBlock) * 8 * 16) return ma_set_error_message(MA_ERR_ARG, "probe needs at least 32 KiB per stream");
  int cus = 0;
  if (int rc = probe_grid(&cus)) return rc;
  ma::probe_two_writes_kernel<<<cus * 4, ma::kBlock, 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<ma::f32x4*>(x), static_cast<ma::f32x4*>(y), bytes_each / 16);
  if (hipGetLastError() != hipSuccess) return ma_set_error_message(MA_ERR_HIP, "probe launch failed");
  return MA_OK;
}

}  // extern "C"
