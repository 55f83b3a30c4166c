// Declarations shared by the translation units of libma_step.so (not installed).
#pragma once

#include <type_traits>

#include "ma_device.h"

#ifndef MA_NORM_BLOCKS_PER_CU
#define MA_NORM_BLOCKS_PER_CU 2  // persistent blocks per compute unit, scan kernel (8.03e9 elements: 2.37 ms with 4, 2.33 with 3, 2.27 with 2)
#endif
#ifndef MA_STEP_BLOCKS_PER_CU
#define MA_STEP_BLOCKS_PER_CU 1  // persistent blocks per compute unit, update kernel
#endif
#ifndef MA_STEP_BLOCKS_PER_CU_BF16
#define MA_STEP_BLOCKS_PER_CU_BF16 1  // the same for states held in bf16
#endif

namespace ma {

// Upper bound of the scan kernel's grid; fixes the workspace size independently of the device.
constexpr uint32_t kMaxNormBlocks = 8192;

// Exactly one of row_host (flat sub-group, row passed by value) and table_dev (tensor list) is
// non-null.  `chunks` is the number of work items over all rows.  With a scaler state the
// finalize kernel takes the loss scale from device memory instead of inv_scale_sq.
// grid_out != null: no finalize launch; *grid_out receives the number of partials written, for a
// following launch that adds them up itself (StepControl::partials).
hipError_t launch_norm(const Desc* row_host, const Desc* table_dev, uint32_t rows, uint64_t chunks,
                       int gdt, double inv_scale_sq, const ScalerState* scaler, NormPartial* partials,
                       NormResult* out, int device_cus, hipStream_t stream, uint32_t* grid_out = nullptr);

// Sign-stripped bit pattern of infinity in the gradient format (the scan's overflow threshold).
uint32_t norm_threshold(int gdt);

// Second level of the scan: one block adds `count` per-block partials in index order.
hipError_t launch_norm_finalize(const NormPartial* partials, uint32_t count, int gdt, double inv_scale_sq,
                                const ScalerState* scaler, NormResult* out, hipStream_t stream);

hipError_t launch_norm_combine(const NormResult* parts, uint32_t count, NormResult* out,
                               hipStream_t stream);

// sdt: dtype of p, m, v (kF32, or kBF16 for states stored by truncation).  queue: the counters at
// the head of a tensor list's table (null for a flat sub-group, which has no such memory).
hipError_t launch_step(const Desc* row_host, const Desc* table_dev, uint32_t rows, uint64_t chunks,
                       int sdt, int gdt, int pdt, const StepScalars& s, const StepControl& ctl,
                       StepQueue* queue, int device_cus, hipStream_t stream);

// Two write-only streams of bytes_each bytes (the measurement aid behind ma_probe_two_writes).
hipError_t launch_probe_two_writes(void* x, void* y, size_t bytes_each, hipStream_t stream);

// A tensor list's device table: the counters, then one row per non-empty tensor.
constexpr size_t kTableHeadBytes = sizeof(StepQueue);

hipError_t launch_scaler_init(ScalerState* state, float scale, int64_t step, hipStream_t stream);
hipError_t launch_scaler_update(ScalerState* state, const NormResult* gate, const ScalerConfig& cfg,
                                hipStream_t stream);

// acc (fp32) = first ? widen(g) : acc + widen(g) over n elements; head / vec as planned by the host.
// With partials != null the same pass also scans the NEW contents of acc (flag and sum of squares
// of fp32 values) and `out` receives the result.
hipError_t launch_accumulate(float* acc, const void* g, int gdt, uint64_t n, uint32_t head,
                             uint32_t vec, int first, NormPartial* partials, double inv_scale_sq,
                             const ScalerState* scaler, NormResult* out, int device_cus,
                             hipStream_t stream);

}  // namespace ma
