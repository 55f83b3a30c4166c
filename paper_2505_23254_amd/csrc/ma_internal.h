// Declarations shared by the translation units of libma_step.so (not installed).
#pragma once

#include <type_traits>

#include "ma_device.h"

#ifndef MA_NORM_BLOCKS_PER_CU
#define MA_NORM_BLOCKS_PER_CU 4  // persistent blocks per compute unit, scan kernel
#endif
#ifndef MA_STEP_BLOCKS_PER_CU
#define MA_STEP_BLOCKS_PER_CU 1  // persistent blocks per compute unit, update kernel
#endif

namespace ma {

// Upper bound of the scan kernel's grid; fixes the workspace size independently of the device.
constexpr uint32_t kMaxNormBlocks = 8192;

// Exactly one of row_host (flat sub-group, row passed by value) and table_dev (tensor list) is
// non-null.  `chunks` is the number of work items over all rows.
hipError_t launch_norm(const Desc* row_host, const Desc* table_dev, uint32_t rows, uint64_t chunks,
                       int gdt, double inv_scale_sq, NormPartial* partials, NormResult* out,
                       int device_cus, hipStream_t stream);

hipError_t launch_norm_combine(const NormResult* parts, uint32_t count, NormResult* out,
                               hipStream_t stream);

// gate == nullptr: s.gscale is final.  Otherwise the kernel reads the gate on the device.
hipError_t launch_step(const Desc* row_host, const Desc* table_dev, uint32_t rows, uint64_t chunks,
                       int gdt, int pdt, const StepScalars& s, const NormResult* gate, float max_norm,
                       float loss_scale, int device_cus, hipStream_t stream);

}  // namespace ma
