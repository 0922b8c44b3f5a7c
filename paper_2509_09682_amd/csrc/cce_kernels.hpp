// Host-side launch entry points of the kernel families (internal to the library).
#pragma once
#include <hip/hip_runtime.h>

#include "cce_device.hpp"

namespace cce {

// One wavefront per position, rows gathered one by one; any mode, fp32 or bf16 inputs.
hipError_t launch_gather(bool backward, bool bf16, const Params &p, hipStream_t stream);

// Clears `words` 32-bit words at dst with a fill kernel (no memset node).
hipError_t launch_fill_zero(int32_t *dst, size_t words, hipStream_t stream);

}  // namespace cce
