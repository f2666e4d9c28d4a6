#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace tg {
// dst[r * dpitch + b] = src[r * spitch + b] for r < height, b < width_bytes.  Either side may be
// page-locked host memory mapped into the GPU's address space.  Asynchronous on `stream`.
hipError_t launch_copy_2d(void* dst, size_t dpitch, const void* src, size_t spitch, size_t width_bytes,
                          size_t height, hipStream_t stream);
}  // namespace tg
