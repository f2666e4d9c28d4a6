// Strided tile copy kernel: moves one tile between a row-major matrix in pinned host memory and
// a contiguous slot in HBM (Algorithm 1 of the paper: "Get A[i,k] from host RAM", "harvest
// C[i,j]").  The GPU reads (or writes) the page-locked host memory directly over the host link,
// so a tile transfer is an ordinary kernel launch: fully asynchronous on its stream and free to
// overlap with tile products running on the other streams.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "copy_kernel.h"

namespace tg {

template <typename V>
__global__ __launch_bounds__(256) void copy_tile_2d(const char* __restrict__ src, size_t spitch,
                                                    char* __restrict__ dst, size_t dpitch,
                                                    int64_t units_per_row, int64_t rows)
{
    const int64_t total = units_per_row * rows;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    // four independent loads in flight per thread before the first store: the host link has
    // microseconds of latency
    for (; i + 3 * stride < total; i += 4 * stride) {
        V v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t j = i + u * stride;
            const int64_t r = j / units_per_row, c = j - r * units_per_row;
            v[u] = *reinterpret_cast<const V*>(src + r * spitch + c * sizeof(V));
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t j = i + u * stride;
            const int64_t r = j / units_per_row, c = j - r * units_per_row;
            *reinterpret_cast<V*>(dst + r * dpitch + c * sizeof(V)) = v[u];
        }
    }
    for (; i < total; i += stride) {
        const int64_t r = i / units_per_row, c = i - r * units_per_row;
        *reinterpret_cast<V*>(dst + r * dpitch + c * sizeof(V)) =
            *reinterpret_cast<const V*>(src + r * spitch + c * sizeof(V));
    }
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

hipError_t launch_copy_2d(void* dst, size_t dpitch, const void* src, size_t spitch, size_t width_bytes,
                          size_t height, hipStream_t stream)
{
    if (width_bytes == 0 || height == 0) return hipSuccess;
    const uintptr_t mix = (uintptr_t)dst | (uintptr_t)src | dpitch | spitch | width_bytes;
    static const int blocks = [] {
        const char* e = getenv("TGEMM_COPY_BLOCKS");
        const int v = e ? atoi(e) : 0;
        return (v >= 1 && v <= 4096) ? v : 128;
    }();
    if ((mix & 15) == 0) {
        hipLaunchKernelGGL(copy_tile_2d<u32x4>, dim3(blocks), dim3(256), 0, stream, (const char*)src, spitch,
                           (char*)dst, dpitch, (int64_t)(width_bytes / 16), (int64_t)height);
    } else if ((mix & 3) == 0) {
        hipLaunchKernelGGL(copy_tile_2d<uint32_t>, dim3(blocks), dim3(256), 0, stream, (const char*)src, spitch,
                           (char*)dst, dpitch, (int64_t)(width_bytes / 4), (int64_t)height);
    } else if ((mix & 1) == 0) {
        hipLaunchKernelGGL(copy_tile_2d<uint16_t>, dim3(blocks), dim3(256), 0, stream, (const char*)src, spitch,
                           (char*)dst, dpitch, (int64_t)(width_bytes / 2), (int64_t)height);
    } else {
        hipLaunchKernelGGL(copy_tile_2d<uint8_t>, dim3(blocks), dim3(256), 0, stream, (const char*)src, spitch,
                           (char*)dst, dpitch, (int64_t)width_bytes, (int64_t)height);
    }
    return hipGetLastError();
}

}  // namespace tg
