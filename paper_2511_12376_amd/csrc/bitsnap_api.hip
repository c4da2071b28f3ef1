// Version and error text of libbitsnap, and a plain streaming copy used to calibrate HBM counters
// and to show what a dependency-free kernel sustains on the same box.
#include <hip/hip_runtime.h>

#include "../../include/bitsnap.h"
#include "host_util.hpp"

namespace bitsnap {
__global__ __launch_bounds__(256) void stream_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
        dst[i] = src[i];
}
}  // namespace bitsnap

extern "C" int bitsnap_debug_stream_copy(void *dst, const void *src, int64_t bytes, bitsnap_stream_t stream)
{
    if (bytes < 0 || (bytes & 15))
        return BITSNAP_E_SIZE;
    if (bytes == 0)
        return BITSNAP_OK;
    if (!dst || !src)
        return BITSNAP_E_NULL;
    if (!bitsnap::aligned16(dst) || !bitsnap::aligned16(src))
        return BITSNAP_E_ALIGN;
    const int grid = bitsnap::device_info().cu_count * 8;
    hipLaunchKernelGGL(bitsnap::stream_copy_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const uint4 *)src,
                       (uint4 *)dst, bytes / 16);
    return bitsnap::launch_status();
}

extern "C" int bitsnap_version(void) { return 100; /* 0.1.0 */ }

extern "C" const char *bitsnap_error_string(int code)
{
    switch (code) {
    case BITSNAP_OK: return "ok";
    case BITSNAP_E_NULL: return "a required pointer is NULL";
    case BITSNAP_E_SIZE: return "unsupported size, element width, cluster count or group length";
    case BITSNAP_E_ALIGN: return "a pointer is not aligned as required";
    case BITSNAP_E_WORKSPACE: return "workspace missing or too small";
    case BITSNAP_E_OFFSETS: return "tile_offsets requested for a tensor of 2^32 elements or more";
    case BITSNAP_E_LAUNCH: return "the HIP runtime refused the kernel launch";
    default: return "unknown bitsnap error code";
    }
}
