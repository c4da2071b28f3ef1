// Version and error text of libbitsnap, and a plain streaming copy used to calibrate HBM counters
// and to show what a dependency-free kernel sustains on the same box.
#include <hip/hip_runtime.h>

#include "../../include/bitsnap.h"
#include "host_util.hpp"

namespace bitsnap {
// One-shot workgroups of 256 threads, 4 x 16 bytes per lane, non-temporal: the form of copy that streams best on
// this chip (6.2 TB/s read + write where a persistent grid-stride loop reaches 4.7-5.1).
constexpr int kCopyThreads = 256, kCopyVecs = 4;
typedef uint32_t copy_u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) copy_u32x4 copy_global_u32x4;
__global__ __launch_bounds__(kCopyThreads) void stream_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int64_t n16)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t base = ((int64_t)blockIdx.x * (kCopyThreads / 64) + wave) * (64 * kCopyVecs);
    if (base + 64 * kCopyVecs <= n16) {
        copy_u32x4 v[kCopyVecs];
#pragma unroll
        for (int k = 0; k < kCopyVecs; ++k)
            v[k] = __builtin_nontemporal_load((const copy_global_u32x4 *)(src + base + k * 64 + lane));
#pragma unroll
        for (int k = 0; k < kCopyVecs; ++k)
            __builtin_nontemporal_store(v[k], (copy_global_u32x4 *)(dst + base + k * 64 + lane));
    } else {
        for (int64_t i = base + lane; i < n16; i += 64)
            dst[i] = src[i];
    }
}

// Streaming kernels with the byte mix and the access pattern of the cluster codecs and next to
// no arithmetic: one wave per 4096 elements, 16 bytes of fp32 per lane and access, non-temporal.
//   to_small: reads 4 bytes per element, writes 1 + 1/2      (quantize_cluster's traffic)
//   else:     reads 1 + 1/2 bytes per element, writes 4      (dequantize_cluster's traffic)
typedef float mix_float4 __attribute__((ext_vector_type(4)));
#define BITSNAP_MIX_GLOBAL __attribute__((address_space(1)))
// kThreads: the workgroup size of the codec whose traffic is imitated (it changes what the memory system delivers)
template <bool kToSmall, int kThreads>
__global__ __launch_bounds__(kThreads) void stream_mix_kernel(float *wide, uint8_t *bytes, uint8_t *halves, int64_t groups)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t g = (int64_t)blockIdx.x * (kThreads / 64) + wave;
    if (g >= groups)
        return;
    const int64_t lo = g * 4096;
    if (kToSmall) {
        mix_float4 v[16];
#pragma unroll
        for (int k = 0; k < 16; ++k)
            v[k] = __builtin_nontemporal_load((const BITSNAP_MIX_GLOBAL mix_float4 *)(wide + lo + k * 256 + lane * 4));
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const uint32_t c4 = __float_as_uint(v[k].x) ^ __float_as_uint(v[k].y) ^ __float_as_uint(v[k].z) ^ __float_as_uint(v[k].w);
            __builtin_nontemporal_store(c4, (BITSNAP_MIX_GLOBAL uint32_t *)(bytes + lo + k * 256 + lane * 4));
            __builtin_nontemporal_store((uint16_t)(c4 >> 7), (BITSNAP_MIX_GLOBAL uint16_t *)(halves + ((lo + k * 256 + lane * 4) >> 1)));
        }
    } else {
        uint32_t c4[16], l4[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            c4[k] = __builtin_nontemporal_load((const BITSNAP_MIX_GLOBAL uint32_t *)(bytes + lo + k * 256 + lane * 4));
            l4[k] = __builtin_nontemporal_load((const BITSNAP_MIX_GLOBAL uint16_t *)(halves + ((lo + k * 256 + lane * 4) >> 1)));
        }
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            mix_float4 r;
            r.x = (float)(c4[k] & 255u) + (float)(l4[k] & 15u);
            r.y = (float)((c4[k] >> 8) & 255u);
            r.z = (float)((c4[k] >> 16) & 255u);
            r.w = (float)(c4[k] >> 24);
            __builtin_nontemporal_store(r, (BITSNAP_MIX_GLOBAL mix_float4 *)(wide + lo + k * 256 + lane * 4));
        }
    }
}
}  // namespace bitsnap

extern "C" int bitsnap_debug_stream_mix(void *wide, void *bytes, void *halves, int64_t n, int to_small,
                                        bitsnap_stream_t stream)
{
    if (n < 0 || (n % 4096) != 0 || n / 4096 > 0x7FFFFFFF)
        return BITSNAP_E_SIZE;
    if (n == 0)
        return BITSNAP_OK;
    if (!wide || !bytes || !halves)
        return BITSNAP_E_NULL;
    if (!bitsnap::aligned16(wide) || !bitsnap::aligned16(bytes) || !bitsnap::aligned16(halves))
        return BITSNAP_E_ALIGN;
    const int64_t groups = n / 4096;
    constexpr int kSmallThreads = 64, kWideThreads = 1024;  // as the batched quantiser and dequantiser
    if (to_small)
        hipLaunchKernelGGL((bitsnap::stream_mix_kernel<true, kSmallThreads>), dim3((unsigned)groups), dim3(kSmallThreads), 0,
                           (hipStream_t)stream, (float *)wide, (uint8_t *)bytes, (uint8_t *)halves, groups);
    else
        hipLaunchKernelGGL((bitsnap::stream_mix_kernel<false, kWideThreads>), dim3((unsigned)((groups + 15) / 16)),
                           dim3(kWideThreads), 0, (hipStream_t)stream, (float *)wide, (uint8_t *)bytes, (uint8_t *)halves,
                           groups);
    return bitsnap::launch_status();
}

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
    const int64_t per_block = (int64_t)bitsnap::kCopyThreads * bitsnap::kCopyVecs, blocks = (bytes / 16 + per_block - 1) / per_block;
    if (blocks > 0x7FFFFFFF)
        return BITSNAP_E_SIZE;
    hipLaunchKernelGGL(bitsnap::stream_copy_kernel, dim3((unsigned)blocks), dim3(bitsnap::kCopyThreads), 0, (hipStream_t)stream,
                       (const uint4 *)src, (uint4 *)dst, bytes / 16);
    return bitsnap::launch_status();
}

extern "C" int bitsnap_version(void) { return 200; /* 0.2.0: bitsnap_encode_sparse_static, the opt-in of the test knob */ }

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
    case BITSNAP_E_STATIC_LIMIT: return "tensor has more tiles than the library's built-in scan buffer serves (BITSNAP_STATIC_MAX_TILES)";
    default: return "unknown bitsnap error code";
    }
}
