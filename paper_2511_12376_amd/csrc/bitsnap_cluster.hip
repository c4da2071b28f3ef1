// quantize_cluster / dequantize_cluster: cluster-based 8-bit quantisation of fp32 optimizer
// states (paper: "Cluster Based Quantization for Optimizer States", Eq. qmap-distance, S and b
// per cluster, Eq. decluster; Algorithm 2).
//
// One wavefront owns one group of G = 256*K elements and keeps it in registers (K float4 per
// lane), so HBM is read once.  Nothing in the kernel crosses waves: no workgroup barrier.
//   step 1  mean / deviation: fp64 partial sums per lane, DPP tree across the wave
//   step 2  the 15 edges mu + sigma*z_k, laid out in LDS as an implicit binary search tree
//   step 3  label = 4 tree steps (compare, shift-in the result)
//   step 4  per-cluster min/max: every lane owns a private column of a [32][64] LDS table
//           (bank = lane mod 32, so the read-modify-writes never conflict), reduced at the end
//   step 5-6  code = rint((x-b) * (255/S)) with (b, 255/S) fetched from a 16-entry LDS table
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/bitsnap.h"
#include "cluster_general.hpp"
#include "cluster_items.hpp"
#include "cluster_wave.hpp"
#include "host_util.hpp"
#include "wave.hpp"

namespace bitsnap {

static const double kZHost[17][16] = {
#include "z_table.inc"
};

// Waves do not cooperate in these kernels, so the workgroup is only the unit in which wave slots and LDS are handed
// out and given back.  Measured on the batched pass of a 6.7 G-element state: the quantiser (reads 4 bytes per
// element, writes 1.5) runs at 73-74 % of HBM peak in 256-thread workgroups, 75-76 % in 128-thread ones and 77 % as
// single waves, whose slots are refilled one by one; the dequantiser (reads 1.5, writes 4) is the other way
// round: 67-68 % in 64- or 128-thread workgroups, 70-72 % in 256-thread ones, 73-75 % in 512- or 1024-thread
// ones - its stores profit from neighbouring groups being written at about the same time.  A single tensor of
// a few thousand groups is one round of waves whatever the workgroup, and there the larger ones lose 4 %
// (they start and end later), so only the batched dequantiser uses them.
constexpr int kQBlock = 64;     // quantize_cluster kernels
constexpr int kQWaves = kQBlock / kWave;
constexpr int kDBlock = 256;    // dequantize_cluster kernel, one tensor
constexpr int kDWaves = kDBlock / kWave;
constexpr int kDListBlock = 1024;  // dequantize_cluster kernel, list of tensors
constexpr int kDListWaves = kDListBlock / kWave;

// Algorithm 2 for one group of len <= 256*K elements, by one wave.
template <int K, bool kFull>
__device__ __forceinline__ void quantize_group(const float *__restrict__ x, int64_t lo, int len, int m, int64_t g,
                                               uint8_t *__restrict__ codes, uint8_t *__restrict__ labels,
                                               float *__restrict__ params, float *__restrict__ fit_out,
                                               const float *__restrict__ fit_in, uint32_t *__restrict__ status,
                                               WaveShared &ws, int lane)
{
    float4 v[K];
    load_elements<K, kFull>(x, lo, len, lane, v);
    reset_ranges(ws, lane);

    // ---- step 1: mean and population standard deviation
    double sum, dev;
    wave_stats<K, kFull>(v, len, lane, sum, dev);
    float mu = (float)(sum / (double)len);
    float sigma = (float)sqrt(dev / (double)len);
    if (fit_in) {
        mu = global_ptr(fit_in)[2 * g];
        sigma = global_ptr(fit_in)[2 * g + 1];
    }
    if (status && lane == 0 && !(isfinite(mu) && isfinite(sigma)))
        atomicOr(status, 1u);

    // ---- step 2: edges and the search tables
    float edge;
    const LabelSearch ls = build_search(mu, sigma, m, ws, lane, edge);
    if (fit_out) {
        if (lane >= 1 && lane < m)
            global_ptr(fit_out)[g * (m + 1) + 1 + lane] = edge;
        if (lane == 0) {
            global_ptr(fit_out)[g * (m + 1) + 0] = mu;
            global_ptr(fit_out)[g * (m + 1) + 1] = sigma;
        }
    }

    // ---- steps 3-4: labels, per-cluster (S, b)
    uint32_t packed[(K + 1) / 2];
    label_pass<K, kFull, true, true>(v, lo, len, ls, ws, lane, labels, packed);
    float mn, mx;
    reduce_ranges(ws, lane, mn, mx);
    if (lane < kMaxClusters) {
        float S, b, inv;
        cluster_coder(mn, mx, S, b, inv);
        ws.coder[lane] = make_float2(b, inv);
        if (lane < m)
            *(BITSNAP_GLOBAL float2v *)(global_ptr(params) + (g * m + lane) * 2) = float2v{S, b};
    }
    wave_lds_sync();

    // ---- steps 5-6: codes
    code_pass<K, kFull>(v, lo, len, packed, ws, lane, codes);
}

// One wave per group.  A tensor's short last group (if it has one) goes through the same code with bounds
// checks, in the same launch: both forms fit the register budget of four waves per SIMD, and a launch of
// its own for one wave costs as much as a launch for a few thousand.
template <int K>
__global__ __launch_bounds__(kQBlock) void quantize_cluster_kernel(
    const float *__restrict__ x, int64_t n, int64_t groups, int m, uint8_t *__restrict__ codes,
    uint8_t *__restrict__ labels, float *__restrict__ params, float *__restrict__ fit_out,
    const float *__restrict__ fit_in, uint32_t *__restrict__ status)
{
    __shared__ WaveShared shared[kQWaves];
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t g = (int64_t)blockIdx.x * kQWaves + wave;
    if (g >= groups)
        return;  // whole wave leaves; the kernel has no workgroup barrier
    constexpr int G = 256 * K;
    const int64_t lo = g * G;
    const int64_t rest = n - lo;
    if (rest >= G)
        quantize_group<K, true>(x, lo, G, m, g, codes, labels, params, fit_out, fit_in, status, shared[wave], lane);
    else
        quantize_group<K, false>(x, lo, (int)rest, m, g, codes, labels, params, fit_out, fit_in, status, shared[wave], lane);
}

// Tensors of few groups (at most kSharedGroups, far fewer than the device has wave slots): the four waves of a
// workgroup share a group, 1024 elements each, instead of one wave walking through all of it.  A call for such
// a tensor is nothing but a wave's chain of load, statistics, tables, labels, ranges and codes; four waves cut it
// from 6.6 to about 4 us.  The statistics of the four parts are combined with the pairwise update formula (every
// term non-negative), the ranges by min / max; every wave builds its own copy of the search tables.
constexpr int kSmallWaves = 4, kSmallK = 4, kSmallPart = 256 * kSmallK;
constexpr int64_t kSharedGroups = 1024;  // beyond a few hundred groups the one-wave kernel is as fast; at 4096 it is 8 % faster
struct SharedGroupLds {
    WaveShared shared[kSmallWaves];
    double part_sum[kSmallWaves], part_dev[kSmallWaves];
    float part_range[kSmallWaves][2 * kMaxClusters];
};

// kFull: the group has all its 4096 elements, so every wave's part is whole (16-byte loads, no bounds checks)
template <bool kFull>
__device__ __forceinline__ void quantize_shared_group(SharedGroupLds &lds, const float *__restrict__ x, int64_t g, int64_t g_lo,
                                                      int g_len, int m, uint8_t *__restrict__ codes, uint8_t *__restrict__ labels,
                                                      float *__restrict__ params, float *__restrict__ fit_out,
                                                      const float *__restrict__ fit_in, uint32_t *__restrict__ status, int lane,
                                                      int wave)
{
    WaveShared &ws = lds.shared[wave];
    double *part_sum = lds.part_sum, *part_dev = lds.part_dev;
    float(*part_range)[2 * kMaxClusters] = lds.part_range;
    auto part_len = [&](int w) { return g_len - w * kSmallPart >= kSmallPart ? kSmallPart : (g_len > w * kSmallPart ? g_len - w * kSmallPart : 0); };
    const int64_t lo = g_lo + wave * kSmallPart;
    const int len = part_len(wave);
    float4 v[kSmallK];
    load_elements<kSmallK, kFull>(x, lo, len, lane, v);
    reset_ranges(ws, lane);

    // ---- step 1
    double sum = 0.0, dev = 0.0;
    if (kFull || len > 0)
        wave_stats<kSmallK, kFull>(v, len, lane, sum, dev);
    if (lane == 0) {
        part_sum[wave] = sum;
        part_dev[wave] = dev;
    }
    __syncthreads();
    double total = 0.0;
#pragma unroll
    for (int w = 0; w < kSmallWaves; ++w)
        total += part_sum[w];
    const double mean = total / (double)g_len;
    double about = 0.0;
#pragma unroll
    for (int w = 0; w < kSmallWaves; ++w) {
        const int part = part_len(w);
        if (part > 0) {
            const double shift = part_sum[w] / (double)part - mean;
            about += part_dev[w] + (double)part * shift * shift;
        }
    }
    float mu = (float)mean;
    float sigma = (float)sqrt(about / (double)g_len);
    if (fit_in) {
        mu = global_ptr(fit_in)[2 * g];
        sigma = global_ptr(fit_in)[2 * g + 1];
    }
    if (status && wave == 0 && lane == 0 && !(isfinite(mu) && isfinite(sigma)))
        atomicOr(status, 1u);

    // ---- step 2
    float edge;
    const LabelSearch ls = build_search(mu, sigma, m, ws, lane, edge);
    if (fit_out && wave == 0) {
        if (lane >= 1 && lane < m)
            global_ptr(fit_out)[g * (m + 1) + 1 + lane] = edge;
        if (lane == 0) {
            global_ptr(fit_out)[g * (m + 1) + 0] = mu;
            global_ptr(fit_out)[g * (m + 1) + 1] = sigma;
        }
    }

    // ---- steps 3-4
    uint32_t packed[(kSmallK + 1) / 2];
    label_pass<kSmallK, kFull, true, true>(v, lo, len, ls, ws, lane, labels, packed);
    float mn, mx;
    reduce_ranges(ws, lane, mn, mx);
    if (lane < kMaxClusters) {
        part_range[wave][lane] = mn;
        part_range[wave][kMaxClusters + lane] = mx;
    }
    __syncthreads();
    if (lane < kMaxClusters) {
#pragma unroll
        for (int w = 0; w < kSmallWaves; ++w) {
            mn = fminf(mn, part_range[w][lane]);
            mx = fmaxf(mx, part_range[w][kMaxClusters + lane]);
        }
        float S, b, inv;
        cluster_coder(mn, mx, S, b, inv);
        ws.coder[lane] = make_float2(b, inv);
        if (wave == 0 && lane < m)
            *(BITSNAP_GLOBAL float2v *)(global_ptr(params) + (g * m + lane) * 2) = float2v{S, b};
    }
    wave_lds_sync();

    // ---- steps 5-6
    code_pass<kSmallK, kFull>(v, lo, len, packed, ws, lane, codes);
}

__global__ __launch_bounds__(kSmallWaves *kWave) void quantize_cluster_shared_kernel(
    const float *__restrict__ x, int64_t n, int G, int m, uint8_t *__restrict__ codes, uint8_t *__restrict__ labels,
    float *__restrict__ params, float *__restrict__ fit_out, const float *__restrict__ fit_in,
    uint32_t *__restrict__ status)
{
    __shared__ SharedGroupLds lds;
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t g = blockIdx.x, g_lo = g * G;
    const int g_len = n - g_lo >= G ? G : (int)(n - g_lo);        // 1 .. 4096
    if (g_len == kSmallWaves * kSmallPart)
        quantize_shared_group<true>(lds, x, g, g_lo, g_len, m, codes, labels, params, fit_out, fit_in, status, lane, wave);
    else
        quantize_shared_group<false>(lds, x, g, g_lo, g_len, m, codes, labels, params, fit_out, fit_in, status, lane, wave);
}

template <int K>
__global__ __launch_bounds__(kDBlock) void dequantize_cluster_kernel(
    const uint8_t *__restrict__ codes, const uint8_t *__restrict__ labels, const float *__restrict__ params,
    int64_t n, int64_t groups, int m, float *__restrict__ out)
{
    __shared__ float2 coder[kDWaves][kMaxClusters];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int64_t g = (int64_t)blockIdx.x * kDWaves + wave;
    if (g >= groups)
        return;
    constexpr int G = 256 * K;
    const int64_t lo = g * G;
    const int64_t rest = n - lo;
    dequantize_group<K>(codes, labels, params, lo, rest >= G ? G : (int)rest, true, m, g, out, coder[wave], lane);
}

// The dequantiser for groups of 2048 or 4096 elements: one wave per 512 elements, one workgroup (4 or 8 waves) per
// group; the parts share nothing but the group's 16 (S, b) pairs, which every wave fetches for itself.  Many light,
// short-lived waves keep reads and writes mixed evenly: with this kernel's traffic and no arithmetic, 256 elements
// per wave stream at 78-81 % of HBM peak, 512 at 74-78 %, 1024 and 4096 at 63-71 %; with the arithmetic and the
// fetch of the pairs 512 is best (a 537 M-element tensor: 79.7 % against 68 % for 256, 73-74 % for 1024 and 70-74 %
// for 4096 elements per wave).
constexpr int kDeqPartK = 2, kDeqPart = 256 * kDeqPartK;
template <int W>  // W = waves per group: the group holds W * 512 elements
__global__ __launch_bounds__(W *kWave) void dequantize_cluster_parts_kernel(
    const uint8_t *__restrict__ codes, const uint8_t *__restrict__ labels, const float *__restrict__ params, int64_t n,
    int m, float *__restrict__ out)
{
    __shared__ float2 coder[W][kMaxClusters];
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t g = blockIdx.x;
    const int64_t lo = g * (W * kDeqPart) + wave * kDeqPart;
    const int64_t rest = n - lo;
    if (rest <= 0)
        return;  // whole wave leaves; no workgroup barrier in this kernel
    dequantize_group<kDeqPartK>(codes, labels, params, lo, rest >= kDeqPart ? kDeqPart : (int)rest, true, m, g, out, coder[wave], lane);
}

// ---------------------------------------------------------------------------------------------
// Batched forms: one launch for a list of tensors.  Groups are numbered across the list
// (item.first_group = groups of all earlier items) and the grid has one wave per group of the
// whole list, so the device works through many rounds of waves whose load, compute and store
// phases overlap; a single tensor of a few thousand groups is one round (one group per wave slot)
// whose phases cannot overlap.
// ---------------------------------------------------------------------------------------------

__device__ __forceinline__ int64_t uniform_i64(int64_t v)
{
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)(uint64_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

template <int K>
__global__ __launch_bounds__(kQBlock) void quantize_cluster_batched_kernel(
    const bitsnap_cluster_item *__restrict__ items, int64_t count, int64_t total_groups, int m,
    uint32_t *__restrict__ status)
{
    __shared__ WaveShared shared[kQWaves];
    // the wave index as a scalar: group and item bookkeeping then lives in SGPRs
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr int G = 256 * K;
    const int64_t gg = (int64_t)blockIdx.x * kQWaves + wave;
    if (gg >= total_groups)
        return;
    const bitsnap_cluster_item &it = items[find_item(items, count, gg)];
    const int64_t g = gg - it.first_group;
    const int64_t lo = g * G;
    const int64_t rest = it.n - lo;
    if (rest >= G)
        quantize_group<K, true>((const float *)it.values, lo, G, m, g, it.codes, it.labels, it.params, it.fit_out,
                                it.fit_in, status, shared[wave], lane);
    else if (rest > 0)  // the tensor's short last group
        quantize_group<K, false>((const float *)it.values, lo, (int)rest, m, g, it.codes, it.labels, it.params,
                                 it.fit_out, it.fit_in, status, shared[wave], lane);
}

template <int K>
__global__ __launch_bounds__(kDListBlock) void dequantize_cluster_batched_kernel(
    const bitsnap_cluster_item *__restrict__ items, int64_t count, int64_t total_groups, int m)
{
    __shared__ float2 coder[kDListWaves][kMaxClusters];
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr int G = 256 * K;
    const int64_t gg = (int64_t)blockIdx.x * kDListWaves + wave;
    if (gg >= total_groups)
        return;
    const bitsnap_cluster_item &it = items[find_item(items, count, gg)];
    const int64_t g = gg - it.first_group;
    const int64_t lo = g * G;
    const int64_t rest = it.n - lo;
    if (rest > 0)
        dequantize_group<K>(it.codes, it.labels, it.params, lo, rest >= G ? G : (int)rest, true, m, g, (float *)it.values,
                            coder[wave], lane);
}

// The same for a list of tensors: one workgroup per group of the whole list, one wave per 512 elements; every wave
// looks its item up itself (a binary search on the scalar unit: nine dependent loads for the 291 items of a
// Llama-2-7B-shaped list, most of them hits in the scalar cache).  One lookup per workgroup handed on through LDS,
// and an eight-way search with fewer round trips but more loads, were slower; so were workgroups that walk several
// groups with one lookup.  Llama-2-7B-shaped states: 70.9 -> 76-77 % of HBM peak against one wave per group.
template <int W>
__global__ __launch_bounds__(W *kWave) void dequantize_cluster_batched_parts_kernel(
    const bitsnap_cluster_item *__restrict__ items, int64_t count, int64_t total_groups, int m)
{
    __shared__ float2 coder[W][kMaxClusters];
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t gg = blockIdx.x;
    if (gg >= total_groups)
        return;
    const bitsnap_cluster_item &it = items[find_item(items, count, gg)];
    const int64_t g = gg - it.first_group;
    const int64_t lo = g * (W * kDeqPart) + wave * kDeqPart;
    const int64_t rest = it.n - lo;
    if (rest > 0)
        dequantize_group<kDeqPartK>(it.codes, it.labels, it.params, lo, rest >= kDeqPart ? kDeqPart : (int)rest, true, m, g,
                                    (float *)it.values, coder[wave], lane);
}

}  // namespace bitsnap

using namespace bitsnap;

extern "C" size_t bitsnap_cluster_groups(int64_t n, int64_t group)
{
    if (n <= 0)
        return 0;
    if (group <= 0 || group > n)
        group = n;
    return (size_t)((n + group - 1) / group);
}

extern "C" size_t bitsnap_cluster_param_bytes(int64_t n, int64_t group, int m)
{
    return bitsnap_cluster_groups(n, group) * (size_t)(m > 0 ? m : 0) * 2 * sizeof(float);
}

extern "C" size_t bitsnap_cluster_label_bytes(int64_t n) { return n <= 0 ? 0 : (size_t)((n + 1) / 2); }

extern "C" size_t bitsnap_cluster_fit_floats(int64_t n, int64_t group, int m)
{
    return bitsnap_cluster_groups(n, group) * (size_t)(m > 0 ? m + 1 : 0);
}

extern "C" size_t bitsnap_cluster_workspace_bytes(int64_t n, int64_t group, int m)
{
    (void)m;
    if (n <= 0 || one_wave_group_k(group) != 0)
        return 0;
    return cluster_general_workspace_bytes(n, group);
}

extern "C" double bitsnap_cluster_z(int k, int m)
{
    if (m < 2 || m > kMaxClusters || k < 1 || k >= m)
        return 0.0;
    return kZHost[m][k];
}

extern "C" int bitsnap_quantize_cluster(const float *x, int64_t n, int64_t group, int m, uint8_t *codes,
                                        uint8_t *labels, float *params, float *fit_out, const float *fit_in,
                                        uint32_t *status, void *workspace, size_t workspace_bytes,
                                        bitsnap_stream_t stream)
{
    if (n < 0 || m < 1 || m > kMaxClusters || group < 0)
        return BITSNAP_E_SIZE;
    if (n == 0)
        return BITSNAP_OK;
    const int K = one_wave_group_k(group);
    if (K == 0 && !cluster_general_supported(n, group))
        return BITSNAP_E_SIZE;
    if (!x || !codes || !labels || !params)
        return BITSNAP_E_NULL;
    if (!aligned16(x) || !aligned16(codes) || !aligned16(labels) || !aligned16(params) || ((uintptr_t)fit_out & 3u) ||
        ((uintptr_t)fit_in & 3u) || ((uintptr_t)status & 3u))
        return BITSNAP_E_ALIGN;
    if (K == 0) {
        if (!workspace)
            return BITSNAP_E_NULL;
        if (!aligned16(workspace))
            return BITSNAP_E_ALIGN;
        if (workspace_bytes < cluster_general_workspace_bytes(n, group))
            return BITSNAP_E_WORKSPACE;
        return cluster_general_quantize(x, n, group, m, codes, labels, params, fit_out, fit_in, status, workspace,
                                        (hipStream_t)stream);
    }
    const int64_t G = 256 * (int64_t)K;
    const int64_t groups = (n + G - 1) / G;      // the last one may be short
    const int64_t blocks = (groups + kQWaves - 1) / kQWaves;
    if (blocks > 0x7FFFFFFF)
        return BITSNAP_E_SIZE;
    const dim3 block(kQBlock);
    hipStream_t s = (hipStream_t)stream;
    // few groups of more than one wave's quarter: four waves share each group
    if (groups <= kSharedGroups && G > kSmallPart && n > kSmallPart) {
        hipLaunchKernelGGL(quantize_cluster_shared_kernel, dim3((unsigned)groups), dim3(kSmallWaves * kWave), 0, s, x, n, (int)G, m,
                           codes, labels, params, fit_out, fit_in, status);
        return launch_status();
    }
#define BITSNAP_LAUNCH_Q(KK)                                                                              \
    hipLaunchKernelGGL((quantize_cluster_kernel<KK>), dim3((unsigned)blocks), block, 0, s, x, n, groups, \
                       m, codes, labels, params, fit_out, fit_in, status)
    switch (K) {
    case 1: BITSNAP_LAUNCH_Q(1); break;
    case 2: BITSNAP_LAUNCH_Q(2); break;
    case 4: BITSNAP_LAUNCH_Q(4); break;
    case 8: BITSNAP_LAUNCH_Q(8); break;
    default: BITSNAP_LAUNCH_Q(16); break;
    }
#undef BITSNAP_LAUNCH_Q
    return launch_status();
}

extern "C" int bitsnap_dequantize_cluster(const uint8_t *codes, const uint8_t *labels, const float *params, int64_t n,
                                          int64_t group, int m, float *out, bitsnap_stream_t stream)
{
    if (n < 0 || m < 1 || m > kMaxClusters || group < 0)
        return BITSNAP_E_SIZE;
    if (n == 0)
        return BITSNAP_OK;
    const int K = one_wave_group_k(group);
    if (K == 0 && !cluster_general_supported(n, group))
        return BITSNAP_E_SIZE;
    if (!codes || !labels || !params || !out)
        return BITSNAP_E_NULL;
    if (!aligned16(codes) || !aligned16(labels) || !aligned16(params) || !aligned16(out))
        return BITSNAP_E_ALIGN;
    if (K == 0)
        return cluster_general_dequantize(codes, labels, params, n, group, m, out, (hipStream_t)stream);
    const int64_t groups = (int64_t)bitsnap_cluster_groups(n, group);
    const int64_t blocks = (groups + kDWaves - 1) / kDWaves;
    if (blocks > 0x7FFFFFFF)
        return BITSNAP_E_SIZE;
    const dim3 grid((unsigned)blocks), block(kDBlock);
    hipStream_t s = (hipStream_t)stream;
    if (256 * K >= 4 * kDeqPart && groups <= 0x7FFFFFFF) {  // groups of 2048 or 4096 elements: one wave per 512 of them
        if (256 * K == 8 * kDeqPart)
            hipLaunchKernelGGL(dequantize_cluster_parts_kernel<8>, dim3((unsigned)groups), dim3(8 * kWave), 0, s, codes, labels,
                               params, n, m, out);
        else
            hipLaunchKernelGGL(dequantize_cluster_parts_kernel<4>, dim3((unsigned)groups), dim3(4 * kWave), 0, s, codes, labels,
                               params, n, m, out);
        return launch_status();
    }
#define BITSNAP_LAUNCH_D(KK) \
    hipLaunchKernelGGL(dequantize_cluster_kernel<KK>, grid, block, 0, s, codes, labels, params, n, groups, m, out)
    switch (K) {
    case 1: BITSNAP_LAUNCH_D(1); break;
    case 2: BITSNAP_LAUNCH_D(2); break;
    case 4: BITSNAP_LAUNCH_D(4); break;
    case 8: BITSNAP_LAUNCH_D(8); break;
    default: BITSNAP_LAUNCH_D(16); break;
    }
#undef BITSNAP_LAUNCH_D
    return launch_status();
}

static int64_t batched_blocks(int64_t total_groups, int waves) { return (total_groups + waves - 1) / waves; }

extern "C" int bitsnap_quantize_cluster_batched(const bitsnap_cluster_item *items, int64_t count, int64_t total_groups,
                                                int64_t group, int m, uint32_t *status, bitsnap_stream_t stream)
{
    if (count < 0 || total_groups < 0 || m < 1 || m > kMaxClusters)
        return BITSNAP_E_SIZE;
    const int K = one_wave_group_k(group);
    if (K == 0)
        return BITSNAP_E_SIZE;  // the batched form exists for the one-wave-per-group lengths only
    if (count == 0 || total_groups == 0)
        return BITSNAP_OK;
    if (!items)
        return BITSNAP_E_NULL;
    if (((uintptr_t)items & 7u) || ((uintptr_t)status & 3u))
        return BITSNAP_E_ALIGN;
    if (batched_blocks(total_groups, kQWaves) > 0x7FFFFFFF)
        return BITSNAP_E_SIZE;
    const dim3 block(kQBlock), grid((unsigned)batched_blocks(total_groups, kQWaves));
    hipStream_t s = (hipStream_t)stream;
#define BITSNAP_LAUNCH_QB(KK) \
    hipLaunchKernelGGL((quantize_cluster_batched_kernel<KK>), grid, block, 0, s, items, count, total_groups, m, status)
    switch (K) {
    case 1: BITSNAP_LAUNCH_QB(1); break;
    case 2: BITSNAP_LAUNCH_QB(2); break;
    case 4: BITSNAP_LAUNCH_QB(4); break;
    case 8: BITSNAP_LAUNCH_QB(8); break;
    default: BITSNAP_LAUNCH_QB(16); break;
    }
#undef BITSNAP_LAUNCH_QB
    return launch_status();
}

extern "C" int bitsnap_dequantize_cluster_batched(const bitsnap_cluster_item *items, int64_t count,
                                                  int64_t total_groups, int64_t group, int m, bitsnap_stream_t stream)
{
    if (count < 0 || total_groups < 0 || m < 1 || m > kMaxClusters)
        return BITSNAP_E_SIZE;
    const int K = one_wave_group_k(group);
    if (K == 0)
        return BITSNAP_E_SIZE;
    if (count == 0 || total_groups == 0)
        return BITSNAP_OK;
    if (!items)
        return BITSNAP_E_NULL;
    if ((uintptr_t)items & 7u)
        return BITSNAP_E_ALIGN;
    if (batched_blocks(total_groups, kDListWaves) > 0x7FFFFFFF)
        return BITSNAP_E_SIZE;
    const dim3 block(kDListBlock), grid((unsigned)batched_blocks(total_groups, kDListWaves));
    hipStream_t s = (hipStream_t)stream;
    if (256 * K >= 4 * kDeqPart && total_groups <= 0x7FFFFFFF) {  // groups of 2048 or 4096 elements: a workgroup each
        if (256 * K == 8 * kDeqPart)
            hipLaunchKernelGGL(dequantize_cluster_batched_parts_kernel<8>, dim3((unsigned)total_groups), dim3(8 * kWave), 0, s,
                               items, count, total_groups, m);
        else
            hipLaunchKernelGGL(dequantize_cluster_batched_parts_kernel<4>, dim3((unsigned)total_groups), dim3(4 * kWave), 0, s,
                               items, count, total_groups, m);
        return launch_status();
    }
#define BITSNAP_LAUNCH_DB(KK) \
    hipLaunchKernelGGL(dequantize_cluster_batched_kernel<KK>, grid, block, 0, s, items, count, total_groups, m)
    switch (K) {
    case 1: BITSNAP_LAUNCH_DB(1); break;
    case 2: BITSNAP_LAUNCH_DB(2); break;
    case 4: BITSNAP_LAUNCH_DB(4); break;
    case 8: BITSNAP_LAUNCH_DB(8); break;
    default: BITSNAP_LAUNCH_DB(16); break;
    }
#undef BITSNAP_LAUNCH_DB
    return launch_status();
}
