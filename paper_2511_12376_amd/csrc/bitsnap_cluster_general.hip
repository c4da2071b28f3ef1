// quantize_cluster / dequantize_cluster for group lengths the one-wave-per-group kernels do not
// take: any even G and G = 0 (one group spanning the tensor, the paper's own formulation of
// Algorithm 2).  A group is cut into chunks of 4096 elements, one 256-thread workgroup per chunk,
// and Algorithm 2's steps become passes over HBM with the per-group state in the workspace:
//   pass 1  sum per chunk                 -> finalize: mean
//   pass 2  sum of (x-mean)^2 per chunk   -> finalize: mu, sigma, edges; min/max tables reset
//   pass 3  labels; per-cluster min/max (LDS per chunk, then integer atomics on ordered keys)
//           -> finalize: (S, b), 255/S
//   pass 4  codes
// Chunk partials are written out and summed in chunk order, so the fit does not depend on the
// order in which workgroups run.  This path favours being right over being fast (x is read four
// times).
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/bitsnap.h"
#include "cluster_general.hpp"
#include "host_util.hpp"
#include "wave.hpp"

namespace bitsnap {

constexpr int kGBlock = 256;
constexpr int kGChunk = 4096;
constexpr int kGMaxClusters = 16;

// the same quantile table as the one-wave-per-group kernels (a copy per translation unit)
__constant__ double kZGeneral[17][16] = {
#include "z_table.inc"
};

struct GroupState {  // one per group, in the workspace
    double sum;
    double dev;
    float mu, sigma;
    float edges[kGMaxClusters];      // [k] = e_k, [0] unused
    int32_t kmin[kGMaxClusters];     // ordered keys of the cluster minima / maxima
    int32_t kmax[kGMaxClusters];
    float2 coder[kGMaxClusters];     // (b, 255/S)
};

// float <-> int key whose signed order is the float order (-0 sorts below +0); an involution
__device__ __forceinline__ int32_t ordered_key(float x)
{
    const int32_t b = __float_as_int(x);
    return b ^ ((b >> 31) & 0x7FFFFFFF);
}
__device__ __forceinline__ float from_key(int32_t k) { return __int_as_float(k ^ ((k >> 31) & 0x7FFFFFFF)); }

struct ChunkRef {
    int64_t group, lo;  // group index, first element (global)
    int len;            // elements in this chunk
};

// chunk c of the tensor: groups are cut into ceil(G/4096) chunks each (the last group may have fewer)
__device__ __forceinline__ ChunkRef chunk_ref(int64_t c, int64_t n, int64_t G, int64_t chunks_per_group)
{
    ChunkRef r;
    r.group = c / chunks_per_group;
    const int64_t within = (c % chunks_per_group) * kGChunk;
    const int64_t g_lo = r.group * G;
    const int64_t g_len = (g_lo + G <= n) ? G : (n - g_lo);
    r.lo = g_lo + within;
    const int64_t rest = g_len - within;
    r.len = rest <= 0 ? 0 : (rest < kGChunk ? (int)rest : kGChunk);
    return r;
}

__device__ __forceinline__ double block_sum(double v, double *scratch)
{
    v = wave_sum(v);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0)
        scratch[wave] = v;
    __syncthreads();
    return (scratch[0] + scratch[1]) + (scratch[2] + scratch[3]);
}

template <bool kDeviation>
__global__ __launch_bounds__(kGBlock) void general_partial_kernel(const float *__restrict__ x, int64_t n, int64_t G,
                                                                  int64_t chunks_per_group, int64_t chunks,
                                                                  const GroupState *__restrict__ gs,
                                                                  double *__restrict__ partial)
{
    __shared__ double scratch[kGBlock / kWave];
    for (int64_t c = blockIdx.x; c < chunks; c += gridDim.x) {
        const ChunkRef r = chunk_ref(c, n, G, chunks_per_group);
        const double mean = kDeviation ? gs[r.group].sum : 0.0;  // after pass 1, .sum holds the mean
        double acc = 0.0;
        for (int e = threadIdx.x; e < r.len; e += kGBlock) {
            const double v = (double)x[r.lo + e];
            if (kDeviation) {
                const double d = v - mean;
                acc = fma(d, d, acc);
            } else {
                acc += v;
            }
        }
        acc = block_sum(acc, scratch);
        if (threadIdx.x == 0)
            partial[c] = acc;
    }
}

// One workgroup per group: add the chunk partials in chunk order.
//   stage 0: sum -> mean (kept in .sum)
//   stage 1: deviation -> mu, sigma, edges, reset of the min/max keys
__global__ __launch_bounds__(kGBlock) void general_finalize_fit_kernel(int stage, int64_t n, int64_t G,
                                                                       int64_t chunks_per_group, int64_t groups, int m,
                                                                       const double *__restrict__ partial, GroupState *gs,
                                                                       float *__restrict__ fit_out,
                                                                       const float *__restrict__ fit_in,
                                                                       uint32_t *__restrict__ status)
{
    __shared__ double scratch[kGBlock / kWave];
    for (int64_t g = blockIdx.x; g < groups; g += gridDim.x) {
        const int64_t g_lo = g * G;
        const int64_t g_len = (g_lo + G <= n) ? G : (n - g_lo);
        const int64_t nch = (g_len + kGChunk - 1) / kGChunk;
        // fixed association: thread t takes chunks t, t+256, ... in order, then the block tree
        double acc = 0.0;
        for (int64_t c = threadIdx.x; c < nch; c += kGBlock)
            acc += partial[g * chunks_per_group + c];
        acc = block_sum(acc, scratch);
        if (stage == 0) {
            if (threadIdx.x == 0)
                gs[g].sum = acc / (double)g_len;
        } else {
            float mu = (float)gs[g].sum;
            float sigma = (float)sqrt(acc / (double)g_len);
            if (fit_in) {
                mu = fit_in[2 * g];
                sigma = fit_in[2 * g + 1];
            }
            const int t = threadIdx.x;
            if (t == 0) {
                gs[g].mu = mu;
                gs[g].sigma = sigma;
                if (status && !(isfinite(mu) && isfinite(sigma)))
                    atomicOr(status, 1u);
                if (fit_out) {
                    fit_out[g * (m + 1) + 0] = mu;
                    fit_out[g * (m + 1) + 1] = sigma;
                }
            }
            if (t < kGMaxClusters) {
                float e = INFINITY;
                if (t >= 1 && t < m)
                    e = (float)__dadd_rn((double)mu, __dmul_rn((double)sigma, kZGeneral[m][t]));
                gs[g].edges[t] = e;
                if (fit_out && t >= 1 && t < m)
                    fit_out[g * (m + 1) + 1 + t] = e;
                gs[g].kmin[t] = 0x7FFFFFFF;
                gs[g].kmax[t] = (int32_t)0x80000000;
            }
        }
        __syncthreads();
    }
}

// Algorithm 2 step 3 as a plain count (the edges that do not exist are +inf)
__device__ __forceinline__ int label_by_count(const float *edges, float x)
{
    int l = 0;
#pragma unroll
    for (int k = 1; k < kGMaxClusters; ++k)
        l += (edges[k] <= x) ? 1 : 0;
    return l;
}

__global__ __launch_bounds__(kGBlock) void general_label_kernel(const float *__restrict__ x, int64_t n, int64_t G,
                                                                int64_t chunks_per_group, int64_t chunks,
                                                                GroupState *gs, uint8_t *__restrict__ labels)
{
    __shared__ float edges[kGMaxClusters];
    __shared__ int32_t kmin[kGMaxClusters], kmax[kGMaxClusters];
    for (int64_t c = blockIdx.x; c < chunks; c += gridDim.x) {
        const ChunkRef r = chunk_ref(c, n, G, chunks_per_group);
        __syncthreads();
        if (threadIdx.x < kGMaxClusters) {
            edges[threadIdx.x] = gs[r.group].edges[threadIdx.x];
            kmin[threadIdx.x] = 0x7FFFFFFF;
            kmax[threadIdx.x] = (int32_t)0x80000000;
        }
        __syncthreads();
        // two elements per thread and step: r.lo is even, so a pair shares one label byte
        for (int p = threadIdx.x; 2 * p < r.len; p += kGBlock) {
            uint32_t byte = 0;
            for (int j = 0; j < 2; ++j) {
                const int e = 2 * p + j;
                if (e < r.len) {
                    const float v = x[r.lo + e];
                    const int l = label_by_count(edges, v);
                    byte |= (uint32_t)l << (4 * j);
                    const int32_t key = ordered_key(v);
                    atomicMin(&kmin[l], key);
                    atomicMax(&kmax[l], key);
                }
            }
            labels[(r.lo >> 1) + p] = (uint8_t)byte;
        }
        __syncthreads();
        if (threadIdx.x < kGMaxClusters && kmin[threadIdx.x] <= kmax[threadIdx.x]) {
            atomicMin(&gs[r.group].kmin[threadIdx.x], kmin[threadIdx.x]);
            atomicMax(&gs[r.group].kmax[threadIdx.x], kmax[threadIdx.x]);
        }
    }
}

__global__ __launch_bounds__(kGBlock) void general_finalize_params_kernel(int64_t groups, int m, GroupState *gs,
                                                                          float *__restrict__ params)
{
    const int64_t i = (int64_t)blockIdx.x * kGBlock + threadIdx.x;
    const int64_t g = i / kGMaxClusters;
    const int c = (int)(i % kGMaxClusters);
    if (g >= groups)
        return;
    float S = 0.0f, b = 0.0f, inv = 0.0f;
    const int32_t lo = gs[g].kmin[c], hi = gs[g].kmax[c];
    if (lo <= hi) {  // the cluster has members
        b = from_key(lo);
        S = __fsub_rn(from_key(hi), b);
        if (S > 0.0f) {
            inv = __fdiv_rn(255.0f, S);
            if (!isfinite(inv))
                inv = 0.0f;
        }
    }
    gs[g].coder[c] = make_float2(b, inv);
    if (c < m)
        *reinterpret_cast<float2 *>(params + (g * m + c) * 2) = make_float2(S, b);
}

__global__ __launch_bounds__(kGBlock) void general_code_kernel(const float *__restrict__ x, int64_t n, int64_t G,
                                                               int64_t chunks_per_group, int64_t chunks,
                                                               const GroupState *__restrict__ gs,
                                                               const uint8_t *__restrict__ labels,
                                                               uint8_t *__restrict__ codes)
{
    __shared__ float2 coder[kGMaxClusters];
    for (int64_t c = blockIdx.x; c < chunks; c += gridDim.x) {
        const ChunkRef r = chunk_ref(c, n, G, chunks_per_group);
        __syncthreads();
        if (threadIdx.x < kGMaxClusters)
            coder[threadIdx.x] = gs[r.group].coder[threadIdx.x];
        __syncthreads();
        for (int e = threadIdx.x; e < r.len; e += kGBlock) {
            const int64_t idx = r.lo + e;
            const int l = (labels[idx >> 1] >> (4 * (int)(idx & 1))) & 15;
            const float2 bi = coder[l];
            const float y = __fmul_rn(__fsub_rn(x[idx], bi.x), bi.y);
            codes[idx] = (uint8_t)__builtin_amdgcn_cvt_pk_u8_f32(y, 0, 0u);  // rint, saturate, NaN -> 0
        }
    }
}

__global__ __launch_bounds__(kGBlock) void general_dequantize_kernel(const uint8_t *__restrict__ codes,
                                                                     const uint8_t *__restrict__ labels,
                                                                     const float *__restrict__ params, int64_t n,
                                                                     int64_t G, int64_t chunks_per_group, int64_t chunks,
                                                                     int m, float *__restrict__ out)
{
    __shared__ float2 coder[kGMaxClusters];  // (S/255, b)
    for (int64_t c = blockIdx.x; c < chunks; c += gridDim.x) {
        const ChunkRef r = chunk_ref(c, n, G, chunks_per_group);
        __syncthreads();
        if (threadIdx.x < kGMaxClusters) {
            float2 sb = make_float2(0.0f, 0.0f);
            if ((int)threadIdx.x < m)
                sb = *reinterpret_cast<const float2 *>(params + (r.group * m + threadIdx.x) * 2);
            coder[threadIdx.x] = make_float2(__fdiv_rn(sb.x, 255.0f), sb.y);
        }
        __syncthreads();
        for (int e = threadIdx.x; e < r.len; e += kGBlock) {
            const int64_t idx = r.lo + e;
            const int l = (labels[idx >> 1] >> (4 * (int)(idx & 1))) & 15;
            const float2 sb = coder[l];
            out[idx] = __fadd_rn(__fmul_rn((float)codes[idx], sb.x), sb.y);
        }
    }
}

static void general_shape(int64_t n, int64_t group, int64_t &G, int64_t &groups, int64_t &cpg, int64_t &chunks)
{
    G = (group <= 0 || group > n) ? n : group;
    groups = (n + G - 1) / G;
    cpg = (G + kGChunk - 1) / kGChunk;
    chunks = groups * cpg;
}

bool cluster_general_supported(int64_t n, int64_t group)
{
    if (n <= 0)
        return true;
    return group <= 0 || group >= n || (group % 2) == 0;  // a group boundary must not split a label byte
}

size_t cluster_general_workspace_bytes(int64_t n, int64_t group)
{
    if (n <= 0)
        return 0;
    int64_t G, groups, cpg, chunks;
    general_shape(n, group, G, groups, cpg, chunks);
    const size_t bytes = (size_t)groups * sizeof(GroupState) + (size_t)chunks * sizeof(double);
    return (bytes + 255) / 256 * 256;
}

static int general_grid(int64_t work)
{
    const int64_t cap = (int64_t)device_info().cu_count * 16;
    return (int)(work < 1 ? 1 : (work < cap ? work : cap));
}

int cluster_general_quantize(const float *x, int64_t n, int64_t group, int m, uint8_t *codes, uint8_t *labels,
                             float *params, float *fit_out, const float *fit_in, uint32_t *status, void *workspace,
                             hipStream_t s)
{
    int64_t G, groups, cpg, chunks;
    general_shape(n, group, G, groups, cpg, chunks);
    GroupState *gs = reinterpret_cast<GroupState *>(workspace);
    double *partial = reinterpret_cast<double *>(gs + groups);
    const dim3 block(kGBlock), cgrid(general_grid(chunks)), ggrid(general_grid(groups));
    hipLaunchKernelGGL(general_partial_kernel<false>, cgrid, block, 0, s, x, n, G, cpg, chunks, gs, partial);
    hipLaunchKernelGGL(general_finalize_fit_kernel, ggrid, block, 0, s, 0, n, G, cpg, groups, m, partial, gs, fit_out,
                       fit_in, status);
    hipLaunchKernelGGL(general_partial_kernel<true>, cgrid, block, 0, s, x, n, G, cpg, chunks, gs, partial);
    hipLaunchKernelGGL(general_finalize_fit_kernel, ggrid, block, 0, s, 1, n, G, cpg, groups, m, partial, gs, fit_out,
                       fit_in, status);
    hipLaunchKernelGGL(general_label_kernel, cgrid, block, 0, s, x, n, G, cpg, chunks, gs, labels);
    const int64_t pthreads = groups * kGMaxClusters;
    hipLaunchKernelGGL(general_finalize_params_kernel, dim3((unsigned)((pthreads + kGBlock - 1) / kGBlock)), block, 0, s,
                       groups, m, gs, params);
    hipLaunchKernelGGL(general_code_kernel, cgrid, block, 0, s, x, n, G, cpg, chunks, gs, labels, codes);
    return launch_status();
}

int cluster_general_dequantize(const uint8_t *codes, const uint8_t *labels, const float *params, int64_t n,
                               int64_t group, int m, float *out, hipStream_t s)
{
    int64_t G, groups, cpg, chunks;
    general_shape(n, group, G, groups, cpg, chunks);
    hipLaunchKernelGGL(general_dequantize_kernel, dim3(general_grid(chunks)), dim3(kGBlock), 0, s, codes, labels, params,
                       n, G, cpg, chunks, m, out);
    return launch_status();
}

}  // namespace bitsnap
