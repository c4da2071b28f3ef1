// quantize_cluster / dequantize_cluster for group lengths the one-wave-per-group kernels do not
// take: any even G and G = 0 (one group spanning the tensor, the paper's own formulation of
// Algorithm 2).  A group is cut into chunks of 4096 elements, one wavefront per chunk with the
// chunk in registers (the building blocks of cluster_wave.hpp), and Algorithm 2's steps become
// three passes over x with the per-group state in the workspace:
//   pass 1  per chunk: sum and, about the chunk's own mean, the sum of squared deviations
//           -> per slice of 256 chunks -> per group: mean, deviation (pairwise update formula), edges
//   pass 2  per chunk: labels (not stored), per-cluster min/max
//           -> per slice -> per group: (S, b), 255/S
//   pass 3  per chunk: labels again, codes; both stored
// x is read three times and 1.5 bytes per element are written: 13.5 bytes per element.  Chunk
// results are written out and combined in chunk order, so nothing depends on the order in which
// the waves run.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/bitsnap.h"
#include "cluster_general.hpp"
#include "cluster_wave.hpp"
#include "host_util.hpp"
#include "wave.hpp"

namespace bitsnap {

constexpr int kGBlock = 256;
constexpr int kGWaves = kGBlock / kWave;
constexpr int kGK = 16;                  // float4 per lane
constexpr int kGChunk = 256 * kGK;       // 4096 elements per wave

struct GroupState {  // one per group, in the workspace
    float mu, sigma;
    float2 coder[kMaxClusters];  // (b, 255/S)
};

struct ChunkStats {  // one per chunk, in the workspace
    double sum, dev;
};

struct ChunkRanges {  // one per chunk, in the workspace
    float mn[kMaxClusters], mx[kMaxClusters];
};

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

// A whole chunk whose first element is 16-byte aligned takes the vector loads and stores.
__device__ __forceinline__ bool chunk_is_full(const ChunkRef &r) { return r.len == kGChunk && (r.lo & 3) == 0; }

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

// ---- pass 1
__global__ __launch_bounds__(kGBlock) void wide_stats_kernel(const float *__restrict__ x, int64_t n, int64_t G,
                                                             int64_t chunks_per_group, int64_t chunks,
                                                             ChunkStats *__restrict__ stats)
{
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t c = (int64_t)blockIdx.x * kGWaves + wave;
    if (c >= chunks)
        return;
    const ChunkRef r = chunk_ref(c, n, G, chunks_per_group);
    double sum = 0.0, dev = 0.0;
    if (r.len > 0) {
        float4 v[kGK];
        if (chunk_is_full(r)) {
            load_elements<kGK, true>(x, r.lo, r.len, lane, v);
            wave_stats<kGK, true>(v, r.len, lane, sum, dev);
        } else {
            load_elements<kGK, false>(x, r.lo, r.len, lane, v);
            wave_stats<kGK, false>(v, r.len, lane, sum, dev);
        }
    }
    if (lane == 0) {
        stats[c].sum = sum;
        stats[c].dev = dev;
    }
}

// The statistics of the chunks are combined in two levels, slices of 256 chunks and then the
// group, each time with the pairwise update formula
//   sum = sum of the parts' sums,   dev = sum over parts of  dev_p + n_p * (mean_p - mean)^2
// (every term non-negative, nothing cancels), in a fixed association: a tensor-wide group of a
// 131 M-element tensor has 32000 chunks, too many for one workgroup to walk through.
constexpr int kGSlice = kGBlock;  // chunks per slice: one per thread

// Elements in chunks [c0, c1) of a group of g_len elements.
__device__ __forceinline__ double chunk_span_elems(int64_t c0, int64_t c1, int64_t g_len)
{
    const int64_t lo = c0 * kGChunk, hi = c1 * kGChunk;
    return (double)((hi < g_len ? hi : g_len) - lo);
}

// grid: groups * slices_per_group workgroups
__global__ __launch_bounds__(kGBlock) void wide_slice_stats_kernel(int64_t n, int64_t G, int64_t chunks_per_group,
                                                                   int64_t slices_per_group, int64_t groups,
                                                                   const ChunkStats *__restrict__ stats,
                                                                   ChunkStats *__restrict__ slice_stats)
{
    __shared__ double scratch[kGBlock / kWave];
    const int64_t g = blockIdx.x / slices_per_group, sl = blockIdx.x % slices_per_group;
    if (g >= groups)
        return;
    const int64_t g_lo = g * G;
    const int64_t g_len = (g_lo + G <= n) ? G : (n - g_lo);
    const int64_t nch = (g_len + kGChunk - 1) / kGChunk;
    const int64_t c = sl * kGSlice + threadIdx.x, c_end = (sl + 1) * kGSlice < nch ? (sl + 1) * kGSlice : nch;
    const bool have = c < nch;
    const ChunkStats mine = have ? stats[g * chunks_per_group + c] : ChunkStats{0.0, 0.0};
    const double sum = block_sum(mine.sum, scratch);
    double term = 0.0;
    if (have && sl * kGSlice < nch) {
        const double mean = sum / chunk_span_elems(sl * kGSlice, c_end, g_len);
        const double n_c = chunk_span_elems(c, c + 1, g_len);
        const double d = mine.sum / n_c - mean;
        term = mine.dev + n_c * d * d;
    }
    const double dev = block_sum(term, scratch);
    if (threadIdx.x == 0) {
        slice_stats[g * slices_per_group + sl].sum = sum;
        slice_stats[g * slices_per_group + sl].dev = dev;
    }
}

// One workgroup per group: slices -> mean, deviation -> mu, sigma (Algorithm 2 step 1), edges.
// Thread t takes slices t, t+256, ... in order, then the block tree.
__global__ __launch_bounds__(kGBlock) void wide_fit_kernel(int64_t n, int64_t G, int64_t slices_per_group, int64_t groups,
                                                           int m, const ChunkStats *__restrict__ slice_stats,
                                                           GroupState *gs, float *__restrict__ fit_out,
                                                           const float *__restrict__ fit_in, uint32_t *__restrict__ status)
{
    __shared__ double scratch[kGBlock / kWave];
    for (int64_t g = blockIdx.x; g < groups; g += gridDim.x) {
        const int64_t g_lo = g * G;
        const int64_t g_len = (g_lo + G <= n) ? G : (n - g_lo);
        const int64_t nch = (g_len + kGChunk - 1) / kGChunk;
        const int64_t nsl = (nch + kGSlice - 1) / kGSlice;
        const ChunkStats *ss = slice_stats + g * slices_per_group;
        double acc = 0.0;
        for (int64_t k = threadIdx.x; k < nsl; k += kGBlock)
            acc += ss[k].sum;
        const double mean = block_sum(acc, scratch) / (double)g_len;
        acc = 0.0;
        for (int64_t k = threadIdx.x; k < nsl; k += kGBlock) {
            const int64_t c_end = (k + 1) * kGSlice < nch ? (k + 1) * kGSlice : nch;
            const double n_k = chunk_span_elems(k * kGSlice, c_end, g_len);
            const double d = ss[k].sum / n_k - mean;
            acc += ss[k].dev + n_k * d * d;
        }
        const double dev = block_sum(acc, scratch);
        float mu = (float)mean;
        float sigma = (float)sqrt(dev / (double)g_len);
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
        if (fit_out && t >= 1 && t < m)  // the same expression as build_search
            fit_out[g * (m + 1) + 1 + t] = (float)__dadd_rn((double)mu, __dmul_rn((double)sigma, kZDev[m][t]));
        __syncthreads();
    }
}

// ---- pass 2
template <bool kFull>
__device__ __forceinline__ void chunk_ranges(const float *__restrict__ x, const ChunkRef &r, int m, float mu, float sigma,
                                             WaveShared &ws, int lane, float &mn, float &mx)
{
    float4 v[kGK];
    load_elements<kGK, kFull>(x, r.lo, r.len, lane, v);
    reset_ranges(ws, lane);
    float edge;
    const LabelSearch ls = build_search(mu, sigma, m, ws, lane, edge);
    uint32_t packed[(kGK + 1) / 2];
    label_pass<kGK, kFull, false, true>(v, r.lo, r.len, ls, ws, lane, nullptr, packed);
    reduce_ranges(ws, lane, mn, mx);
    wave_lds_sync();
}

__global__ __launch_bounds__(kGBlock) void wide_range_kernel(const float *__restrict__ x, int64_t n, int64_t G,
                                                             int64_t chunks_per_group, int64_t chunks, int m,
                                                             const GroupState *__restrict__ gs,
                                                             ChunkRanges *__restrict__ ranges)
{
    __shared__ WaveShared shared[kGWaves];
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t c = (int64_t)blockIdx.x * kGWaves + wave;
    if (c >= chunks)
        return;
    const ChunkRef r = chunk_ref(c, n, G, chunks_per_group);
    float mn = INFINITY, mx = -INFINITY;
    if (r.len > 0) {
        const float mu = gs[r.group].mu, sigma = gs[r.group].sigma;
        if (chunk_is_full(r))
            chunk_ranges<true>(x, r, m, mu, sigma, shared[wave], lane, mn, mx);
        else
            chunk_ranges<false>(x, r, m, mu, sigma, shared[wave], lane, mn, mx);
    }
    if (lane < kMaxClusters) {
        ranges[c].mn[lane] = mn;
        ranges[c].mx[lane] = mx;
    }
}

// Min / max of every cluster over `count` rows of 32 floats (16 minima, 16 maxima), by one
// workgroup: thread t looks at column t % 32 of rows t/32, t/32 + 8, ...; the result is left in
// part[0..32).
__device__ __forceinline__ void reduce_range_rows(const float *__restrict__ rows, int64_t count, float *part)
{
    const int col = threadIdx.x & 31, row = threadIdx.x >> 5;
    const bool is_min = col < kMaxClusters;
    float acc = is_min ? INFINITY : -INFINITY;
    for (int64_t c = row; c < count; c += kGBlock / 32) {
        const float t = rows[c * 32 + col];
        acc = is_min ? fminf(acc, t) : fmaxf(acc, t);
    }
    __syncthreads();
    part[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x < 32) {
        for (int k = 1; k < kGBlock / 32; ++k) {
            const float t = part[k * 32 + col];
            acc = is_min ? fminf(acc, t) : fmaxf(acc, t);
        }
    }
    __syncthreads();
    if (threadIdx.x < 32)
        part[threadIdx.x] = acc;
    __syncthreads();
}

// grid: groups * slices_per_group workgroups, each over the (up to) 256 chunks of its slice
__global__ __launch_bounds__(kGBlock) void wide_slice_ranges_kernel(int64_t n, int64_t G, int64_t chunks_per_group,
                                                                    int64_t slices_per_group, int64_t groups,
                                                                    const ChunkRanges *__restrict__ ranges,
                                                                    ChunkRanges *__restrict__ slice_ranges)
{
    __shared__ float part[kGBlock];
    const int64_t g = blockIdx.x / slices_per_group, sl = blockIdx.x % slices_per_group;
    if (g >= groups)
        return;
    const int64_t g_lo = g * G;
    const int64_t g_len = (g_lo + G <= n) ? G : (n - g_lo);
    const int64_t nch = (g_len + kGChunk - 1) / kGChunk;
    const int64_t c0 = sl * kGSlice;
    const int64_t cnt = c0 >= nch ? 0 : (nch - c0 < kGSlice ? nch - c0 : kGSlice);
    reduce_range_rows(reinterpret_cast<const float *>(ranges + g * chunks_per_group + c0), cnt, part);
    if (threadIdx.x < 32)
        reinterpret_cast<float *>(slice_ranges + g * slices_per_group + sl)[threadIdx.x] = part[threadIdx.x];
}

// One workgroup per group: slices -> min / max of every cluster -> (S, b), 255/S (Algorithm 2 step 4).
__global__ __launch_bounds__(kGBlock) void wide_params_kernel(int64_t n, int64_t G, int64_t slices_per_group,
                                                              int64_t groups, int m,
                                                              const ChunkRanges *__restrict__ slice_ranges, GroupState *gs,
                                                              float *__restrict__ params)
{
    __shared__ float part[kGBlock];
    for (int64_t g = blockIdx.x; g < groups; g += gridDim.x) {
        const int64_t g_lo = g * G;
        const int64_t g_len = (g_lo + G <= n) ? G : (n - g_lo);
        const int64_t nch = (g_len + kGChunk - 1) / kGChunk;
        const int64_t nsl = (nch + kGSlice - 1) / kGSlice;
        reduce_range_rows(reinterpret_cast<const float *>(slice_ranges + g * slices_per_group), nsl, part);
        if (threadIdx.x < kMaxClusters) {
            float S, b, inv;
            cluster_coder(part[threadIdx.x], part[kMaxClusters + threadIdx.x], S, b, inv);
            gs[g].coder[threadIdx.x] = make_float2(b, inv);
            if ((int)threadIdx.x < m)
                *reinterpret_cast<float2 *>(params + (g * m + threadIdx.x) * 2) = make_float2(S, b);
        }
    }
}

// ---- pass 3
template <bool kFull>
__device__ __forceinline__ void chunk_codes(const float *__restrict__ x, const ChunkRef &r, int m, const GroupState &st,
                                            WaveShared &ws, int lane, uint8_t *__restrict__ labels,
                                            uint8_t *__restrict__ codes)
{
    float4 v[kGK];
    load_elements<kGK, kFull>(x, r.lo, r.len, lane, v);
    if (lane < kMaxClusters)
        ws.coder[lane] = st.coder[lane];
    float edge;
    const LabelSearch ls = build_search(st.mu, st.sigma, m, ws, lane, edge);
    uint32_t packed[(kGK + 1) / 2];
    label_pass<kGK, kFull, true, false>(v, r.lo, r.len, ls, ws, lane, labels, packed);
    code_pass<kGK, kFull>(v, r.lo, r.len, packed, ws, lane, codes);
}

__global__ __launch_bounds__(kGBlock) void wide_code_kernel(const float *__restrict__ x, int64_t n, int64_t G,
                                                            int64_t chunks_per_group, int64_t chunks, int m,
                                                            const GroupState *__restrict__ gs, uint8_t *__restrict__ labels,
                                                            uint8_t *__restrict__ codes)
{
    __shared__ WaveShared shared[kGWaves];
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t c = (int64_t)blockIdx.x * kGWaves + wave;
    if (c >= chunks)
        return;
    const ChunkRef r = chunk_ref(c, n, G, chunks_per_group);
    if (r.len == 0)
        return;
    if (chunk_is_full(r))
        chunk_codes<true>(x, r, m, gs[r.group], shared[wave], lane, labels, codes);
    else
        chunk_codes<false>(x, r, m, gs[r.group], shared[wave], lane, labels, codes);
}

__global__ __launch_bounds__(kGBlock) void wide_dequantize_kernel(const uint8_t *__restrict__ codes,
                                                                  const uint8_t *__restrict__ labels,
                                                                  const float *__restrict__ params, int64_t n, int64_t G,
                                                                  int64_t chunks_per_group, int64_t chunks, int m,
                                                                  float *__restrict__ out)
{
    __shared__ float2 coder[kGWaves][kMaxClusters];
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t c = (int64_t)blockIdx.x * kGWaves + wave;
    if (c >= chunks)
        return;
    const ChunkRef r = chunk_ref(c, n, G, chunks_per_group);
    if (r.len == 0)
        return;
    dequantize_group<kGK>(codes, labels, params, r.lo, r.len, (r.lo & 3) == 0, m, r.group, out, coder[wave], lane);
}

static void general_shape(int64_t n, int64_t group, int64_t &G, int64_t &groups, int64_t &cpg, int64_t &chunks,
                          int64_t &spg)
{
    G = (group <= 0 || group > n) ? n : group;
    groups = (n + G - 1) / G;
    cpg = (G + kGChunk - 1) / kGChunk;
    chunks = groups * cpg;
    spg = (cpg + kGSlice - 1) / kGSlice;
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
    int64_t G, groups, cpg, chunks, spg;
    general_shape(n, group, G, groups, cpg, chunks, spg);
    const size_t bytes = (size_t)groups * sizeof(GroupState) +
                         (size_t)(chunks + groups * spg) * (sizeof(ChunkStats) + sizeof(ChunkRanges));
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
    int64_t G, groups, cpg, chunks, spg;
    general_shape(n, group, G, groups, cpg, chunks, spg);
    const int64_t blocks = (chunks + kGWaves - 1) / kGWaves, slices = groups * spg;
    if (blocks > 0x7FFFFFFF || slices > 0x7FFFFFFF)
        return BITSNAP_E_SIZE;
    static_assert(sizeof(GroupState) % 8 == 0 && sizeof(ChunkStats) % 8 == 0, "workspace parts stay 8-byte aligned");
    GroupState *gs = reinterpret_cast<GroupState *>(workspace);
    ChunkStats *stats = reinterpret_cast<ChunkStats *>(gs + groups);
    ChunkStats *slice_stats = stats + chunks;
    ChunkRanges *ranges = reinterpret_cast<ChunkRanges *>(slice_stats + slices);
    ChunkRanges *slice_ranges = ranges + chunks;
    const dim3 block(kGBlock), cgrid((unsigned)blocks), sgrid((unsigned)slices), ggrid(general_grid(groups));
    hipLaunchKernelGGL(wide_stats_kernel, cgrid, block, 0, s, x, n, G, cpg, chunks, stats);
    hipLaunchKernelGGL(wide_slice_stats_kernel, sgrid, block, 0, s, n, G, cpg, spg, groups, stats, slice_stats);
    hipLaunchKernelGGL(wide_fit_kernel, ggrid, block, 0, s, n, G, spg, groups, m, slice_stats, gs, fit_out, fit_in,
                       status);
    hipLaunchKernelGGL(wide_range_kernel, cgrid, block, 0, s, x, n, G, cpg, chunks, m, gs, ranges);
    hipLaunchKernelGGL(wide_slice_ranges_kernel, sgrid, block, 0, s, n, G, cpg, spg, groups, ranges, slice_ranges);
    hipLaunchKernelGGL(wide_params_kernel, ggrid, block, 0, s, n, G, spg, groups, m, slice_ranges, gs, params);
    hipLaunchKernelGGL(wide_code_kernel, cgrid, block, 0, s, x, n, G, cpg, chunks, m, gs, labels, codes);
    return launch_status();
}

int cluster_general_dequantize(const uint8_t *codes, const uint8_t *labels, const float *params, int64_t n,
                               int64_t group, int m, float *out, hipStream_t s)
{
    int64_t G, groups, cpg, chunks, spg;
    general_shape(n, group, G, groups, cpg, chunks, spg);
    const int64_t blocks = (chunks + kGWaves - 1) / kGWaves;
    if (blocks > 0x7FFFFFFF)
        return BITSNAP_E_SIZE;
    hipLaunchKernelGGL(wide_dequantize_kernel, dim3((unsigned)blocks), dim3(kGBlock), 0, s, codes, labels, params, n, G,
                       cpg, chunks, m, out);
    return launch_status();
}

}  // namespace bitsnap
