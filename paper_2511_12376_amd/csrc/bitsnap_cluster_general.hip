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
//
// Format variants (a table for Q^map, cluster-major codes; see cluster_variants.hpp).  The table
// only changes how pass 3 turns (x-b)/S into a code.  Cluster-major codes of a wide group are a
// stable 16-way partition across all its chunks: pass 2 also leaves the number of members of
// every cluster per chunk, the two reduction levels turn these into exclusive prefix sums
// (chunk within slice, slice within group, cluster within group), and pass 3 partitions its
// chunk inside the wave and copies each cluster's run of codes to
//   group start + cluster base + slice base + chunk offset.
// Dequantisation rebuilds the same sums from the stored labels and collects the runs again.
//
// Every kernel takes its chunks, slices and groups from a "source": one tensor with any group
// length, or a list of tensors with one group each, numbered across the list, so that a pass
// over a whole checkpoint state is one launch.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/bitsnap.h"
#include "cluster_general.hpp"
#include "cluster_items.hpp"
#include "cluster_variants.hpp"
#include "cluster_wave.hpp"
#include "host_util.hpp"
#include "wave.hpp"

namespace bitsnap {

constexpr int kGBlock = 256;
constexpr int kGWaves = kGBlock / kWave;
// The three passes that stream over x (statistics, ranges, codes) run one wave per workgroup, as the one-wave
// quantiser does: their waves share nothing, and single-wave workgroups stream reads best on this chip.
constexpr int kStreamBlock = 64;
constexpr int kStreamWaves = kStreamBlock / kWave;
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

struct ChunkCounts {  // one per chunk, per slice and per group, in the workspace (cluster-major codes only)
    uint32_t cnt[kMaxClusters];
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

constexpr int kGSlice = kGBlock;  // chunks per slice of the two-level reductions: one per thread

// One tensor as the kernels see it, and where its chunks, slices and groups sit in the workspace arrays.
struct WideTensor {
    void *values;  // x (quantise) or out (dequantise)
    uint8_t *codes, *labels;
    float *params, *fit_out;
    const float *fit_in;
    int64_t n, G, cpg, spg, groups;     // elements, group length, chunks per group, slices per group, groups
    int64_t chunk0, slice0, group0;     // index of its first chunk / slice / group in the workspace arrays
};

__host__ __device__ inline WideTensor wide_tensor(void *values, uint8_t *codes, uint8_t *labels, float *params,
                                                  float *fit_out, const float *fit_in, int64_t n, int64_t group)
{
    WideTensor t;
    t.values = values, t.codes = codes, t.labels = labels, t.params = params, t.fit_out = fit_out, t.fit_in = fit_in;
    t.n = n;
    t.G = (group <= 0 || group > n) ? n : group;
    t.groups = (n + t.G - 1) / t.G;
    t.cpg = (t.G + kGChunk - 1) / kGChunk;
    t.spg = (t.cpg + kGSlice - 1) / kGSlice;
    t.chunk0 = t.slice0 = t.group0 = 0;
    return t;
}

// Where a kernel's work items come from: one tensor (any group length), or a list of tensors with
// one group each (the batched form of group = 0).  Work is numbered across the whole source:
// chunk gc, slice gs, group gg; the of_* calls name the tensor and the index inside it.
struct OneTensor {
    WideTensor t;
    __device__ int64_t chunks() const { return t.groups * t.cpg; }
    __device__ int64_t slices() const { return t.groups * t.spg; }
    __device__ int64_t groups() const { return t.groups; }
    __device__ WideTensor of_chunk(int64_t gc, int64_t &c) const
    {
        c = gc;
        return t;
    }
    __device__ WideTensor of_slice(int64_t gs, int64_t &g, int64_t &sl) const
    {
        g = gs / t.spg, sl = gs % t.spg;
        return t;
    }
    __device__ WideTensor of_group(int64_t gg, int64_t &g) const
    {
        g = gg;
        return t;
    }
};

struct TensorList {
    const bitsnap_cluster_item *items;  // first_group counts chunks here
    int64_t count, total_chunks;
    const int64_t *slice0;              // [count + 1], written by wide_list_slices_kernel; the last entry is the total
    __device__ int64_t chunks() const { return total_chunks; }
    __device__ int64_t slices() const { return slice0[count]; }
    __device__ int64_t groups() const { return count; }
    __device__ WideTensor tensor(int64_t i) const
    {
        const bitsnap_cluster_item &it = items[i];
        WideTensor t = wide_tensor(it.values, it.codes, it.labels, it.params, it.fit_out, it.fit_in, it.n, 0);
        t.chunk0 = it.first_group, t.slice0 = slice0 ? slice0[i] : 0, t.group0 = i;  // no slice list where no reduction runs
        return t;
    }
    __device__ WideTensor of_chunk(int64_t gc, int64_t &c) const
    {
        const WideTensor t = tensor(find_item(items, count, gc));
        c = gc - t.chunk0;
        return t;
    }
    __device__ WideTensor of_slice(int64_t gs, int64_t &g, int64_t &sl) const
    {
        int64_t lo = 0, hi = count - 1;  // the last tensor whose first slice is <= gs
        while (lo < hi) {
            const int64_t mid = (lo + hi + 1) >> 1;
            if (slice0[mid] <= gs)
                lo = mid;
            else
                hi = mid - 1;
        }
        const WideTensor t = tensor(lo);
        g = 0, sl = gs - t.slice0;
        return t;
    }
    __device__ WideTensor of_group(int64_t gg, int64_t &g) const
    {
        g = 0;
        return tensor(gg);
    }
};

// The workspace, cut up.
struct WideSpace {
    GroupState *gs;
    ChunkStats *stats, *slice_stats;
    ChunkRanges *ranges, *slice_ranges;
    ChunkCounts *counts, *slice_counts, *cluster_base;  // cluster-major codes only
};

// slice0[i] = slices of all tensors before i (one group each), slice0[count] = all of them.  One workgroup.
__global__ __launch_bounds__(kGBlock) void wide_list_slices_kernel(const bitsnap_cluster_item *__restrict__ items,
                                                                   int64_t count, int64_t *__restrict__ slice0)
{
    __shared__ uint32_t wave_total[kGWaves];
    __shared__ int64_t running;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    if (threadIdx.x == 0)
        running = 0;
    __syncthreads();
    for (int64_t base = 0; base < count; base += kGBlock) {
        const int64_t i = base + threadIdx.x;
        uint32_t v = 0;
        if (i < count) {
            const int64_t chunks = (items[i].n + kGChunk - 1) / kGChunk;
            v = (uint32_t)((chunks + kGSlice - 1) / kGSlice);
        }
        const uint32_t inc = wave_inclusive_add(v);
        if (lane == kWave - 1)
            wave_total[wave] = inc;
        __syncthreads();
        uint32_t before = 0;
        for (int w = 0; w < wave; ++w)
            before += wave_total[w];
        const int64_t start = running;
        if (i < count)
            slice0[i] = start + before + inc - v;
        __syncthreads();
        if (threadIdx.x == kGBlock - 1)
            running = start + before + inc;
        __syncthreads();
    }
    if (threadIdx.x == 0)
        slice0[count] = running;
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

// ---- pass 1
template <typename Src>
__global__ __launch_bounds__(kStreamBlock) void wide_stats_kernel(Src src, WideSpace sp)
{
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t gc = (int64_t)blockIdx.x * kStreamWaves + wave;
    if (gc >= src.chunks())
        return;
    int64_t c;
    const WideTensor t = src.of_chunk(gc, c);
    const float *x = (const float *)t.values;
    const ChunkRef r = chunk_ref(c, t.n, t.G, t.cpg);
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
        sp.stats[t.chunk0 + c].sum = sum;
        sp.stats[t.chunk0 + c].dev = dev;
    }
}

// The statistics of the chunks are combined in two levels, slices of 256 chunks and then the
// group, each time with the pairwise update formula
//   sum = sum of the parts' sums,   dev = sum over parts of  dev_p + n_p * (mean_p - mean)^2
// (every term non-negative, nothing cancels), in a fixed association: a tensor-wide group of a
// 131 M-element tensor has 32000 chunks, too many for one workgroup to walk through.
// Elements in chunks [c0, c1) of a group of g_len elements.
__device__ __forceinline__ double chunk_span_elems(int64_t c0, int64_t c1, int64_t g_len)
{
    const int64_t lo = c0 * kGChunk, hi = c1 * kGChunk;
    return (double)((hi < g_len ? hi : g_len) - lo);
}

// The elements of group g of a tensor.
__device__ __forceinline__ int64_t group_len(const WideTensor &t, int64_t g)
{
    const int64_t g_lo = g * t.G;
    return (g_lo + t.G <= t.n) ? t.G : (t.n - g_lo);
}

// grid: one workgroup per slice (a list of tensors may be launched with more: they leave at once)
template <typename Src>
__global__ __launch_bounds__(kGBlock) void wide_slice_stats_kernel(Src src, WideSpace sp)
{
    __shared__ double scratch[kGBlock / kWave];
    if ((int64_t)blockIdx.x >= src.slices())
        return;
    int64_t g, sl;
    const WideTensor t = src.of_slice(blockIdx.x, g, sl);
    const int64_t g_len = group_len(t, g);
    const int64_t nch = (g_len + kGChunk - 1) / kGChunk;
    const int64_t c = sl * kGSlice + threadIdx.x, c_end = (sl + 1) * kGSlice < nch ? (sl + 1) * kGSlice : nch;
    const bool have = c < nch;
    const ChunkStats mine = have ? sp.stats[t.chunk0 + g * t.cpg + c] : ChunkStats{0.0, 0.0};
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
        sp.slice_stats[t.slice0 + g * t.spg + sl].sum = sum;
        sp.slice_stats[t.slice0 + g * t.spg + sl].dev = dev;
    }
}

// One workgroup per group: slices -> mean, deviation -> mu, sigma (Algorithm 2 step 1), edges.
// Thread t takes slices t, t+256, ... in order, then the block tree.
template <typename Src>
__global__ __launch_bounds__(kGBlock) void wide_fit_kernel(Src src, WideSpace sp, int m, uint32_t *__restrict__ status)
{
    __shared__ double scratch[kGBlock / kWave];
    for (int64_t gg = blockIdx.x; gg < src.groups(); gg += gridDim.x) {
        int64_t g;
        const WideTensor t = src.of_group(gg, g);
        float *fit_out = t.fit_out;
        const float *fit_in = t.fit_in;
        GroupState *gs = sp.gs + t.group0;
        const int64_t g_len = group_len(t, g);
        const int64_t nch = (g_len + kGChunk - 1) / kGChunk;
        const int64_t nsl = (nch + kGSlice - 1) / kGSlice;
        const ChunkStats *ss = sp.slice_stats + t.slice0 + g * t.spg;
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
        const int tid = threadIdx.x;
        if (tid == 0) {
            gs[g].mu = mu;
            gs[g].sigma = sigma;
            if (status && !(isfinite(mu) && isfinite(sigma)))
                atomicOr(status, 1u);
            if (fit_out) {
                fit_out[g * (m + 1) + 0] = mu;
                fit_out[g * (m + 1) + 1] = sigma;
            }
        }
        if (fit_out && tid >= 1 && tid < m)  // the same expression as build_search
            fit_out[g * (m + 1) + 1 + tid] = (float)__dadd_rn((double)mu, __dmul_rn((double)sigma, kZDev[m][tid]));
        __syncthreads();
    }
}

// Members of every cluster among the wave's elements: lane c < 16 (every lane with lane % 16 == c)
// returns the count of cluster c.  label(k, j) = the label of element k*256 + lane*4 + j;
// `counters` is a [16][64] LDS table, one private column per lane.
template <int K, bool kFull, typename Label>
__device__ __forceinline__ uint32_t wave_label_counts(Label label, int len, int lane, uint32_t *counters)
{
#pragma unroll
    for (int c = 0; c < kMaxClusters; ++c)
        counters[c * kWave + lane] = 0;
#pragma unroll
    for (int k = 0; k < K; ++k)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (kFull || k * 256 + lane * 4 + j < len)
                lds_fetch_add(&counters[label(k, j) * kWave + lane], 1u);
    wave_lds_sync();
    const int row = lane & 15, quarter = lane >> 4;
    uint32_t v = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j)
        v += counters[row * kWave + quarter * 16 + ((j + lane) & 15)];
    v += (uint32_t)__shfl_xor((int)v, 16, kWave);
    v += (uint32_t)__shfl_xor((int)v, 32, kWave);
    wave_lds_sync();
    return v;
}

// ---- pass 2
template <bool kFull, bool kCounts>
__device__ __forceinline__ void chunk_ranges(const float *__restrict__ x, const ChunkRef &r, int m, float mu, float sigma,
                                             WaveShared &ws, uint32_t *counters, int lane, float &mn, float &mx,
                                             uint32_t &count)
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
    if (kCounts)
        count = wave_label_counts<kGK, kFull>(
            [&](int k, int j) { return (packed[k >> 1] >> (16 * (k & 1) + 4 * j)) & 15u; }, r.len, lane, counters);
}

template <typename Src, bool kCounts>
__global__ __launch_bounds__(kStreamBlock) void wide_range_kernel(Src src, WideSpace sp, int m)
{
    __shared__ WaveShared shared[kStreamWaves];
    __shared__ uint32_t counters[kCounts ? kStreamWaves : 1][kMaxClusters * kWave];
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t gc = (int64_t)blockIdx.x * kStreamWaves + wave;
    if (gc >= src.chunks())
        return;
    int64_t c;
    const WideTensor t = src.of_chunk(gc, c);
    const float *x = (const float *)t.values;
    const ChunkRef r = chunk_ref(c, t.n, t.G, t.cpg);
    float mn = INFINITY, mx = -INFINITY;
    uint32_t count = 0;
    if (r.len > 0) {
        const float mu = sp.gs[t.group0 + r.group].mu, sigma = sp.gs[t.group0 + r.group].sigma;
        uint32_t *col = counters[kCounts ? wave : 0];
        if (chunk_is_full(r))
            chunk_ranges<true, kCounts>(x, r, m, mu, sigma, shared[wave], col, lane, mn, mx, count);
        else
            chunk_ranges<false, kCounts>(x, r, m, mu, sigma, shared[wave], col, lane, mn, mx, count);
    }
    if (lane < kMaxClusters) {
        sp.ranges[t.chunk0 + c].mn[lane] = mn;
        sp.ranges[t.chunk0 + c].mx[lane] = mx;
        if (kCounts)
            sp.counts[t.chunk0 + c].cnt[lane] = count;
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

// The per-chunk member counts of one slice (thread t holds chunk t of `cnt` chunks) become, in
// place, the members in earlier chunks of the slice; *total receives the slice's own counts.
// Called by a whole workgroup.
__device__ __forceinline__ void slice_counts_scan(ChunkCounts *__restrict__ chunk, int64_t cnt, ChunkCounts *__restrict__ total)
{
    __shared__ uint32_t wave_total[kGWaves][kMaxClusters];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const bool have = (int64_t)threadIdx.x < cnt;
    uint32_t v[kMaxClusters], inc[kMaxClusters];
#pragma unroll
    for (int c = 0; c < kMaxClusters; ++c) {
        v[c] = have ? chunk[threadIdx.x].cnt[c] : 0u;
        inc[c] = wave_inclusive_add(v[c]);
        if (lane == kWave - 1)
            wave_total[wave][c] = inc[c];
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kMaxClusters; ++c) {
        uint32_t before = 0;
        for (int w = 0; w < wave; ++w)
            before += wave_total[w][c];
        if (have)
            chunk[threadIdx.x].cnt[c] = before + inc[c] - v[c];
        if (threadIdx.x == kGBlock - 1)
            total->cnt[c] = before + inc[c];
    }
}

// The per-slice member counts of one group (`nsl` slices) become, in place, the members in
// earlier slices; *base receives, per cluster, the members of all lower clusters of the group.
// Called by a whole workgroup; thread t works on cluster t % 16 and on every 16th slice.
__device__ __forceinline__ void group_counts_scan(ChunkCounts *__restrict__ slice, int64_t nsl, ChunkCounts *__restrict__ base)
{
    __shared__ uint32_t tile[16][kMaxClusters];
    __shared__ uint32_t running[kMaxClusters];
    const int c = threadIdx.x & 15, s = threadIdx.x >> 4;
    if (threadIdx.x < kMaxClusters)
        running[threadIdx.x] = 0;
    __syncthreads();
    for (int64_t sl0 = 0; sl0 < nsl; sl0 += 16) {
        const int64_t sl = sl0 + s;
        const uint32_t v = sl < nsl ? slice[sl].cnt[c] : 0u;
        tile[s][c] = v;
        __syncthreads();
        uint32_t before = running[c];
        for (int k = 0; k < s; ++k)
            before += tile[k][c];
        if (sl < nsl)
            slice[sl].cnt[c] = before;
        __syncthreads();
        if (s == 15)
            running[c] = before + v;
        __syncthreads();
    }
    if (threadIdx.x < kMaxClusters) {
        uint32_t lower = 0;
        for (int k = 0; k < (int)threadIdx.x; ++k)
            lower += running[k];
        base->cnt[threadIdx.x] = lower;
    }
    __syncthreads();
}

// grid: one workgroup per slice, each over the (up to) 256 chunks of its slice
template <typename Src, bool kRanges, bool kCounts>
__global__ __launch_bounds__(kGBlock) void wide_slice_kernel(Src src, WideSpace sp)
{
    __shared__ float part[kGBlock];
    if ((int64_t)blockIdx.x >= src.slices())
        return;
    int64_t g, sl;
    const WideTensor t = src.of_slice(blockIdx.x, g, sl);
    const int64_t nch = (group_len(t, g) + kGChunk - 1) / kGChunk;
    const int64_t c0 = sl * kGSlice;
    const int64_t cnt = c0 >= nch ? 0 : (nch - c0 < kGSlice ? nch - c0 : kGSlice);
    const int64_t chunk = t.chunk0 + g * t.cpg + c0, slice = t.slice0 + g * t.spg + sl;
    if (kRanges) {
        reduce_range_rows(reinterpret_cast<const float *>(sp.ranges + chunk), cnt, part);
        if (threadIdx.x < 32)
            reinterpret_cast<float *>(sp.slice_ranges + slice)[threadIdx.x] = part[threadIdx.x];
    }
    if (kCounts)
        slice_counts_scan(sp.counts + chunk, cnt, sp.slice_counts + slice);
}

// One workgroup per group: slices -> min / max of every cluster -> (S, b), 255/S (Algorithm 2 step 4);
// with kCounts also the slices' and clusters' places in the cluster-major arrangement.
template <typename Src, bool kRanges, bool kCounts>
__global__ __launch_bounds__(kGBlock) void wide_group_kernel(Src src, WideSpace sp, int m)
{
    __shared__ float part[kGBlock];
    for (int64_t gg = blockIdx.x; gg < src.groups(); gg += gridDim.x) {
        int64_t g;
        const WideTensor t = src.of_group(gg, g);
        const int64_t nch = (group_len(t, g) + kGChunk - 1) / kGChunk;
        const int64_t nsl = (nch + kGSlice - 1) / kGSlice;
        const int64_t slice = t.slice0 + g * t.spg;
        if (kRanges) {
            reduce_range_rows(reinterpret_cast<const float *>(sp.slice_ranges + slice), nsl, part);
            if (threadIdx.x < kMaxClusters) {
                float S, b, inv;
                cluster_coder(part[threadIdx.x], part[kMaxClusters + threadIdx.x], S, b, inv);
                sp.gs[t.group0 + g].coder[threadIdx.x] = make_float2(b, inv);
                if ((int)threadIdx.x < m)
                    *reinterpret_cast<float2 *>(t.params + (g * m + threadIdx.x) * 2) = make_float2(S, b);
            }
        }
        if (kCounts)
            group_counts_scan(sp.slice_counts + slice, nsl, sp.cluster_base + t.group0 + g);
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

template <typename Src>
__global__ __launch_bounds__(kStreamBlock) void wide_code_kernel(Src src, WideSpace sp, int m)
{
    __shared__ WaveShared shared[kStreamWaves];
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t gc = (int64_t)blockIdx.x * kStreamWaves + wave;
    if (gc >= src.chunks())
        return;
    int64_t c;
    const WideTensor t = src.of_chunk(gc, c);
    const ChunkRef r = chunk_ref(c, t.n, t.G, t.cpg);
    if (r.len == 0)
        return;
    const GroupState &st = sp.gs[t.group0 + r.group];
    if (chunk_is_full(r))
        chunk_codes<true>((const float *)t.values, r, m, st, shared[wave], lane, t.labels, t.codes);
    else
        chunk_codes<false>((const float *)t.values, r, m, st, shared[wave], lane, t.labels, t.codes);
}

template <typename Src>
__global__ __launch_bounds__(kGBlock) void wide_dequantize_kernel(Src src, int m)
{
    __shared__ float2 coder[kGWaves][kMaxClusters];
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t gc = (int64_t)blockIdx.x * kGWaves + wave;
    if (gc >= src.chunks())
        return;
    int64_t c;
    const WideTensor t = src.of_chunk(gc, c);
    const ChunkRef r = chunk_ref(c, t.n, t.G, t.cpg);
    if (r.len == 0)
        return;
    dequantize_group<kGK>(t.codes, t.labels, t.params, r.lo, r.len, (r.lo & 3) == 0, m, r.group, (float *)t.values,
                          coder[wave], lane);
}

// ---- format variants: pass 3 and the dequantiser with a table and / or cluster-major codes

// Where the chunk's run of cluster `lane` (< 16) starts, relative to the group's first code.
__device__ __forceinline__ uint32_t segment_dest(const WideSpace &sp, const WideTensor &t, int64_t c, int64_t group, int lane)
{
    if (lane >= kMaxClusters)
        return 0;
    const int64_t sl = (c % t.cpg) / kGSlice;
    return sp.cluster_base[t.group0 + group].cnt[lane] + sp.slice_counts[t.slice0 + group * t.spg + sl].cnt[lane] +
           sp.counts[t.chunk0 + c].cnt[lane];
}

template <bool kFull, bool kTable, bool kMajor>
__device__ __forceinline__ void chunk_codes_ex(const float *__restrict__ x, const ChunkRef &r, int m, const GroupState &st,
                                               const float *__restrict__ params, int64_t g_lo, int64_t g_len, uint32_t dest,
                                               WaveShared &ws, const TableShared &table, int lane,
                                               uint8_t *__restrict__ labels, uint8_t *__restrict__ codes)
{
    float4 v[kGK];
    load_elements<kGK, kFull>(x, r.lo, r.len, lane, v);
    if (lane < kMaxClusters) {
        float2 coder = st.coder[lane];  // (b, 255/S)
        if (kTable) {
            // (b, 1/S) from the stored S, with the same rule for a range that cannot be coded
            const float S = lane < m ? global_ptr(params)[(r.group * m + lane) * 2] : 0.0f;
            float inv = S > 0.0f ? __fdiv_rn(1.0f, S) : 0.0f;
            if (!isfinite(inv))
                inv = 0.0f;
            coder.y = inv;
        }
        ws.coder[lane] = coder;
    }
    float edge;
    const LabelSearch ls = build_search(st.mu, st.sigma, m, ws, lane, edge);
    uint32_t packed[(kGK + 1) / 2];
    label_pass<kGK, kFull, true, false>(v, r.lo, r.len, ls, ws, lane, labels, packed);
    uint32_t c4[kGK];
    codes_to_registers<kGK, kTable>(v, packed, ws, table, c4);
    if (!kMajor) {
        store_codes<kGK, kFull>(c4, r.lo, r.len, lane, codes);
        wave_lds_sync();
        return;
    }
    const MajorView mv = major_view(ws);
    uint16_t *l16 = (uint16_t *)mv.labels;
#pragma unroll
    for (int k = 0; k < kGK; ++k) {
        mv.bytes[k * kWave + lane] = c4[k];
        l16[k * kWave + lane] = (uint16_t)(packed[k >> 1] >> (16 * (k & 1)));
    }
    wave_lds_sync();
    uint32_t start;
    to_cluster_major<kGK, kFull>(mv, r.len, lane, start);
    // every cluster's run of the chunk goes to its place in the group's arrangement
    const uint8_t *b8 = (const uint8_t *)mv.bytes;
#pragma unroll
    for (int cl = 0; cl < kMaxClusters; ++cl) {
        const uint32_t s0 = read_lane(start, cl), s1 = read_lane(start, cl + 1);  // lane 16 holds len
        const uint32_t d = read_lane(dest, cl);
        for (uint32_t i = (uint32_t)lane; i < s1 - s0; i += kWave)
            if ((int64_t)d + i < g_len)  // holds whenever the counts are consistent; keeps any store inside the group
                global_ptr(codes)[g_lo + d + i] = b8[s0 + i];
    }
    wave_lds_sync();
}

template <typename Src, bool kTable, bool kMajor>
__global__ __launch_bounds__(kGBlock, 3) void wide_code_ex_kernel(Src src, WideSpace sp, int m, const float *__restrict__ qmap)
{
    __shared__ WaveShared shared[kGWaves];
    __shared__ TableShared table;
    if (kTable)
        load_table(table, qmap);
    // no workgroup barrier from here on
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t chunks = src.chunks();
    for (int64_t gc = (int64_t)blockIdx.x * kGWaves + wave; gc < chunks; gc += (int64_t)gridDim.x * kGWaves) {
        int64_t c;
        const WideTensor t = src.of_chunk(gc, c);
        const ChunkRef r = chunk_ref(c, t.n, t.G, t.cpg);
        if (r.len == 0)
            continue;
        const int64_t g_lo = r.group * t.G;
        const int64_t g_len = group_len(t, r.group);
        const uint32_t dest = kMajor ? segment_dest(sp, t, c, r.group, lane) : 0u;
        const GroupState &st = sp.gs[t.group0 + r.group];
        if (chunk_is_full(r))
            chunk_codes_ex<true, kTable, kMajor>((const float *)t.values, r, m, st, t.params, g_lo, g_len, dest, shared[wave],
                                                 table, lane, t.labels, t.codes);
        else
            chunk_codes_ex<false, kTable, kMajor>((const float *)t.values, r, m, st, t.params, g_lo, g_len, dest, shared[wave],
                                                  table, lane, t.labels, t.codes);
    }
}

// Labels of a chunk as stored (two per byte), four per float4 position: l4[k] = elements
// k*256 + lane*4 .. + 3.  `aligned`: the chunk starts at a multiple of 4 elements.
__device__ __forceinline__ void load_chunk_labels(const uint8_t *__restrict__ labels, int64_t lo, int len, bool aligned,
                                                  int lane, uint32_t (&l4)[kGK])
{
#pragma unroll
    for (int k = 0; k < kGK; ++k) {
        const int off = k * 256 + lane * 4;
        l4[k] = 0;
        if (aligned && off + 3 < len) {
            l4[k] = __builtin_nontemporal_load((const BITSNAP_GLOBAL uint16_t *)(global_ptr(labels) + ((lo + off) >> 1)));
        } else {
            for (int j = 0; j < 4; ++j)
                if (off + j < len)
                    l4[k] |= (uint32_t)((global_ptr(labels)[(lo + off + j) >> 1] >> (4 * ((lo + off + j) & 1))) & 15u) << (4 * j);
        }
    }
}

// Dequantisation of cluster-major codes, first pass: members of every cluster per chunk, from the labels.
template <typename Src>
__global__ __launch_bounds__(kGBlock) void wide_label_counts_kernel(Src src, WideSpace sp)
{
    __shared__ uint32_t counters[kGWaves][kMaxClusters * kWave];
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t gc = (int64_t)blockIdx.x * kGWaves + wave;
    if (gc >= src.chunks())
        return;
    int64_t c;
    const WideTensor t = src.of_chunk(gc, c);
    const ChunkRef r = chunk_ref(c, t.n, t.G, t.cpg);
    uint32_t count = 0;
    if (r.len > 0) {
        uint32_t l4[kGK];
        load_chunk_labels(t.labels, r.lo, r.len, (r.lo & 3) == 0, lane, l4);
        count = wave_label_counts<kGK, false>([&](int k, int j) { return (l4[k] >> (4 * j)) & 15u; }, r.len, lane,
                                              counters[wave]);
    }
    if (lane < kMaxClusters)
        sp.counts[t.chunk0 + c].cnt[lane] = count;
}

template <typename Src, bool kTable, bool kMajor>
__global__ __launch_bounds__(kGBlock, 2) void wide_dequantize_ex_kernel(Src src, WideSpace sp, int m,
                                                                        const float *__restrict__ qmap)
{
    __shared__ DequantizeShared shared[kGWaves];
    __shared__ float table[kLevels];
    if (kTable)
        load_levels(table, qmap);
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t gc = (int64_t)blockIdx.x * kGWaves + wave;
    if (gc >= src.chunks())
        return;
    int64_t c;
    const WideTensor t = src.of_chunk(gc, c);
    const uint8_t *codes = t.codes, *labels = t.labels;
    const float *params = t.params;
    float *out = (float *)t.values;
    const ChunkRef r = chunk_ref(c, t.n, t.G, t.cpg);
    if (r.len == 0)
        return;
    DequantizeShared &sh = shared[wave];
    const bool aligned = (r.lo & 3) == 0;
    const int64_t g_lo = r.group * t.G;
    const int64_t g_len = group_len(t, r.group);
    uint32_t c4[kGK], l4[kGK];
    load_chunk_labels(labels, r.lo, r.len, aligned, lane, l4);
    if (!kMajor) {
#pragma unroll
        for (int k = 0; k < kGK; ++k) {
            const int off = k * 256 + lane * 4;
            c4[k] = 0;
            if (aligned && off + 3 < r.len) {
                c4[k] = __builtin_nontemporal_load((const BITSNAP_GLOBAL uint32_t *)(global_ptr(codes) + r.lo + off));
            } else {
                for (int j = 0; j < 4; ++j)
                    if (off + j < r.len)
                        c4[k] |= (uint32_t)global_ptr(codes)[r.lo + off + j] << (8 * j);
            }
        }
    }
    if (lane < kMaxClusters) {
        float2 sb = make_float2(0.0f, 0.0f);
        if (lane < m) {
            const float2v t = *(const BITSNAP_GLOBAL float2v *)(global_ptr(params) + (r.group * m + lane) * 2);
            sb = make_float2(t.x, t.y);
        }
        sh.coder[lane] = kTable ? sb : make_float2(__fdiv_rn(sb.x, 255.0f), sb.y);  // (S or S/255, b)
    }
    if (kMajor) {
        MajorView mv;
        mv.counters = sh.counters;
        mv.bytes = sh.bytes;
        mv.labels = sh.labels;
        uint16_t *l16 = (uint16_t *)mv.labels;
#pragma unroll
        for (int k = 0; k < kGK; ++k)
            l16[k * kWave + lane] = (uint16_t)l4[k];
        wave_lds_sync();
        const uint32_t dest = segment_dest(sp, t, c, r.group, lane);
        uint8_t *b8 = (uint8_t *)mv.bytes;
        const int len = r.len;
        // The chunk's 16 runs of codes, collected once their places inside the chunk are known.  Lane l takes the
        // chunk's cluster-major positions l, l + 64, ...: the run a position belongs to only moves forward, and
        // all of a lane's loads are issued before the first of them is used.
        uint32_t *seg_start = sh.seg_start, *seg_delta = sh.seg_delta;
        auto collect = [&](uint32_t start) {
            if (lane <= kMaxClusters)
                seg_start[lane] = start;  // lane 16 holds len
            if (lane < kMaxClusters)
                seg_delta[lane] = dest - start;  // position in the chunk -> place in the group
            wave_lds_sync();
            uint32_t cl = 0, next = seg_start[1], delta = seg_delta[0];
            uint32_t src[4 * kGK], b[4 * kGK];
#pragma unroll
            for (int it = 0; it < 4 * kGK; ++it) {
                const uint32_t p = (uint32_t)lane + (uint32_t)it * kWave;
                src[it] = 0xFFFFFFFFu;
                if (p < (uint32_t)len) {
                    while (p >= next) {
                        ++cl;
                        next = seg_start[cl + 1];
                        delta = seg_delta[cl];
                    }
                    src[it] = delta + p;
                }
            }
#pragma unroll
            for (int it = 0; it < 4 * kGK; ++it)  // holds whenever the counts are consistent; keeps any load inside the group
                b[it] = (int64_t)src[it] < g_len ? (uint32_t)global_ptr(codes)[g_lo + src[it]] : 0u;
#pragma unroll
            for (int it = 0; it < 4 * kGK; ++it) {
                const uint32_t p = (uint32_t)lane + (uint32_t)it * kWave;
                if (p < (uint32_t)len)
                    b8[p] = (uint8_t)b[it];
            }
            wave_lds_sync();
        };
        if (len == kGChunk)
            from_cluster_major<kGK, true>(mv, len, lane, collect);
        else
            from_cluster_major<kGK, false>(mv, len, lane, collect);
#pragma unroll
        for (int k = 0; k < kGK; ++k)
            c4[k] = mv.bytes[k * kWave + lane];
    } else {
        wave_lds_sync();
    }
#pragma unroll
    for (int k = 0; k < kGK; ++k) {
        const int off = k * 256 + lane * 4;
        float v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float2 sb = sh.coder[(l4[k] >> (4 * j)) & 15u];
            const uint32_t q = (c4[k] >> (8 * j)) & 255u;
            const float level = kTable ? table[q] : (float)q;
            v[j] = __fadd_rn(__fmul_rn(level, sb.x), sb.y);
        }
        if (aligned && off + 3 < r.len) {
            __builtin_nontemporal_store(float4v{v[0], v[1], v[2], v[3]}, (BITSNAP_GLOBAL float4v *)(global_ptr(out) + r.lo + off));
        } else {
            for (int j = 0; j < 4; ++j)
                if (off + j < r.len)
                    global_ptr(out)[r.lo + off + j] = v[j];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------

bool cluster_general_supported(int64_t n, int64_t group)
{
    if (n <= 0)
        return true;
    return group <= 0 || group >= n || (group % 2) == 0;  // a group boundary must not split a label byte
}

// Workspace for `chunks` chunks in `slices` slices and `groups` groups; `major`: with the cluster
// counts.  `extra` bytes (a multiple of 8) come first.
static size_t space_bytes(int64_t chunks, int64_t slices, int64_t groups, bool major, size_t extra)
{
    size_t bytes = extra + (size_t)groups * sizeof(GroupState) +
                   (size_t)(chunks + slices) * (sizeof(ChunkStats) + sizeof(ChunkRanges));
    if (major)
        bytes += (size_t)(chunks + slices + groups) * sizeof(ChunkCounts);
    return (bytes + 255) / 256 * 256;
}

static WideSpace cut_space(void *workspace, int64_t chunks, int64_t slices, int64_t groups, size_t extra)
{
    static_assert(sizeof(GroupState) % 8 == 0 && sizeof(ChunkStats) % 8 == 0 && sizeof(ChunkRanges) % 8 == 0,
                  "workspace parts stay 8-byte aligned");
    WideSpace sp;
    sp.gs = reinterpret_cast<GroupState *>((char *)workspace + extra);
    sp.stats = reinterpret_cast<ChunkStats *>(sp.gs + groups);
    sp.slice_stats = sp.stats + chunks;
    sp.ranges = reinterpret_cast<ChunkRanges *>(sp.slice_stats + slices);
    sp.slice_ranges = sp.ranges + chunks;
    sp.counts = reinterpret_cast<ChunkCounts *>(sp.slice_ranges + slices);  // present only with cluster-major codes
    sp.slice_counts = sp.counts + chunks;
    sp.cluster_base = sp.slice_counts + slices;
    return sp;
}

size_t cluster_general_workspace_bytes_ex(int64_t n, int64_t group, bool major)
{
    if (n <= 0)
        return 0;
    const WideTensor t = wide_tensor(nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, n, group);
    return space_bytes(t.groups * t.cpg, t.groups * t.spg, t.groups, major, 0);
}

size_t cluster_general_workspace_bytes(int64_t n, int64_t group) { return cluster_general_workspace_bytes_ex(n, group, false); }

size_t cluster_list_workspace_bytes(int64_t total_chunks, int64_t count, bool major)
{
    if (total_chunks <= 0 || count <= 0)
        return 0;
    // every tensor has at most chunks/256 + 1 slices; the list of first slices comes first
    return space_bytes(total_chunks, total_chunks / kGSlice + count, count, major, (size_t)(count + 1) * sizeof(int64_t));
}

static int general_grid(int64_t work)
{
    const int64_t cap = (int64_t)device_info().cu_count * 16;
    return (int)(work < 1 ? 1 : (work < cap ? work : cap));
}

// Grid of the persistent pass-3 kernel when a table has to be prepared per workgroup.
template <typename Src, bool kTable, bool kMajor>
static unsigned code_ex_grid(int64_t blocks)
{
    if (!kTable)
        return (unsigned)blocks;
    const void *kernel = (const void *)wide_code_ex_kernel<Src, kTable, kMajor>;
    const int64_t resident = (int64_t)device_info().cu_count * occupancy_blocks_per_cu(kernel, kGBlock);
    return (unsigned)(blocks < resident ? blocks : resident);
}

// The three passes over `chunks` chunks, at most `slices` slices and `groups` groups of `src`.
template <typename Src>
static int quantize_passes(const Src &src, const WideSpace &sp, int64_t chunks, int64_t slices, int64_t groups, int m,
                           bool major, const float *qmap, uint32_t *status, hipStream_t s)
{
    const int64_t blocks = (chunks + kGWaves - 1) / kGWaves, stream_blocks = (chunks + kStreamWaves - 1) / kStreamWaves;
    if (blocks > 0x7FFFFFFF || stream_blocks > 0x7FFFFFFF || slices > 0x7FFFFFFF)
        return BITSNAP_E_SIZE;
    const dim3 block(kGBlock), sgrid((unsigned)slices), ggrid(general_grid(groups));
    const dim3 stream_block(kStreamBlock), stream_grid((unsigned)stream_blocks);
    hipLaunchKernelGGL(wide_stats_kernel<Src>, stream_grid, stream_block, 0, s, src, sp);
    hipLaunchKernelGGL(wide_slice_stats_kernel<Src>, sgrid, block, 0, s, src, sp);
    hipLaunchKernelGGL(wide_fit_kernel<Src>, ggrid, block, 0, s, src, sp, m, status);
    if (major) {
        hipLaunchKernelGGL((wide_range_kernel<Src, true>), stream_grid, stream_block, 0, s, src, sp, m);
        hipLaunchKernelGGL((wide_slice_kernel<Src, true, true>), sgrid, block, 0, s, src, sp);
        hipLaunchKernelGGL((wide_group_kernel<Src, true, true>), ggrid, block, 0, s, src, sp, m);
    } else {
        hipLaunchKernelGGL((wide_range_kernel<Src, false>), stream_grid, stream_block, 0, s, src, sp, m);
        hipLaunchKernelGGL((wide_slice_kernel<Src, true, false>), sgrid, block, 0, s, src, sp);
        hipLaunchKernelGGL((wide_group_kernel<Src, true, false>), ggrid, block, 0, s, src, sp, m);
    }
#define BITSNAP_CODE_EX(T, M)                                                                                     \
    hipLaunchKernelGGL((wide_code_ex_kernel<Src, T, M>), dim3(code_ex_grid<Src, T, M>(blocks)), block, 0, s, src, sp, m, qmap)
    if (qmap && major)
        BITSNAP_CODE_EX(true, true);
    else if (qmap)
        BITSNAP_CODE_EX(true, false);
    else if (major)
        BITSNAP_CODE_EX(false, true);
    else
        hipLaunchKernelGGL(wide_code_kernel<Src>, stream_grid, stream_block, 0, s, src, sp, m);
#undef BITSNAP_CODE_EX
    return launch_status();
}

template <typename Src>
static int dequantize_passes(const Src &src, const WideSpace &sp, int64_t chunks, int64_t slices, int64_t groups, int m,
                             bool major, const float *qmap, hipStream_t s)
{
    const int64_t blocks = (chunks + kGWaves - 1) / kGWaves;
    if (blocks > 0x7FFFFFFF || slices > 0x7FFFFFFF)
        return BITSNAP_E_SIZE;
    const dim3 block(kGBlock), cgrid((unsigned)blocks), sgrid((unsigned)slices), ggrid(general_grid(groups));
    if (major) {
        hipLaunchKernelGGL(wide_label_counts_kernel<Src>, cgrid, block, 0, s, src, sp);
        hipLaunchKernelGGL((wide_slice_kernel<Src, false, true>), sgrid, block, 0, s, src, sp);
        hipLaunchKernelGGL((wide_group_kernel<Src, false, true>), ggrid, block, 0, s, src, sp, m);
    }
#define BITSNAP_DEQ_EX(T, M) hipLaunchKernelGGL((wide_dequantize_ex_kernel<Src, T, M>), cgrid, block, 0, s, src, sp, m, qmap)
    if (qmap && major)
        BITSNAP_DEQ_EX(true, true);
    else if (qmap)
        BITSNAP_DEQ_EX(true, false);
    else if (major)
        BITSNAP_DEQ_EX(false, true);
    else
        hipLaunchKernelGGL(wide_dequantize_kernel<Src>, cgrid, block, 0, s, src, m);
#undef BITSNAP_DEQ_EX
    return launch_status();
}

int cluster_general_quantize_ex(const float *x, int64_t n, int64_t group, int m, bool major, const float *qmap,
                                uint8_t *codes, uint8_t *labels, float *params, float *fit_out, const float *fit_in,
                                uint32_t *status, void *workspace, hipStream_t s)
{
    if (major && n > 0xFFFFFFFFll)
        return BITSNAP_E_SIZE;  // places inside a group are 32-bit
    OneTensor src;
    src.t = wide_tensor(const_cast<float *>(x), codes, labels, params, fit_out, fit_in, n, group);
    const int64_t chunks = src.t.groups * src.t.cpg, slices = src.t.groups * src.t.spg;
    return quantize_passes(src, cut_space(workspace, chunks, slices, src.t.groups, 0), chunks, slices, src.t.groups, m, major,
                           qmap, status, s);
}

int cluster_general_quantize(const float *x, int64_t n, int64_t group, int m, uint8_t *codes, uint8_t *labels,
                             float *params, float *fit_out, const float *fit_in, uint32_t *status, void *workspace,
                             hipStream_t s)
{
    return cluster_general_quantize_ex(x, n, group, m, false, nullptr, codes, labels, params, fit_out, fit_in, status,
                                       workspace, s);
}

int cluster_general_dequantize_ex(const uint8_t *codes, const uint8_t *labels, const float *params, int64_t n,
                                  int64_t group, int m, bool major, const float *qmap, float *out, void *workspace,
                                  hipStream_t s)
{
    if (major && n > 0xFFFFFFFFll)
        return BITSNAP_E_SIZE;
    OneTensor src;
    src.t = wide_tensor(out, const_cast<uint8_t *>(codes), const_cast<uint8_t *>(labels), const_cast<float *>(params), nullptr,
                        nullptr, n, group);
    const int64_t chunks = src.t.groups * src.t.cpg, slices = src.t.groups * src.t.spg;
    WideSpace sp = {};
    if (major)
        sp = cut_space(workspace, chunks, slices, src.t.groups, 0);
    return dequantize_passes(src, sp, chunks, slices, src.t.groups, m, major, qmap, s);
}

int cluster_general_dequantize(const uint8_t *codes, const uint8_t *labels, const float *params, int64_t n,
                               int64_t group, int m, float *out, hipStream_t s)
{
    return cluster_general_dequantize_ex(codes, labels, params, n, group, m, false, nullptr, out, nullptr, s);
}

// A list of tensors, one group each.  The workspace starts with the list of first slices.
static TensorList list_source(const bitsnap_cluster_item *items, int64_t count, int64_t total_chunks, void *workspace,
                              hipStream_t s)
{
    TensorList src;
    src.items = items, src.count = count, src.total_chunks = total_chunks;
    src.slice0 = reinterpret_cast<const int64_t *>(workspace);
    hipLaunchKernelGGL(wide_list_slices_kernel, dim3(1), dim3(kGBlock), 0, s, items, count, reinterpret_cast<int64_t *>(workspace));
    return src;
}

int cluster_list_quantize(const bitsnap_cluster_item *items, int64_t count, int64_t total_chunks, int m, bool major,
                          const float *qmap, uint32_t *status, void *workspace, hipStream_t s)
{
    const int64_t slices = total_chunks / kGSlice + count;
    const TensorList src = list_source(items, count, total_chunks, workspace, s);
    return quantize_passes(src, cut_space(workspace, total_chunks, slices, count, (size_t)(count + 1) * sizeof(int64_t)),
                           total_chunks, slices, count, m, major, qmap, status, s);
}

int cluster_list_dequantize(const bitsnap_cluster_item *items, int64_t count, int64_t total_chunks, int m, bool major,
                            const float *qmap, void *workspace, hipStream_t s)
{
    const int64_t slices = total_chunks / kGSlice + count;
    TensorList src;
    src.items = items, src.count = count, src.total_chunks = total_chunks, src.slice0 = nullptr;
    WideSpace sp = {};
    if (major) {
        src = list_source(items, count, total_chunks, workspace, s);
        sp = cut_space(workspace, total_chunks, slices, count, (size_t)(count + 1) * sizeof(int64_t));
    }
    return dequantize_passes(src, sp, total_chunks, slices, count, m, major, qmap, s);
}

}  // namespace bitsnap
