// Format variants of the cluster quantiser (paper: "Cluster Based Quantization for Optimizer
// States") for the group lengths that one wavefront handles:
//   * a general map Q^map in Eq. qmap-distance: code = the entry of a 256-entry table nearest to
//     (x-b)/S, and T^D = Q(T^Q)*S + b on the way back;
//   * the cluster-major arrangement of Eq. decluster: inside a group the codes of cluster 0 come
//     first, then cluster 1, ..., each cluster's codes in element order.
// Steps 1-4 of Algorithm 2 are the plain kernels' code; the table search and the partition are
// in cluster_variants.hpp.  Wide groups go to the multi-pass kernels.
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

// Algorithm 2 with the format options for one group of len <= 256*K elements, by one wave.
template <int K, bool kFull, bool kTable, bool kMajor>
__device__ __forceinline__ void quantize_group_ex(const float *__restrict__ x, int64_t lo, int len, int m, int64_t g,
                                                  uint8_t *__restrict__ codes, uint8_t *__restrict__ labels,
                                                  float *__restrict__ params, float *__restrict__ fit_out,
                                                  const float *__restrict__ fit_in, uint32_t *__restrict__ status,
                                                  WaveShared &ws, const TableShared &table, int lane)
{

    // ---- steps 1-4 of Algorithm 2, as in the plain kernel
    float4 v[K];
    load_elements<K, kFull>(x, lo, len, lane, v);
    reset_ranges(ws, lane);
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
    uint32_t packed[(K + 1) / 2];
    label_pass<K, kFull, true, true>(v, lo, len, ls, ws, lane, labels, packed);
    float mn, mx;
    reduce_ranges(ws, lane, mn, mx);
    if (lane < kMaxClusters) {
        float S, b, inv;
        cluster_coder(mn, mx, S, b, inv);
        if (kTable) {
            inv = S > 0.0f ? __fdiv_rn(1.0f, S) : 0.0f;
            if (!isfinite(inv))
                inv = 0.0f;
        }
        ws.coder[lane] = make_float2(b, inv);
        if (lane < m)
            *(BITSNAP_GLOBAL float2v *)(global_ptr(params) + (g * m + lane) * 2) = float2v{S, b};
    }
    wave_lds_sync();

    // ---- steps 5-6
    uint32_t c4[K];
    codes_to_registers<K, kTable>(v, packed, ws, table, c4);
    if (kMajor) {
        const MajorView mv = major_view(ws);  // the min/max table is done with
        uint16_t *l16 = (uint16_t *)mv.labels;
#pragma unroll
        for (int k = 0; k < K; ++k) {
            mv.bytes[k * kWave + lane] = c4[k];
            l16[k * kWave + lane] = (uint16_t)(packed[k >> 1] >> (16 * (k & 1)));
        }
        wave_lds_sync();
        uint32_t start;
        to_cluster_major<K, kFull>(mv, len, lane, start);
#pragma unroll
        for (int k = 0; k < K; ++k)
            c4[k] = mv.bytes[k * kWave + lane];
    }
    store_codes<K, kFull>(c4, lo, len, lane, codes);
    wave_lds_sync();  // this wave may go on to another group and rewrite the tables
}

// Every wave walks over groups first_group + w, + w + W, ... (w = its index among the W waves of
// the grid): the grid is sized to the device when a table has to be prepared per workgroup, and
// to one group per wave otherwise.
template <int K, bool kFull, bool kTable, bool kMajor>
__global__ __launch_bounds__(kVBlock, kTable ? 3 : 4) void quantize_cluster_ex_kernel(
    const float *__restrict__ x, int64_t n, int64_t first_group, int64_t groups, int m, const float *__restrict__ qmap,
    uint8_t *__restrict__ codes, uint8_t *__restrict__ labels, float *__restrict__ params, float *__restrict__ fit_out,
    const float *__restrict__ fit_in, uint32_t *__restrict__ status)
{
    __shared__ WaveShared shared[kVWaves];
    __shared__ TableShared table;
    if (kTable)
        load_table(table, qmap);
    // no workgroup barrier from here on: waves leave when they run out of groups
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    constexpr int G = 256 * K;
    int64_t g = first_group + (int64_t)blockIdx.x * kVWaves + wave;
    if (!kTable) {  // one group per wave: written without the loop, which costs registers
        if (g < first_group + groups) {
            const int64_t lo = g * G;
            const int64_t rest = n - lo;
            quantize_group_ex<K, kFull, kTable, kMajor>(x, lo, kFull ? G : (int)(rest < G ? rest : G), m, g, codes, labels,
                                                        params, fit_out, fit_in, status, shared[wave], table, lane);
        }
        return;
    }
    for (; g < first_group + groups; g += (int64_t)gridDim.x * kVWaves) {
        const int64_t lo = g * G;
        const int64_t rest = n - lo;
        const int len = kFull ? G : (int)(rest < G ? rest : G);
        quantize_group_ex<K, kFull, kTable, kMajor>(x, lo, len, m, g, codes, labels, params, fit_out, fit_in, status,
                                                    shared[wave], table, lane);
    }
}

// The inverse for one group of len <= 256*K elements, by one wave.
template <int K, bool kTable, bool kMajor>
__device__ __forceinline__ void dequantize_group_ex(const uint8_t *__restrict__ codes, const uint8_t *__restrict__ labels,
                                                    const float *__restrict__ params, int64_t lo, int len, int m, int64_t g,
                                                    float *__restrict__ out, DequantizeShared &sh, const float *table, int lane)
{
    constexpr int G = 256 * K;
    uint32_t c4[K], l4[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int off = k * 256 + lane * 4;
        c4[k] = 0, l4[k] = 0;
        if (off + 3 < len) {
            c4[k] = __builtin_nontemporal_load((const BITSNAP_GLOBAL uint32_t *)(global_ptr(codes) + lo + off));
            l4[k] = __builtin_nontemporal_load((const BITSNAP_GLOBAL uint16_t *)(global_ptr(labels) + ((lo + off) >> 1)));
        } else {
            for (int j = 0; j < 4; ++j)
                if (off + j < len) {
                    c4[k] |= (uint32_t)global_ptr(codes)[lo + off + j] << (8 * j);
                    l4[k] |= (uint32_t)((global_ptr(labels)[(lo + off + j) >> 1] >> (4 * ((lo + off + j) & 1))) & 15u) << (4 * j);
                }
        }
    }
    if (lane < kMaxClusters) {
        float2 sb = make_float2(0.0f, 0.0f);
        if (lane < m) {
            const float2v t = *(const BITSNAP_GLOBAL float2v *)(global_ptr(params) + (g * m + lane) * 2);
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
        for (int k = 0; k < K; ++k) {
            mv.bytes[k * kWave + lane] = c4[k];
            l16[k * kWave + lane] = (uint16_t)l4[k];
        }
        wave_lds_sync();
        if (len == G)
            from_cluster_major<K, true>(mv, len, lane);
        else
            from_cluster_major<K, false>(mv, len, lane);
#pragma unroll
        for (int k = 0; k < K; ++k)
            c4[k] = mv.bytes[k * kWave + lane];
    } else {
        wave_lds_sync();
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int off = k * 256 + lane * 4;
        float r[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float2 sb = sh.coder[(l4[k] >> (4 * j)) & 15u];
            const uint32_t q = (c4[k] >> (8 * j)) & 255u;
            const float level = kTable ? table[q] : (float)q;
            r[j] = __fadd_rn(__fmul_rn(level, sb.x), sb.y);
        }
        if (off + 3 < len) {
            __builtin_nontemporal_store(float4v{r[0], r[1], r[2], r[3]}, (BITSNAP_GLOBAL float4v *)(global_ptr(out) + lo + off));
        } else {
            for (int j = 0; j < 4; ++j)
                if (off + j < len)
                    global_ptr(out)[lo + off + j] = r[j];
        }
    }
    wave_lds_sync();  // this wave may go on to another group and rewrite the tables
}

template <int K, bool kTable, bool kMajor>
__global__ __launch_bounds__(kVBlock, 4) void dequantize_cluster_ex_kernel(
    const uint8_t *__restrict__ codes, const uint8_t *__restrict__ labels, const float *__restrict__ params, int64_t n,
    int64_t groups, int m, const float *__restrict__ qmap, float *__restrict__ out)
{
    __shared__ DequantizeShared shared[kVWaves];
    __shared__ float table[kLevels];
    if (kTable)
        load_levels(table, qmap);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int64_t g = (int64_t)blockIdx.x * kVWaves + wave;
    if (g >= groups)
        return;
    constexpr int G = 256 * K;
    const int64_t lo = g * G;
    const int64_t rest = n - lo;
    dequantize_group_ex<K, kTable, kMajor>(codes, labels, params, lo, rest >= G ? G : (int)rest, m, g, out, shared[wave], table,
                                           lane);
}

// ---------------------------------------------------------------------------------------------
// Batched forms: groups are numbered across the list of tensors as in the plain batched kernels.
// ---------------------------------------------------------------------------------------------
template <int K, bool kFull, bool kTable, bool kMajor>
__global__ __launch_bounds__(kVBlock, kTable ? 3 : 4) void quantize_cluster_ex_batched_kernel(
    const bitsnap_cluster_item *__restrict__ items, int64_t count, int64_t total_groups, int m,
    const float *__restrict__ qmap, uint32_t *__restrict__ status)
{
    __shared__ WaveShared shared[kVWaves];
    __shared__ TableShared table;
    if (kTable)
        load_table(table, qmap);
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr int G = 256 * K;
    // list-wide group gg (kFull) or the short last group of tensor gg (!kFull)
    auto one = [&](int64_t gg) {
        if (kFull) {
            const bitsnap_cluster_item &it = items[find_item(items, count, gg)];
            const int64_t g = gg - it.first_group;
            const int64_t lo = g * G;
            if (it.n - lo >= G)  // a short last group is left to the tail launch
                quantize_group_ex<K, true, kTable, kMajor>((const float *)it.values, lo, G, m, g, it.codes, it.labels,
                                                           it.params, it.fit_out, it.fit_in, status, shared[wave], table,
                                                           lane);
        } else {
            const bitsnap_cluster_item &it = items[gg];
            const int64_t g = it.n / G;
            const int rest = (int)(it.n - g * G);
            if (rest > 0)
                quantize_group_ex<K, false, kTable, kMajor>((const float *)it.values, g * G, rest, m, g, it.codes, it.labels,
                                                            it.params, it.fit_out, it.fit_in, status, shared[wave], table,
                                                            lane);
        }
    };
    const int64_t end = kFull ? total_groups : count;
    int64_t gg = (int64_t)blockIdx.x * kVWaves + wave;
    if (!kTable) {  // one turn per wave: written without the loop, which costs registers
        if (gg < end)
            one(gg);
        return;
    }
    for (; gg < end; gg += (int64_t)gridDim.x * kVWaves)
        one(gg);
}

template <int K, bool kTable, bool kMajor>
__global__ __launch_bounds__(kVBlock, 4) void dequantize_cluster_ex_batched_kernel(
    const bitsnap_cluster_item *__restrict__ items, int64_t count, int64_t total_groups, int m,
    const float *__restrict__ qmap)
{
    __shared__ DequantizeShared shared[kVWaves];
    __shared__ float table[kLevels];
    if (kTable)
        load_levels(table, qmap);
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr int G = 256 * K;
    const int64_t gg = (int64_t)blockIdx.x * kVWaves + wave;
    if (gg >= total_groups)
        return;
    const bitsnap_cluster_item &it = items[find_item(items, count, gg)];
    const int64_t g = gg - it.first_group;
    const int64_t lo = g * G;
    const int64_t rest = it.n - lo;
    if (rest > 0)
        dequantize_group_ex<K, kTable, kMajor>(it.codes, it.labels, it.params, lo, rest >= G ? G : (int)rest, m, g,
                                               (float *)it.values, shared[wave], table, lane);
}

template <int K, bool kTable, bool kMajor>
static void launch_quantize_ex(const float *x, int64_t n, int m, const float *qmap, uint8_t *codes, uint8_t *labels,
                               float *params, float *fit_out, const float *fit_in, uint32_t *status, hipStream_t s)
{
    const int64_t G = 256 * (int64_t)K;
    const int64_t full = n / G;
    const bool tail = (n % G) != 0;
    int64_t blocks = (full + kVWaves - 1) / kVWaves;
    if (kTable) {
        const void *kernel = (const void *)quantize_cluster_ex_kernel<K, true, kTable, kMajor>;
        const int64_t resident = (int64_t)device_info().cu_count * occupancy_blocks_per_cu(kernel, kVBlock);
        if (blocks > resident)
            blocks = resident;
    }
    if (full > 0)
        hipLaunchKernelGGL((quantize_cluster_ex_kernel<K, true, kTable, kMajor>), dim3((unsigned)blocks), dim3(kVBlock), 0, s,
                           x, n, (int64_t)0, full, m, qmap, codes, labels, params, fit_out, fit_in, status);
    if (tail)
        hipLaunchKernelGGL((quantize_cluster_ex_kernel<K, false, kTable, kMajor>), dim3(1), dim3(kVBlock), 0, s, x, n, full,
                           (int64_t)1, m, qmap, codes, labels, params, fit_out, fit_in, status);
}

template <int K, bool kTable, bool kMajor>
static void launch_dequantize_ex(const uint8_t *codes, const uint8_t *labels, const float *params, int64_t n, int m,
                                 const float *qmap, float *out, hipStream_t s)
{
    const int64_t G = 256 * (int64_t)K;
    const int64_t groups = (n + G - 1) / G;
    const int64_t blocks = (groups + kVWaves - 1) / kVWaves;
    hipLaunchKernelGGL((dequantize_cluster_ex_kernel<K, kTable, kMajor>), dim3((unsigned)blocks), dim3(kVBlock), 0, s, codes,
                       labels, params, n, groups, m, qmap, out);
}

}  // namespace bitsnap

using namespace bitsnap;

#define BITSNAP_BY_K(K, CALL)          \
    switch (K) {                       \
    case 1: CALL(1); break;            \
    case 2: CALL(2); break;            \
    case 4: CALL(4); break;            \
    case 8: CALL(8); break;            \
    default: CALL(16); break;          \
    }

extern "C" size_t bitsnap_cluster_workspace_bytes_ex(int64_t n, int64_t group, int m, uint32_t flags)
{
    (void)m;
    if (n <= 0 || group < 0 || one_wave_group_k(group) != 0)
        return 0;
    return cluster_general_workspace_bytes_ex(n, group, (flags & BITSNAP_CLUSTER_MAJOR) != 0);
}

// Checks shared by the two calls; 1 = go on, else the value to return.
static int check_ex(int64_t n, int64_t group, int m, uint32_t flags, const void *workspace, size_t workspace_bytes,
                    bool need_workspace, int &K)
{
    if (n < 0 || m < 1 || m > kMaxClusters || group < 0 || (flags & ~(uint32_t)BITSNAP_CLUSTER_MAJOR))
        return BITSNAP_E_SIZE;
    K = one_wave_group_k(group);
    if (K != 0 && (n + 256 * (int64_t)K - 1) / (256 * (int64_t)K) / kVWaves > 0x7FFFFFFF)
        return BITSNAP_E_SIZE;
    if (K == 0 && !cluster_general_supported(n, group))
        return BITSNAP_E_SIZE;
    if (n == 0)
        return BITSNAP_OK;
    if (K == 0 && need_workspace) {
        if (!workspace)
            return BITSNAP_E_NULL;
        if (!aligned16(workspace))
            return BITSNAP_E_ALIGN;
        if (workspace_bytes < bitsnap_cluster_workspace_bytes_ex(n, group, m, flags))
            return BITSNAP_E_WORKSPACE;
    }
    return 1;
}

extern "C" int bitsnap_quantize_cluster_ex(const float *x, int64_t n, int64_t group, int m, uint32_t flags,
                                           const float *qmap, uint8_t *codes, uint8_t *labels, float *params,
                                           float *fit_out, const float *fit_in, uint32_t *status, void *workspace,
                                           size_t workspace_bytes, bitsnap_stream_t stream)
{
    const bool major = (flags & BITSNAP_CLUSTER_MAJOR) != 0;
    if (!qmap && !major && !(flags & ~(uint32_t)BITSNAP_CLUSTER_MAJOR))
        return bitsnap_quantize_cluster(x, n, group, m, codes, labels, params, fit_out, fit_in, status, workspace,
                                        workspace_bytes, stream);
    int K = 0;
    const int rc = check_ex(n, group, m, flags, workspace, workspace_bytes, true, K);
    if (rc <= 0)
        return rc;
    if (!x || !codes || !labels || !params)
        return BITSNAP_E_NULL;
    if (!aligned16(x) || !aligned16(codes) || !aligned16(labels) || !aligned16(params) || ((uintptr_t)fit_out & 3u) ||
        ((uintptr_t)fit_in & 3u) || ((uintptr_t)status & 3u) || ((uintptr_t)qmap & 3u))
        return BITSNAP_E_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    if (K == 0)
        return cluster_general_quantize_ex(x, n, group, m, major, qmap, codes, labels, params, fit_out, fit_in, status,
                                           workspace, s);
#define BITSNAP_Q_TM(KK) launch_quantize_ex<KK, true, true>(x, n, m, qmap, codes, labels, params, fit_out, fit_in, status, s)
#define BITSNAP_Q_T(KK) launch_quantize_ex<KK, true, false>(x, n, m, qmap, codes, labels, params, fit_out, fit_in, status, s)
#define BITSNAP_Q_M(KK) launch_quantize_ex<KK, false, true>(x, n, m, qmap, codes, labels, params, fit_out, fit_in, status, s)
    if (qmap && major) {
        BITSNAP_BY_K(K, BITSNAP_Q_TM)
    } else if (qmap) {
        BITSNAP_BY_K(K, BITSNAP_Q_T)
    } else {
        BITSNAP_BY_K(K, BITSNAP_Q_M)
    }
#undef BITSNAP_Q_TM
#undef BITSNAP_Q_T
#undef BITSNAP_Q_M
    return launch_status();
}

extern "C" int bitsnap_dequantize_cluster_ex(const uint8_t *codes, const uint8_t *labels, const float *params,
                                             int64_t n, int64_t group, int m, uint32_t flags, const float *qmap,
                                             float *out, void *workspace, size_t workspace_bytes,
                                             bitsnap_stream_t stream)
{
    const bool major = (flags & BITSNAP_CLUSTER_MAJOR) != 0;
    if (!qmap && !major && !(flags & ~(uint32_t)BITSNAP_CLUSTER_MAJOR))
        return bitsnap_dequantize_cluster(codes, labels, params, n, group, m, out, stream);
    int K = 0;
    const int rc = check_ex(n, group, m, flags, workspace, workspace_bytes, major, K);  // only the partition needs it
    if (rc <= 0)
        return rc;
    if (!codes || !labels || !params || !out)
        return BITSNAP_E_NULL;
    if (!aligned16(codes) || !aligned16(labels) || !aligned16(params) || !aligned16(out) || ((uintptr_t)qmap & 3u))
        return BITSNAP_E_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    if (K == 0)
        return cluster_general_dequantize_ex(codes, labels, params, n, group, m, major, qmap, out, workspace, s);
#define BITSNAP_D_TM(KK) launch_dequantize_ex<KK, true, true>(codes, labels, params, n, m, qmap, out, s)
#define BITSNAP_D_T(KK) launch_dequantize_ex<KK, true, false>(codes, labels, params, n, m, qmap, out, s)
#define BITSNAP_D_M(KK) launch_dequantize_ex<KK, false, true>(codes, labels, params, n, m, qmap, out, s)
    if (qmap && major) {
        BITSNAP_BY_K(K, BITSNAP_D_TM)
    } else if (qmap) {
        BITSNAP_BY_K(K, BITSNAP_D_T)
    } else {
        BITSNAP_BY_K(K, BITSNAP_D_M)
    }
#undef BITSNAP_D_TM
#undef BITSNAP_D_T
#undef BITSNAP_D_M
    return launch_status();
}

static int64_t ex_batched_blocks(int64_t total_groups) { return (total_groups + kVWaves - 1) / kVWaves; }

template <int K, bool kTable, bool kMajor>
static void launch_quantize_ex_batched(const bitsnap_cluster_item *items, int64_t count, int64_t total_groups, int m,
                                       const float *qmap, uint32_t *status, hipStream_t s)
{
    int64_t blocks = ex_batched_blocks(total_groups), tblocks = (count + kVWaves - 1) / kVWaves;
    if (kTable) {
        const void *kernel = (const void *)quantize_cluster_ex_batched_kernel<K, true, kTable, kMajor>;
        const int64_t resident = (int64_t)device_info().cu_count * occupancy_blocks_per_cu(kernel, kVBlock);
        blocks = blocks < resident ? blocks : resident;
        tblocks = tblocks < resident ? tblocks : resident;
    }
    hipLaunchKernelGGL((quantize_cluster_ex_batched_kernel<K, true, kTable, kMajor>), dim3((unsigned)blocks), dim3(kVBlock), 0,
                       s, items, count, total_groups, m, qmap, status);
    hipLaunchKernelGGL((quantize_cluster_ex_batched_kernel<K, false, kTable, kMajor>), dim3((unsigned)tblocks), dim3(kVBlock),
                       0, s, items, count, total_groups, m, qmap, status);
}

template <int K, bool kTable, bool kMajor>
static void launch_dequantize_ex_batched(const bitsnap_cluster_item *items, int64_t count, int64_t total_groups, int m,
                                         const float *qmap, hipStream_t s)
{
    hipLaunchKernelGGL((dequantize_cluster_ex_batched_kernel<K, kTable, kMajor>), dim3((unsigned)ex_batched_blocks(total_groups)),
                       dim3(kVBlock), 0, s, items, count, total_groups, m, qmap);
}

extern "C" size_t bitsnap_cluster_chunk_elems(void) { return 4096; }

extern "C" size_t bitsnap_cluster_batch_workspace_bytes(int64_t total_groups, int64_t count, int64_t group, uint32_t flags)
{
    if (group != 0)
        return 0;
    return cluster_list_workspace_bytes(total_groups, count, (flags & BITSNAP_CLUSTER_MAJOR) != 0);
}

// Checks shared by the two calls; 1 = go on, else the value to return.  group == 0 (one group per
// tensor) takes the multi-pass kernels over the whole list and needs the workspace.
static int check_ex_batched(const bitsnap_cluster_item *items, int64_t count, int64_t total_groups, int64_t group, int m,
                            uint32_t flags, const float *qmap, const uint32_t *status, const void *workspace,
                            size_t workspace_bytes, bool need_workspace, int &K)
{
    if (count < 0 || total_groups < 0 || m < 1 || m > kMaxClusters || (flags & ~(uint32_t)BITSNAP_CLUSTER_MAJOR))
        return BITSNAP_E_SIZE;
    K = one_wave_group_k(group);
    if ((K == 0 && group != 0) || ex_batched_blocks(total_groups) > 0x7FFFFFFF)
        return BITSNAP_E_SIZE;
    if (K == 0 && (count > 0x3FFFFFFF || total_groups / 256 + count > 0x7FFFFFFF))  // grid of the slice kernels
        return BITSNAP_E_SIZE;
    if (count == 0 || total_groups == 0)
        return BITSNAP_OK;
    if (!items)
        return BITSNAP_E_NULL;
    if (((uintptr_t)items & 7u) || ((uintptr_t)status & 3u) || ((uintptr_t)qmap & 3u))
        return BITSNAP_E_ALIGN;
    if (K == 0 && need_workspace) {
        if (!workspace)
            return BITSNAP_E_NULL;
        if (!aligned16(workspace))
            return BITSNAP_E_ALIGN;
        if (workspace_bytes < bitsnap_cluster_batch_workspace_bytes(total_groups, count, group, flags))
            return BITSNAP_E_WORKSPACE;
    }
    return 1;
}

extern "C" int bitsnap_quantize_cluster_batched_ex(const bitsnap_cluster_item *items, int64_t count, int64_t total_groups,
                                                   int64_t group, int m, uint32_t flags, const float *qmap,
                                                   uint32_t *status, void *workspace, size_t workspace_bytes,
                                                   bitsnap_stream_t stream)
{
    int K = 0;
    const int rc = check_ex_batched(items, count, total_groups, group, m, flags, qmap, status, workspace, workspace_bytes,
                                    true, K);
    if (rc <= 0)
        return rc;
    const bool major = (flags & BITSNAP_CLUSTER_MAJOR) != 0;
    hipStream_t s = (hipStream_t)stream;
    if (K == 0)
        return cluster_list_quantize(items, count, total_groups, m, major, qmap, status, workspace, s);
    if (!qmap && !major)
        return bitsnap_quantize_cluster_batched(items, count, total_groups, group, m, status, stream);
#define BITSNAP_QB_TM(KK) launch_quantize_ex_batched<KK, true, true>(items, count, total_groups, m, qmap, status, s)
#define BITSNAP_QB_T(KK) launch_quantize_ex_batched<KK, true, false>(items, count, total_groups, m, qmap, status, s)
#define BITSNAP_QB_M(KK) launch_quantize_ex_batched<KK, false, true>(items, count, total_groups, m, qmap, status, s)
    if (qmap && major) {
        BITSNAP_BY_K(K, BITSNAP_QB_TM)
    } else if (qmap) {
        BITSNAP_BY_K(K, BITSNAP_QB_T)
    } else {
        BITSNAP_BY_K(K, BITSNAP_QB_M)
    }
#undef BITSNAP_QB_TM
#undef BITSNAP_QB_T
#undef BITSNAP_QB_M
    return launch_status();
}

extern "C" int bitsnap_dequantize_cluster_batched_ex(const bitsnap_cluster_item *items, int64_t count, int64_t total_groups,
                                                     int64_t group, int m, uint32_t flags, const float *qmap,
                                                     void *workspace, size_t workspace_bytes, bitsnap_stream_t stream)
{
    int K = 0;
    const bool major = (flags & BITSNAP_CLUSTER_MAJOR) != 0;
    const int rc = check_ex_batched(items, count, total_groups, group, m, flags, qmap, nullptr, workspace, workspace_bytes,
                                    major, K);
    if (rc <= 0)
        return rc;
    hipStream_t s = (hipStream_t)stream;
    if (K == 0)
        return cluster_list_dequantize(items, count, total_groups, m, major, qmap, workspace, s);
    if (!qmap && !major)
        return bitsnap_dequantize_cluster_batched(items, count, total_groups, group, m, stream);
#define BITSNAP_DB_TM(KK) launch_dequantize_ex_batched<KK, true, true>(items, count, total_groups, m, qmap, s)
#define BITSNAP_DB_T(KK) launch_dequantize_ex_batched<KK, true, false>(items, count, total_groups, m, qmap, s)
#define BITSNAP_DB_M(KK) launch_dequantize_ex_batched<KK, false, true>(items, count, total_groups, m, qmap, s)
    if (qmap && major) {
        BITSNAP_BY_K(K, BITSNAP_DB_TM)
    } else if (qmap) {
        BITSNAP_BY_K(K, BITSNAP_DB_T)
    } else {
        BITSNAP_BY_K(K, BITSNAP_DB_M)
    }
#undef BITSNAP_DB_TM
#undef BITSNAP_DB_T
#undef BITSNAP_DB_M
    return launch_status();
}
