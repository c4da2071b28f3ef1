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

#include <type_traits>

#include "../../include/bitsnap.h"
#include "cluster_general.hpp"
#include "host_util.hpp"
#include "wave.hpp"

namespace bitsnap {

static const double kZHost[17][16] = {
#include "z_table.inc"
};
__constant__ double kZDev[17][16] = {
#include "z_table.inc"
};

constexpr int kQBlock = 256;
constexpr int kQWaves = kQBlock / kWave;
constexpr int kMaxClusters = 16;
// Label search by bins.  bin(x) = min(63, sat_u8(rne(x*r + c))) with r = 16/sigma and
// c = 32 - mu*r is a non-decreasing function of x whatever the rounding (r > 0), so
//   bin(x) < bin(e)  =>  x < e      and      bin(x) > bin(e)  =>  x > e
// for every edge e, and the label of x, #{k : e_k <= x}, is the number of edges in lower bins
// plus one comparison with the edge in x's own bin - provided no bin holds two edges, which is
// checked per group on the actual edges; a group that fails the check takes the tree search.
// 16 bins per sigma put the 15 normal quantiles of m = 16 at least 2.5 bins apart.
constexpr int kBins = 64;
constexpr float kBinsPerSigma = 16.0f, kBinOffset = 32.0f;

struct alignas(16) WaveShared {
    float tab[2 * kMaxClusters][kWave];  // rows 0..15: running min per cluster, rows 16..31: running max
    float tree[kMaxClusters];            // node i of the edge search tree (node 1 = root), [0] unused
    float2 coder[kMaxClusters];          // (b, 255/S) for quantize, (S/255, b) for dequantize
    float2 bins[kBins];                  // label search by bins: (the edge inside the bin or +inf, edges below the bin)
};

// Orders this wave's LDS writes before its later LDS reads (lanes exchange data through LDS).
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ float comp(const float4 &v, int j) { return j == 0 ? v.x : j == 1 ? v.y : j == 2 ? v.z : v.w; }

typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float2v __attribute__((ext_vector_type(2)));
#define BITSNAP_LDS __attribute__((address_space(3)))
// Device buffers are addressed as global memory explicitly.  Through a generic pointer every
// access is a flat instruction, which also counts as an LDS operation in flight, so each wait
// for an LDS read would wait for the HBM traffic issued before it as well.
#define BITSNAP_GLOBAL __attribute__((address_space(1)))
template <typename T>
__device__ __forceinline__ BITSNAP_GLOBAL T *global_ptr(T *p)
{
    return (BITSNAP_GLOBAL T *)p;
}

// Byte address of an LDS object, and LDS accesses by byte address.  The label search and the
// min/max table below carry addresses, not indices, so that one shift-add per step does both the
// tree descent and the address arithmetic.
__device__ __forceinline__ uint32_t lds_addr(const void *p) { return (uint32_t)(uintptr_t)(const BITSNAP_LDS void *)p; }
__device__ __forceinline__ float lds_read_f32(uint32_t a) { return *(const BITSNAP_LDS float *)(uintptr_t)a; }
__device__ __forceinline__ float2 lds_read_f32x2(uint32_t a)
{
    const float2v t = *(const BITSNAP_LDS float2v *)(uintptr_t)a;
    return make_float2(t.x, t.y);
}

__device__ __forceinline__ uint32_t bin_of(float x, float r, float c)
{
    const uint32_t i = __builtin_amdgcn_cvt_pk_u8_f32(__fmaf_rn(x, r, c), 0, 0u);
    return i < (uint32_t)(kBins - 1) ? i : (uint32_t)(kBins - 1);
}

// Inputs and outputs are touched once, so they are loaded and stored non-temporally (measured on
// the batched 7B pass: 67.5 % -> 72 % of HBM peak for quantize, 66.5 % -> 69.5 % for dequantize).
// streaming 16-byte load
__device__ __forceinline__ float4 load_stream(const float *p)
{
    const float4v t = __builtin_nontemporal_load((const BITSNAP_GLOBAL float4v *)p);
    return make_float4(t.x, t.y, t.z, t.w);
}

template <int K, bool kFull>
__device__ __forceinline__ void quantize_group(const float *__restrict__ x, int64_t lo, int len, int m, int64_t g,
                                               uint8_t *__restrict__ codes, uint8_t *__restrict__ labels,
                                               float *__restrict__ params, float *__restrict__ fit_out,
                                               const float *__restrict__ fit_in, uint32_t *__restrict__ status,
                                               WaveShared &ws, int lane)
{
    // ---- load: lane owns elements lo + k*256 + lane*4 + {0..3}
    float4 v[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int off = k * 256 + lane * 4;
        if (kFull) {
            v[k] = load_stream(x + lo + off);
        } else {
            v[k].x = off + 0 < len ? global_ptr(x)[lo + off + 0] : 0.0f;
            v[k].y = off + 1 < len ? global_ptr(x)[lo + off + 1] : 0.0f;
            v[k].z = off + 2 < len ? global_ptr(x)[lo + off + 2] : 0.0f;
            v[k].w = off + 3 < len ? global_ptr(x)[lo + off + 3] : 0.0f;
        }
    }
    // running min/max table: this lane's column
#pragma unroll
    for (int c = 0; c < kMaxClusters; ++c) {
        ws.tab[c][lane] = INFINITY;
        ws.tab[kMaxClusters + c][lane] = -INFINITY;
    }

    // ---- step 1: mean and population standard deviation, fp64
    double s = 0.0;
#pragma unroll
    for (int k = 0; k < K; ++k)
        s += ((double)v[k].x + (double)v[k].y) + ((double)v[k].z + (double)v[k].w);  // padding adds 0
    s = wave_sum(s);
    const double mean = s / (double)len;
    // Keep the group as fp32 in registers: without this the compiler holds on to the fp64 copies
    // made for the sum above, which doubles the register footprint and halves the occupancy.
#pragma unroll
    for (int k = 0; k < K; ++k)
        asm volatile("" : "+v"(v[k].x), "+v"(v[k].y), "+v"(v[k].z), "+v"(v[k].w));
    double q = 0.0;
#pragma unroll
    for (int k = 0; k < K; ++k) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (kFull || k * 256 + lane * 4 + j < len) {
                const double d = (double)comp(v[k], j) - mean;
                q = fma(d, d, q);
            }
        }
    }
    q = wave_sum(q);
    float mu = (float)mean;
    float sigma = (float)sqrt(q / (double)len);
    if (fit_in) {
        mu = global_ptr(fit_in)[2 * g];
        sigma = global_ptr(fit_in)[2 * g + 1];
    }
    if (status && lane == 0 && !(isfinite(mu) && isfinite(sigma)))
        atomicOr(status, 1u);

    // ---- step 2: edges e_k = fl32(mu + sigma * z_k), product and sum rounded separately in fp64
    float edge = INFINITY;  // edges that do not exist (m < 16) are never <= x
    if (lane >= 1 && lane < m)
        edge = (float)__dadd_rn((double)mu, __dmul_rn((double)sigma, kZDev[m][lane]));
    if (lane >= 1 && lane < kMaxClusters) {
        const int tz = __ffs(lane) - 1;
        ws.tree[(1 << (3 - tz)) + (lane >> (tz + 1))] = edge;
        if (fit_out && lane < m)
            global_ptr(fit_out)[g * (m + 1) + 1 + lane] = edge;
    }
    if (fit_out && lane == 0) {
        global_ptr(fit_out)[g * (m + 1) + 0] = mu;
        global_ptr(fit_out)[g * (m + 1) + 1] = sigma;
    }
    const float root = read_lane(edge, 8);  // the middle edge, e_8: first step of every search
    const float bin_r = __fdiv_rn(kBinsPerSigma, sigma);
    const float bin_c = __fsub_rn(kBinOffset, __fmul_rn(mu, bin_r));
    ws.bins[lane] = make_float2(INFINITY, 0.0f);
    wave_lds_sync();
    if (lane >= 1 && lane < m)
        ws.bins[bin_of(edge, bin_r, bin_c)].x = edge;
    wave_lds_sync();
    bool by_bins;
    {
        const uint64_t occupied = __ballot(ws.bins[lane].x < INFINITY);
        by_bins = (int)__popcll(occupied) == m - 1 && bin_r > 0.0f;  // every edge alone in its bin
        const uint32_t below = __builtin_amdgcn_mbcnt_hi((uint32_t)(occupied >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)occupied, 0u));
        ws.bins[lane].y = __uint_as_float(below);
    }
    wave_lds_sync();

    // ---- steps 3-4: labels, per-cluster min and max.
    // Tree search: the state a = byte address of tree node `node`: a = T + 4*node, so the step
    // node' = 2*node + c is a' = 2a + (c ? 4 - T : -T).  The last step also subtracts T + 64,
    // which leaves 4*label.
    const uint32_t T = lds_addr(&ws.tree[0]);
    const uint32_t a_lo = T + 8u, a_hi = T + 12u;                  // nodes 2 and 3
    const uint32_t k0 = 0u - T, k1 = 4u - T;
    const uint32_t k0_last = 0u - 2u * T - 64u, k1_last = 4u - 2u * T - 64u;
    const uint32_t bins0 = lds_addr(&ws.bins[0]);
    const uint32_t tab0 = lds_addr(&ws.tab[0][lane]);              // + 256*label: this lane's min of the cluster
    // The searches run in batches of kBatch float4 (4*kBatch elements): all LDS reads of one step
    // are issued together and waited for once.  Left to itself the compiler's scheduler
    // finishes one element's read-compare-step chain before starting the next, which exposes
    // the LDS latency once per element and step; the scheduling barriers keep the batches intact.
    constexpr int kBatch = K >= 2 ? 2 : 1;
    constexpr int kB = 4 * kBatch;
    uint32_t packed[(K + 1) / 2];
#pragma unroll
    for (int i = 0; i < (K + 1) / 2; ++i)
        packed[i] = 0;
    auto label_pass = [&](auto by_bins_c) {
        constexpr bool kByBins = decltype(by_bins_c)::value;
#pragma unroll
        for (int kb = 0; kb < K; kb += kBatch) {
            float xs[kB];
            uint32_t label[kB];
#pragma unroll
            for (int i = 0; i < kB; ++i)
                xs[i] = comp(v[kb + i / 4], i % 4);
            if (kByBins) {
                uint32_t a[kB];
                float2 cb[kB];
#pragma unroll
                for (int i = 0; i < kB; ++i)
                    a[i] = bins0 + (bin_of(xs[i], bin_r, bin_c) << 3);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < kB; ++i)
                    cb[i] = lds_read_f32x2(a[i]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < kB; ++i)
                    label[i] = __float_as_uint(cb[i].y) + (xs[i] >= cb[i].x ? 1u : 0u);
            } else {
                uint32_t a[kB];
#pragma unroll
                for (int i = 0; i < kB; ++i)
                    a[i] = xs[i] >= root ? a_hi : a_lo;
#pragma unroll
                for (int st = 0; st < 3; ++st) {
                    float e[kB];
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int i = 0; i < kB; ++i)
                        e[i] = lds_read_f32(a[i]);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int i = 0; i < kB; ++i)
                        a[i] = (a[i] << 1) + (xs[i] >= e[i] ? (st == 2 ? k1_last : k1) : (st == 2 ? k0_last : k0));
                }
#pragma unroll
                for (int i = 0; i < kB; ++i)
                    label[i] = a[i] >> 2;
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < kBatch; ++b) {
                const int k = kb + b;
                uint32_t l4 = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t l = label[4 * b + j];
                    if (kFull || k * 256 + lane * 4 + j < len) {
                        // LDS float min/max without return value: no round trip, no conflict (private column)
                        float *pmin = (float *)(BITSNAP_LDS float *)(uintptr_t)(tab0 + (l << 8));
                        __hip_atomic_fetch_min(pmin, xs[4 * b + j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
                        __hip_atomic_fetch_max(pmin + kMaxClusters * kWave, xs[4 * b + j], __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_WAVEFRONT);
                        l4 |= l << (4 * j);
                    }
                }
                packed[k >> 1] |= l4 << (16 * (k & 1));
                // labels: two per byte, even element in the low nibble
                const int off = k * 256 + lane * 4;
                BITSNAP_GLOBAL uint8_t *lp = global_ptr(labels) + ((lo + off) >> 1);
                if (kFull || off + 3 < len) {
                    __builtin_nontemporal_store((uint16_t)l4, (BITSNAP_GLOBAL uint16_t *)lp);
                } else {
                    if (off < len)
                        lp[0] = (uint8_t)l4;
                    if (off + 2 < len)
                        lp[1] = (uint8_t)(l4 >> 8);
                }
            }
        }
    };
    if (by_bins)
        label_pass(std::true_type{});
    else
        label_pass(std::false_type{});
    wave_lds_sync();

    // ---- reduce the table over its 64 columns: lane handles row (lane & 31), half (lane >> 5)
    {
        const int row = lane & 31, half = lane >> 5;
        float mn = INFINITY, mx = -INFINITY;
#pragma unroll 8
        for (int j = 0; j < 32; ++j) {
            const float t = ws.tab[row][half * 32 + ((j + lane) & 31)];
            mn = fminf(mn, t);
            mx = fmaxf(mx, t);
        }
        float r = row < kMaxClusters ? mn : mx;
        const float o = __shfl_xor(r, 32, kWave);
        r = row < kMaxClusters ? fminf(r, o) : fmaxf(r, o);
        const float hi = __shfl_down(r, kMaxClusters, kWave);  // lane c receives max of cluster c
        if (lane < kMaxClusters) {
            float S = 0.0f, b = 0.0f, inv = 0.0f;
            if (r <= hi) {  // the cluster has members
                b = r;
                S = __fsub_rn(hi, r);
                if (S > 0.0f) {
                    inv = __fdiv_rn(255.0f, S);
                    if (!isfinite(inv))
                        inv = 0.0f;
                }
            }
            ws.coder[lane] = make_float2(b, inv);
            if (lane < m)
                *(BITSNAP_GLOBAL float2v *)(global_ptr(params) + (g * m + lane) * 2) = float2v{S, b};
        }
    }
    wave_lds_sync();

    // ---- steps 5-6: nearest of the 256 levels inside the element's cluster.  v_cvt_pk_u8_f32
    // rounds to nearest even, saturates to [0, 255], maps NaN to 0 and inserts the byte.
    const uint32_t coder0 = lds_addr(&ws.coder[0]);
#pragma unroll
    for (int kb = 0; kb < K; kb += kBatch) {
        float2 bi[kB];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < kB; ++i) {
            const int k = kb + i / 4;
            const uint32_t l4 = (packed[k >> 1] >> (16 * (k & 1))) & 0xFFFFu;
            bi[i] = lds_read_f32x2(coder0 + (((l4 >> (4 * (i % 4))) & 15u) << 3));
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
            const int k = kb + b;
            uint32_t c4 = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float y = __fmul_rn(__fsub_rn(comp(v[k], j), bi[4 * b + j].x), bi[4 * b + j].y);
                c4 = __builtin_amdgcn_cvt_pk_u8_f32(y, j, c4);
            }
            const int off = k * 256 + lane * 4;
            BITSNAP_GLOBAL uint8_t *cp = global_ptr(codes) + lo + off;
            if (kFull || off + 3 < len) {
                __builtin_nontemporal_store(c4, (BITSNAP_GLOBAL uint32_t *)cp);
            } else {
                for (int j = 0; j < 4; ++j)
                    if (off + j < len)
                        cp[j] = (uint8_t)(c4 >> (8 * j));
            }
        }
    }
    wave_lds_sync();  // this wave may start its next group and rewrite the tables
}

// Full groups: one wave per group, `groups` of them.  The short last group of a tensor (if any)
// goes through the same code with bounds checks, as a launch of its own (kFull = false, one wave).
template <int K, bool kFull>
__global__ __launch_bounds__(kQBlock) void quantize_cluster_kernel(
    const float *__restrict__ x, int64_t n, int64_t first_group, int64_t groups, int m, uint8_t *__restrict__ codes,
    uint8_t *__restrict__ labels, float *__restrict__ params, float *__restrict__ fit_out,
    const float *__restrict__ fit_in, uint32_t *__restrict__ status)
{
    __shared__ WaveShared shared[kQWaves];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int64_t g = first_group + (int64_t)blockIdx.x * kQWaves + wave;
    if (g >= first_group + groups)
        return;  // whole wave leaves; the kernel has no workgroup barrier
    constexpr int G = 256 * K;
    const int64_t lo = g * G;
    const int64_t rest = n - lo;
    const int len = kFull ? G : (int)(rest < G ? rest : G);
    quantize_group<K, kFull>(x, lo, len, m, g, codes, labels, params, fit_out, fit_in, status, shared[wave], lane);
}

// Dequantisation of one group by one wave: codes[lo..lo+len) -> out[lo..lo+len).
template <int K>
__device__ __forceinline__ void dequantize_group(const uint8_t *__restrict__ codes, const uint8_t *__restrict__ labels,
                                                 const float *__restrict__ params, int64_t lo, int len, int m, int64_t g,
                                                 float *__restrict__ out, float2 *coder, int lane)
{
    if (lane < kMaxClusters) {
        float2 sb = make_float2(0.0f, 0.0f);
        if (lane < m)
        {
            const float2v t = *(const BITSNAP_GLOBAL float2v *)(global_ptr(params) + (g * m + lane) * 2);
            sb = make_float2(t.x, t.y);
        }
        coder[lane] = make_float2(__fdiv_rn(sb.x, 255.0f), sb.y);  // (S/255, b)
    }
    wave_lds_sync();
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int off = k * 256 + lane * 4;
        if (off >= len)
            break;
        const bool full = off + 3 < len;
        uint32_t c4 = 0, l4 = 0;
        if (full) {
            c4 = __builtin_nontemporal_load((const BITSNAP_GLOBAL uint32_t *)(global_ptr(codes) + lo + off));
            l4 = __builtin_nontemporal_load((const BITSNAP_GLOBAL uint16_t *)(global_ptr(labels) + ((lo + off) >> 1)));
        } else {
            for (int j = 0; j < 4; ++j)
                if (off + j < len) {
                    c4 |= (uint32_t)global_ptr(codes)[lo + off + j] << (8 * j);
                    l4 |= (uint32_t)((global_ptr(labels)[(lo + off + j) >> 1] >> (4 * (j & 1))) & 15u) << (4 * j);
                }
        }
        float r[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float2 sb = coder[(l4 >> (4 * j)) & 15u];
            r[j] = __fadd_rn(__fmul_rn((float)((c4 >> (8 * j)) & 255u), sb.x), sb.y);
        }
        if (full) {
            __builtin_nontemporal_store(float4v{r[0], r[1], r[2], r[3]}, (BITSNAP_GLOBAL float4v *)(global_ptr(out) + lo + off));
        } else {
            for (int j = 0; j < 4; ++j)
                if (off + j < len)
                    global_ptr(out)[lo + off + j] = r[j];
        }
    }
    wave_lds_sync();  // the coder table may be rewritten by this wave's next group
}

template <int K>
__global__ __launch_bounds__(kQBlock) void dequantize_cluster_kernel(
    const uint8_t *__restrict__ codes, const uint8_t *__restrict__ labels, const float *__restrict__ params,
    int64_t n, int64_t groups, int m, float *__restrict__ out)
{
    __shared__ float2 coder[kQWaves][kMaxClusters];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int64_t g = (int64_t)blockIdx.x * kQWaves + wave;
    if (g >= groups)
        return;
    constexpr int G = 256 * K;
    const int64_t lo = g * G;
    const int64_t rest = n - lo;
    dequantize_group<K>(codes, labels, params, lo, rest >= G ? G : (int)rest, m, g, out, coder[wave], lane);
}

// ---------------------------------------------------------------------------------------------
// Batched forms: one launch for a list of tensors.  Groups are numbered across the list
// (item.first_group = groups of all earlier items) and the grid has one wave per group of the
// whole list, so the device works through many rounds of waves whose load, compute and store
// phases overlap; a single tensor of a few thousand groups is one round (one group per wave slot)
// whose phases cannot overlap.
// ---------------------------------------------------------------------------------------------

// The item that holds list-wide group gg: the last one whose first_group <= gg (binary search;
// every operand is wave-uniform, so this runs on the scalar unit).
__device__ __forceinline__ int64_t find_item(const bitsnap_cluster_item *__restrict__ items, int64_t count, int64_t gg)
{
    int64_t lo = 0, hi = count - 1;
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if (items[mid].first_group <= gg)
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo;
}

__device__ __forceinline__ int64_t uniform_i64(int64_t v)
{
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)(uint64_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

template <int K, bool kFull>
__global__ __launch_bounds__(kQBlock) void quantize_cluster_batched_kernel(
    const bitsnap_cluster_item *__restrict__ items, int64_t count, int64_t total_groups, int m,
    uint32_t *__restrict__ status)
{
    __shared__ WaveShared shared[kQWaves];
    // the wave index as a scalar: group and item bookkeeping then lives in SGPRs
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr int G = 256 * K;
    if (kFull) {
        const int64_t gg = (int64_t)blockIdx.x * kQWaves + wave;
        if (gg >= total_groups)
            return;
        const bitsnap_cluster_item &it = items[find_item(items, count, gg)];
        const int64_t g = gg - it.first_group;
        const int64_t lo = g * G;
        if (it.n - lo >= G)  // a short last group is left to the tail launch
            quantize_group<K, true>((const float *)it.values, lo, G, m, g, it.codes, it.labels, it.params, it.fit_out,
                                    it.fit_in, status, shared[wave], lane);
    } else {
        // one wave per tensor: its short last group, if it has one
        const int64_t t = (int64_t)blockIdx.x * kQWaves + wave;
        if (t >= count)
            return;
        const bitsnap_cluster_item &it = items[t];
        const int64_t g = it.n / G;
        const int rest = (int)(it.n - g * G);
        if (rest > 0)
            quantize_group<K, false>((const float *)it.values, g * G, rest, m, g, it.codes, it.labels, it.params,
                                     it.fit_out, it.fit_in, status, shared[wave], lane);
    }
}

template <int K>
__global__ __launch_bounds__(kQBlock) void dequantize_cluster_batched_kernel(
    const bitsnap_cluster_item *__restrict__ items, int64_t count, int64_t total_groups, int m)
{
    __shared__ float2 coder[kQWaves][kMaxClusters];
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr int G = 256 * K;
    const int64_t gg = (int64_t)blockIdx.x * kQWaves + wave;
    if (gg >= total_groups)
        return;
    const bitsnap_cluster_item &it = items[find_item(items, count, gg)];
    const int64_t g = gg - it.first_group;
    const int64_t lo = g * G;
    const int64_t rest = it.n - lo;
    if (rest > 0)
        dequantize_group<K>(it.codes, it.labels, it.params, lo, rest >= G ? G : (int)rest, m, g, (float *)it.values,
                            coder[wave], lane);
}

// K (float4 per lane) of the one-wave-per-group kernels, or 0 when the group length needs the
// multi-pass path
static int group_k(int64_t n, int64_t group)
{
    (void)n;
    switch (group) {
    case 256: return 1;
    case 512: return 2;
    case 1024: return 4;
    case 2048: return 8;
    case 4096: return 16;
    default: return 0;
    }
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
    if (n <= 0 || group_k(n, group) != 0)
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
    const int K = group_k(n, group);
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
    const int64_t full = n / G;                  // groups that are complete
    const bool tail = (n % G) != 0;              // plus one short group
    const int64_t blocks = (full + kQWaves - 1) / kQWaves;
    if (blocks > 0x7FFFFFFF)
        return BITSNAP_E_SIZE;
    const dim3 block(kQBlock);
    hipStream_t s = (hipStream_t)stream;
#define BITSNAP_LAUNCH_Q(KK)                                                                                       \
    do {                                                                                                           \
        if (full > 0)                                                                                              \
            hipLaunchKernelGGL((quantize_cluster_kernel<KK, true>), dim3((unsigned)blocks), block, 0, s, x, n,     \
                               (int64_t)0, full, m, codes, labels, params, fit_out, fit_in, status);               \
        if (tail)                                                                                                  \
            hipLaunchKernelGGL((quantize_cluster_kernel<KK, false>), dim3(1), block, 0, s, x, n, full, (int64_t)1, \
                               m, codes, labels, params, fit_out, fit_in, status);                                 \
    } while (0)
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
    const int K = group_k(n, group);
    if (K == 0 && !cluster_general_supported(n, group))
        return BITSNAP_E_SIZE;
    if (!codes || !labels || !params || !out)
        return BITSNAP_E_NULL;
    if (!aligned16(codes) || !aligned16(labels) || !aligned16(params) || !aligned16(out))
        return BITSNAP_E_ALIGN;
    if (K == 0)
        return cluster_general_dequantize(codes, labels, params, n, group, m, out, (hipStream_t)stream);
    const int64_t groups = (int64_t)bitsnap_cluster_groups(n, group);
    const int64_t blocks = (groups + kQWaves - 1) / kQWaves;
    if (blocks > 0x7FFFFFFF)
        return BITSNAP_E_SIZE;
    const dim3 grid((unsigned)blocks), block(kQBlock);
    hipStream_t s = (hipStream_t)stream;
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

static int64_t batched_blocks(int64_t total_groups) { return (total_groups + kQWaves - 1) / kQWaves; }

extern "C" int bitsnap_quantize_cluster_batched(const bitsnap_cluster_item *items, int64_t count, int64_t total_groups,
                                                int64_t group, int m, uint32_t *status, bitsnap_stream_t stream)
{
    if (count < 0 || total_groups < 0 || m < 1 || m > kMaxClusters)
        return BITSNAP_E_SIZE;
    const int K = group_k(0, group);
    if (K == 0)
        return BITSNAP_E_SIZE;  // the batched form exists for the one-wave-per-group lengths only
    if (count == 0 || total_groups == 0)
        return BITSNAP_OK;
    if (!items)
        return BITSNAP_E_NULL;
    if (((uintptr_t)items & 7u) || ((uintptr_t)status & 3u))
        return BITSNAP_E_ALIGN;
    if (batched_blocks(total_groups) > 0x7FFFFFFF)
        return BITSNAP_E_SIZE;
    const dim3 block(kQBlock), grid((unsigned)batched_blocks(total_groups)), tgrid((unsigned)((count + kQWaves - 1) / kQWaves));
    hipStream_t s = (hipStream_t)stream;
#define BITSNAP_LAUNCH_QB(KK)                                                                                     \
    do {                                                                                                          \
        hipLaunchKernelGGL((quantize_cluster_batched_kernel<KK, true>), grid, block, 0, s, items, count,          \
                           total_groups, m, status);                                                              \
        hipLaunchKernelGGL((quantize_cluster_batched_kernel<KK, false>), tgrid, block, 0, s, items, count,        \
                           total_groups, m, status);                                                              \
    } while (0)
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
    const int K = group_k(0, group);
    if (K == 0)
        return BITSNAP_E_SIZE;
    if (count == 0 || total_groups == 0)
        return BITSNAP_OK;
    if (!items)
        return BITSNAP_E_NULL;
    if ((uintptr_t)items & 7u)
        return BITSNAP_E_ALIGN;
    if (batched_blocks(total_groups) > 0x7FFFFFFF)
        return BITSNAP_E_SIZE;
    const dim3 block(kQBlock), grid((unsigned)batched_blocks(total_groups));
    hipStream_t s = (hipStream_t)stream;
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
