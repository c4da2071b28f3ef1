// Building blocks of the cluster quantiser (paper: "Cluster Based Quantization for Optimizer
// States", Algorithm 2) for one wavefront that holds up to 256*K consecutive fp32 elements in
// registers, K float4 per lane: lane l owns elements k*256 + l*4 + {0..3}, k = 0..K-1.
//
//   load_elements   HBM -> registers
//   wave_stats      step 1: sum and sum of squared deviations, fp64
//   build_search    step 2: edges e_k = mu + sigma*z_k; the two label-search structures in LDS
//   label_pass      steps 3-4: labels (packed, optionally stored), per-cluster min/max in LDS
//   reduce_ranges   step 4: min and max of every cluster over the wave's elements
//   code_pass       steps 5-6: codes, stored
//   dequantize_group  the inverse
//
// The one-wave-per-group kernels run all of them on one group; the wide-group kernels (a group
// spans many waves) run them in three passes with the group's state in a workspace.
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <type_traits>

#include "wave.hpp"

namespace bitsnap {

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

// Phi^-1(k/m), correctly rounded (one copy per translation unit)
static __constant__ double kZDev[17][16] = {
#include "z_table.inc"
};

struct alignas(16) WaveShared {
    float tab[2 * kMaxClusters][kWave];  // rows 0..15: running min per cluster, rows 16..31: running max
    float tree[kMaxClusters];            // node i of the edge search tree (node 1 = root), [0] unused
    float2 coder[kMaxClusters];          // (b, 255/S) for quantize, (S/255, b) for dequantize
    float2 bins[kBins];                  // label search by bins: (the edge inside the bin or NaN, edges below the bin)
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
// table lookup and the address arithmetic.
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
__device__ __forceinline__ float4 load_stream(const float *p)
{
    const float4v t = __builtin_nontemporal_load((const BITSNAP_GLOBAL float4v *)p);
    return make_float4(t.x, t.y, t.z, t.w);
}

// ---- load: x[lo .. lo+len) -> v; elements at or beyond len read as 0.  kFull: len == 256*K and
// x + lo is 16-byte aligned.
template <int K, bool kFull>
__device__ __forceinline__ void load_elements(const float *__restrict__ x, int64_t lo, int len, int lane, float4 (&v)[K])
{
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
}

// ---- step 1: sum of the elements and, about their mean, the sum of squared deviations; fp64
// per-lane partial sums, then a DPP tree across the wave (fixed association: reproducible).
// The deviations come from one pass where that is safe: the square of an fp32 number is exact in fp64, so
// Q = sum of x^2 carries only the rounding of its 4096 additions (below 1e-14 relative), and
// Q - S^2/n loses log2(Q / result) of the 53 bits to cancellation.  Where the result keeps more than 1/64 of
// Q (|mean| below 8 deviations) its relative error stays under 1e-12, far below what changes the fp32
// rounding of the deviation in more than one group in a million; every other group (and every group whose
// elements are all equal, where the result must be an exact zero) takes the second pass over x - mean.
template <int K, bool kFull>
__device__ __forceinline__ void wave_stats(float4 (&v)[K], int len, int lane, double &sum, double &dev)
{
    double s0 = 0.0, s1 = 0.0, q0 = 0.0, q1 = 0.0;
#pragma unroll
    for (int k = 0; k < K; ++k) {  // padding adds 0 to both
        const double x = (double)v[k].x, y = (double)v[k].y, z = (double)v[k].z, w = (double)v[k].w;
        s0 += x + y;
        s1 += z + w;
        q0 = fma(x, x, q0);
        q1 = fma(y, y, q1);
        q0 = fma(z, z, q0);
        q1 = fma(w, w, q1);
    }
    const double s = wave_sum(s0 + s1), q = wave_sum(q0 + q1);
    const double mean = s / (double)len;
    double d = fma(-s, mean, q);
    if (!(d > q * 0x1p-6)) {  // wave-uniform
        // Keep the elements as fp32 in registers: without this the compiler holds on to the fp64 copies
        // made above, which doubles the register footprint and halves the occupancy.
#pragma unroll
        for (int k = 0; k < K; ++k)
            asm volatile("" : "+v"(v[k].x), "+v"(v[k].y), "+v"(v[k].z), "+v"(v[k].w));
        double t = 0.0;
#pragma unroll
        for (int k = 0; k < K; ++k) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (kFull || k * 256 + lane * 4 + j < len) {
                    const double e = (double)comp(v[k], j) - mean;
                    t = fma(e, e, t);
                }
            }
        }
        d = wave_sum(t);
    }
    sum = s;
    dev = d;
}

// Running min/max table: this lane's column back to "no members" (call before label_pass with
// kRanges; best right after the loads are issued, the writes then hide under the load latency).
__device__ __forceinline__ void reset_ranges(WaveShared &ws, int lane)
{
#pragma unroll
    for (int c = 0; c < kMaxClusters; ++c) {
        ws.tab[c][lane] = INFINITY;
        ws.tab[kMaxClusters + c][lane] = -INFINITY;
    }
}

// What the label search needs besides the LDS tables.
struct LabelSearch {
    float root;          // the middle edge e_8: first step of the tree search
    float bin_r, bin_c;  // bin(x) = min(63, sat_u8(rne(x*bin_r + bin_c)))
    bool by_bins;        // every edge alone in its bin: the bin table is valid
};

// ---- step 2: edges e_k = fl32(mu + sigma * z_k), product and sum rounded separately in fp64;
// lane k holds e_k (returned through `edge`; NaN where there is no edge: never <= x, whatever x).
// Fills ws.tree and ws.bins.
__device__ __forceinline__ LabelSearch build_search(float mu, float sigma, int m, WaveShared &ws, int lane, float &edge)
{
    edge = __uint_as_float(0x7FC00000u);
    if (lane >= 1 && lane < m)
        edge = (float)__dadd_rn((double)mu, __dmul_rn((double)sigma, kZDev[m][lane]));
    if (lane >= 1 && lane < kMaxClusters) {
        const int tz = __ffs(lane) - 1;
        ws.tree[(1 << (3 - tz)) + (lane >> (tz + 1))] = edge;
    }
    LabelSearch ls;
    ls.root = read_lane(edge, 8);
    ls.bin_r = __fdiv_rn(kBinsPerSigma, sigma);
    ls.bin_c = __fsub_rn(kBinOffset, __fmul_rn(mu, ls.bin_r));
    ws.bins[lane] = make_float2(__uint_as_float(0x7FC00000u), 0.0f);  // NaN: no edge here, and x >= NaN never holds
    wave_lds_sync();
    if (lane >= 1 && lane < m)
        ws.bins[bin_of(edge, ls.bin_r, ls.bin_c)].x = edge;
    wave_lds_sync();
    const float mine = ws.bins[lane].x;
    const uint64_t occupied = __ballot(mine == mine);
    ls.by_bins = (int)__popcll(occupied) == m - 1 && ls.bin_r > 0.0f;
    const uint32_t below = __builtin_amdgcn_mbcnt_hi((uint32_t)(occupied >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)occupied, 0u));
    ws.bins[lane].y = __uint_as_float(below);
    wave_lds_sync();
    return ls;
}

// ---- steps 3-4: labels of the wave's elements -> packed (4 bits each, 8 elements of two
// consecutive float4 per word); kStore: also written to labels[] (two per byte, even element in
// the low nibble; lo is even); kRanges: per-cluster min/max into this lane's column of ws.tab.
//
// Tree search: the state a = byte address of tree node `node`: a = T + 4*node, so the step
// node' = 2*node + c is a' = 2a + (c ? 4 - T : -T).  The last step also subtracts T + 64, which
// leaves 4*label.
// The searches run in batches of kBatch float4 (4*kBatch elements): all LDS reads of one step are
// issued together and waited for once.  Left to itself the compiler's scheduler finishes one
// element's read-compare-step chain before starting the next, which exposes the LDS latency
// once per element and step; the scheduling barriers keep the batches intact.
template <int K, bool kFull, bool kStore, bool kRanges, bool kByBins>
__device__ __forceinline__ void label_pass_impl(const float4 (&v)[K], int64_t lo, int len, const LabelSearch &ls,
                                                WaveShared &ws, int lane, uint8_t *__restrict__ labels,
                                                uint32_t (&packed)[(K + 1) / 2])
{
    const uint32_t T = lds_addr(&ws.tree[0]);
    const uint32_t a_lo = T + 8u, a_hi = T + 12u;  // nodes 2 and 3
    const uint32_t k0 = 0u - T, k1 = 4u - T;
    const uint32_t k0_last = 0u - 2u * T - 64u, k1_last = 4u - 2u * T - 64u;
    const uint32_t bins0 = lds_addr(&ws.bins[0]);
    const uint32_t tab0 = lds_addr(&ws.tab[0][lane]);  // + 256*label: this lane's min of the cluster
    constexpr int kBatch = K >= 2 ? 2 : 1;
    constexpr int kB = 4 * kBatch;
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
                a[i] = bins0 + (bin_of(xs[i], ls.bin_r, ls.bin_c) << 3);
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
                a[i] = xs[i] >= ls.root ? a_hi : a_lo;
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
                    if (kRanges) {
                        // LDS float min/max without return value: no round trip, no conflict (private column)
                        float *pmin = (float *)(BITSNAP_LDS float *)(uintptr_t)(tab0 + (l << 8));
                        __hip_atomic_fetch_min(pmin, xs[4 * b + j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
                        __hip_atomic_fetch_max(pmin + kMaxClusters * kWave, xs[4 * b + j], __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_WAVEFRONT);
                    }
                    l4 |= l << (4 * j);
                }
            }
            packed[k >> 1] |= l4 << (16 * (k & 1));
            if (kStore) {
                const int off = k * 256 + lane * 4;
                // lo and off are even; written as a sum, the constant part of off becomes the store's offset field
                BITSNAP_GLOBAL uint8_t *lp = global_ptr(labels) + (lo >> 1) + (lane * 2) + k * 128;
                if (kFull || (off + 3 < len && (lo & 3) == 0)) {  // four whole elements at an aligned place
                    __builtin_nontemporal_store((uint16_t)l4, (BITSNAP_GLOBAL uint16_t *)lp);
                } else {
                    if (off < len)
                        lp[0] = (uint8_t)l4;
                    if (off + 2 < len)
                        lp[1] = (uint8_t)(l4 >> 8);
                }
            }
        }
    }
}

template <int K, bool kFull, bool kStore, bool kRanges>
__device__ __forceinline__ void label_pass(const float4 (&v)[K], int64_t lo, int len, const LabelSearch &ls, WaveShared &ws,
                                           int lane, uint8_t *__restrict__ labels, uint32_t (&packed)[(K + 1) / 2])
{
#pragma unroll
    for (int i = 0; i < (K + 1) / 2; ++i)
        packed[i] = 0;
    if (ls.by_bins)
        label_pass_impl<K, kFull, kStore, kRanges, true>(v, lo, len, ls, ws, lane, labels, packed);
    else
        label_pass_impl<K, kFull, kStore, kRanges, false>(v, lo, len, ls, ws, lane, labels, packed);
    wave_lds_sync();
}

// ---- step 4: reduce the min/max table over its 64 columns.  Lane c < 16 returns the minimum of
// cluster c in `mn` and its maximum in `mx` (+inf / -inf for a cluster without members).
__device__ __forceinline__ void reduce_ranges(WaveShared &ws, int lane, float &mn_out, float &mx_out)
{
    const int row = lane & 31, half = lane >> 5;  // lane handles row (lane & 31), half (lane >> 5)
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
    mn_out = r;
    mx_out = __shfl_down(r, kMaxClusters, kWave);  // lane c receives the max of cluster c
}

// (S, b, 255/S) of a cluster from its minimum and maximum (Algorithm 2 step 4; S = max - min,
// b = min; a cluster without members gets (0, 0); a range too small to code gets 255/S = 0).
__device__ __forceinline__ void cluster_coder(float mn, float mx, float &S, float &b, float &inv)
{
    S = 0.0f, b = 0.0f, inv = 0.0f;
    if (mn <= mx) {  // the cluster has members
        b = mn;
        S = __fsub_rn(mx, mn);
        if (S > 0.0f) {
            inv = __fdiv_rn(255.0f, S);
            if (!isfinite(inv))
                inv = 0.0f;
        }
    }
}

// ---- steps 5-6: nearest of the 256 levels inside the element's cluster, (b, 255/S) per cluster
// from ws.coder.  v_cvt_pk_u8_f32 rounds to nearest even, saturates to [0, 255], maps NaN to 0
// and inserts the byte.
template <int K, bool kFull>
__device__ __forceinline__ void code_pass(const float4 (&v)[K], int64_t lo, int len, const uint32_t (&packed)[(K + 1) / 2],
                                          WaveShared &ws, int lane, uint8_t *__restrict__ codes)
{
    constexpr int kBatch = K >= 2 ? 2 : 1;
    constexpr int kB = 4 * kBatch;
    const uint32_t coder0 = lds_addr(&ws.coder[0]);
#pragma unroll
    for (int kb = 0; kb < K; kb += kBatch) {
        float2 bi[kB];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < kB; ++i) {
            const int k = kb + i / 4;
            // bit-field extract + shift-add: two instructions per address
            uint32_t label;
            asm("v_bfe_u32 %0, %1, %2, 4" : "=v"(label) : "v"(packed[k >> 1]), "n"(16 * (k & 1) + 4 * (i % 4)));
            bi[i] = lds_read_f32x2((label << 3) + coder0);
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
            if (kFull || (off + 3 < len && (lo & 3) == 0)) {
                __builtin_nontemporal_store(c4, (BITSNAP_GLOBAL uint32_t *)cp);
            } else {
                for (int j = 0; j < 4; ++j)
                    if (off + j < len)
                        cp[j] = (uint8_t)(c4 >> (8 * j));
            }
        }
    }
    wave_lds_sync();  // this wave may go on to other elements and rewrite the tables
}

// Dequantisation (x^ = q * (S/255) + b, product and sum rounded separately) of len <= 256*K
// consecutive elements of group g by one wave: codes[lo..lo+len) -> out[lo..lo+len).  `aligned`:
// lo is a multiple of 4, so four elements are one 4-byte, 2-byte and 16-byte access.
template <int K>
__device__ __forceinline__ void dequantize_group(const uint8_t *__restrict__ codes, const uint8_t *__restrict__ labels,
                                                 const float *__restrict__ params, int64_t lo, int len, bool aligned,
                                                 int m, int64_t g, float *__restrict__ out, float2 *coder, int lane)
{
    // codes and labels are requested first, the 16 (S, b) pairs next: one memory latency, not two
    uint32_t c4[K], l4[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int off = k * 256 + lane * 4;
        c4[k] = 0, l4[k] = 0;
        if (aligned && off + 3 < len) {
            c4[k] = __builtin_nontemporal_load((const BITSNAP_GLOBAL uint32_t *)(global_ptr(codes) + lo + off));
            l4[k] = __builtin_nontemporal_load((const BITSNAP_GLOBAL uint16_t *)(global_ptr(labels) + (lo >> 1) + lane * 2 + k * 128));
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
        coder[lane] = make_float2(__fdiv_rn(sb.x, 255.0f), sb.y);  // (S/255, b)
    }
    wave_lds_sync();
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int off = k * 256 + lane * 4;
        float r[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float2 sb = coder[(l4[k] >> (4 * j)) & 15u];
            r[j] = __fadd_rn(__fmul_rn((float)((c4[k] >> (8 * j)) & 255u), sb.x), sb.y);
        }
        if (aligned && off + 3 < len) {
            __builtin_nontemporal_store(float4v{r[0], r[1], r[2], r[3]}, (BITSNAP_GLOBAL float4v *)(global_ptr(out) + lo + off));
        } else {
            for (int j = 0; j < 4; ++j)
                if (off + j < len)
                    global_ptr(out)[lo + off + j] = r[j];
        }
    }
    wave_lds_sync();  // the coder table may be rewritten by this wave's next group
}

}  // namespace bitsnap
