// Format variants of the cluster quantiser (paper: "Cluster Based Quantization for Optimizer
// States"):
//   * a general map Q^map in Eq. qmap-distance: code = the entry of a 256-entry table nearest to
//     (x-b)/S, and T^D = Q(T^Q)*S + b on the way back;
//   * the cluster-major arrangement of Eq. decluster: inside a group the codes of cluster 0 come
//     first, then cluster 1, ..., each cluster's codes in element order.
//
// One wavefront per group, as in the plain kernels, and steps 1-4 of Algorithm 2 are the same
// code.  The table lives in LDS once per workgroup, turned into a step function over 1024 bins
// of (x-b)/S where its levels are far enough apart for that, and searched by bisection otherwise.
// The
// cluster-major arrangement is a stable 16-way partition of the group's codes done inside the
// wave through LDS: the codes and the labels are laid down in element order; then lane l takes
// the 4K consecutive elements l*4K .. l*4K+4K-1, counts its labels into a private column of a
// [16][64] counter table, an exclusive prefix sum over that table read row by row (cluster, then
// lane) turns every counter into the position of the lane's first member of the cluster, and a
// second walk over the same elements hands out consecutive positions.
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

constexpr int kVBlock = 256;
constexpr int kVWaves = kVBlock / kWave;
constexpr int kLevels = 256;

// LDS of one wave for the partition.
struct MajorView {
    uint32_t *counters;  // [16][64]: cluster c, lane l at c*64 + l
    uint32_t *bytes;     // [256*K] bytes: the group's codes (element order on one side, cluster-major on the other)
    uint32_t *labels;    // [256*K] nibbles: the group's labels in element order
};

struct alignas(16) QuantizeShared {
    WaveShared ws;
    uint32_t labels[kMaxClusters * 256 / 8];
};

struct alignas(16) DequantizeShared {
    uint32_t counters[kMaxClusters][kWave];
    uint32_t bytes[kMaxClusters * 256 / 4];
    uint32_t labels[kMaxClusters * 256 / 8];
    float2 coder[kMaxClusters];
};

__device__ __forceinline__ uint32_t lds_fetch_add(uint32_t *p, uint32_t v)
{
    return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
}

// The lane's own labels: halfword i holds those of elements lane*4K + 4i .. + 3.
template <int K>
__device__ __forceinline__ void own_labels(const MajorView &mv, int lane, uint32_t (&lh)[K])
{
    const uint16_t *l16 = (const uint16_t *)mv.labels;
#pragma unroll
    for (int i = 0; i < K; ++i)
        lh[i] = l16[lane * K + i];
}

// Counts the lane's labels and turns the counter table into first positions: afterwards
// counters[c][lane] = members of clusters < c in the group + members of c in lower lanes.
template <int K, bool kFull>
__device__ __forceinline__ void major_positions(const MajorView &mv, const uint32_t (&lh)[K], int len, int lane)
{
#pragma unroll
    for (int c = 0; c < kMaxClusters; ++c)
        mv.counters[c * kWave + lane] = 0;
#pragma unroll
    for (int i = 0; i < K; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (kFull || lane * 4 * K + 4 * i + j < len)
                lds_fetch_add(&mv.counters[((lh[i] >> (4 * j)) & 15u) * kWave + lane], 1u);
    wave_lds_sync();
    // exclusive prefix over the 1024 counters in row order: 16 consecutive ones per lane
    uint32_t c[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
        c[i] = mv.counters[lane * 16 + i];
    uint32_t total = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint32_t t = c[i];
        c[i] = total;
        total += t;
    }
    const uint32_t before = wave_inclusive_add(total) - total;
    wave_lds_sync();  // every lane has read its 16 counters (other lanes' columns) before any is rewritten
#pragma unroll
    for (int i = 0; i < 16; ++i)
        mv.counters[lane * 16 + i] = c[i] + before;
    wave_lds_sync();
}

// Element order -> cluster-major.  In: mv.bytes and mv.labels hold the group in element order.
// Out: mv.bytes holds the cluster-major arrangement.
template <int K, bool kFull>
__device__ __forceinline__ void to_cluster_major(const MajorView &mv, int len, int lane)
{
    uint32_t lh[K], cw[K];
    own_labels<K>(mv, lane, lh);
#pragma unroll
    for (int i = 0; i < K; ++i)
        cw[i] = mv.bytes[lane * K + i];
    major_positions<K, kFull>(mv, lh, len, lane);  // its barriers also order the reads above before the writes below
    uint8_t *b8 = (uint8_t *)mv.bytes;
#pragma unroll
    for (int i = 0; i < K; ++i) {
        uint32_t pos[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            pos[j] = 0;
            if (kFull || lane * 4 * K + 4 * i + j < len)
                pos[j] = lds_fetch_add(&mv.counters[((lh[i] >> (4 * j)) & 15u) * kWave + lane], 1u);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (kFull || lane * 4 * K + 4 * i + j < len)
                b8[pos[j]] = (uint8_t)(cw[i] >> (8 * j));
    }
    wave_lds_sync();
}

// Cluster-major -> element order.  In: mv.bytes cluster-major, mv.labels element order.
// Out: mv.bytes in element order.
template <int K, bool kFull>
__device__ __forceinline__ void from_cluster_major(const MajorView &mv, int len, int lane)
{
    uint32_t lh[K], cw[K];
    own_labels<K>(mv, lane, lh);
    major_positions<K, kFull>(mv, lh, len, lane);
    const uint8_t *b8 = (const uint8_t *)mv.bytes;
#pragma unroll
    for (int i = 0; i < K; ++i) {
        uint32_t pos[4];
        cw[i] = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            pos[j] = 0;
            if (kFull || lane * 4 * K + 4 * i + j < len)
                pos[j] = lds_fetch_add(&mv.counters[((lh[i] >> (4 * j)) & 15u) * kWave + lane], 1u);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (kFull || lane * 4 * K + 4 * i + j < len)
                cw[i] |= (uint32_t)b8[pos[j]] << (8 * j);
    }
    wave_lds_sync();  // every lane has fetched its codes before the element-order copy overwrites them
#pragma unroll
    for (int i = 0; i < K; ++i)
        mv.bytes[lane * K + i] = cw[i];
    wave_lds_sync();
}

// ---------------------------------------------------------------------------------------------
// Eq. qmap-distance with a table, decided in fp32: code(t) = the index of the entry nearest to
// t in rounded distance fl32(|Q_j - t|), the lowest index where several are equally near.
//
// General search.  The table is non-decreasing, so the nearest entry is one of the two that
// bracket t: p = the last entry <= t among entries 1..255 (0 if there is none; 8 bisection
// steps) and its successor.  Entries below p can only tie with it, never beat it; the walk down
// at the end finds the first of such a run.
//
// Search by bins.  Let L_0 < L_1 < ... be the distinct levels of the table and f_k the first
// index of level k.  For a well-separated table code(t) = f_k with k = #{i >= 1 : theta_i <= t},
// where theta_i is the smallest fp32 t that is nearer (in rounded distance) to L_i than to
// L_{i-1}: a step function, evaluated like the label search - bin(t) = min(1023, floor(1024 t))
// is non-decreasing, every bin stores the threshold inside it (or NaN) and the codes below and
// at that threshold, so an element costs one 8-byte LDS read and a compare.  It needs
//   * at most one threshold per bin, and every threshold found within a few ulps of the midpoint;
//   * no two levels so close that, seen from a t whose nearest level is the upper of them, their
//     rounded distances coincide (the reference then answers with the lower one's index): with
//     t <= 1 + 2^-22, which holds for every element because x - b <= S, it is enough that
//     L_k - L_{k-1} >= 2^-20 (min(L_{k+1}, 1 + 2^-22) - L_{k-1}) for all k.
// Both are checked on the table itself, once per workgroup; a table that fails takes the
// general search.
// ---------------------------------------------------------------------------------------------
constexpr int kTableBins = 1024;
constexpr float kTMax = 1.0f + 0x1p-22f;

struct alignas(16) TableShared {
    float q[kLevels];
    float2 bins[kTableBins];     // (threshold in the bin or NaN, code below it | code at and above it << 16)
    uint16_t bin_of_entry[kLevels];  // bin of the threshold that starts entry j's level (first entries only)
    uint32_t general;            // != 0: this table takes the general search
};

__device__ __forceinline__ uint32_t table_bin(float t)
{
    // floor(1024 t) held to 0..1023; NaN goes to bin 0
    return (uint32_t)fminf(fmaxf(__fmul_rn(t, (float)kTableBins), 0.0f), (float)(kTableBins - 1));
}

__device__ __forceinline__ float next_up(float x)
{
    if (x == 0.0f)
        return __uint_as_float(1u);
    const uint32_t u = __float_as_uint(x);
    return __uint_as_float(x > 0.0f ? u + 1u : u - 1u);
}

__device__ __forceinline__ float next_down(float x)
{
    if (x == 0.0f)
        return __uint_as_float(0x80000001u);
    const uint32_t u = __float_as_uint(x);
    return __uint_as_float(x > 0.0f ? u - 1u : u + 1u);
}

// Fills the workgroup's copy of the table and its bins; thread j of the kVBlock == kLevels
// threads takes entry j.  Contains workgroup barriers: call with every thread.
__device__ __forceinline__ void load_table(TableShared &ts, const float *__restrict__ qmap)
{
    const int j = threadIdx.x;
    const float nan = __uint_as_float(0x7FC00000u);
    ts.q[j] = global_ptr(qmap)[j];
    for (int i = 0; i < kTableBins / kLevels; ++i)
        ts.bins[j * (kTableBins / kLevels) + i] = make_float2(nan, 0.0f);
    if (j == 0)
        ts.general = 0;
    __syncthreads();
    const float B = ts.q[j];
    const bool first = j == 0 || ts.q[j - 1] != B;  // entry j starts a level
    int below = 0, above = j + 1;                   // first entry of the level below, first entry of the level above
    float theta = nan;
    bool bad = !(B == B) || (j > 0 && ts.q[j - 1] > B);  // NaN entry or a decreasing step
    if (first) {
        while (above < kLevels && ts.q[above] == B)
            ++above;
        if (j > 0) {
            const float A = ts.q[j - 1];
            below = j - 1;
            while (below > 0 && ts.q[below - 1] == A)
                --below;
            // theta: the smallest t with fl|B - t| < fl|A - t|; the predicate is monotone in t
            float c = __fadd_rn(__fmul_rn(0.5f, A), __fmul_rn(0.5f, B));
            bool found = false;
            for (int it = 0; it < 32 && !found; ++it) {
                if (fabsf(__fsub_rn(B, c)) < fabsf(__fsub_rn(A, c))) {
                    const float d = next_down(c);
                    if (fabsf(__fsub_rn(B, d)) < fabsf(__fsub_rn(A, d)))
                        c = d;
                    else
                        found = true;
                } else {
                    c = next_up(c);
                }
            }
            theta = c;
            const float next_level = above < kLevels ? ts.q[above] : kTMax;
            const float span = __fsub_rn(fminf(next_level, kTMax), A);
            bad = bad || !found || !(__fsub_rn(B, A) >= __fmul_rn(span, 0x1p-20f));
            const uint32_t bin = table_bin(theta);
            ts.bin_of_entry[j] = (uint16_t)bin;
            ts.bins[bin].y = __uint_as_float((uint32_t)j);  // claim the bin
        }
    }
    __syncthreads();
    if (first && j > 0 && __float_as_uint(ts.bins[ts.bin_of_entry[j]].y) != (uint32_t)j)
        bad = true;  // another threshold claimed the same bin
    if (bad)
        atomicOr(&ts.general, 1u);
    __syncthreads();
    if (first && ts.general == 0) {
        // entry j's level answers from just after its own threshold up to the next level's threshold
        const int from = j == 0 ? 0 : (int)ts.bin_of_entry[j] + 1;
        const int to = above < kLevels ? (int)ts.bin_of_entry[above] : kTableBins;  // the next threshold's bin, or the end
        for (int b = from; b < to; ++b)
            ts.bins[b] = make_float2(nan, __uint_as_float((uint32_t)j | ((uint32_t)j << 16)));
        if (j > 0)
            ts.bins[ts.bin_of_entry[j]] = make_float2(theta, __uint_as_float((uint32_t)below | ((uint32_t)j << 16)));
    }
    __syncthreads();
}

constexpr int kTableBatch = 8;

__device__ __forceinline__ void table_codes_by_bins(const TableShared &ts, const float (&t)[kTableBatch],
                                                    uint32_t (&code)[kTableBatch])
{
    float2 e[kTableBatch];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < kTableBatch; ++i)
        e[i] = ts.bins[table_bin(t[i])];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < kTableBatch; ++i) {
        const uint32_t c = __float_as_uint(e[i].y);
        code[i] = t[i] >= e[i].x ? c >> 16 : c & 0xFFFFu;
    }
}

__device__ __forceinline__ void table_codes_general(const TableShared &ts, const float (&t)[kTableBatch],
                                                    uint32_t (&code)[kTableBatch])
{
    uint32_t p[kTableBatch];
#pragma unroll
    for (int i = 0; i < kTableBatch; ++i)
        p[i] = 0;
#pragma unroll
    for (int s = kLevels / 2; s >= 1; s >>= 1) {
        float q[kTableBatch];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < kTableBatch; ++i)
            q[i] = ts.q[p[i] + s];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < kTableBatch; ++i)
            p[i] += q[i] <= t[i] ? (uint32_t)s : 0u;
    }
    float ql[kTableBatch], qh[kTableBatch], qb[kTableBatch];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < kTableBatch; ++i) {
        ql[i] = ts.q[p[i]];
        qh[i] = ts.q[p[i] < kLevels - 1 ? p[i] + 1 : kLevels - 1];
        qb[i] = ts.q[p[i] > 0 ? p[i] - 1 : 0];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < kTableBatch; ++i) {
        const float dl = fabsf(__fsub_rn(ql[i], t[i])), dh = fabsf(__fsub_rn(qh[i], t[i]));
        uint32_t w = p[i];
        if (dh < dl) {
            w = p[i] < kLevels - 1 ? p[i] + 1 : kLevels - 1;
        } else if (w > 0 && fabsf(__fsub_rn(qb[i], t[i])) <= dl) {
            --w;  // a run of equally near entries (repeated entries, or a distance that rounds the same)
            while (w > 0 && fabsf(__fsub_rn(ts.q[w - 1], t[i])) <= dl)
                --w;
        }
        code[i] = w;
    }
}

// Codes of the wave's elements into registers: c4[k] = the four codes of float4 k.
// ws.coder holds (b, 255/S) for the linear map and (b, 1/S) for a table.
template <int K, bool kTable>
__device__ __forceinline__ void codes_to_registers(const float4 (&v)[K], const uint32_t (&packed)[(K + 1) / 2], WaveShared &ws,
                                                   const TableShared &table, uint32_t (&c4)[K])
{
    constexpr int kF = kTableBatch / 4 < K ? kTableBatch / 4 : K;  // float4 per batch
#pragma unroll
    for (int kb = 0; kb < K; kb += kF) {
        float t[kTableBatch];
        uint32_t code[kTableBatch];
#pragma unroll
        for (int i = 0; i < kTableBatch; ++i) {
            t[i] = 0.0f;
            if (i < 4 * kF) {
                const int k = kb + i / 4;
                const uint32_t l4 = (packed[k >> 1] >> (16 * (k & 1))) & 0xFFFFu;
                const float2 bi = ws.coder[(l4 >> (4 * (i % 4))) & 15u];
                t[i] = __fmul_rn(__fsub_rn(comp(v[k], i % 4), bi.x), bi.y);
                if (kTable && bi.y == 0.0f)
                    t[i] = __uint_as_float(0x7FC00000u);  // a range that cannot be coded: NaN finds entry 0
            }
        }
        if (kTable) {
            if (table.general)
                table_codes_general(table, t, code);
            else
                table_codes_by_bins(table, t, code);
#pragma unroll
            for (int f = 0; f < kF; ++f)
                c4[kb + f] = code[4 * f] | (code[4 * f + 1] << 8) | (code[4 * f + 2] << 16) | (code[4 * f + 3] << 24);
        } else {
#pragma unroll
            for (int f = 0; f < kF; ++f) {
                uint32_t c = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    c = __builtin_amdgcn_cvt_pk_u8_f32(t[4 * f + j], j, c);
                c4[kb + f] = c;
            }
        }
    }
}

template <int K, bool kFull>
__device__ __forceinline__ void store_codes(const uint32_t (&c4)[K], int64_t lo, int len, int lane, uint8_t *__restrict__ codes)
{
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int off = k * 256 + lane * 4;
        BITSNAP_GLOBAL uint8_t *cp = global_ptr(codes) + lo + off;
        if (kFull || off + 3 < len) {
            __builtin_nontemporal_store(c4[k], (BITSNAP_GLOBAL uint32_t *)cp);
        } else {
            for (int j = 0; j < 4; ++j)
                if (off + j < len)
                    cp[j] = (uint8_t)(c4[k] >> (8 * j));
        }
    }
}

// Algorithm 2 with the format options for one group of len <= 256*K elements, by one wave.
template <int K, bool kFull, bool kTable, bool kMajor>
__device__ __forceinline__ void quantize_group_ex(const float *__restrict__ x, int64_t lo, int len, int m, int64_t g,
                                                  uint8_t *__restrict__ codes, uint8_t *__restrict__ labels,
                                                  float *__restrict__ params, float *__restrict__ fit_out,
                                                  const float *__restrict__ fit_in, uint32_t *__restrict__ status,
                                                  QuantizeShared &shared, const TableShared &table, int lane)
{
    WaveShared &ws = shared.ws;

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
        // the min/max table is done with: its first half becomes the counters, its second half the codes
        MajorView mv;
        mv.counters = (uint32_t *)&ws.tab[0][0];
        mv.bytes = (uint32_t *)&ws.tab[kMaxClusters][0];
        mv.labels = shared.labels;
        uint16_t *l16 = (uint16_t *)mv.labels;
#pragma unroll
        for (int k = 0; k < K; ++k) {
            mv.bytes[k * kWave + lane] = c4[k];
            l16[k * kWave + lane] = (uint16_t)(packed[k >> 1] >> (16 * (k & 1)));
        }
        wave_lds_sync();
        to_cluster_major<K, kFull>(mv, len, lane);
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
__global__ __launch_bounds__(kVBlock, 3) void quantize_cluster_ex_kernel(
    const float *__restrict__ x, int64_t n, int64_t first_group, int64_t groups, int m, const float *__restrict__ qmap,
    uint8_t *__restrict__ codes, uint8_t *__restrict__ labels, float *__restrict__ params, float *__restrict__ fit_out,
    const float *__restrict__ fit_in, uint32_t *__restrict__ status)
{
    __shared__ QuantizeShared shared[kVWaves];
    __shared__ TableShared table;
    if (kTable)
        load_table(table, qmap);
    // no workgroup barrier from here on: waves leave when they run out of groups
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    constexpr int G = 256 * K;
    for (int64_t g = first_group + (int64_t)blockIdx.x * kVWaves + wave; g < first_group + groups;
         g += (int64_t)gridDim.x * kVWaves) {
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
        mv.counters = &sh.counters[0][0];
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

// The table of the dequantisers: one copy per workgroup (kVBlock == kLevels threads).
__device__ __forceinline__ void load_levels(float *table, const float *__restrict__ qmap)
{
    table[threadIdx.x] = global_ptr(qmap)[threadIdx.x];
    __syncthreads();
}

template <int K, bool kTable, bool kMajor>
__global__ __launch_bounds__(kVBlock) void dequantize_cluster_ex_kernel(
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
__global__ __launch_bounds__(kVBlock, 3) void quantize_cluster_ex_batched_kernel(
    const bitsnap_cluster_item *__restrict__ items, int64_t count, int64_t total_groups, int m,
    const float *__restrict__ qmap, uint32_t *__restrict__ status)
{
    __shared__ QuantizeShared shared[kVWaves];
    __shared__ TableShared table;
    if (kTable)
        load_table(table, qmap);
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr int G = 256 * K;
    const int64_t stride = (int64_t)gridDim.x * kVWaves;
    if (kFull) {
        for (int64_t gg = (int64_t)blockIdx.x * kVWaves + wave; gg < total_groups; gg += stride) {
            const bitsnap_cluster_item &it = items[find_item(items, count, gg)];
            const int64_t g = gg - it.first_group;
            const int64_t lo = g * G;
            if (it.n - lo >= G)  // a short last group is left to the tail launch
                quantize_group_ex<K, true, kTable, kMajor>((const float *)it.values, lo, G, m, g, it.codes, it.labels,
                                                           it.params, it.fit_out, it.fit_in, status, shared[wave], table,
                                                           lane);
        }
    } else {
        // one wave per tensor: its short last group, if it has one
        for (int64_t t = (int64_t)blockIdx.x * kVWaves + wave; t < count; t += stride) {
            const bitsnap_cluster_item &it = items[t];
            const int64_t g = it.n / G;
            const int rest = (int)(it.n - g * G);
            if (rest > 0)
                quantize_group_ex<K, false, kTable, kMajor>((const float *)it.values, g * G, rest, m, g, it.codes, it.labels,
                                                            it.params, it.fit_out, it.fit_in, status, shared[wave], table,
                                                            lane);
        }
    }
}

template <int K, bool kTable, bool kMajor>
__global__ __launch_bounds__(kVBlock) void dequantize_cluster_ex_batched_kernel(
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

extern "C" int bitsnap_quantize_cluster_ex(const float *x, int64_t n, int64_t group, int m, uint32_t flags,
                                           const float *qmap, uint8_t *codes, uint8_t *labels, float *params,
                                           float *fit_out, const float *fit_in, uint32_t *status,
                                           bitsnap_stream_t stream)
{
    if (n < 0 || m < 1 || m > kMaxClusters || (flags & ~(uint32_t)BITSNAP_CLUSTER_MAJOR))
        return BITSNAP_E_SIZE;
    const int K = one_wave_group_k(group);
    if (K == 0 || (n + 256 * (int64_t)K - 1) / (256 * (int64_t)K) / kVWaves > 0x7FFFFFFF)
        return BITSNAP_E_SIZE;
    if (n == 0)
        return BITSNAP_OK;
    const bool major = (flags & BITSNAP_CLUSTER_MAJOR) != 0;
    if (!qmap && !major)
        return bitsnap_quantize_cluster(x, n, group, m, codes, labels, params, fit_out, fit_in, status, nullptr, 0, stream);
    if (!x || !codes || !labels || !params)
        return BITSNAP_E_NULL;
    if (!aligned16(x) || !aligned16(codes) || !aligned16(labels) || !aligned16(params) || ((uintptr_t)fit_out & 3u) ||
        ((uintptr_t)fit_in & 3u) || ((uintptr_t)status & 3u) || ((uintptr_t)qmap & 3u))
        return BITSNAP_E_ALIGN;
    hipStream_t s = (hipStream_t)stream;
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
                                             float *out, bitsnap_stream_t stream)
{
    if (n < 0 || m < 1 || m > kMaxClusters || (flags & ~(uint32_t)BITSNAP_CLUSTER_MAJOR))
        return BITSNAP_E_SIZE;
    const int K = one_wave_group_k(group);
    if (K == 0 || (n + 256 * (int64_t)K - 1) / (256 * (int64_t)K) / kVWaves > 0x7FFFFFFF)
        return BITSNAP_E_SIZE;
    if (n == 0)
        return BITSNAP_OK;
    const bool major = (flags & BITSNAP_CLUSTER_MAJOR) != 0;
    if (!qmap && !major)
        return bitsnap_dequantize_cluster(codes, labels, params, n, group, m, out, stream);
    if (!codes || !labels || !params || !out)
        return BITSNAP_E_NULL;
    if (!aligned16(codes) || !aligned16(labels) || !aligned16(params) || !aligned16(out) || ((uintptr_t)qmap & 3u))
        return BITSNAP_E_ALIGN;
    hipStream_t s = (hipStream_t)stream;
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

static int check_ex_batched(const bitsnap_cluster_item *items, int64_t count, int64_t total_groups, int64_t group, int m,
                            uint32_t flags, const float *qmap, const uint32_t *status, int &K)
{
    if (count < 0 || total_groups < 0 || m < 1 || m > kMaxClusters || (flags & ~(uint32_t)BITSNAP_CLUSTER_MAJOR))
        return BITSNAP_E_SIZE;
    K = one_wave_group_k(group);
    if (K == 0 || ex_batched_blocks(total_groups) > 0x7FFFFFFF)
        return BITSNAP_E_SIZE;
    if (count == 0 || total_groups == 0)
        return BITSNAP_OK;
    if (!items)
        return BITSNAP_E_NULL;
    if (((uintptr_t)items & 7u) || ((uintptr_t)status & 3u) || ((uintptr_t)qmap & 3u))
        return BITSNAP_E_ALIGN;
    return 1;  // go on
}

extern "C" int bitsnap_quantize_cluster_batched_ex(const bitsnap_cluster_item *items, int64_t count, int64_t total_groups,
                                                   int64_t group, int m, uint32_t flags, const float *qmap,
                                                   uint32_t *status, bitsnap_stream_t stream)
{
    int K = 0;
    const int rc = check_ex_batched(items, count, total_groups, group, m, flags, qmap, status, K);
    if (rc <= 0)
        return rc;
    const bool major = (flags & BITSNAP_CLUSTER_MAJOR) != 0;
    if (!qmap && !major)
        return bitsnap_quantize_cluster_batched(items, count, total_groups, group, m, status, stream);
    hipStream_t s = (hipStream_t)stream;
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
                                                     bitsnap_stream_t stream)
{
    int K = 0;
    const int rc = check_ex_batched(items, count, total_groups, group, m, flags, qmap, nullptr, K);
    if (rc <= 0)
        return rc;
    const bool major = (flags & BITSNAP_CLUSTER_MAJOR) != 0;
    if (!qmap && !major)
        return bitsnap_dequantize_cluster_batched(items, count, total_groups, group, m, stream);
    hipStream_t s = (hipStream_t)stream;
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
