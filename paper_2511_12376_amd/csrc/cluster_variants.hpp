// Per-wave building blocks of the cluster quantiser's format variants (paper: "Cluster Based
// Quantization for Optimizer States"): the search of a 256-entry map Q^map in Eq.
// qmap-distance, and the stable 16-way partition that turns element-order codes into the
// cluster-major arrangement of Eq. decluster and back.  Used by the one-wave-per-group kernels
// and by the multi-pass kernels for wide groups.
//
// The table lives in LDS once per workgroup, turned into a step function over 1024 bins of
// (x-b)/S where its levels are far enough apart for that, and searched by bisection otherwise.
// The partition runs inside the wave through LDS: the codes and the labels are laid down in
// element order; then lane l takes the 4K consecutive elements l*4K .. l*4K+4K-1, counts its
// labels into a private column of a [16][64] counter table, an exclusive prefix sum over that
// table read row by row (cluster, then lane) turns every counter into the position of the lane's
// first member of the cluster, and a second walk over the same elements hands out consecutive
// positions.
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "cluster_wave.hpp"
#include "wave.hpp"

namespace bitsnap {

constexpr int kVBlock = 256;
constexpr int kVWaves = kVBlock / kWave;
constexpr int kLevels = 256;

// LDS of one wave for the partition: 8 KB, so that sixteen waves fit a CU next to their other tables.
struct MajorView {
    uint32_t *counters;  // [16][32] words of two 16-bit counters: cluster c, lane l in word c*32 + l%32, upper half for l >= 32
    uint32_t *bytes;     // [256*K] bytes: the group's codes (element order on one side, cluster-major on the other)
    uint32_t *labels;    // [256*K] nibbles: the group's labels in element order
};
constexpr int kCounterWords = kMaxClusters * kWave / 2;

// In the quantiser the partition runs when the min/max table is done with, and takes its place:
// rows 0-7 the counters, rows 8-15 the labels, rows 16-31 the code bytes.
__device__ __forceinline__ MajorView major_view(WaveShared &ws)
{
    MajorView mv;
    mv.counters = (uint32_t *)&ws.tab[0][0];
    mv.labels = (uint32_t *)&ws.tab[kMaxClusters / 2][0];
    mv.bytes = (uint32_t *)&ws.tab[kMaxClusters][0];
    return mv;
}

struct alignas(16) DequantizeShared {
    uint32_t counters[kCounterWords];
    uint32_t bytes[kMaxClusters * 256 / 4];
    uint32_t labels[kMaxClusters * 256 / 8];
    float2 coder[kMaxClusters];
    uint32_t seg_start[kMaxClusters + 4], seg_delta[kMaxClusters];  // wide groups: the chunk's runs and where they come from
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

// The counter of (cluster, lane): a 16-bit half of a word that lanes l and l + 32 share.  Counts and
// positions stay below 2^13, so an add to the lower half never carries into the upper one.
__device__ __forceinline__ uint32_t counter_word(uint32_t cluster, int lane) { return cluster * (kWave / 2) + (uint32_t)(lane & 31); }
__device__ __forceinline__ uint32_t counter_shift(int lane) { return (uint32_t)(lane >> 5) * 16u; }

// Takes the next position of `cluster` in this lane's counter.
__device__ __forceinline__ uint32_t take_position(const MajorView &mv, uint32_t cluster, int lane)
{
    const uint32_t shift = counter_shift(lane);
    return (lds_fetch_add(&mv.counters[counter_word(cluster, lane)], 1u << shift) >> shift) & 0xFFFFu;
}

// Counts the lane's labels and turns the counter table into first positions: afterwards the
// counter of (c, lane) = members of clusters < c in the group + members of c in lower lanes.
template <int K, bool kFull>
__device__ __forceinline__ void major_positions(const MajorView &mv, const uint32_t (&lh)[K], int len, int lane)
{
    if (lane < kWave / 2) {
#pragma unroll
        for (int c = 0; c < kMaxClusters; ++c)
            mv.counters[c * (kWave / 2) + lane] = 0;
    }
    wave_lds_sync();
    const uint32_t one = 1u << counter_shift(lane);
#pragma unroll
    for (int i = 0; i < K; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (kFull || lane * 4 * K + 4 * i + j < len)
                lds_fetch_add(&mv.counters[counter_word((lh[i] >> (4 * j)) & 15u, lane)], one);
    wave_lds_sync();
    // Exclusive prefix over the 1024 counters in (cluster, lane) order, 16 consecutive ones per lane:
    // lane L takes cluster L/4, lanes 16*(L%4) .. +15, i.e. 16 consecutive words and one half of each.
    const uint32_t w0 = (uint32_t)(lane >> 2) * (kWave / 2) + (uint32_t)(lane & 1) * 16u, upper = (uint32_t)(lane >> 1) & 1u;
    uint32_t c[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
        c[i] = (mv.counters[w0 + i] >> (16u * upper)) & 0xFFFFu;
    uint32_t total = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint32_t t = c[i];
        c[i] = total;
        total += t;
    }
    const uint32_t before = wave_inclusive_add(total) - total;
    wave_lds_sync();  // every lane has read its 16 counters (other lanes' columns) before any is rewritten
    uint16_t *c16 = (uint16_t *)mv.counters;
#pragma unroll
    for (int i = 0; i < 16; ++i)
        c16[2u * (w0 + i) + upper] = (uint16_t)(c[i] + before);
    wave_lds_sync();
}

// After major_positions and before any position is handed out: lane c < 16 gets the position of
// cluster c's first member (lane 0's counter of that cluster), the other lanes get len.
__device__ __forceinline__ uint32_t cluster_start(const MajorView &mv, int len, int lane)
{
    return lane < kMaxClusters ? (mv.counters[lane * (kWave / 2)] & 0xFFFFu) : (uint32_t)len;
}

// Element order -> cluster-major.  In: mv.bytes and mv.labels hold the group in element order.
// Out: mv.bytes holds the cluster-major arrangement; `start` as from cluster_start.
template <int K, bool kFull>
__device__ __forceinline__ void to_cluster_major(const MajorView &mv, int len, int lane, uint32_t &start)
{
    uint32_t lh[K], cw[K];
    own_labels<K>(mv, lane, lh);
#pragma unroll
    for (int i = 0; i < K; ++i)
        cw[i] = mv.bytes[lane * K + i];
    major_positions<K, kFull>(mv, lh, len, lane);  // its barriers also order the reads above before the writes below
    start = cluster_start(mv, len, lane);
    uint8_t *b8 = (uint8_t *)mv.bytes;
    // positions are handed out kWalk elements at a time: one LDS round trip per batch, not per element
    constexpr int kWalk = 4 * (K >= 4 ? 4 : K);
#pragma unroll
    for (int e0 = 0; e0 < 4 * K; e0 += kWalk) {
        uint32_t pos[kWalk];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int e = 0; e < kWalk; ++e) {
            const int i = (e0 + e) >> 2, j = (e0 + e) & 3;
            pos[e] = 0;
            if (kFull || lane * 4 * K + e0 + e < len)
                pos[e] = take_position(mv, (lh[i] >> (4 * j)) & 15u, lane);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int e = 0; e < kWalk; ++e) {
            const int i = (e0 + e) >> 2, j = (e0 + e) & 3;
            if (kFull || lane * 4 * K + e0 + e < len)
                b8[pos[e]] = (uint8_t)(cw[i] >> (8 * j));
        }
    }
    wave_lds_sync();
}

struct BytesInPlace {
    __device__ __forceinline__ void operator()(uint32_t) const {}
};

// Cluster-major -> element order.  In: mv.labels in element order; mv.bytes cluster-major, either
// already there or brought in by `fill(start)` (start as from cluster_start; fill ends with a
// wave_lds_sync of its own), which is how a chunk of a wide group collects its 16 segments once
// their places inside the chunk are known.  Out: mv.bytes in element order.
template <int K, bool kFull, typename Fill = BytesInPlace>
__device__ __forceinline__ void from_cluster_major(const MajorView &mv, int len, int lane, Fill fill = Fill())
{
    uint32_t lh[K], cw[K];
    own_labels<K>(mv, lane, lh);
    major_positions<K, kFull>(mv, lh, len, lane);
    fill(cluster_start(mv, len, lane));
    const uint8_t *b8 = (const uint8_t *)mv.bytes;
    constexpr int kWalk = 4 * (K >= 4 ? 4 : K);
#pragma unroll
    for (int i = 0; i < K; ++i)
        cw[i] = 0;
#pragma unroll
    for (int e0 = 0; e0 < 4 * K; e0 += kWalk) {
        uint32_t pos[kWalk], got[kWalk];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int e = 0; e < kWalk; ++e) {
            const int i = (e0 + e) >> 2, j = (e0 + e) & 3;
            pos[e] = 0;
            if (kFull || lane * 4 * K + e0 + e < len)
                pos[e] = take_position(mv, (lh[i] >> (4 * j)) & 15u, lane);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int e = 0; e < kWalk; ++e)
            got[e] = b8[pos[e]];  // position 0 for an element that does not exist: in bounds, ignored
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int e = 0; e < kWalk; ++e) {
            const int i = (e0 + e) >> 2, j = (e0 + e) & 3;
            if (kFull || lane * 4 * K + e0 + e < len)
                cw[i] |= got[e] << (8 * j);
        }
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
        if (kFull || (off + 3 < len && (lo & 3) == 0)) {
            __builtin_nontemporal_store(c4[k], (BITSNAP_GLOBAL uint32_t *)cp);
        } else {
            for (int j = 0; j < 4; ++j)
                if (off + j < len)
                    cp[j] = (uint8_t)(c4[k] >> (8 * j));
        }
    }
}

// The table of the dequantisers: one copy per workgroup (kVBlock == kLevels threads).
__device__ __forceinline__ void load_levels(float *table, const float *__restrict__ qmap)
{
    table[threadIdx.x] = global_ptr(qmap)[threadIdx.x];
    __syncthreads();
}

}  // namespace bitsnap
