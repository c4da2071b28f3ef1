// encode_sparse / decode_sparse: bitmask-based delta sparsification of 16-bit model states
// (paper: "Bitmask Based Sparsification for Model States", improved bitmask; Algorithm 1) and
// its inverse.  Encode is one kernel and one pass over HBM; decode is three kernels, of which
// only the last touches more than the mask (one kernel for tensors of a few tiles, or when the
// encoder's tile offsets come with the mask).
//
// Elements are 2 bytes (fp16 / bf16 model states) or 4 bytes (fp32 states); E is the element width.
// A tile is 64 KB of each input - 32768 2-byte or 16384 4-byte elements, in rounds of 8192 - and
// is processed by one 512-thread workgroup; all of a tile's loads are issued before anything
// waits on them.  A lane owns pieces of 8 consecutive elements (one mask byte; one or two 16-byte
// loads); in the encoder a wavefront owns, in each round, two consecutive 512-element chunks, in the
// decoder's merge one contiguous segment of 1024 elements.  Per-lane popcounts are scanned with DPP inside
// the wave, and in the encoder through LDS across the eight waves and the rounds and by the
// scanning wave of scan_state.hpp across tiles.  The tile is large because every tile costs the machine one
// same-address atomic (the ticket; the chip serves 88 million of them per second, one every 11.4 ns)
// and two words of scan state.  Changed values are staged in LDS so
// that the payload leaves (encode) or enters (decode) HBM as 16-byte accesses aligned on the
// payload buffer, whatever the tile's (decode: the wave's) offset.
#include <hip/hip_runtime.h>
#include <stdlib.h>
#include <stdint.h>

#include <atomic>
#include <mutex>
#include <type_traits>

#include "../../include/bitsnap.h"
#include "host_util.hpp"
#include "scan_state.hpp"
#include "wave.hpp"

namespace bitsnap {

constexpr int kBlock = 512;
constexpr int kWaves = kBlock / kWave;
constexpr int kLaneElems = 8;                              // one 16-byte load of 16-bit elements
constexpr int kChunkElems = kWave * kLaneElems;            // 512: what one wave covers with one load
constexpr int kRoundChunks = 2 * kWaves;                   // a round: every wave takes two consecutive chunks
constexpr int kRoundElems = kRoundChunks * kChunkElems;    // 8192

template <int E>
struct Geom {
    static_assert(E == 2 || E == 4, "16-bit or 32-bit elements");
    typedef typename std::conditional<E == 2, uint16_t, uint32_t>::type elem_t;
    typedef __attribute__((address_space(1))) elem_t global_elem_t;
    static constexpr int kVecs = E / 2;                       // 16-byte loads per 8-element piece
    static constexpr int kRounds = 8 / E;                     // rounds per tile, all loaded before the scan
    static constexpr int kTileElems = kRounds * kRoundElems;  // one ticket, one status word, one look-back
    static constexpr int kVecElems = 16 / E;                  // elements per 16 bytes
};

// The lane's 8 consecutive elements
template <int E>
struct Piece {
    uint4 v[Geom<E>::kVecs];
};

// The tile's changed values pass through `stage`: at their rank inside the tile in the encoder
// (before the tile's place in the payload is known), as the aligned payload segment in the decoder.
template <int E>
struct TileShared {
    alignas(16) typename Geom<E>::elem_t stage[Geom<E>::kTileElems + 16];  // + what realigning (encode) or a shifted segment (decode) adds
    uint32_t wave_total[Geom<E>::kRounds][kWaves];
    uint64_t excl;
    int64_t next_tile;
    int aborted;
};

// Device buffers are addressed as global memory explicitly: a generic (flat) access would also
// count as an LDS operation in flight, and every wait for LDS would then wait for HBM.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) u32x4 global_u32x4;
typedef __attribute__((address_space(1))) uint16_t global_u16;
typedef __attribute__((address_space(1))) uint8_t global_u8;

// kStream: non-temporal access, for data that is touched once.  Measured on the batched 7B pass:
// streaming loads of cur/base and streaming stores of the payload are worth about 2 % to the
// encoder; the decoder is about 2 % faster with ordinary stores of its output.
template <bool kStream>
__device__ __forceinline__ uint4 load_global16(const void *p)
{
    const u32x4 v = kStream ? __builtin_nontemporal_load((const global_u32x4 *)p) : *(const global_u32x4 *)p;
    return make_uint4(v.x, v.y, v.z, v.w);
}
template <bool kStream>
__device__ __forceinline__ void store_global16(void *p, uint4 v)
{
    u32x4 t;
    t.x = v.x, t.y = v.y, t.z = v.z, t.w = v.w;
    if (kStream)
        __builtin_nontemporal_store(t, (global_u32x4 *)p);
    else
        *(global_u32x4 *)p = t;
}

__device__ __forceinline__ uint32_t word_of(const uint4 &v, int k) { return k == 0 ? v.x : k == 1 ? v.y : k == 2 ? v.z : v.w; }

// element t (0..7) of a piece
template <int E>
__device__ __forceinline__ typename Geom<E>::elem_t piece_elem(const Piece<E> &pc, int t)
{
    if (E == 2)
        return (typename Geom<E>::elem_t)(word_of(pc.v[0], t >> 1) >> ((t & 1) * 16));
    return (typename Geom<E>::elem_t)word_of(pc.v[(E == 4) ? (t >> 2) : 0], t & 3);
}

// 8 elements to p[e0 .. e0+8) (e0 a multiple of 8), clipped at n
template <bool kStream, int E>
__device__ __forceinline__ void store8(typename Geom<E>::elem_t *p, int64_t e0, int64_t n, const Piece<E> &pc)
{
    if (e0 + kLaneElems <= n) {
#pragma unroll
        for (int k = 0; k < Geom<E>::kVecs; ++k)
            store_global16<kStream>(p + e0 + k * Geom<E>::kVecElems, pc.v[k]);
        return;
    }
    for (int t = 0; t < kLaneElems; ++t)
        if (e0 + t < n)
            ((typename Geom<E>::global_elem_t *)p)[e0 + t] = piece_elem<E>(pc, t);
}

// bit t = 1 iff element t of x is non-zero; with x = cur XOR base: the element changed
// (Algorithm 1 steps 1-2)
template <int E>
__device__ __forceinline__ uint32_t nonzero_bits(const Piece<E> &x)
{
    uint32_t m = 0;
    if (E == 2) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t w = word_of(x.v[0], j);
            m |= ((w & 0xFFFFu) != 0u ? 1u : 0u) << (2 * j);
            m |= ((w >> 16) != 0u ? 1u : 0u) << (2 * j + 1);
        }
    } else {
#pragma unroll
        for (int t = 0; t < 8; ++t)
            m |= (word_of(x.v[(E == 4) ? (t >> 2) : 0], t & 3) != 0u ? 1u : 0u) << t;
    }
    return m;
}

// Where the calling lane's 8-element pieces sit inside a tile: round r, piece j (0 or 1)
//   chunk  = tile*16R + r*16 + wave*2 + j        element = chunk*512 + lane*8
// so element order is round-major, then wave, then piece, then lane.
template <int E>
__device__ __forceinline__ int64_t piece_chunk(int64_t tile, int r, int wave, int j)
{
    return tile * (Geom<E>::kRounds * kRoundChunks) + r * kRoundChunks + wave * 2 + j;
}

// Per-lane popcounts cnt[r][j] -> this lane's exclusive rank of each piece inside the tile;
// returns the tile total.  Contains one __syncthreads.
template <int E>
__device__ __forceinline__ uint32_t tile_ranks(TileShared<E> &sh, const uint32_t (&cnt)[Geom<E>::kRounds][2], int lane,
                                               int wave, uint32_t (&rank)[Geom<E>::kRounds][2])
{
    constexpr int kRounds = Geom<E>::kRounds;
    uint32_t ex[kRounds], t0[kRounds];
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const uint32_t pk = cnt[r][0] | (cnt[r][1] << 16);
        const uint32_t incl = wave_inclusive_add(pk);
        const uint32_t tot = read_lane(incl, 63);
        ex[r] = incl - pk;
        t0[r] = tot & 0xFFFFu;
        if (lane == 0)
            sh.wave_total[r][wave] = t0[r] + (tot >> 16);
    }
    __syncthreads();
    uint32_t run = 0;
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        uint32_t before = 0, all = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const uint32_t v = sh.wave_total[r][w];
            before += (w < wave) ? v : 0u;
            all += v;
        }
        rank[r][0] = run + before + (ex[r] & 0xFFFFu);
        rank[r][1] = run + before + t0[r] + (ex[r] >> 16);
        run += all;
    }
    return run;
}

// All of a tile's loads for the calling lane (issued back to back, nothing waits here): a
// wave-uniform tile base plus a 32-bit offset each.  A 16-byte load whose first element lies at or
// beyond the end of the tensor reads the tile's first 16 bytes instead, and one that straddles the
// end is made whole: the buffer is 16-byte aligned, so an aligned 16-byte load never leaves the
// page its first element is in.  The caller ignores what lies at or beyond n (piece_valid_bits).
template <int E>
__device__ __forceinline__ void load_tile(const typename Geom<E>::elem_t *__restrict__ p, int64_t tile, int wave, int lane,
                                          int64_t n, Piece<E> (&v)[Geom<E>::kRounds][2])
{
    constexpr int kTileElems = Geom<E>::kTileElems;
    const int64_t t0 = tile * kTileElems;
    const typename Geom<E>::elem_t *__restrict__ tp = p + t0;  // wave-uniform
    const uint32_t rem = n - t0 >= kTileElems ? (uint32_t)kTileElems : (uint32_t)(n - t0);
    const uint32_t e0 = (uint32_t)(wave * (2 * kChunkElems) + lane * kLaneElems);
#pragma unroll
    for (int r = 0; r < Geom<E>::kRounds; ++r)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint32_t e = e0 + (uint32_t)((r * kRoundChunks + j) * kChunkElems);
#pragma unroll
            for (int k = 0; k < Geom<E>::kVecs; ++k) {
                const uint32_t ek = e + (uint32_t)(k * Geom<E>::kVecElems);
                v[r][j].v[k] = load_global16<true>(tp + (ek < rem ? ek : 0u));
            }
        }
}

// Which of the 8 elements of the lane's piece (r, j) exist, in a tile that holds `rem` elements.
__device__ __forceinline__ uint32_t piece_valid_bits(int r, int j, int wave, int lane, uint32_t rem)
{
    const int32_t left = (int32_t)rem - (r * kRoundChunks + wave * 2 + j) * kChunkElems - lane * kLaneElems;
    return left >= kLaneElems ? 0xFFu : left > 0 ? (1u << left) - 1u : 0u;
}

// A value every lane holds alike, moved to scalar registers.
__device__ __forceinline__ uint64_t uniform64(uint64_t t)
{
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)t), hi = __builtin_amdgcn_readfirstlane((uint32_t)(t >> 32));
    return ((uint64_t)hi << 32) | lo;
}

// The value thread 0 left in sh.next_tile, as a scalar in every thread (call after a barrier).
template <int E>
__device__ __forceinline__ int64_t claimed_tile(const TileShared<E> &sh)
{
    return (int64_t)uniform64((uint64_t)sh.next_tile);
}

// The tensor a launch-wide tile number belongs to.  Tickets only grow, so a workgroup moves through the item
// list forwards - but between two tiles of one workgroup lie all the tiles the other workgroups took meanwhile,
// which in a list of small tensors are dozens or hundreds of items.  So the next seven items are looked at at once
// (one round trip of scalar loads), and if the tile lies beyond them the rest of the list is searched eight ways per
// round trip.  (Walked item by item, a list with 1600 one-tile tensors among 160 large ones took a quarter longer.)
// With kBatched == false there is one tensor, passed by value.
template <bool kBatched>
struct ItemCursor {
    const bitsnap_sparse_item *items;
    int64_t count, t, next_first;
    bitsnap_sparse_item it;

    __device__ __forceinline__ ItemCursor(const bitsnap_sparse_item &single, const bitsnap_sparse_item *list, int64_t n)
        : items(list), count(n), t(0), next_first(INT64_MAX), it(single)
    {
        if (kBatched) {
            it = items[0];
            next_first = count > 1 ? items[1].first_tile : INT64_MAX;
        }
    }
    __device__ __forceinline__ void seek(int64_t tile)
    {
        if (!kBatched || tile < next_first)
            return;
        // items[lo].first_tile <= tile, and the answer lies in [lo, hi)
        int64_t lo = t + 1, hi = count;
        bool near = true;
        while (hi - lo > 1) {
            const int64_t step = near ? 1 : (hi - lo + 7) >> 3;
            int64_t first[7];
#pragma unroll
            for (int k = 0; k < 7; ++k) {
                const int64_t idx = lo + (k + 1) * step;
                first[k] = idx < hi ? items[idx].first_tile : INT64_MAX;
            }
            int reached = 0;  // first_tile grows along the list: the probes at or below the tile are the leading ones
#pragma unroll
            for (int k = 0; k < 7; ++k)
                reached += first[k] <= tile ? 1 : 0;
            if (near && reached == 7) {  // beyond the next items: search what is left
                lo += 7;
                near = false;
                continue;
            }
            near = false;
            const int64_t up = lo + (reached + 1) * step;
            lo += reached * step;
            hi = up < hi ? up : hi;
        }
        t = lo;
        it = items[t];
        next_first = (t + 1 < count) ? items[t + 1].first_tile : INT64_MAX;
    }
};

// After the scan: what only the workgroup that finished last may write.
__device__ __forceinline__ void report_failures(int epilogue, const bitsnap_sparse_item &single,
                                                const bitsnap_sparse_item *items, int64_t count, bool batched,
                                                int64_t num_tiles)
{
    if (!(epilogue & kEpilogueLast))
        return;
    if (epilogue & kEpilogueError) {  // some workgroup gave up waiting: every count of this launch is void
        if (batched) {
            for (int64_t t = threadIdx.x; t < count; t += blockDim.x)
                if (items[t].n_changed)
                    *items[t].n_changed = ~0ull;
        } else if (threadIdx.x == 0 && single.n_changed) {
            *single.n_changed = ~0ull;
        }
    } else if (!batched && num_tiles == 0 && threadIdx.x == 0 && single.n_changed) {
        *single.n_changed = 0;  // an empty tensor has no tile that could report its count
    }
}

// Algorithm 1 step 5, second half: payload[excl + i] = stage[i], i < total.  With P = 16 / E
// elements per 16 bytes, payload element excl - shift (shift = excl mod P) is 16-byte aligned;
// piece q covers payload elements [dst0 + P*q, dst0 + P*q + P), i.e. stage elements from P*q - shift,
// read as dwords and, for 2-byte elements and an odd shift, moved by one element.  The ragged
// ends of the tile's segment, and whatever would cross the payload capacity, go out element by
// element.
template <int E>
__device__ __forceinline__ void copy_out_stage(const TileShared<E> &sh, typename Geom<E>::elem_t *__restrict__ payload,
                                               int64_t capacity, uint64_t excl, uint32_t total, int tid)
{
    constexpr uint32_t P = Geom<E>::kVecElems;
    const uint32_t shift = (uint32_t)(excl & (P - 1u));
    const uint32_t first = shift, last = shift + total;
    const int64_t dst0 = (int64_t)(excl - shift);
    const uint32_t pieces = (last + P - 1u) / P;
    const uint32_t odd_bytes = (E == 2) ? (shift & 1u) * 2u : 0u;
    const uint32_t *stage32 = reinterpret_cast<const uint32_t *>(sh.stage);
    uint64_t base_bits = (uint64_t)payload;
    asm volatile("" : "+s"(base_bits));                                             // stays in scalar registers
    typename Geom<E>::elem_t *__restrict__ dst = (typename Geom<E>::elem_t *)base_bits + dst0;  // wave-uniform, 16-byte aligned
    const int64_t room = capacity - dst0;                                            // elements of dst that may be written
    constexpr int64_t kMost = Geom<E>::kTileElems + (int64_t)P;
    const uint32_t fits = room >= kMost ? (uint32_t)kMost : room > 0 ? (uint32_t)room : 0u;
    for (uint32_t q = tid; q < pieces; q += kBlock) {
        const uint32_t lo = q * P;
        if (lo >= first && lo + P <= last && lo + P <= fits) {
            const uint32_t w0 = ((lo - shift) * (uint32_t)E) >> 2;
            uint32_t w[5];
#pragma unroll
            for (int k = 0; k < (E == 2 ? 5 : 4); ++k)
                w[k] = stage32[w0 + k];
            uint4 v;
            if (E == 2) {
                v.x = __builtin_amdgcn_alignbyte(w[1], w[0], odd_bytes);
                v.y = __builtin_amdgcn_alignbyte(w[2], w[1], odd_bytes);
                v.z = __builtin_amdgcn_alignbyte(w[3], w[2], odd_bytes);
                v.w = __builtin_amdgcn_alignbyte(w[4], w[3], odd_bytes);
            } else {
                v = make_uint4(w[0], w[1], w[2], w[3]);
            }
            store_global16<true>(dst + lo, v);
        } else {
            for (uint32_t t = 0; t < P; ++t) {
                const uint32_t i = lo + t;
                if (i >= first && i < last && i < fits)
                    ((typename Geom<E>::global_elem_t *)dst)[i] = sh.stage[i - shift];
            }
        }
    }
}

// What a workgroup remembers of the tile whose values wait in its stage.
template <int E>
struct StagedTile {
    typename Geom<E>::elem_t *payload;
    int64_t capacity;
    uint32_t *offsets;
    uint64_t *count_out;
    int64_t gtile, tile;  // launch-wide number, number inside the tensor
    uint32_t total;       // number of staged values
    bool first, last;     // the tensor's first / last tile
};

// The workgroup that draws ticket 0 lends its first wave to the scan (scan_state.hpp) and does nothing else; the
// others take tiles.  Order of work in one turn of a tile workgroup's loop:
//   the tile's loads are issued -> thread 0 fetches the previous tile's place in the payload (its count went
//   to the scanning wave a whole scatter, ticket and load issue ago) -> the previous tile's staged values go
//   out as 16-byte stores aligned on the payload buffer, realigned on the way out of LDS -> mask bytes and
//   counts -> ranks inside the tile -> the tile's count goes to the scanning wave -> changed values are
//   scattered into LDS at their rank inside the tile -> ticket for the next tile.
// So a tile's HBM reads overlap the wait for, and the copy-out of, the tile before it, and between a ticket and
// the count of its tile lies one load latency and nothing that waits on another workgroup: the scanning wave
// answers tiles in ticket order, so a count that comes late holds up every tile behind it.
// launch_bounds: 4 waves per SIMD, i.e. two 512-thread workgroups per CU (128 registers per lane).
// kDelta: the payload holds cur XOR base (the non-zero elements of the delta states) instead of
// cur.  refresh: item.out, where set, receives a copy of cur (it may be the base buffer itself: a
// tile's base is in registers before the tile's copy of cur is stored, and no other tile touches it).
// kSolo: the launch is one workgroup for a tensor of one tile, which needs no ticket, no scan and no
// last-workgroup bookkeeping: the workspace is not touched at all.
template <bool kBatched, bool kDelta, int E, bool kSolo = false>
__global__ __launch_bounds__(kBlock, 4) void encode_sparse_kernel(bitsnap_sparse_item single,
                                                               const bitsnap_sparse_item *__restrict__ items,
                                                               int64_t count, ScanHeader *hdr, uint64_t *status,
                                                               int64_t status_cap, int64_t num_tiles, uint32_t spin_limit,
                                                               int refresh)
{
    typedef typename Geom<E>::elem_t elem_t;
    constexpr int kRounds = Geom<E>::kRounds, kTileElems = Geom<E>::kTileElems;
    __shared__ TileShared<E> sh;
    __shared__ StagedTile<E> st;
    const int tid0 = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid0 >> 6);
    const uint32_t epoch = kSolo ? 0u : hdr->epoch;
    bool aborted = false;
    ItemCursor<kBatched> cursor(single, items, count);

    if (tid0 == 0)
        sh.next_tile = kSolo ? 0 : (int64_t)atomicAdd(&hdr->ticket, 1u) - 1;
    __syncthreads();
    if (!kSolo && claimed_tile(sh) < 0) {  // ticket 0: the scan
        if (wave == 0)
            aborted = serve_scan(hdr, status, num_tiles, epoch, spin_limit);
        const int epilogue = scan_epilogue(hdr, status, status_cap, epoch, aborted);  // thread 0 is in wave 0
        report_failures(epilogue, single, items, count, kBatched, num_tiles);
        return;
    }
    bool staged = false;  // the previous tile of this workgroup is in the stage (and described in st), still to be copied out
    for (;;) {
        // The thread's index is made opaque once per turn: otherwise every per-piece offset derived
        // from it counts as loop-invariant and is kept in (or spilled from) a register of its own.
        int tid = tid0;
        asm volatile("" : "+v"(tid));
        const int lane = tid & (kWave - 1);
        const int64_t gtile = claimed_tile(sh);
        const bool valid = gtile < num_tiles;
        Piece<E> c[kRounds][2], b[kRounds][2];
        if (valid) {  // this tile's loads fly while the previous tile's values leave
            cursor.seek(gtile);
            load_tile<E>((const elem_t *)cursor.it.src, gtile - cursor.it.first_tile, wave, lane, cursor.it.n, c);
            load_tile<E>((const elem_t *)cursor.it.base, gtile - cursor.it.first_tile, wave, lane, cursor.it.n, b);
        }
        if (staged) {
            if (tid == 0) {
                uint32_t zero = 0;
                asm volatile("" : "+v"(zero));  // made here, not kept in registers across the loop
                uint64_t before = zero;         // a tensor's first tile starts its payload
                bool ok = true;
                if (!st.first)
                    ok = await_prefix(hdr, status, num_tiles, st.gtile, epoch, spin_limit, before);
                sh.excl = before;
                sh.aborted = ok ? 0 : 1;
                if (ok) {
                    if (st.offsets)
                        st.offsets[st.tile] = (uint32_t)before;
                    if (st.last)  // the tensor's last tile knows the total
                        *st.count_out = before + st.total;
                }
            }
            __syncthreads();  // sh.excl / sh.aborted are set
            if (sh.aborted) {
                aborted = true;
                break;
            }
            copy_out_stage<E>(sh, (elem_t *)uniform64((uint64_t)st.payload), (int64_t)uniform64((uint64_t)st.capacity),
                              uniform64(sh.excl), __builtin_amdgcn_readfirstlane(st.total), tid);
        }
        if (!valid)
            break;

        const bitsnap_sparse_item &it = cursor.it;
        const int64_t n = it.n, tile = gtile - it.first_tile;
        const int64_t mask_bytes = (((n + 7) >> 3) + 15) & ~(int64_t)15;
        uint8_t *__restrict__ wave_mask = it.mask + tile * (kTileElems / 8) + wave * (2 * kWave);
        const bool full_tile = (tile + 1) * kTileElems <= n;
        const int32_t wave_mask_bytes =
            (full_tile ? (int32_t)(kTileElems / 8) : (int32_t)(mask_bytes - tile * (kTileElems / 8))) - wave * (2 * kWave);
        const uint32_t tile_elems = full_tile ? (uint32_t)kTileElems : (uint32_t)(n - tile * kTileElems);
        elem_t *new_base = refresh ? (elem_t *)it.out : nullptr;

        uint32_t m[kRounds][2], cnt[kRounds][2], rank[kRounds][2];
#pragma unroll
        for (int r = 0; r < kRounds; ++r)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                if (new_base)
                    store8<false, E>(new_base, piece_chunk<E>(tile, r, wave, j) * kChunkElems + lane * kLaneElems, n, c[r][j]);
                Piece<E> x;
#pragma unroll
                for (int k = 0; k < Geom<E>::kVecs; ++k)
                    x.v[k] = make_uint4(c[r][j].v[k].x ^ b[r][j].v[k].x, c[r][j].v[k].y ^ b[r][j].v[k].y,
                                        c[r][j].v[k].z ^ b[r][j].v[k].z, c[r][j].v[k].w ^ b[r][j].v[k].w);
                m[r][j] = nonzero_bits<E>(x) & piece_valid_bits(r, j, wave, lane, tile_elems);
                if (kDelta)
                    c[r][j] = x;
                cnt[r][j] = __popc(m[r][j]);
                // Algorithm 1 steps 3-4: one mask byte per lane; bytes past ceil(n/8) come out as 0
                const int32_t mb = (r * kRoundChunks + j) * kWave;  // + lane, in this wave's part of the tile's mask
                if (mb + lane < wave_mask_bytes)
                    ((global_u8 *)(wave_mask + mb))[(uint32_t)lane] = (uint8_t)m[r][j];
            }
        // the barrier inside: every thread has also finished reading the stage and st for the tile that left above
        const uint32_t total = tile_ranks<E>(sh, cnt, lane, wave, rank);
        if (!kSolo && tid == 0)
            publish_count(status, gtile, tile == 0, epoch, total);

        // Algorithm 1 step 5, first half: changed values in index order, at their rank inside the tile
#pragma unroll
        for (int r = 0; r < kRounds; ++r)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                uint32_t p = rank[r][j];
#pragma unroll
                for (int t = 0; t < kLaneElems; ++t)
                    if ((m[r][j] >> t) & 1u)
                        sh.stage[p++] = piece_elem<E>(c[r][j], t);
            }
        staged = true;
        if (tid == 0) {
            st.payload = (elem_t *)it.payload;
            st.capacity = it.capacity;
            st.offsets = it.tile_offsets;
            st.count_out = it.n_changed;
            st.gtile = gtile;
            st.tile = tile;
            st.total = total;
            st.first = tile == 0;
            st.last = (tile + 1) * kTileElems >= n;
            sh.next_tile = kSolo ? 1 : (int64_t)atomicAdd(&hdr->ticket, 1u) - 1;
        }
        __syncthreads();  // the stage is complete, the next tile is known
    }
    if (kSolo)
        return;
    const int epilogue = scan_epilogue(hdr, status, status_cap, epoch, aborted);
    report_failures(epilogue, single, items, count, kBatched, num_tiles);
}

// ---------------------------------------------------------------------------------------------
// decode_sparse.  The ranks of the inverse only depend on the mask, which is 1/33 of the data, so
// the decoder does not scan while it streams: a first kernel counts the set bits of every tile and
// of every wave's segment inside it, a second turns the tile counts into per-tile payload offsets
// (one workgroup per tensor), and the third, which moves all the bytes, has no dependency between
// workgroups, and none between the waves of a workgroup either.
// ---------------------------------------------------------------------------------------------

// The item that holds launch-wide tile gt (binary search on wave-uniform operands).
__device__ __forceinline__ int64_t find_sparse_item(const bitsnap_sparse_item *__restrict__ items, int64_t count, int64_t gt)
{
    int64_t lo = 0, hi = count - 1;
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) >> 1;
        if (items[mid].first_tile <= gt)
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo;
}

// Where a tile's offset in the payload comes from in the merge (see decode_merge_kernel).
enum { kFromWorkspace = 0, kFromEncoder = 1, kFromMask = 2, kFromCounts = 3 };
// Segments per tile in the decoder: a wave of the merge owns one.  The lighter the waves, the more evenly reads and
// writes mix: a plain copy streams at 72-76 % of HBM peak with 4 KB per wave, at 75-80 % with 2 KB; with 16 segments
// of two-byte elements instead of 32 a pass over a list decodes at 73 instead of 77 % where 71 % of the elements
// changed (74 and 75 % where 6 % did), with 8 segments single tensors lose another 2 to 10 %.  That holds where a
// wave is handed its place (kFromWorkspace).  Where it works its place out itself - from the counts of the earlier
// tiles, from the mask of its own tile or of the tensor before it - twice the waves do twice that work, and 32
// segments are slower than 16: the 131 M-element tensor decodes in 0.156 instead of 0.120 ms, a list with the
// encoder's tile offsets at 58 instead of 73 % of peak.
template <int E, int kSource>
constexpr int kDecSegsOf = (E == 2 && kSource == kFromWorkspace) ? 32 : 16;
constexpr int kMaxDecSegs = 32;
// The segments' places inside their tile are kept as 16-bit numbers, three to a 64-bit word whose upper 16 bits stay
// zero: whatever a decode leaves in the workspace then reads as "not written" to the encoder's scan (scan_state.hpp).
template <int S>
constexpr int kSegWordsOf = (S + 2) / 3;
__device__ __forceinline__ int seg_slot(int k) { return (k / 3) * 4 + k % 3; }

// One wave per tile: popcount of the tile's 4 or 2 KB of mask (bits at or beyond n do not count), and the
// places of the tile's segments inside the tile.
constexpr int kCountWaves = 2;  // tiles per workgroup of the counting kernel (small workgroups: see kMergeWaves)
template <bool kBatched, int E, int S>  // S: segments per tile
__global__ __launch_bounds__(kCountWaves * kWave) void decode_count_kernel(bitsnap_sparse_item single,
                                                              const bitsnap_sparse_item *__restrict__ items,
                                                              int64_t count, int64_t num_tiles,
                                                              uint32_t *__restrict__ tile_count,
                                                              uint16_t *__restrict__ seg_place)
{
    const int lane = threadIdx.x & (kWave - 1), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t gt = (int64_t)blockIdx.x * kCountWaves + wave;
    if (gt >= num_tiles)
        return;
    const bitsnap_sparse_item &it = kBatched ? items[find_sparse_item(items, count, gt)] : single;
    const int64_t tile = gt - it.first_tile, n = it.n;
    const int64_t mask_bytes = (n + 7) >> 3;
    constexpr int kTileMaskBytes = Geom<E>::kTileElems / 8, kPerLane = kTileMaskBytes / kWave;
    static_assert(kPerLane % 8 == 0, "a lane reads whole 8-byte pieces of the mask");
    // Pass q covers 512 consecutive mask bytes, i.e. one or two whole segments (a wave's part of the tile in
    // the merge): the running sums at the segments' last lanes are the segments' places inside the tile.
    constexpr int kDecSegs = S;
    constexpr int kSegsPerPass = (kWave * 8) / (Geom<E>::kTileElems / kDecSegs / 8);
    // All of the lane's loads are issued before the first is used.  An 8-byte piece that straddles the end of the
    // mask is read whole (the buffer is 16-byte aligned, so the load stays inside the 16-byte block of the mask's
    // last byte); one that lies beyond it reads the tile's first bytes instead; what is not mask is cleared below.
    uint2 loaded[kPerLane / 8];
#pragma unroll
    for (int q = 0; q < kPerLane / 8; ++q) {
        const int64_t b0 = tile * kTileMaskBytes + (int64_t)(q * kWave + lane) * 8;  // byte offset, 8-aligned
        loaded[q] = *reinterpret_cast<const uint2 *>(it.mask + (b0 < mask_bytes ? b0 : tile * kTileMaskBytes));
    }
    uint32_t run = 0;
#pragma unroll
    for (int q = 0; q < kPerLane / 8; ++q) {
        const int64_t b0 = tile * kTileMaskBytes + (int64_t)(q * kWave + lane) * 8;
        uint32_t w[2] = {loaded[q].x, loaded[q].y};
        // bits at or beyond n carry no element
        const int64_t e0 = b0 * 8;
        uint32_t c = 0;
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int64_t ek = e0 + 32 * k;
            if (ek + 32 > n)
                w[k] &= (ek < n) ? ((1u << (uint32_t)(n - ek)) - 1u) : 0u;
            c += __popc(w[k]);
        }
        const uint32_t incl = wave_inclusive_add(c);
#pragma unroll
        for (int sgm = 0; sgm < kSegsPerPass; ++sgm) {
            const uint32_t inside = sgm == 0 ? 0u : read_lane(incl, sgm == 0 ? 0 : sgm * (kWave / kSegsPerPass) - 1);
            if (lane == 0)  // below the tile's 2^15 elements
                seg_place[gt * (4 * kSegWordsOf<S>) + seg_slot(q * kSegsPerPass + sgm)] = (uint16_t)(run + inside);
        }
        run += read_lane(incl, kWave - 1);
    }
    if (lane == 0)
        tile_count[gt] = run;
    if (lane < kSegWordsOf<S>) {  // the upper 16 bits of every word, and what the last word has beyond the last segment
        seg_place[gt * (4 * kSegWordsOf<S>) + 4 * lane + 3] = 0;
        if (lane == kSegWordsOf<S> - 1)
            for (int k = kDecSegs; k < 3 * kSegWordsOf<S>; ++k)
                seg_place[gt * (4 * kSegWordsOf<S>) + seg_slot(k)] = 0;
    }
}

// One workgroup per tensor: exclusive scan of its tiles' counts -> payload offset of every tile,
// and the tensor's total.
template <bool kBatched, int E>
__global__ __launch_bounds__(kBlock) void decode_scan_kernel(bitsnap_sparse_item single,
                                                             const bitsnap_sparse_item *__restrict__ items,
                                                             const uint32_t *__restrict__ tile_count,
                                                             uint64_t *__restrict__ tile_offset)
{
    __shared__ uint64_t wave_sum_s[kWaves];
    __shared__ uint64_t carry_s;
    const bitsnap_sparse_item &it = kBatched ? items[blockIdx.x] : single;
    const int64_t ntiles = (it.n + Geom<E>::kTileElems - 1) / Geom<E>::kTileElems, first = it.first_tile;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    if (tid == 0)
        carry_s = 0;
    __syncthreads();
    for (int64_t base = 0; base < ntiles; base += kBlock) {
        const int64_t i = base + tid;
        const uint32_t c = i < ntiles ? tile_count[first + i] : 0u;
        const uint32_t incl = wave_inclusive_add(c);  // a wave covers 64 tiles: at most 2^20 elements
        if (lane == kWave - 1)
            wave_sum_s[wave] = incl;
        __syncthreads();
        uint64_t before = carry_s;
        for (int w = 0; w < wave; ++w)
            before += wave_sum_s[w];
        if (i < ntiles)
            tile_offset[first + i] = before + incl - c;
        __syncthreads();
        if (tid == kBlock - 1)
            carry_s = before + incl;
        __syncthreads();
    }
    if (tid == 0 && it.n_changed)
        *it.n_changed = carry_s;
}

// The merge: out = bit ? next payload element : base.  One wavefront per segment (1024 or 2048 elements, see
// kDecSegsOf), each entirely on its own - no barrier anywhere; kMergeWaves of them make a workgroup.  A wave
// requests its base pieces, its own mask bytes and the mask bytes between the start of the
// tile and its segment at once; the popcount of the latter is the segment's place behind the tile's offset
// (the other waves of the tile read the same few KB, from L2).  Then it fetches its part of the payload as
// aligned 16-byte pieces into its private region of LDS (region[i] holds payload element src0 + i, src0 a
// multiple of 16 / E), from where every lane picks its elements by rank.  With the eight waves of a tile
// in one workgroup, meeting at two barriers per tile, and ordinary instead of non-temporal accesses to payload
// and output, this kernel ran 5 to 8 points of HBM peak slower.
// kDelta: the payload holds cur XOR base; the element is base XOR payload.
// kSource: where the tile's offset in the payload comes from - the counting and scanning kernels
// (kFromWorkspace), the counting kernel alone (kFromCounts: the wave adds up the counts of the tensor's earlier
// tiles itself, a few KB from L2, which saves a single tensor of moderate size the scanning launch), the
// encoder's tile_offsets (kFromEncoder), or nowhere: the wave counts the tensor's whole mask before its
// segment itself (kFromMask; tensors of a few tiles, decoded by this one launch).
constexpr int kSoloTiles = 8;        // single tensors of up to this many tiles take kFromMask
constexpr int kCountsTiles = 4096;   // single tensors of up to this many tiles take kFromCounts (offsets stay below 2^32)
constexpr int kOffsetsTiles = 2048;  // a call with the encoder's tile offsets uses them (kFromEncoder) up to this many tiles
// Waves of a tile do not cooperate, so the workgroup is only the unit in which the hardware hands out wave
// slots and LDS: a new workgroup starts when a whole one has left.  With the byte mix of this kernel and no
// logic, 16 waves per CU stream at 67-70 % of HBM peak as 512-thread workgroups, 72-74 % as 256-thread ones,
// 77-78 % as 128-thread ones and 74-75 % as single waves.
constexpr int kMergeWaves = 2;                          // waves (segments) per workgroup
constexpr int kMergeBlock = kMergeWaves * kWave;
template <int E, int kSource>
constexpr int kMergeBlocksPerTileOf = kDecSegsOf<E, kSource> / kMergeWaves;

template <int E, int S>
struct DecGeom {
    static constexpr int kSegElems = Geom<E>::kTileElems / S;           // 1024 or 2048 two-byte, 1024 four-byte elements
    static constexpr int kPieces = kSegElems / kChunkElems;             // 512-element pieces per segment: 2 or 4
    static constexpr int kSegMaskBytes = kSegElems / 8;
    static constexpr int kVecsPerLane = kSegElems / Geom<E>::kVecElems / kWave;  // 16-byte payload pieces per lane: 4
    static_assert(kPieces % 2 == 0, "counts are scanned two to a word");
};

template <bool kBatched, bool kDelta, int kSource, int E>
__global__ __launch_bounds__(kMergeBlock) void decode_merge_kernel(bitsnap_sparse_item single,
                                                                 const bitsnap_sparse_item *__restrict__ items,
                                                                 int64_t count, const uint64_t *__restrict__ tile_offset,
                                                                 const uint32_t *__restrict__ tile_count,
                                                                 const uint16_t *__restrict__ seg_place)
{
    typedef typename Geom<E>::elem_t elem_t;
    typedef typename Geom<E>::global_elem_t global_elem_t;
    constexpr int kDecSegs = kDecSegsOf<E, kSource>, kMergeBlocksPerTile = kMergeBlocksPerTileOf<E, kSource>;
    typedef DecGeom<E, kDecSegs> SegGeom;
    constexpr int kTileElems = Geom<E>::kTileElems, kSegElems = SegGeom::kSegElems, kPieces = SegGeom::kPieces,
                  kVecs = Geom<E>::kVecs, kVecElems = Geom<E>::kVecElems, kVecsPerLane = SegGeom::kVecsPerLane;
    constexpr uint32_t P = Geom<E>::kVecElems;
    __shared__ alignas(16) elem_t regions[kMergeWaves][kSegElems + 4 * P];  // + a shifted segment's end + what the merge reads past it
    const int tid = threadIdx.x, lane = tid & (kWave - 1), local_wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t gtile = blockIdx.x / kMergeBlocksPerTile;
    const int wave = (int)(blockIdx.x % kMergeBlocksPerTile) * kMergeWaves + local_wave;  // the segment inside the tile
    const bitsnap_sparse_item &it = kBatched ? items[find_sparse_item(items, count, gtile)] : single;
    const int64_t n = it.n, payload_elems = it.capacity, tile = gtile - it.first_tile;
    const int64_t seg0 = tile * kTileElems + (int64_t)wave * kSegElems;  // first element of the wave's segment
    if (seg0 >= n)
        return;
    // every field of the item that is needed is fetched here, not where it is used: a word of the item array
    // read late would be waited for on its own
    const elem_t *base = (const elem_t *)it.base + seg0;  // may alias out
    const uint8_t *__restrict__ mask = it.mask;
    const elem_t *__restrict__ payload = (const elem_t *)it.payload;
    const uint32_t *__restrict__ encoder_offsets = it.tile_offsets;
    uint64_t *count_out = it.n_changed;
    elem_t *out = (elem_t *)it.out;
    elem_t *region = regions[local_wave];
    const int64_t mask_bytes = (n + 7) >> 3;
    const uint32_t rem = n - seg0 >= kSegElems ? (uint32_t)kSegElems : (uint32_t)(n - seg0);
    const uint32_t e0 = (uint32_t)(lane * kLaneElems);
    // What the counting and scanning kernels left: the place and the length of every segment.  Read before
    // anything else is requested, so that waiting for these few words does not mean waiting for the base as well
    // (loads return in the order they were issued).
    uint64_t known_start = 0;
    if (kSource == kFromWorkspace || kSource == kFromCounts) {
        uint64_t tile_excl;
        if (kSource == kFromCounts) {
            // the counts of the tensor's earlier tiles (at most kCountsTiles of them), two per lane and load, a
            // batch of loads in flight at a time; the array is 8-byte aligned and holds an entry for this tile
            // too, so the second word of a pair is always there
            const uint32_t *__restrict__ counts = tile_count + it.first_tile;
            constexpr int kBatch = 16;
            uint32_t partial = 0;
            for (int64_t lo = 0; lo < tile; lo += kBatch * kWave * 2) {
                uint2 pair[kBatch];
#pragma unroll
                for (int k = 0; k < kBatch; ++k) {
                    const int64_t i = lo + (int64_t)(k * kWave + lane) * 2;
                    pair[k] = make_uint2(0u, 0u);
                    if (i < tile)
                        pair[k] = *reinterpret_cast<const uint2 *>(counts + i);
                }
#pragma unroll
                for (int k = 0; k < kBatch; ++k) {
                    const int64_t i = lo + (int64_t)(k * kWave + lane) * 2;
                    partial += pair[k].x + (i + 1 < tile ? pair[k].y : 0u);
                }
            }
            tile_excl = read_lane(wave_inclusive_add(partial), kWave - 1);
        } else {
            tile_excl = uniform64(tile_offset[gtile]);
        }
        known_start = tile_excl;
    }
    uint32_t seg_before = 0, seg_mine = 0;
    if (kSource == kFromWorkspace || kSource == kFromCounts) {
        const uint16_t *__restrict__ places = seg_place + gtile * (4 * kSegWordsOf<kDecSegs>);
        seg_before = __builtin_amdgcn_readfirstlane(places[seg_slot(wave)]);
        const uint32_t next = __builtin_amdgcn_readfirstlane(wave + 1 < kDecSegs ? places[seg_slot(wave + 1)] : tile_count[gtile]);
        seg_mine = next - seg_before;
    }

    // base: a 16-byte load whose first element lies at or beyond the end of the tensor reads the segment's first
    // 16 bytes instead; one that straddles the end is made whole (the buffer is 16-byte aligned)
    Piece<E> v[kPieces];
#pragma unroll
    for (int q = 0; q < kPieces; ++q)
#pragma unroll
        for (int k = 0; k < kVecs; ++k) {
            const uint32_t ek = e0 + (uint32_t)(q * kChunkElems + k * kVecElems);
            v[q].v[k] = load_global16<true>(base + (ek < rem ? ek : 0u));
        }
    // the segment's own mask bytes, one per lane and piece; bits at or beyond n carry no element
    uint32_t m[kPieces];
#pragma unroll
    for (int q = 0; q < kPieces; ++q) {
        const int64_t mb = (seg0 >> 3) + q * kWave + lane;
        uint32_t bits = (mb < mask_bytes) ? ((const global_u8 *)mask)[mb] : 0u;
        const int32_t left = (int32_t)rem - (int32_t)(q * kChunkElems) - (int32_t)e0;
        bits &= left >= kLaneElems ? 0xFFu : left > 0 ? (1u << left) - 1u : 0u;
        m[q] = bits;
    }
    // The segment's changed values, payload elements [start, start + seg_count), as aligned 16-byte pieces.
    uint64_t start = 0;
    uint32_t seg_count = 0, shift = 0, pieces = 0;
    uint4 pv[kVecsPerLane];
    const elem_t *__restrict__ seg = nullptr;
    int64_t seg_elems = 0;
    // Base, payload and output are touched once: non-temporal accesses throughout (66 -> 69-70 % of HBM peak on
    // checkpoints with 6 % changed; where most elements changed the hints make no difference beyond the noise
    // between runs in a batched pass, and one call per tensor gains 3-4 %).
    auto request_payload = [&]() {
        shift = (uint32_t)(start & (P - 1u));
        const int64_t src0 = (int64_t)(start - shift);
        pieces = (shift + seg_count + P - 1u) / P;           // at most kSegElems / P + 1
        seg = payload + src0;                                // wave-uniform, 16-byte aligned
        seg_elems = payload_elems - src0;                    // elements of seg that may be read
#pragma unroll
        for (int i = 0; i < kVecsPerLane; ++i) {
            const uint32_t q = (uint32_t)(i * kWave + lane);
            pv[i] = make_uint4(0, 0, 0, 0);  // never read at or beyond payload_elems: what is missing decodes to 0
            if (q < pieces) {
                if ((int64_t)(q * P + P) <= seg_elems) {
                    pv[i] = load_global16<true>(seg + q * P);
                } else {
                    uint32_t w[4] = {0, 0, 0, 0};
                    for (uint32_t t = 0; t < P; ++t)
                        if ((int64_t)(q * P + t) < seg_elems)
                            w[(t * E) >> 2] |= (uint32_t)((const global_elem_t *)seg)[q * P + t] << (((t * E) & 3u) * 8u);
                    pv[i] = make_uint4(w[0], w[1], w[2], w[3]);
                }
            }
        }
    };
    if (kSource == kFromWorkspace || kSource == kFromCounts) {
        start = known_start + seg_before;
        seg_count = seg_mine;
        request_payload();
    }
    // ranks inside the segment
    uint32_t rank[kPieces], counted = 0;
#pragma unroll
    for (int q = 0; q < kPieces; q += 2) {
        const uint32_t c0 = __popc(m[q]), c1 = __popc(m[q + 1]);
        const uint32_t pk = c0 | (c1 << 16);
        const uint32_t incl = wave_inclusive_add(pk);
        const uint32_t tot = read_lane(incl, kWave - 1);
        const uint32_t ex = incl - pk;
        rank[q] = counted + (ex & 0xFFFFu);
        rank[q + 1] = counted + (tot & 0xFFFFu) + (ex >> 16);
        counted += (tot & 0xFFFFu) + (tot >> 16);
    }
    if (kSource == kFromEncoder || kSource == kFromMask) {
        // set bits between the point the known offset refers to and the segment (whole bytes of whole segments)
        const int64_t from = kSource == kFromMask ? 0 : tile * (int64_t)(kTileElems / 8);
        const int32_t prior_bytes = (int32_t)((seg0 >> 3) - from);
        uint32_t before = 0;
#pragma unroll 8
        for (int32_t o = lane * 8; o < prior_bytes; o += kWave * 8) {
            const uint2 w = *reinterpret_cast<const uint2 *>(mask + from + o);
            before += __popc(w.x) + __popc(w.y);
        }
        before = read_lane(wave_inclusive_add(before), kWave - 1);
        const uint64_t tile_excl = kSource == kFromEncoder ? (uint64_t)__builtin_amdgcn_readfirstlane(encoder_offsets[tile]) : 0ull;
        start = tile_excl + before;
        seg_count = counted;
        request_payload();
    }
#pragma unroll
    for (int i = 0; i < kVecsPerLane; ++i)
        *reinterpret_cast<uint4 *>(&region[(uint32_t)(i * kWave + lane) * P]) = pv[i];
    if (lane == 0 && pieces > (uint32_t)(kVecsPerLane * kWave)) {  // a full segment that starts off the 16-byte grid
        const uint32_t q = (uint32_t)(kVecsPerLane * kWave);
        for (uint32_t t = 0; t < P; ++t)
            region[q * P + t] = (int64_t)(q * P + t) < seg_elems ? ((const global_elem_t *)seg)[q * P + t] : (elem_t)0;
    }
    __builtin_amdgcn_wave_barrier();  // the region is read by other lanes of this wave than wrote it
    // Element t of a piece takes region[p + (set bits below t)] if its bit is set.  Straight-line code: the value
    // is read whether or not the bit is set (the region is long enough for that) and then kept or dropped
    // through a mask of the bit; with a branch per element the merge was four times as many instructions.
#pragma unroll
    for (int q = 0; q < kPieces; ++q) {
        const uint32_t p = shift + rank[q];
        uint32_t w[2 * E];  // the piece's dwords
#pragma unroll
        for (int k = 0; k < 2 * E; ++k)
            w[k] = word_of(v[q].v[k >> 2], k & 3);
        uint32_t val[kLaneElems], keep[kLaneElems];
#pragma unroll
        for (int t = 0; t < kLaneElems; ++t) {
            val[t] = region[p + __popc(m[q] & ((1u << t) - 1u))];
            keep[t] = (uint32_t)(-(int32_t)((m[q] >> t) & 1u));  // all ones where the element changed
        }
        if (E == 4) {
#pragma unroll
            for (int t = 0; t < kLaneElems; ++t)
                w[t] = kDelta ? (w[t] ^ (val[t] & keep[t])) : ((val[t] & keep[t]) | (w[t] & ~keep[t]));
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t pair = (val[2 * k] & 0xFFFFu) | (val[2 * k + 1] << 16);
                const uint32_t km = (keep[2 * k] & 0xFFFFu) | (keep[2 * k + 1] << 16);
                w[k] = kDelta ? (w[k] ^ (pair & km)) : ((pair & km) | (w[k] & ~km));
            }
        }
        Piece<E> res;
#pragma unroll
        for (int k = 0; k < kVecs; ++k)
            res.v[k] = make_uint4(w[4 * k + 0], w[4 * k + 1], w[4 * k + 2], w[4 * k + 3]);
        store8<true, E>(out, seg0 + q * kChunkElems + e0, n, res);
    }
    // no scan kernel ran to report the count: the wave that holds the tensor's last element knows it
    if (kSource != kFromWorkspace && lane == 0 && count_out && seg0 + kSegElems >= n)
        *count_out = start + seg_count;
}

// Workspace after the header: encode keeps its count and prefix words there (scan_state.hpp: 8 bytes per tile,
// then, from a 128-byte boundary, 64 bytes per tile); decode keeps the tiles' payload offsets (8 bytes each)
// followed by their counts (4 bytes each) and the places of their segments (up to 11 words of three 16-bit places).
// A raw offset is below 2^40, a tile's count at most 2^15 in 32 bits, and the upper 16 bits of a word of places are
// zero, so as scan words their two flag bits read "not written": a decode never confuses a later encode.
constexpr size_t kWorkspaceBytesPerTile = kScanBytesPerTile;
static_assert(kWorkspaceBytesPerTile >= 16 + 8 * kSegWordsOf<kMaxDecSegs>,
              "decode keeps 8 + 4 (+ 4 once) + 8 * ceil(segments / 3) bytes per tile");

static std::atomic<uint32_t> g_spin_limit{kDefaultSpinLimit};

// Persistent grid of the scan kernel.  Tiles are handed out by ticket, so nothing depends on every
// workgroup being resident: a workgroup that only starts after others have finished finds no tile
// left and exits.  Registers and LDS allow two workgroups per CU.
static int sparse_grid(const void *kernel, int64_t num_tiles)
{
    const DeviceInfo &di = device_info();
    int per_cu = occupancy_blocks_per_cu(kernel, kBlock);
    if (per_cu < 2)
        per_cu = 2;
    int64_t resident = (int64_t)di.cu_count * per_cu;
    int64_t g = num_tiles < resident ? num_tiles : resident;
    return (int)(g < 1 ? 1 : g);
}

static int64_t tile_elems_of(int elem_bytes) { return elem_bytes == 4 ? Geom<4>::kTileElems : Geom<2>::kTileElems; }
static int64_t tiles_of(int64_t n, int elem_bytes)
{
    return n <= 0 ? 0 : (n + tile_elems_of(elem_bytes) - 1) / tile_elems_of(elem_bytes);
}
static size_t workspace_bytes_for_tiles(int64_t tiles)
{
    const size_t bytes = kScanHeaderBytes + (size_t)(tiles < 0 ? 0 : tiles) * kWorkspaceBytesPerTile;
    return (bytes + 255) / 256 * 256;
}

static int check_workspace(void *workspace, size_t workspace_bytes, int64_t n, int elem_bytes)
{
    if (!workspace)
        return BITSNAP_E_NULL;
    if (!aligned16(workspace))
        return BITSNAP_E_ALIGN;
    if (workspace_bytes < workspace_bytes_for_tiles(tiles_of(n, elem_bytes)))
        return BITSNAP_E_WORKSPACE;
    return BITSNAP_OK;
}

}  // namespace bitsnap

using namespace bitsnap;

extern "C" size_t bitsnap_sparse_tile_elems(void) { return (size_t)Geom<2>::kTileElems; }

extern "C" size_t bitsnap_sparse_tile_elems_for(int elem_bytes)
{
    return (elem_bytes == 2 || elem_bytes == 4) ? (size_t)tile_elems_of(elem_bytes) : 0;
}

extern "C" size_t bitsnap_sparse_mask_bytes(int64_t n)
{
    if (n <= 0)
        return 0;
    return (size_t)((((n + 7) / 8) + 15) / 16 * 16);
}

extern "C" size_t bitsnap_sparse_workspace_bytes(int64_t n) { return workspace_bytes_for_tiles(tiles_of(n, 2)); }

extern "C" size_t bitsnap_sparse_workspace_bytes_for(int64_t n, int elem_bytes)
{
    return (elem_bytes == 2 || elem_bytes == 4) ? workspace_bytes_for_tiles(tiles_of(n, elem_bytes)) : 0;
}

extern "C" void bitsnap_debug_set_spin_limit(uint32_t polls)
{
    // opt-in: a stray call in a production process must not be able to make encodes give up
    const char *knobs = getenv("BITSNAP_DEBUG_KNOBS");
    if (!knobs || knobs[0] != '1' || knobs[1] != '\0')
        return;
    g_spin_limit.store(polls ? polls : kDefaultSpinLimit, std::memory_order_relaxed);
}

template <typename Kernel>
static int launch_scan(Kernel kernel, const bitsnap_sparse_item &single, const bitsnap_sparse_item *items, int64_t count,
                       int64_t num_tiles, void *workspace, size_t workspace_bytes, bitsnap_stream_t stream, int refresh)
{
    ScanHeader *hdr = reinterpret_cast<ScanHeader *>(workspace);
    uint64_t *status = reinterpret_cast<uint64_t *>(reinterpret_cast<char *>(workspace) + kScanHeaderBytes);
    const int64_t status_cap = (int64_t)((workspace_bytes - kScanHeaderBytes) / sizeof(uint64_t));
    const int grid = sparse_grid(reinterpret_cast<const void *>(kernel), num_tiles + 1);  // + the workgroup of the scanning wave
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(kBlock), 0, (hipStream_t)stream, single, items, count, hdr, status,
                       status_cap, num_tiles, g_spin_limit.load(std::memory_order_relaxed), refresh);
    return launch_status();
}

static int check_scan_workspace(void *workspace, size_t workspace_bytes, int64_t num_tiles)
{
    if (!workspace)
        return BITSNAP_E_NULL;
    if (!aligned16(workspace))
        return BITSNAP_E_ALIGN;
    if (workspace_bytes < kScanHeaderBytes + (size_t)num_tiles * kWorkspaceBytesPerTile)
        return BITSNAP_E_WORKSPACE;
    return BITSNAP_OK;
}

// The segments' places follow the tiles' counts, from the next 8-byte boundary: their words must be words of the scan too.
static uint16_t *seg_places_of(const uint32_t *tile_count, int64_t num_tiles)
{
    return reinterpret_cast<uint16_t *>(const_cast<uint32_t *>(tile_count) + ((num_tiles + 1) & ~(int64_t)1));
}

template <bool kBatched, bool kDelta, int kSource, int E>
static void launch_merge(const bitsnap_sparse_item &single, const bitsnap_sparse_item *items, int64_t count,
                         int64_t num_tiles, const uint64_t *tile_offset, hipStream_t s)
{
    const uint32_t *tile_count = reinterpret_cast<const uint32_t *>(tile_offset + num_tiles);
    hipLaunchKernelGGL((decode_merge_kernel<kBatched, kDelta, kSource, E>), dim3((unsigned)(num_tiles * kMergeBlocksPerTileOf<E, kSource>)),
                       dim3(kMergeBlock), 0, s, single, items, count, tile_offset, tile_count,
                       seg_places_of(tile_count, num_tiles));
}

template <bool kBatched, int E>
static int launch_decode_e(const bitsnap_sparse_item &single, const bitsnap_sparse_item *items, int64_t count,
                           int64_t num_tiles, void *workspace, bitsnap_stream_t stream, bool delta, bool offsets)
{
    uint64_t *tile_offset = reinterpret_cast<uint64_t *>(reinterpret_cast<char *>(workspace) + kScanHeaderBytes);
    uint32_t *tile_count = reinterpret_cast<uint32_t *>(tile_offset + num_tiles);
    hipStream_t s = (hipStream_t)stream;
    if (num_tiles > 0x7FFFFFFF / (kMaxDecSegs / kMergeWaves))
        return BITSNAP_E_SIZE;
    // The encoder's tile offsets are given: one launch, in which every wave counts inside its tile.  That saves a
    // tensor (or a list) of up to a few thousand tiles 2-3 us; beyond, the launches that hand every wave its place
    // are faster (131 M two-byte elements: 114-133 against 117-140 us, 6.7 G in a list: 6.4 against 6.7 ms), and
    // the offsets are left unused.
    if (offsets && num_tiles > 0 && num_tiles <= kOffsetsTiles) {
        if (delta)
            launch_merge<kBatched, true, kFromEncoder, E>(single, items, count, num_tiles, tile_offset, s);
        else
            launch_merge<kBatched, false, kFromEncoder, E>(single, items, count, num_tiles, tile_offset, s);
        return launch_status();
    }
    if (!kBatched && num_tiles > kSoloTiles && num_tiles <= kCountsTiles) {  // counting kernel, then the merge adds up the counts
        hipLaunchKernelGGL((decode_count_kernel<kBatched, E, kDecSegsOf<E, kFromCounts>>), dim3((unsigned)((num_tiles + kCountWaves - 1) / kCountWaves)),
                           dim3(kCountWaves * kWave), 0, s, single, items, count, num_tiles, tile_count,
                           seg_places_of(tile_count, num_tiles));
        if (delta)
            launch_merge<kBatched, true, kFromCounts, E>(single, items, count, num_tiles, tile_offset, s);
        else
            launch_merge<kBatched, false, kFromCounts, E>(single, items, count, num_tiles, tile_offset, s);
        return launch_status();
    }
    if (!kBatched && num_tiles > 0 && num_tiles <= kSoloTiles) {  // a small tensor: every wave counts for itself
        if (delta)
            launch_merge<kBatched, true, kFromMask, E>(single, items, count, num_tiles, tile_offset, s);
        else
            launch_merge<kBatched, false, kFromMask, E>(single, items, count, num_tiles, tile_offset, s);
        return launch_status();
    }
    if (num_tiles > 0)
        hipLaunchKernelGGL((decode_count_kernel<kBatched, E, kDecSegsOf<E, kFromWorkspace>>), dim3((unsigned)((num_tiles + kCountWaves - 1) / kCountWaves)),
                           dim3(kCountWaves * kWave), 0, s, single, items, count, num_tiles, tile_count,
                           seg_places_of(tile_count, num_tiles));
    // the scan also reports n_changed, for an empty tensor too
    hipLaunchKernelGGL((decode_scan_kernel<kBatched, E>), dim3((unsigned)(kBatched ? count : 1)), dim3(kBlock), 0, s,
                       single, items, tile_count, tile_offset);
    if (num_tiles > 0 && delta)
        launch_merge<kBatched, true, kFromWorkspace, E>(single, items, count, num_tiles, tile_offset, s);
    else if (num_tiles > 0)
        launch_merge<kBatched, false, kFromWorkspace, E>(single, items, count, num_tiles, tile_offset, s);
    return launch_status();
}

template <bool kBatched>
static int launch_decode(const bitsnap_sparse_item &single, const bitsnap_sparse_item *items, int64_t count,
                         int64_t num_tiles, void *workspace, bitsnap_stream_t stream, bool delta, bool offsets,
                         int elem_bytes)
{
    if (elem_bytes == 4)
        return launch_decode_e<kBatched, 4>(single, items, count, num_tiles, workspace, stream, delta, offsets);
    return launch_decode_e<kBatched, 2>(single, items, count, num_tiles, workspace, stream, delta, offsets);
}

template <bool kBatched>
static int launch_encode(const bitsnap_sparse_item &single, const bitsnap_sparse_item *items, int64_t count,
                         int64_t num_tiles, void *workspace, size_t workspace_bytes, bitsnap_stream_t stream, bool delta,
                         int refresh, int elem_bytes)
{
    if (!kBatched && num_tiles == 1) {  // one workgroup, nothing to coordinate
        ScanHeader *hdr = reinterpret_cast<ScanHeader *>(workspace);
        const dim3 one(1), block(kBlock);
        hipStream_t s = (hipStream_t)stream;
#define BITSNAP_LAUNCH_SOLO(D, EB)                                                                                   \
    hipLaunchKernelGGL((encode_sparse_kernel<false, D, EB, true>), one, block, 0, s, single, items, count, hdr, nullptr, \
                       (int64_t)0, num_tiles, 0u, refresh)
        if (elem_bytes == 4) {
            if (delta)
                BITSNAP_LAUNCH_SOLO(true, 4);
            else
                BITSNAP_LAUNCH_SOLO(false, 4);
        } else {
            if (delta)
                BITSNAP_LAUNCH_SOLO(true, 2);
            else
                BITSNAP_LAUNCH_SOLO(false, 2);
        }
#undef BITSNAP_LAUNCH_SOLO
        return launch_status();
    }
    if (elem_bytes == 4) {
        if (delta)
            return launch_scan(&encode_sparse_kernel<kBatched, true, 4>, single, items, count, num_tiles, workspace,
                               workspace_bytes, stream, refresh);
        return launch_scan(&encode_sparse_kernel<kBatched, false, 4>, single, items, count, num_tiles, workspace,
                           workspace_bytes, stream, refresh);
    }
    if (delta)
        return launch_scan(&encode_sparse_kernel<kBatched, true, 2>, single, items, count, num_tiles, workspace,
                           workspace_bytes, stream, refresh);
    return launch_scan(&encode_sparse_kernel<kBatched, false, 2>, single, items, count, num_tiles, workspace,
                       workspace_bytes, stream, refresh);
}

extern "C" int bitsnap_encode_sparse_ex(const void *cur, const void *base, int64_t n, int elem_bytes, uint32_t flags,
                                        uint8_t *mask, void *payload, int64_t payload_capacity_elems,
                                        uint32_t *tile_offsets, uint64_t *n_changed, void *new_base, void *workspace,
                                        size_t workspace_bytes, bitsnap_stream_t stream)
{
    if (n < 0 || (elem_bytes != 2 && elem_bytes != 4) || payload_capacity_elems < 0 || n >= (int64_t)1 << kValueBits ||
        (flags & ~(uint32_t)BITSNAP_SPARSE_DELTA))
        return BITSNAP_E_SIZE;
    if (!n_changed || (n > 0 && (!cur || !base || !mask)) || (payload_capacity_elems > 0 && !payload))
        return BITSNAP_E_NULL;
    if (!aligned16(cur) || !aligned16(base) || !aligned16(mask) || !aligned16(payload) || !aligned16(new_base) ||
        ((uintptr_t)n_changed & 7u) || ((uintptr_t)tile_offsets & 3u))
        return BITSNAP_E_ALIGN;
    if (int rc = check_workspace(workspace, workspace_bytes, n, elem_bytes))
        return rc;
    if (tile_offsets && n >= (int64_t)1 << 32)
        return BITSNAP_E_OFFSETS;
    bitsnap_sparse_item it = {};
    it.src = cur;
    it.base = base;
    it.mask = mask;
    it.payload = payload;
    it.out = new_base;
    it.n_changed = n_changed;
    it.tile_offsets = tile_offsets;
    it.n = n;
    it.capacity = payload_capacity_elems;
    return launch_encode<false>(it, nullptr, 1, tiles_of(n, elem_bytes), workspace, workspace_bytes, stream,
                                (flags & BITSNAP_SPARSE_DELTA) != 0, new_base != nullptr, elem_bytes);
}

extern "C" int bitsnap_encode_sparse(const void *cur, const void *base, int64_t n, int elem_bytes, uint8_t *mask,
                                     void *payload, int64_t payload_capacity_elems, uint32_t *tile_offsets,
                                     uint64_t *n_changed, void *workspace, size_t workspace_bytes,
                                     bitsnap_stream_t stream)
{
    return bitsnap_encode_sparse_ex(cur, base, n, elem_bytes, 0u, mask, payload, payload_capacity_elems, tile_offsets,
                                    n_changed, nullptr, workspace, workspace_bytes, stream);
}

extern "C" int bitsnap_decode_sparse_ex(const void *base, const uint8_t *mask, const void *payload,
                                        int64_t payload_elems, int64_t n, int elem_bytes, uint32_t flags,
                                        const uint32_t *tile_offsets, void *out, uint64_t *n_changed, void *workspace,
                                        size_t workspace_bytes, bitsnap_stream_t stream)
{
    if (n < 0 || (elem_bytes != 2 && elem_bytes != 4) || payload_elems < 0 || n >= (int64_t)1 << kValueBits ||
        (flags & ~(uint32_t)BITSNAP_SPARSE_DELTA))
        return BITSNAP_E_SIZE;
    if ((n > 0 && (!base || !mask || !out)) || (payload_elems > 0 && !payload))
        return BITSNAP_E_NULL;
    if (!aligned16(base) || !aligned16(mask) || !aligned16(payload) || !aligned16(out) || ((uintptr_t)n_changed & 7u) ||
        ((uintptr_t)tile_offsets & 3u))
        return BITSNAP_E_ALIGN;
    if (int rc = check_workspace(workspace, workspace_bytes, n, elem_bytes))
        return rc;
    if (tile_offsets && n >= (int64_t)1 << 32)
        return BITSNAP_E_OFFSETS;
    bitsnap_sparse_item it = {};
    it.base = base;
    it.mask = const_cast<uint8_t *>(mask);
    it.payload = const_cast<void *>(payload);
    it.out = out;
    it.n_changed = n_changed;
    it.tile_offsets = const_cast<uint32_t *>(tile_offsets);
    it.n = n;
    it.capacity = payload_elems;
    return launch_decode<false>(it, nullptr, 1, tiles_of(n, elem_bytes), workspace, stream,
                                (flags & BITSNAP_SPARSE_DELTA) != 0, tile_offsets != nullptr, elem_bytes);
}

extern "C" int bitsnap_decode_sparse(const void *base, const uint8_t *mask, const void *payload, int64_t payload_elems,
                                     int64_t n, int elem_bytes, void *out, uint64_t *n_changed, void *workspace,
                                     size_t workspace_bytes, bitsnap_stream_t stream)
{
    return bitsnap_decode_sparse_ex(base, mask, payload, payload_elems, n, elem_bytes, 0u, nullptr, out, n_changed, workspace,
                                    workspace_bytes, stream);
}

// ---------------------------------------------------------------------------------------------
// The encoder for callers that cannot allocate: its scan state lives in a device array that is part
// of the library's code object instead of a caller-supplied workspace.
// ---------------------------------------------------------------------------------------------
namespace bitsnap {
constexpr size_t kStaticScratchBytes = kScanHeaderBytes + (size_t)BITSNAP_STATIC_MAX_TILES * kWorkspaceBytesPerTile;
}
// One copy per GPU, at an address of its own on each, held until the process ends.
static __device__ __align__(256) unsigned char scratch[bitsnap::kStaticScratchBytes];

namespace bitsnap {

// Everything the scan state holds (header, epoch and status words) back to "never used".
__global__ __launch_bounds__(256) void clear_scratch_kernel(uint4 *p, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
        p[i] = make_uint4(0, 0, 0, 0);
}

// The device address of `scratch` on the current GPU (the array's name means nothing to host code
// beyond being the handle this lookup takes).  Looked up once per device; *first tells the caller
// that this is the first use on that device.
static int static_scratch(void **ptr, bool *first)
{
    static void *addr[kMaxDevices];
    static std::mutex mu;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return BITSNAP_E_LAUNCH;
    std::lock_guard<std::mutex> lock(mu);
    *first = addr[dev] == nullptr;
    if (!addr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p)
            return BITSNAP_E_LAUNCH;
        addr[dev] = p;
    }
    *ptr = addr[dev];
    return BITSNAP_OK;
}

}  // namespace bitsnap

extern "C" int bitsnap_encode_sparse_static(const void *cur, const void *base, int64_t n, int elem_bytes, uint8_t *mask,
                                            void *payload, int64_t payload_capacity_elems, uint32_t *tile_offsets,
                                            uint64_t *n_changed, bitsnap_stream_t stream)
{
    if (n < 0 || (elem_bytes != 2 && elem_bytes != 4))
        return BITSNAP_E_SIZE;
    if (tiles_of(n, elem_bytes) > (int64_t)BITSNAP_STATIC_MAX_TILES)
        return BITSNAP_E_STATIC_LIMIT;
    void *ws = nullptr;
    bool first = false;
    if (int rc = static_scratch(&ws, &first))
        return rc;
    if (first) {
        // A fill kernel, not a memset: this call may be recorded into a graph.  The array starts out
        // as zeros anyway; clearing it is right at any time no call that uses it is in flight.
        hipLaunchKernelGGL(clear_scratch_kernel, dim3(64), dim3(256), 0, (hipStream_t)stream, (uint4 *)ws,
                           kStaticScratchBytes / 16);
        if (int rc = launch_status())
            return rc;
    }
    return bitsnap_encode_sparse_ex(cur, base, n, elem_bytes, 0u, mask, payload, payload_capacity_elems, tile_offsets,
                                    n_changed, nullptr, ws, kStaticScratchBytes, stream);
}

extern "C" size_t bitsnap_sparse_batch_workspace_bytes(int64_t total_tiles) { return workspace_bytes_for_tiles(total_tiles); }

static int check_batch(const bitsnap_sparse_item *items, int64_t count, int64_t total_tiles, void *workspace,
                       size_t workspace_bytes)
{
    if (count < 0 || total_tiles < 0 || total_tiles >= (int64_t)1 << 32)
        return BITSNAP_E_SIZE;
    if (count > 0 && !items)
        return BITSNAP_E_NULL;
    if ((uintptr_t)items & 7u)
        return BITSNAP_E_ALIGN;
    return check_scan_workspace(workspace, workspace_bytes, total_tiles);
}

static int encode_batched(const bitsnap_sparse_item *items, int64_t count, int64_t total_tiles, int elem_bytes,
                          uint32_t flags, int refresh, void *workspace, size_t workspace_bytes, bitsnap_stream_t stream)
{
    if ((flags & ~(uint32_t)BITSNAP_SPARSE_DELTA) || (elem_bytes != 2 && elem_bytes != 4))
        return BITSNAP_E_SIZE;
    if (int rc = check_batch(items, count, total_tiles, workspace, workspace_bytes))
        return rc;
    if (count == 0 || total_tiles == 0)
        return BITSNAP_OK;
    return launch_encode<true>(bitsnap_sparse_item{}, items, count, total_tiles, workspace, workspace_bytes, stream,
                               (flags & BITSNAP_SPARSE_DELTA) != 0, refresh, elem_bytes);
}

extern "C" int bitsnap_encode_sparse_batched(const bitsnap_sparse_item *items, int64_t count, int64_t total_tiles,
                                             void *workspace, size_t workspace_bytes, bitsnap_stream_t stream)
{
    return encode_batched(items, count, total_tiles, 2, 0u, 0, workspace, workspace_bytes, stream);
}

extern "C" int bitsnap_encode_sparse_batched_ex(const bitsnap_sparse_item *items, int64_t count, int64_t total_tiles,
                                                int elem_bytes, uint32_t flags, void *workspace, size_t workspace_bytes,
                                                bitsnap_stream_t stream)
{
    return encode_batched(items, count, total_tiles, elem_bytes, flags, 1, workspace, workspace_bytes, stream);
}

extern "C" int bitsnap_decode_sparse_batched_ex(const bitsnap_sparse_item *items, int64_t count, int64_t total_tiles,
                                                int elem_bytes, uint32_t flags, void *workspace, size_t workspace_bytes,
                                                bitsnap_stream_t stream)
{
    if ((flags & ~(uint32_t)(BITSNAP_SPARSE_DELTA | BITSNAP_SPARSE_OFFSETS)) || (elem_bytes != 2 && elem_bytes != 4))
        return BITSNAP_E_SIZE;
    if (int rc = check_batch(items, count, total_tiles, workspace, workspace_bytes))
        return rc;
    if (count == 0 || total_tiles == 0)
        return BITSNAP_OK;
    return launch_decode<true>(bitsnap_sparse_item{}, items, count, total_tiles, workspace, stream,
                               (flags & BITSNAP_SPARSE_DELTA) != 0, (flags & BITSNAP_SPARSE_OFFSETS) != 0, elem_bytes);
}

extern "C" int bitsnap_decode_sparse_batched(const bitsnap_sparse_item *items, int64_t count, int64_t total_tiles,
                                             void *workspace, size_t workspace_bytes, bitsnap_stream_t stream)
{
    return bitsnap_decode_sparse_batched_ex(items, count, total_tiles, 2, 0u, workspace, workspace_bytes, stream);
}
