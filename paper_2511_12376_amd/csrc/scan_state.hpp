// Cross-workgroup exclusive scan of per-tile counts, single pass, by a scanning wave.
//
// Every tile leaves its count in a word of its own; one wavefront of the launch (the "scanning
// wave") reads those words in tile order, many at a time, and answers each tile with the count of
// everything before it in its tensor, again in a word of the tile's own.  A tile therefore polls one
// address that nobody else polls, and the chain of the scan is one wave adding up numbers instead of
// every workgroup polling its predecessors.
//
// Workspace layout: a 256-byte header; count words, one per tile, packed (the scanning wave reads 64
// consecutive ones per load); then, from the next 128-byte boundary, prefix words, one per 64 bytes.
//   word = [63:62] flag | [61:40] epoch tag | [39:0] value
//   count word:  kFlagCount (kFlagFirst for the first tile of a tensor: the scan restarts there) | epoch | changed elements
//   prefix word: kFlagPrefix | epoch | changed elements before the tile in its tensor
// A word only counts if its epoch tag equals the header's epoch, so the words a previous call
// left behind read as "not yet written" and nothing has to be cleared between calls.  The
// workgroup that finishes last advances the epoch and resets the counters; when the 22-bit tag
// is about to wrap it clears every word the workspace can hold, so a stale word can never
// be taken for a fresh one.
//
// Roles and tiles are handed out through one atomic ticket: ticket 0 makes its workgroup lend a wave
// to the scan, ticket t > 0 is tile t - 1.  So the scanning wave belongs to a workgroup that is
// running, and a tile only ever waits for tiles that a running workgroup has already claimed:
// forward progress does not depend on the order in which the hardware dispatches workgroups.  Every
// wait is bounded: after `spin_limit` polls without an answer a waiting lane raises header.error
// and its workgroup leaves; the others (the scanning wave included) see the flag within 64 polls
// and leave too, so every wave reaches the end of the kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "wave.hpp"

namespace bitsnap {

constexpr uint32_t kFlagCount = 1;   // count word of a tile inside a tensor
constexpr uint32_t kFlagFirst = 2;   // count word of a tensor's first tile
constexpr uint32_t kFlagPrefix = 3;  // prefix word
constexpr int kEpochBits = 22;
constexpr uint32_t kEpochMask = (1u << kEpochBits) - 1;
constexpr int kValueBits = 40;
constexpr uint64_t kValueMask = (1ull << kValueBits) - 1;
constexpr size_t kScanHeaderBytes = 256;
constexpr uint32_t kDefaultSpinLimit = 1u << 22;

struct ScanHeader {
    uint32_t ticket;  // next ticket to hand out
    uint32_t done;    // workgroups that have finished
    uint32_t epoch;   // tag of the call in flight
    uint32_t error;   // non-zero once a wait has been given up
};

__device__ __forceinline__ uint64_t make_status(uint32_t flag, uint32_t epoch, uint64_t value)
{
    return ((uint64_t)((flag << kEpochBits) | epoch) << kValueBits) | (value & kValueMask);
}

// The flag of a word in the call tagged `epoch` (0: not written in this call).
__device__ __forceinline__ uint32_t status_flag(uint64_t word, uint32_t epoch)
{
    const uint32_t tag = (uint32_t)(word >> kValueBits);
    return ((tag & kEpochMask) == epoch) ? (tag >> kEpochBits) : 0u;
}

// Distance, in 64-bit words, between the prefix words of consecutive tiles (64 bytes: a tile's poll
// shares its 128-byte line with one neighbour at most), and the bytes of workspace per tile that
// hold both kinds of words for any number of tiles >= 2.
constexpr int kPrefixStride = 8;
constexpr size_t kScanBytesPerTile = 128;

// First prefix word, counted in words from the first count word.
__device__ __forceinline__ int64_t prefix_words_at(int64_t num_tiles) { return (num_tiles + 15) & ~(int64_t)15; }

__device__ __forceinline__ void publish_count(uint64_t *status, int64_t tile, bool first_of_tensor, uint32_t epoch, uint32_t count)
{
    __hip_atomic_store(&status[tile], make_status(first_of_tensor ? kFlagFirst : kFlagCount, epoch, count), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}

// Count words per lane and round of the scanning wave: 256 tiles per round trip to memory.  A round
// trip takes a few microseconds while the launch streams, and tiles finish every 25 ns or so.
constexpr int kServeLoads = 4;

// The scanning wave (all 64 lanes).  Returns true if it gave up: an error was raised elsewhere, or
// no count arrived within spin_limit rounds.
__device__ __forceinline__ bool serve_scan(ScanHeader *hdr, uint64_t *status, int64_t num_tiles, uint32_t epoch,
                                           uint32_t spin_limit)
{
    const int lane = lane_id();
    uint64_t *prefix = status + prefix_words_at(num_tiles);
    int64_t f = 0;       // tiles answered so far
    uint64_t carry = 0;  // changed elements of the current tensor before tile f
    uint32_t idle = 0;
    while (f < num_tiles) {
        uint64_t w[kServeLoads];
#pragma unroll
        for (int k = 0; k < kServeLoads; ++k) {
            const int64_t idx = f + k * kWave + lane;
            w[k] = idx < num_tiles ? __hip_atomic_load(&status[idx], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0ull;
        }
        bool progressed = false;
#pragma unroll
        for (int k = 0; k < kServeLoads; ++k) {
            const uint32_t flag = status_flag(w[k], epoch);
            const uint64_t ready = __ballot(flag == kFlagCount || flag == kFlagFirst);
            const int nready = ~ready == 0ull ? kWave : __ffsll((long long)~ready) - 1;  // tiles in order, no gap
            if (nready == 0)
                break;
            const bool active = lane < nready;
            const uint32_t v = active ? (uint32_t)(w[k] & kValueMask) : 0u;  // at most a tile's elements: 64 of them fit 32 bits
            const bool first = active && flag == kFlagFirst;
            const uint32_t incl = wave_inclusive_add(v), excl = incl - v;
            // the nearest first-tile-of-a-tensor at or before this lane, if the window holds one
            const uint64_t firsts = __ballot(first);
            const uint64_t upto = firsts & (lane == kWave - 1 ? ~0ull : ((2ull << lane) - 1ull));
            const int fp = upto ? 63 - __builtin_clzll(upto) : 0;
            const uint32_t excl_fp = (uint32_t)__shfl((int)excl, fp, kWave);
            const uint64_t before = upto ? (uint64_t)(excl - excl_fp) : carry + excl;
            if (active && !first)  // a tensor's first tile knows its answer
                __hip_atomic_store(&prefix[(f + lane) * kPrefixStride], make_status(kFlagPrefix, epoch, before), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            const uint64_t through = before + v;
            carry = ((uint64_t)read_lane((uint32_t)(through >> 32), nready - 1) << 32) | read_lane((uint32_t)through, nready - 1);
            f += nready;
            progressed = true;
            if (nready < kWave)
                break;
        }
        if (progressed) {
            idle = 0;
            continue;
        }
        ++idle;
        if (idle > spin_limit || ((idle & 63u) == 0 && __hip_atomic_load(&hdr->error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)))
            return true;
        __builtin_amdgcn_s_sleep(2);
    }
    return false;
}

// One lane waits for the prefix word of a tile.  On give-up raises header.error and returns false.
__device__ __forceinline__ bool await_prefix(ScanHeader *hdr, const uint64_t *status, int64_t num_tiles, int64_t tile, uint32_t epoch,
                                             uint32_t spin_limit, uint64_t &before)
{
    const uint64_t *word = status + prefix_words_at(num_tiles) + tile * kPrefixStride;
    uint32_t polls = 0;
    for (;;) {
        const uint64_t w = __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (status_flag(w, epoch) == kFlagPrefix) {
            before = w & kValueMask;
            return true;
        }
        ++polls;
        if (polls > spin_limit || ((polls & 63u) == 0 && __hip_atomic_load(&hdr->error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
            __hip_atomic_store(&hdr->error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return false;
        }
        __builtin_amdgcn_s_sleep(1);
    }
}

constexpr int kEpilogueLast = 1;   // this workgroup finished last
constexpr int kEpilogueError = 2;  // ... and some wait had been given up

// Last step of every workgroup of a scan kernel (called by all threads, uniformly).  The
// workgroup that arrives last resets the header for the next call.  Returns, to every thread of
// the workgroup, kEpilogueLast (| kEpilogueError) in the last workgroup and 0 elsewhere, so that
// the caller can write what only the last workgroup may write.
//   aborted        this workgroup gave up
//   status_cap     number of status words the workspace holds
__device__ __forceinline__ int scan_epilogue(ScanHeader *hdr, uint64_t *status, int64_t status_cap, uint32_t epoch,
                                             bool aborted)
{
    __shared__ int s_wrap, s_result;
    __syncthreads();
    if (threadIdx.x == 0) {
        int wrap = 0, result = 0;
        if (aborted)
            __hip_atomic_store(&hdr->error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __threadfence();
        const uint32_t prev = atomicAdd(&hdr->done, 1u);
        if (prev == gridDim.x - 1) {
            __threadfence();
            result = kEpilogueLast;
            if (__hip_atomic_load(&hdr->error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
                result |= kEpilogueError;
            hdr->done = 0;
            hdr->ticket = 0;
            hdr->error = 0;
            if (epoch == kEpochMask)
                wrap = 1;
            else
                hdr->epoch = epoch + 1;
        }
        s_wrap = wrap;
        s_result = result;
    }
    __syncthreads();
    if (s_wrap) {
        for (int64_t i = threadIdx.x; i < status_cap; i += blockDim.x)
            status[i] = 0;
        __syncthreads();
        if (threadIdx.x == 0)
            hdr->epoch = 0;
    }
    return s_result;
}

}  // namespace bitsnap
