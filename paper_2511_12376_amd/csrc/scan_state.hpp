// Cross-workgroup exclusive scan of per-tile counts: single pass, decoupled look-back.
//
// Workspace layout: a 256-byte header, then one 64-bit status word per tile, kStatusStride
// words apart.
//   word = [63:62] flag | [61:40] epoch tag | [39:0] value
// A word only counts if its epoch tag equals the header's epoch, so the words a previous call
// left behind read as "not yet written" and nothing has to be cleared between calls.  The
// workgroup that finishes last advances the epoch and resets the counters; when the 22-bit tag
// is about to wrap it clears every status word the workspace can hold, so a stale word can never
// be taken for a fresh one.
//
// Tiles are handed out through an atomic ticket, so a tile only ever waits for tiles that a
// running workgroup has already claimed: forward progress does not depend on the order in which
// the hardware dispatches workgroups.  Every wait is bounded: after `spin_limit` polls a
// workgroup marks its tile aborted, raises header.error, and leaves; the others see either the
// aborted word or the error flag and leave too, so every wave reaches the end of the kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "wave.hpp"

namespace bitsnap {

constexpr uint32_t kFlagAggregate = 1;  // value = the tile's own count
constexpr uint32_t kFlagInclusive = 2;  // value = count of this tile and all before it
constexpr uint32_t kFlagAbort = 3;      // the tile's workgroup gave up
constexpr int kEpochBits = 22;
constexpr uint32_t kEpochMask = (1u << kEpochBits) - 1;
constexpr int kValueBits = 40;
constexpr uint64_t kValueMask = (1ull << kValueBits) - 1;
constexpr size_t kScanHeaderBytes = 256;
constexpr uint32_t kDefaultSpinLimit = 1u << 22;

struct ScanHeader {
    uint32_t ticket;  // next tile to hand out
    uint32_t done;    // workgroups that have finished
    uint32_t epoch;   // tag of the call in flight
    uint32_t error;   // non-zero once a workgroup has given up
};

__device__ __forceinline__ uint64_t make_status(uint32_t flag, uint32_t epoch, uint64_t value)
{
    return ((uint64_t)((flag << kEpochBits) | epoch) << kValueBits) | (value & kValueMask);
}

// Distance, in 64-bit words, between the status words of consecutive tiles: one 128-byte line
// each.  At any moment every workgroup polls the words of the few dozen tiles around the front of
// the scan; packed eight to a 64-byte line those polls queued up on a handful of lines
// (measured: 58 % -> 63 % of HBM peak for the sparse encoder from the spacing alone).
constexpr int kStatusStride = 16;

__device__ __forceinline__ void publish(uint64_t *status, int64_t tile, uint64_t word)
{
    __hip_atomic_store(&status[tile * kStatusStride], word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Lanes of the wave that take part in a poll, one predecessor each (the others stay idle).  A
// polled word is an uncached memory request of its own, and those requests, not the number of
// round trips, are what the scan costs the machine: with 64 lanes the encoder reached 63 % of
// HBM peak, with 16 lanes 65 %, with 8 lanes 67-70 %, with 4 lanes 64 %, with 1 lane 46 %.
constexpr int kLookbackLanes = 8;

// Number of counted items in tiles [first_tile, tile): the scan restarts at first_tile (the first
// tile of the tensor this tile belongs to).  Called by one full wavefront.  On give-up sets
// `aborted` and returns 0.
//
// Lane l < kLookbackLanes inspects tile look - l.  Walking away from the tile, every word must
// carry at least the tile's own count (aggregate) until the first word that carries an
// inclusive prefix; the answer is the sum up to and including that word.
__device__ __forceinline__ uint64_t look_back(uint64_t *status, ScanHeader *hdr, int64_t tile, int64_t first_tile,
                                              uint32_t epoch, uint32_t spin_limit, bool &aborted)
{
    const int lane = lane_id();
    const bool polls_lane = lane < kLookbackLanes;
    uint64_t excl = 0;
    int64_t look = tile - 1;  // nearest predecessor not yet accounted for
    uint32_t polls = 0;
    aborted = false;
    for (;;) {
        const int64_t idx = look - lane;
        uint64_t lane_sum;
        bool stop, blocked, abort_word;
        for (;;) {
            // idle lanes: an aggregate of 0; tiles before the first one: an inclusive prefix of 0
            uint64_t w = make_status(kFlagAggregate, epoch, 0);
            if (polls_lane)
                w = (idx >= first_tile) ? __hip_atomic_load(&status[idx * kStatusStride], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                        : make_status(kFlagInclusive, epoch, 0);
            const uint32_t tag = (uint32_t)(w >> kValueBits);
            const uint32_t flag = ((tag & kEpochMask) == epoch) ? (tag >> kEpochBits) : 0u;
            blocked = flag == 0;
            stop = flag == kFlagInclusive || flag == kFlagAbort;
            abort_word = flag == kFlagAbort;
            lane_sum = blocked ? 0ull : (w & kValueMask);
            const uint64_t halt = __ballot(stop || blocked);
            if (halt == 0)
                break;  // the whole window holds aggregates: take them all and look further back
            const int first = __ffsll((long long)halt) - 1;
            if (!(__ballot(blocked) & (1ull << first)))
                break;  // the nearest halting lane found an inclusive word
            ++polls;
            if (polls > spin_limit ||
                ((polls & 63u) == 0 && __hip_atomic_load(&hdr->error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
                aborted = true;
                return 0;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        const uint64_t halt = __ballot(stop);
        if (halt) {
            const int first = __ffsll((long long)halt) - 1;
            if (__ballot(abort_word) & (1ull << first)) {
                aborted = true;
                return 0;
            }
            excl += wave_sum_u64(lane <= first ? lane_sum : 0ull);
            return excl;
        }
        excl += wave_sum_u64(lane_sum);
        look -= kLookbackLanes;
    }
}

constexpr int kEpilogueLast = 1;   // this workgroup finished last
constexpr int kEpilogueError = 2;  // ... and some workgroup had given up

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
