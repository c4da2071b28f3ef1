// Wave64 cross-lane primitives for gfx950, built on DPP moves.  All of them must be called with
// every lane of the wavefront active.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bitsnap {

constexpr int kWave = 64;

// DPP control words (GFX9 encoding).
constexpr int kDppRowShr1 = 0x111;
constexpr int kDppRowShr2 = 0x112;
constexpr int kDppRowShr4 = 0x114;
constexpr int kDppRowShr8 = 0x118;
constexpr int kDppRowBcast15 = 0x142;  // lane 15 of each row -> every lane of the next row
constexpr int kDppRowBcast31 = 0x143;  // lane 31 -> every lane of rows 2 and 3

__device__ __forceinline__ int lane_id() { return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)); }

// Source lane's value, or 0 where the DPP pattern has no source lane / the row is masked out.
template <int kCtrl, int kRowMask>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, kCtrl, kRowMask, 0xF, false);
}

// Inclusive prefix sum over the 64 lanes (lane i receives v_0 + ... + v_i).
__device__ __forceinline__ uint32_t wave_inclusive_add(uint32_t v)
{
    v += dpp_or_zero<kDppRowShr1, 0xF>(v);
    v += dpp_or_zero<kDppRowShr2, 0xF>(v);
    v += dpp_or_zero<kDppRowShr4, 0xF>(v);
    v += dpp_or_zero<kDppRowShr8, 0xF>(v);
    v += dpp_or_zero<kDppRowBcast15, 0xA>(v);
    v += dpp_or_zero<kDppRowBcast31, 0xC>(v);
    return v;
}

__device__ __forceinline__ uint32_t read_lane(uint32_t v, int lane) { return (uint32_t)__builtin_amdgcn_readlane((int)v, lane); }

__device__ __forceinline__ double read_lane(double v, int lane)
{
    uint64_t u = (uint64_t)__double_as_longlong(v);
    uint32_t lo = read_lane((uint32_t)u, lane), hi = read_lane((uint32_t)(u >> 32), lane);
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}

__device__ __forceinline__ float read_lane(float v, int lane) { return __uint_as_float(read_lane(__float_as_uint(v), lane)); }

template <int kCtrl, int kRowMask>
__device__ __forceinline__ double dpp_or_zero(double v)
{
    uint64_t u = (uint64_t)__double_as_longlong(v);
    uint32_t lo = dpp_or_zero<kCtrl, kRowMask>((uint32_t)u), hi = dpp_or_zero<kCtrl, kRowMask>((uint32_t)(u >> 32));
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));   // +0.0 where there is no source
}

// Sum over the 64 lanes, returned in every lane.  The association order is fixed by the DPP
// tree, so the result is reproducible from run to run.
__device__ __forceinline__ double wave_sum(double v)
{
    v += dpp_or_zero<kDppRowShr1, 0xF>(v);
    v += dpp_or_zero<kDppRowShr2, 0xF>(v);
    v += dpp_or_zero<kDppRowShr4, 0xF>(v);
    v += dpp_or_zero<kDppRowShr8, 0xF>(v);
    v += dpp_or_zero<kDppRowBcast15, 0xA>(v);
    v += dpp_or_zero<kDppRowBcast31, 0xC>(v);
    return read_lane(v, 63);
}

__device__ __forceinline__ uint64_t wave_sum_u64(uint64_t v)
{
    // two independent 32-bit sums would lose the carry; go through shuffles, this runs once per tile
    for (int off = 32; off > 0; off >>= 1)
        v += (uint64_t)__shfl_xor((unsigned long long)v, off, kWave);
    return v;
}

}  // namespace bitsnap
