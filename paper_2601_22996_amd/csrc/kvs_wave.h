/*
 * kvs_wave.h -- wavefront-wide helpers of the gfx950 kernels (64 lanes): rank of
 * a lane inside a ballot, prefix sums, sums and maxima through DPP lane moves.
 */
#ifndef KVS_WAVE_H
#define KVS_WAVE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

/*
 * Wavefront-wide sums and maxima through the VALU's data-parallel lane moves
 * (DPP), which leave the LDS pipeline to the window atomics.  All 64 lanes
 * must be active.  Shifts by 1, 2, 4, 8 lanes inside each row of 16 build the
 * rows' prefixes; the last lane of row 0 / 2 is then broadcast into row
 * 1 / 3, and lane 31 into rows 2 and 3.
 */
template <int CTRL, int ROWS>
__device__ __forceinline__ int32_t dpp_take(int32_t fill, int32_t v)
{
    return __builtin_amdgcn_update_dpp(fill, v, CTRL, ROWS, 0xf, false);
}

/* inclusive prefix sum over the lanes */
__device__ __forceinline__ int32_t wave_prefix_add(int32_t v)
{
    v += dpp_take<0x111, 0xf>(0, v); /* row_shr:1 */
    v += dpp_take<0x112, 0xf>(0, v); /* row_shr:2 */
    v += dpp_take<0x114, 0xf>(0, v); /* row_shr:4 */
    v += dpp_take<0x118, 0xf>(0, v); /* row_shr:8 */
    v += dpp_take<0x142, 0xa>(0, v); /* row_bcast:15 into rows 1 and 3 */
    v += dpp_take<0x143, 0xc>(0, v); /* row_bcast:31 into rows 2 and 3 */
    return v;
}

/* sum over the lanes, the same value in every lane */
__device__ __forceinline__ int32_t wave_sum(int32_t v)
{
    return __builtin_amdgcn_readlane(wave_prefix_add(v), 63);
}

/* maximum over the lanes of values >= 0, the same value in every lane */
__device__ __forceinline__ int32_t wave_max_nonneg(int32_t v)
{
    int32_t u;
    u = dpp_take<0x111, 0xf>(0, v); v = u > v ? u : v;
    u = dpp_take<0x112, 0xf>(0, v); v = u > v ? u : v;
    u = dpp_take<0x114, 0xf>(0, v); v = u > v ? u : v;
    u = dpp_take<0x118, 0xf>(0, v); v = u > v ? u : v;
    u = dpp_take<0x142, 0xa>(0, v); v = u > v ? u : v;
    u = dpp_take<0x143, 0xc>(0, v); v = u > v ? u : v;
    return __builtin_amdgcn_readlane(v, 63);
}

/* bitwise or over the lanes, the same value in every lane */
__device__ __forceinline__ uint32_t wave_or(uint32_t x)
{
    int32_t v = (int32_t)x;
    v |= dpp_take<0x111, 0xf>(0, v);
    v |= dpp_take<0x112, 0xf>(0, v);
    v |= dpp_take<0x114, 0xf>(0, v);
    v |= dpp_take<0x118, 0xf>(0, v);
    v |= dpp_take<0x142, 0xa>(0, v);
    v |= dpp_take<0x143, 0xc>(0, v);
    return (uint32_t)__builtin_amdgcn_readlane(v, 63);
}

/* sum over the lanes of 63-bit values, in three limbs of 21 bits */
__device__ __forceinline__ unsigned long long wave_sum_u63(unsigned long long v)
{
    const uint32_t m = (1u << 21) - 1u;
    const unsigned long long a = (uint32_t)wave_sum((int32_t)((uint32_t)v & m));
    const unsigned long long b = (uint32_t)wave_sum((int32_t)((uint32_t)(v >> 21) & m));
    const unsigned long long c = (uint32_t)wave_sum((int32_t)((uint32_t)(v >> 42) & m));
    return a + (b << 21) + (c << 42);
}

} // namespace

#endif /* KVS_WAVE_H */
