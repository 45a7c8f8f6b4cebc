// Device helpers shared by the kernels of libsentencekv (gfx950, wave64): DPP adds and scans, the block scan
// of the 1024-thread kernels, the order-preserving image of a score.
#pragma once

#include "skv_internal.h"

namespace skv {

constexpr int kBlockWaves = kBlockThreads / kWave;

// x + (x moved by a DPP pattern): quad_perm [1,0,3,2] = 0xB1, [2,3,0,1] = 0x4E, row_ror:n = 0x120 + n
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
    const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false);
    return x + __int_as_float(moved);
}

// Order-preserving 32-bit image of a float: larger score <=> larger key.
__device__ __forceinline__ uint32_t score_key(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;          // NaN ranks below everything
    if (u == 0x80000000u) u = 0u;                             // -0 == +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// v + (v moved by a DPP pattern; lanes without a source, or rows masked out, add 0)
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_add_u32(uint32_t v) {
    return v + (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, true);
}
// inclusive prefix sum over the 64 lanes of a wave: row_shr 1,2,4,8 then row_bcast 15 and 31
__device__ __forceinline__ uint32_t wave_scan_u32(uint32_t v) {
    v = dpp_add_u32<0x111, 0xf>(v);
    v = dpp_add_u32<0x112, 0xf>(v);
    v = dpp_add_u32<0x114, 0xf>(v);
    v = dpp_add_u32<0x118, 0xf>(v);
    v = dpp_add_u32<0x142, 0xa>(v);
    v = dpp_add_u32<0x143, 0xc>(v);
    return v;
}
// v and (v moved by a DPP pattern), the larger of the two; lanes without a source, or rows masked out, keep v
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_max_u32(uint32_t v) {
    return max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, true));
}
// inclusive running maximum over the 64 lanes of a wave (same DPP steps as the prefix sum)
__device__ __forceinline__ uint32_t wave_scan_max_u32(uint32_t v) {
    v = dpp_max_u32<0x111, 0xf>(v);
    v = dpp_max_u32<0x112, 0xf>(v);
    v = dpp_max_u32<0x114, 0xf>(v);
    v = dpp_max_u32<0x118, 0xf>(v);
    v = dpp_max_u32<0x142, 0xa>(v);
    v = dpp_max_u32<0x143, 0xc>(v);
    return v;
}
// Inclusive scan over the block's threads (thread order); one barrier.  A `slot` is used once per call
// of the selection.
__device__ __forceinline__ uint32_t block_scan_u32(uint32_t val, uint32_t* slot, uint32_t* total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const uint32_t x = wave_scan_u32(val);
    if (lane == 63) slot[w] = x;
    __syncthreads();
    // prefix over the 16 wave totals: one more wave scan instead of 16 reads per thread
    const uint32_t t = slot[lane & (kBlockWaves - 1)];
    const uint32_t ti = wave_scan_u32(lane < kBlockWaves ? t : 0u);
    *total = (uint32_t)__builtin_amdgcn_readlane((int)ti, kBlockWaves - 1);
    const uint32_t pre = (uint32_t)__builtin_amdgcn_readlane((int)(ti - t), w);     // lane w < 16 holds slot[w]
    return x + pre;
}

}  // namespace skv
