// Prefix sums over the 64 lanes of a wave without the LDS crossbar that __shfl_up goes through.
#ifndef GBT_WAVE_SCAN_H
#define GBT_WAVE_SCAN_H
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

// Inclusive prefix sum over the 64 lanes of a wave with data-parallel-primitive moves (no LDS crossbar): shifts by
// 1, 2, 4, 8 inside each row of 16 lanes (a lane without a source adds 0), then lane 15 of rows 0 and 2 into rows 1
// and 3, then lane 31 into rows 2 and 3.  A 64-bit value moves as its two halves.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int64_t dpp_i64(int64_t v) {
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(v & 0xffffffff), CTRL, ROW_MASK, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(v >> 32), CTRL, ROW_MASK, 0xf, false);
    return (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}
__device__ __forceinline__ int64_t wave_scan_i64(int64_t x) {
    x += dpp_i64<0x111, 0xf>(x);   // row_shr:1
    x += dpp_i64<0x112, 0xf>(x);   // row_shr:2
    x += dpp_i64<0x114, 0xf>(x);   // row_shr:4
    x += dpp_i64<0x118, 0xf>(x);   // row_shr:8
    x += dpp_i64<0x142, 0xa>(x);   // row_bcast:15 into rows 1 and 3
    x += dpp_i64<0x143, 0xc>(x);   // row_bcast:31 into rows 2 and 3
    return x;
}
__device__ __forceinline__ int64_t last_lane_i64(int64_t v) {
    const int lo = __builtin_amdgcn_readlane((int)(v & 0xffffffff), 63);
    const int hi = __builtin_amdgcn_readlane((int)(v >> 32), 63);
    return (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}

}  // namespace
#endif
