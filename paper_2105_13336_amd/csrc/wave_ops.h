// Wavefront-level building blocks (64 lanes) for 64-bit integers on gfx950: DPP moves,
// inclusive scans, lane reads.  Device code only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tensile {

// One DPP move of a 64-bit value (two 32-bit halves).  Lanes without a source (shifted in from
// outside a row) and lanes masked off by kRowMask receive `ident`.
//   0x111/0x112/0x114/0x118 = row_shr:1/2/4/8 (shift towards higher lanes inside rows of 16)
//   0x101/.../0x108         = row_shl:1..8
//   0x142 = row_bcast:15 (lane 15 of each row to the next row), 0x143 = row_bcast:31
template <int kCtrl, int kRowMask>
__device__ __forceinline__ int64_t dpp_move(int64_t x, int64_t ident) {
    const int lo = __builtin_amdgcn_update_dpp(static_cast<int>(ident), static_cast<int>(x), kCtrl, kRowMask, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(static_cast<int>(ident >> 32), static_cast<int>(x >> 32), kCtrl, kRowMask,
                                               0xf, false);
    return (static_cast<int64_t>(hi) << 32) | static_cast<uint32_t>(lo);
}

// Same with identity 0 (lets the hardware supply the zero).
template <int kCtrl, int kRowMask>
__device__ __forceinline__ int64_t dpp_or_zero(int64_t x) {
    const int lo = __builtin_amdgcn_update_dpp(0, static_cast<int>(x), kCtrl, kRowMask, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, static_cast<int>(x >> 32), kCtrl, kRowMask, 0xf, true);
    return (static_cast<int64_t>(hi) << 32) | static_cast<uint32_t>(lo);
}

// Inclusive add-scan over the 64 lanes: shifts by 1, 2, 4, 8 inside each row of 16 lanes, then
// lane 15 of rows 0 and 2 is added to rows 1 and 3, then lane 31 to rows 2 and 3.
__device__ __forceinline__ int64_t wave_scan_add(int64_t x) {
    x += dpp_or_zero<0x111, 0xf>(x);
    x += dpp_or_zero<0x112, 0xf>(x);
    x += dpp_or_zero<0x114, 0xf>(x);
    x += dpp_or_zero<0x118, 0xf>(x);
    x += dpp_or_zero<0x142, 0xa>(x);
    x += dpp_or_zero<0x143, 0xc>(x);
    return x;
}

__device__ __forceinline__ int64_t max64(int64_t a, int64_t b) { return a > b ? a : b; }

// Inclusive max-scan over the 64 lanes (same network, identity INT64_MIN).
__device__ __forceinline__ int64_t wave_scan_max(int64_t x) {
    x = max64(x, dpp_move<0x111, 0xf>(x, INT64_MIN));
    x = max64(x, dpp_move<0x112, 0xf>(x, INT64_MIN));
    x = max64(x, dpp_move<0x114, 0xf>(x, INT64_MIN));
    x = max64(x, dpp_move<0x118, 0xf>(x, INT64_MIN));
    x = max64(x, dpp_move<0x142, 0xa>(x, INT64_MIN));
    x = max64(x, dpp_move<0x143, 0xc>(x, INT64_MIN));
    return x;
}

// value of lane `src` (wave-uniform index), as a wave-uniform scalar
__device__ __forceinline__ int64_t lane_value(int64_t x, int src) {
    const uint32_t lo = __builtin_amdgcn_readlane(static_cast<int>(x), src);
    const uint32_t hi = __builtin_amdgcn_readlane(static_cast<int>(x >> 32), src);
    return (static_cast<int64_t>(hi) << 32) | lo;
}

__device__ __forceinline__ int64_t last_lane(int64_t x) { return lane_value(x, 63); }

}  // namespace tensile
