// Order-preserving 32-bit keys of fp32 conformity scores (device code; shared by calib.hip and sort.hip).
//
// A key is an unsigned image of the score such that unsigned comparison of keys reproduces the IEEE comparison
// of scores (-0 folded onto +0, +-inf ordinary); every NaN maps to key 0, below the key of -inf, so a NaN
// calibration score is never ">=" anything.  Integer only: sub-normal scores keep their order whatever the
// float mode is.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace atts {

constexpr uint32_t kPadKey = 0xFFFFFFFFu;   // above the key of +inf (0xFF800000): never the key of a score

__device__ __forceinline__ bool score_is_nan(float f) { return (__float_as_uint(f) & 0x7FFFFFFFu) > 0x7F800000u; }
__device__ __forceinline__ uint32_t score_to_key(float f) {
    uint32_t b = __float_as_uint(f);
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) return 0u;   // NaN
    if ((b & 0x7FFFFFFFu) == 0u) b = 0u;              // -0 -> +0
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key_to_score(uint32_t k) {
    if (k == 0u) return __uint_as_float(0x7FC00000u);
    return __uint_as_float((k & 0x80000000u) ? (k ^ 0x80000000u) : ~k);
}

// Number of elements taken from a[] among the first `diag` outputs of the stable merge of two ascending arrays
// (a first on ties).
template <typename Index>
__device__ __forceinline__ Index merge_path(const uint32_t* a, Index na, const uint32_t* b, Index nb, Index diag) {
    Index lo = diag > nb ? diag - nb : 0, hi = diag < na ? diag : na;
    while (lo < hi) {
        Index mid = (lo + hi) >> 1;
        if (a[mid] <= b[diag - 1 - mid]) lo = mid + 1; else hi = mid;
    }
    return lo;
}

}  // namespace atts
