// Integer requantization used by every kernel's epilogue.
//
// The rule is the integer branch of the paper's quantized ReLU listing (section "Emitted OpenCL
// Runtime Code"), applied after the bias:  y = (t * mult) / 2^sb  with C division (truncation
// toward zero), then an arithmetic right shift (floor) by `shift`, or a multiplication by
// 2^-shift when shift is negative; then + z_y and the clamp, whose lower bound is raised to z_y
// for ReLU.
#pragma once

#include "common.h"

namespace mpq {

__device__ __forceinline__ int requant64(long long t, const Epi &e) {
    long long p = t * e.mult;
    // truncating division by 2^sb: bias negatives by 2^sb - 1, then shift
    long long y = (p + ((p >> 63) & ((1ll << e.sb) - 1))) >> e.sb;
    if (e.shift >= 0) y >>= e.shift;
    else y *= (1ll << (-e.shift));
    y += e.zy;
    y = y < e.lo ? e.lo : y;
    y = y > e.hi ? e.hi : y;
    return (int)y;
}

}  // namespace mpq
