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

// The same rule for an int32 accumulator with sb = 31 (8-bit storage), in 32-bit arithmetic:
// t * mult is formed as a (high, low) pair; floor(p / 2^31) = (high << 1) | (low >> 31), and the
// truncation adds one back when p is negative with a non-zero remainder.  |y| <= |t| fits int32.
__device__ __forceinline__ int requant32(int t, const Epi &e) {
    if (e.shift < 0 || e.sb != 31) return requant64((long long)t, e);
    const int mult = (int)e.mult;
    const int hi = __mulhi(t, mult);
    const unsigned lo = (unsigned)t * (unsigned)mult;
    int y = (int)(((unsigned)hi << 1) | (lo >> 31));
    y += (hi < 0 && (lo & 0x7fffffffu) != 0u) ? 1 : 0;
    const int sh = e.shift > 31 ? 31 : e.shift;
    y >>= sh;
    // clamp before adding the zero-point: the bounds are small, y may be anywhere in int32
    const int lo_b = e.lo - e.zy, hi_b = e.hi - e.zy;
    y = y < lo_b ? lo_b : y;
    y = y > hi_b ? hi_b : y;
    return y + e.zy;
}

}  // namespace mpq
