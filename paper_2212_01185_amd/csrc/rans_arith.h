// The row coder's exact division, x / f for a 63-bit state and a 17-bit frequency, done in fp64.
//
// Pure arithmetic on plain integers and doubles: the HIP kernels include this file, and so does a host
// program of the CPU test suite that checks the claim below against 64-bit integer division for every
// frequency (compiled with the host compiler; the two macros below are then empty or plain C).
//
// Claim.  For 1 <= f <= 2^16 and 0 <= x < f * 2^47, with rf_below = rans_recip_below(f) computed in any
// rounding mode and rans_push evaluated with fp64 rounding TOWARD ZERO:
//   x  converted to fp64 is at most x                        (relative error < 2^-52)
//   rf_below lies strictly below 1/f, by at most 2^-49 / f   (two Newton steps leave about 2^-52, the pull is 2^-50)
//   fma(xd, rf_below, 2^52) rounds down to an integer q' + 2^52 with q' = floor(x/f) or floor(x/f) - 1
//       (the quotient is below 2^47 and all errors together are below 2^47 * 2^-48 < 1)
// so the remainder x - q' f lies in [0, 2f), fits 32 bits, and one comparison corrects it.
#pragma once

#include <stdint.h>

#ifndef PCC_RANS_HD
#define PCC_RANS_HD __host__ __device__ __forceinline__
#define PCC_RANS_RCP_SEED(fd) __builtin_amdgcn_rcp(fd)
#endif

namespace pcc {

// A value just below 1/f in fp64 for 1 <= f < 2^17: an estimate (the hardware's reciprocal) plus two
// Newton steps, then pulled down by 2^-50.  Independent of the coder state.
PCC_RANS_HD double rans_recip_below(uint32_t f32) {
    const double fd = (double)f32;
    double rf = PCC_RANS_RCP_SEED(fd);
    rf = __builtin_fma(__builtin_fma(-fd, rf, 1.0), rf, rf);
    rf = __builtin_fma(__builtin_fma(-fd, rf, 1.0), rf, rf);
    return rf * (1.0 - 0x1p-50);
}

// x <- C(x, (start, f)) = ((x / f) << 16) + (x % f) + start for x = xh 2^32 + xl < 2^47 * f.
// Needs fp64 rounding toward zero.  Branch-free.
PCC_RANS_HD void rans_push(uint32_t& xl, uint32_t& xh, uint32_t f, uint32_t start, double rf_below) {
    const double xd = __builtin_fma((double)xh, 4294967296.0, (double)xl);
    const double qd = __builtin_fma(xd, rf_below, 4503599627370496.0);
    uint64_t qb;
    __builtin_memcpy(&qb, &qd, 8);
    const uint32_t rem = xl - (uint32_t)qb * f;
    const uint32_t z = rem + start + (rem >= f ? 65536u - f : 0u);   // a quotient one short: carry 2^16 - f
    const uint64_t x = (qb << 16) + z;                               // the exponent bits of qb leave at the top
    xl = (uint32_t)x;
    xh = (uint32_t)(x >> 32);
}

}  // namespace pcc
