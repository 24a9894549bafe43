// Device-side helpers shared by the kernel translation units: wave-wide reductions, order-preserving
// integer keys of floating-point values, and an fp64 exponential.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ygg {

// ---- wave-wide reductions on DPP (row shifts and row broadcasts of the 64-wide wavefront) --------
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_or_self(uint32_t v) {
    // lanes without a valid source (or outside ROW_MASK) keep their own value
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, ROW_MASK, 0xf, false);
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
    v = max(v, dpp_or_self<0xb1, 0xf>(v));   // quad_perm [1,0,3,2]
    v = max(v, dpp_or_self<0x4e, 0xf>(v));   // quad_perm [2,3,0,1]
    v = max(v, dpp_or_self<0x114, 0xf>(v));  // row_shr:4
    v = max(v, dpp_or_self<0x118, 0xf>(v));  // row_shr:8   -> lane 15 of every row holds the row maximum
    v = max(v, dpp_or_self<0x142, 0xa>(v));  // row_bcast:15 into rows 1 and 3
    v = max(v, dpp_or_self<0x143, 0xc>(v));  // row_bcast:31 into rows 2 and 3 -> lane 63 holds the maximum
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) { return ~wave_max_u32(~v); }

// order-preserving maps to unsigned integers (larger value <-> larger key; -inf is the smallest real key)
__device__ __forceinline__ uint32_t key_of(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float float_of(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}
__device__ __forceinline__ uint64_t key_of(double d) {
    const uint64_t u = (uint64_t)__double_as_longlong(d);
    return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}
__device__ __forceinline__ double double_of(uint64_t k) {
    return __longlong_as_double((long long)((k >> 63) ? (k & 0x7fffffffffffffffull) : ~k));
}

// exp(t) for t <= 0 in fp64: k = round(t/ln 2), r = t - k ln 2 (two-part constant), Taylor series of
// degree 13 on |r| <= ln(2)/2 (remainder < 1e-17), scaled by 2^k.  Relative error about 1e-16.
// Branch-free (0 below the underflow point comes from a select), so independent calls interleave.
__device__ __forceinline__ double exp_nonpos(double t) {
    const double tc = fmax(t, -746.0);
    const double k = rint(tc * 1.4426950408889634074);
    double r = fma(k, -6.93147180369123816490e-01, tc);
    r = fma(k, -1.90821492927058770002e-10, r);
    double p = 1.0 / 6227020800.0;
    p = fma(p, r, 1.0 / 479001600.0);
    p = fma(p, r, 1.0 / 39916800.0);
    p = fma(p, r, 1.0 / 3628800.0);
    p = fma(p, r, 1.0 / 362880.0);
    p = fma(p, r, 1.0 / 40320.0);
    p = fma(p, r, 1.0 / 5040.0);
    p = fma(p, r, 1.0 / 720.0);
    p = fma(p, r, 1.0 / 120.0);
    p = fma(p, r, 1.0 / 24.0);
    p = fma(p, r, 1.0 / 6.0);
    p = fma(p, r, 0.5);
    p = fma(p, r, 1.0);
    p = fma(p, r, 1.0);
    const double e = ldexp(p, (int)k);
    return t < -745.0 ? 0.0 : e;
}

}  // namespace ygg
