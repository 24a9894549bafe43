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

// ---- hand-off of small results between workgroups of one launch ------------------------------------
// "The last workgroup to arrive finishes the job": producers write their partial results, then bump a
// counter; whoever sees the final count reads every partial.  Ordinary stores may stay in the writing
// XCD's L2 and ordinary loads may hit stale lines in the reader's, and a release/acquire fence pair at
// device scope would write back and invalidate whole L2s.  Instead the partials themselves travel by
// device-scope relaxed atomic stores and loads (write-through / always-coherent accesses of 8 bytes),
// the producer waits for its stores to be acknowledged before the counter is touched, and the reader's
// loads are issued only after the counter's value has come back.  Nothing waits or spins.
__device__ __forceinline__ void store_coherent(uint64_t* p, uint64_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t load_coherent(const uint64_t* p) {
    return __hip_atomic_load(const_cast<uint64_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ void store_coherent(T* p, const T& v) {
    static_assert(sizeof(T) % 8 == 0 && alignof(T) >= 8, "moved in 8-byte pieces");
    uint64_t w[sizeof(T) / 8];
    __builtin_memcpy(w, &v, sizeof(T));
#pragma unroll
    for (size_t i = 0; i < sizeof(T) / 8; ++i) store_coherent(reinterpret_cast<uint64_t*>(p) + i, w[i]);
}
template <typename T>
__device__ __forceinline__ T load_coherent(const T* p) {
    static_assert(sizeof(T) % 8 == 0 && alignof(T) >= 8, "moved in 8-byte pieces");
    uint64_t w[sizeof(T) / 8];
#pragma unroll
    for (size_t i = 0; i < sizeof(T) / 8; ++i) w[i] = load_coherent(reinterpret_cast<const uint64_t*>(p) + i);
    T v;
    __builtin_memcpy(&v, w, sizeof(T));
    return v;
}
// Called by every thread of the workgroup after its store_coherent calls.  Returns true in the workgroup
// that arrives last of `total` (the counter must be 0 before the first arrival and is 0 again afterwards).
// `flag` is one word of LDS.
__device__ __forceinline__ bool arrive_and_check_last(uint32_t* counter, uint32_t total, uint32_t* flag) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this thread's stores have been acknowledged
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t old = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool last = old + 1 == total;
        if (last) __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *flag = last;
    }
    __syncthreads();
    return *flag != 0;
}

// exp(t) for t <= 0 in fp64: k = round(t/ln 2), r = t - k ln 2 (two-part constant), Taylor series of
// degree 13 on |r| <= ln(2)/2 (remainder < 1e-17), scaled by 2^k.  Relative error about 1e-16.
__device__ __forceinline__ double exp_nonpos(double t) {
    if (t < -745.0) return 0.0;
    const double k = rint(t * 1.4426950408889634074);
    double r = fma(k, -6.93147180369123816490e-01, t);
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
    return ldexp(p, (int)k);
}

}  // namespace ygg
