// Pieces shared by the matrix-core attention kernels: vector types, the direct-to-LDS tile loads, the LDS
// transpose read and bf16 packing.
#pragma once
#include "ygg_internal.h"
#include "ygg_device.h"

namespace ygg {
namespace attn {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) short i16x2;
typedef __attribute__((ext_vector_type(4))) short i16x4;
typedef __attribute__((ext_vector_type(8))) short i16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// One K or V row of head_dim DH in bf16 is ROWB = 2*DH bytes = ROWB/16 slots of 16 bytes (head_dim 128: 16 slots, 64: 8).
// LDS tiles are filled by direct-to-LDS loads (64 lanes x 16 bytes land contiguously), so rows are
// unpadded and bank conflicts are avoided by permuting the 16-byte slots inside each row instead:
//   K tile: slot' = slot ^ (row & (ROWB/16 - 1))       as many consecutive rows as a row has slots read the same
//                                                      column conflict-free
//   V tile: slot' = slot ^ ((row & (DH/32 - 1)) << 2)  a transpose read of 32 lanes touches 4 rows x 64 bytes: the
//                                                      64-byte chunks of neighbouring rows land on different banks
// The permutation is applied on the global side (which 16 bytes a lane fetches), never in LDS.
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kRescaleGap = 8.f;  // log2 units by which a row maximum may outgrow its softmax reference when one is taken
constexpr float kWeightSumLimit = 1073741824.f;  // 2^30: a lane's 16 weights of one block may sum to this before the reference moves

__device__ __forceinline__ i16x4 lds_read_tr16(const unsigned char* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)(p));
}

// Direct-to-LDS load of 16 bytes per lane: lane l's data lands at LDS byte address lds_base + 16*l
// (lds_base is wave-uniform and goes through M0).  Written as inline assembly so that the compiler
// does not treat every later LDS read as dependent on it (it would wait for the whole prefetch
// before each operand read); completion is awaited explicitly with dma_wait_keep() before the barrier
// that publishes the tile.  The compiler keeps nothing live in M0 on this target.
// NT adds the streaming hint: used when the stream is read by one workgroup only (one row tile), so that
// nothing would ever hit the lines in L2 again.
template <bool NT>
__device__ __forceinline__ void dma_load16(const void* base /* wave-uniform */, uint32_t byte_off, uint32_t lds_base) {
    if constexpr (NT)
        asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(lds_base), "v"(byte_off), "s"(base) : "memory");
    else
        asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(byte_off), "s"(base) : "memory");
}
// Same with a per-lane 64-bit address.
template <bool NT>
__device__ __forceinline__ void dma_load16_flat(const void* gptr, uint32_t lds_base) {
    if constexpr (NT)
        asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off nt" ::"s"(lds_base), "v"(gptr) : "memory");
    else
        asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr) : "memory");
}
// Waits until at most KEEP of this wavefront's vector-memory operations are still outstanding (they
// complete in issue order, so the KEEP youngest may still be in flight).
template <int KEEP>
__device__ __forceinline__ void dma_wait_keep() {
    static_assert(KEEP >= 0 && KEEP <= 63, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(KEEP) : "memory");
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    // round-to-nearest-even on both halves
    uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
    a += 0x7fffu + ((a >> 16) & 1u);
    b += 0x7fffu + ((b >> 16) & 1u);
    return (a >> 16) | (b & 0xffff0000u);
}

// Local-memory barrier: orders this wavefront's LDS traffic with the other wavefronts' without
// waiting for its global loads in flight (a full workgroup fence would drain them).
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <int V>
struct IntC {
    static constexpr int value = V;
};
// f(IntC<I>{}) for I = FROM .. TO-1, unrolled at compile time
template <int FROM, int TO, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (FROM < TO) {
        f(IntC<FROM>{});
        static_for<FROM + 1, TO>(f);
    }
}

}  // namespace attn
}  // namespace ygg
