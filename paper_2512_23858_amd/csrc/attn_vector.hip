// Tree-masked verify attention, fp32 vector-ALU path (paper Sec. 2 "Source of Improvements",
// Sec. 4.2 last paragraph: one parallel pass, mask = the tree's causal dependency), and the
// split-KV combine shared with the matrix-core path.
//
// One wavefront owns one query row (sequence b, node i, query head h) and one split of the key
// range.  Lanes split the keys of a 64-key tile for q.k (one key per lane), the tile's softmax
// statistics are wave reductions, and lanes split head_dim for the value product.  This path is
// exact fp32 throughout and serves the fp32 configuration and any shape the matrix-core kernel
// does not take; it is not the bandwidth path.
#include "ygg_internal.h"

#include <hip/hip_bf16.h>
#include <hip/hip_ext.h>

namespace ygg {
namespace {

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ void load4(const float* p, float (&o)[4]) {
        const float4 v = *reinterpret_cast<const float4*>(p);
        o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    }
    static __device__ __forceinline__ float load1(const float* p) { return *p; }
};
template <> struct Elem<uint16_t> {
    static __device__ __forceinline__ void load4(const uint16_t* p, float (&o)[4]) {
        const uint2 v = *reinterpret_cast<const uint2*>(p);
        o[0] = bf16_bits_to_f32(v.x & 0xffffu); o[1] = bf16_bits_to_f32(v.x >> 16);
        o[2] = bf16_bits_to_f32(v.y & 0xffffu); o[3] = bf16_bits_to_f32(v.y >> 16);
    }
    static __device__ __forceinline__ float load1(const uint16_t* p) { return bf16_bits_to_f32(*p); }
};

template <typename T, int DH>
__global__ __launch_bounds__(256) void attn_vector_kernel(AttnArgs a) {
    constexpr int EPL = DH / 64;  // head_dim elements per lane in the value product
    __shared__ float q_s[4][DH];
    __shared__ uint32_t anc_s[4][kMaxNodes / 32];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t rows = (int64_t)a.B * a.N * a.Hq;
    const int64_t r = (int64_t)blockIdx.x * 4 + wave;
    if (r >= rows) return;  // no barrier below: waves are independent
    const int split = blockIdx.y;
    const int h = (int)(r % a.Hq), i = (int)((r / a.Hq) % a.N), b = (int)(r / ((int64_t)a.Hq * a.N));
    const int hk = h / a.G;
    int L = a.seq_lens[b];
    L = L < 0 ? 0 : (L > a.max_seq_len ? a.max_seq_len : L);
    const int Tk = L + a.N;  // keys of this sequence
    int chunk = (Tk + a.nsplit - 1) / a.nsplit;
    chunk = (chunk + kKeyTile - 1) / kKeyTile * kKeyTile;
    const int k0 = split * chunk;
    const int k1 = min(Tk, k0 + chunk);

    const T* qp = static_cast<const T*>(a.q) + r * DH;
    for (int d = lane; d < DH; d += 64) q_s[wave][d] = Elem<T>::load1(qp + d);
    const int32_t* parent = a.parent_idx + (int64_t)b * a.N;
    if (k1 > L) {  // this split touches tree keys: bitmask of {i, parent[i], ..., root}
        for (int w = lane; w < (a.N + 31) / 32; w += 64) anc_s[wave][w] = 0;
        __builtin_amdgcn_wave_barrier();
        int guard = 0;
        for (int t = i; t >= 0 && t < a.N && guard < a.N; t = parent[t], ++guard)
            if (lane == 0) anc_s[wave][t >> 5] |= 1u << (t & 31);
    }
    __builtin_amdgcn_wave_barrier();

    const T* kc = static_cast<const T*>(a.k_cache) + ((int64_t)b * a.cap * a.Hkv + hk) * DH;
    const T* vc = static_cast<const T*>(a.v_cache) + ((int64_t)b * a.cap * a.Hkv + hk) * DH;
    const T* kt = static_cast<const T*>(a.k_tree) + ((int64_t)b * a.N * a.Hkv + hk) * DH;
    const T* vt = static_cast<const T*>(a.v_tree) + ((int64_t)b * a.N * a.Hkv + hk) * DH;
    const int64_t tok_stride = (int64_t)a.Hkv * DH;

    float m = -INFINITY, l = 0.f, acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;

    for (int t0 = k0; t0 < k1; t0 += 64) {
        const int j = t0 + lane;
        bool ok = j < k1;
        if (ok && j >= L) ok = (anc_s[wave][(j - L) >> 5] >> ((j - L) & 31)) & 1u;
        float s = -INFINITY;
        if (ok) {
            const T* kp = j < L ? kc + (int64_t)j * tok_stride : kt + (int64_t)(j - L) * tok_stride;
            float dot = 0.f;
#pragma unroll 8
            for (int d = 0; d < DH; d += 4) {
                float kv[4];
                Elem<T>::load4(kp + d, kv);
                const float4 qv = *reinterpret_cast<const float4*>(&q_s[wave][d]);
                dot = fmaf(qv.x, kv[0], dot);
                dot = fmaf(qv.y, kv[1], dot);
                dot = fmaf(qv.z, kv[2], dot);
                dot = fmaf(qv.w, kv[3], dot);
            }
            s = dot * a.scale;
        }
        const float tmax = wave_max(s);
        if (tmax == -INFINITY) continue;  // nothing visible in this tile (wave-uniform)
        const float m_new = fmaxf(m, tmax);
        const float alpha = expf(m - m_new);  // m = -inf on the first live tile -> 0
        const float p = ok ? expf(s - m_new) : 0.f;
        l = l * alpha + wave_sum(p);
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] *= alpha;
        m = m_new;

        if (t0 + 64 <= min(k1, L)) {  // whole tile inside the prefix: fixed trip count
#pragma unroll 16
            for (int jj = 0; jj < 64; ++jj) {
                const float pj = __shfl(p, jj);
                const T* vp = vc + (int64_t)(t0 + jj) * tok_stride + lane * EPL;
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[e] = fmaf(pj, Elem<T>::load1(vp + e), acc[e]);
            }
        } else {
            uint64_t live = __ballot(ok);
            while (live) {
                const int jj = __ffsll((unsigned long long)live) - 1;
                live &= live - 1;
                const float pj = __shfl(p, jj);
                const int key = t0 + jj;
                const T* vp = (key < L ? vc + (int64_t)key * tok_stride : vt + (int64_t)(key - L) * tok_stride) + lane * EPL;
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[e] = fmaf(pj, Elem<T>::load1(vp + e), acc[e]);
            }
        }
    }

    float* po = static_cast<float*>(a.part_o) + ((int64_t)split * rows + r) * DH + lane * EPL;
#pragma unroll
    for (int e = 0; e < EPL; ++e) po[e] = acc[e];
    if (lane == 0) {
        float* pml = a.part_ml + ((int64_t)split * rows + r) * 2;
        pml[0] = m;
        pml[1] = l;
    }
}

// Merge of the per-split partials: m* = max_s m_s, l* = sum_s l_s e^{m_s - m*},
// O = sum_s O~_s e^{m_s - m*} / l*, lse = m* + ln l*.  One thread per 4 output elements.
// Splits are taken eight at a time with all of a group's loads issued before any is used, so a
// row costs one memory round trip per group instead of one per split; groups are chained with the
// usual running-maximum rescale.
// PBF16: the partial outputs are bf16 (matrix-core kernels) instead of fp32 (vector kernel).
template <typename T, int DH, bool PBF16>
__global__ __launch_bounds__(256) void attn_combine_kernel(AttnArgs a) {
    constexpr int TPR = DH / 4;  // threads per row
    constexpr int GS = 8;        // splits per group
    const int64_t rows = (int64_t)a.B * a.N * a.Hq;
    const int64_t r = (int64_t)blockIdx.x * (256 / TPR) + threadIdx.x / TPR;
    if (r >= rows) return;
    const int c = (threadIdx.x % TPR) * 4;
    const int nsp = a.nsplit;
    float mstar = -INFINITY, lstar = 0.f;
    float o[4] = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < nsp; s0 += GS) {
        float2 ml[GS];
        float4 v[GS];
#pragma unroll
        for (int u = 0; u < GS; ++u) {
            const int s = min(s0 + u, nsp - 1);  // the tail repeats the last split; its weight is dropped below
            ml[u] = *reinterpret_cast<const float2*>(a.part_ml + ((int64_t)s * rows + r) * 2);
            if constexpr (PBF16) {
                const uint2 h = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(a.part_o) + ((int64_t)s * rows + r) * DH + c);
                v[u] = make_float4(__uint_as_float(h.x << 16), __uint_as_float(h.x & 0xffff0000u),
                                   __uint_as_float(h.y << 16), __uint_as_float(h.y & 0xffff0000u));
            } else {
                v[u] = *reinterpret_cast<const float4*>(static_cast<const float*>(a.part_o) + ((int64_t)s * rows + r) * DH + c);
            }
        }
        float mg = mstar;
#pragma unroll
        for (int u = 0; u < GS; ++u) mg = fmaxf(mg, ml[u].x);
        if (mg == -INFINITY) continue;  // no split so far saw a visible key for this row
        const float carry = expf(mstar - mg);  // 0 when nothing was accumulated yet
        lstar *= carry;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] *= carry;
        mstar = mg;
#pragma unroll
        for (int u = 0; u < GS; ++u) {
            // an empty split wrote only its (m = -inf, l = 0) record: its O~ is whatever the workspace held
            const bool live = s0 + u < nsp && ml[u].x != -INFINITY;
            const float w = live ? expf(ml[u].x - mstar) : 0.f;
            const float4 vv = live ? v[u] : make_float4(0.f, 0.f, 0.f, 0.f);
            lstar = fmaf(live ? ml[u].y : 0.f, w, lstar);
            o[0] = fmaf(vv.x, w, o[0]); o[1] = fmaf(vv.y, w, o[1]);
            o[2] = fmaf(vv.z, w, o[2]); o[3] = fmaf(vv.w, w, o[3]);
        }
    }
    const float inv = 1.f / lstar;
    if constexpr (sizeof(T) == 4) {
        *reinterpret_cast<float4*>(static_cast<float*>(a.out) + r * DH + c) =
            make_float4(o[0] * inv, o[1] * inv, o[2] * inv, o[3] * inv);
    } else {
        __hip_bfloat16 h[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) h[e] = __float2bfloat16(o[e] * inv);  // round to nearest even
        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(a.out) + r * DH + c) = *reinterpret_cast<uint2*>(h);
    }
    if (a.lse && c == 0) a.lse[r] = mstar + logf(lstar);
}

template <typename T>
hipError_t launch_vector_t(const AttnArgs& a, const AttnPlan& p, hipStream_t st) {
    const int64_t rows = (int64_t)a.B * a.N * a.Hq;
    dim3 grid((unsigned)((rows + 3) / 4), (unsigned)p.nsplit);
    if (a.Dh == 128) hipLaunchKernelGGL((attn_vector_kernel<T, 128>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((attn_vector_kernel<T, 64>), grid, dim3(256), 0, st, a);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_combine_t(const AttnArgs& a, bool partials_bf16, hipStream_t st) {
    const int64_t rows = (int64_t)a.B * a.N * a.Hq;
    if (a.Dh == 128) {
        dim3 grid((unsigned)((rows + 7) / 8));
        if (partials_bf16) hipLaunchKernelGGL((attn_combine_kernel<T, 128, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((attn_combine_kernel<T, 128, false>), grid, dim3(256), 0, st, a);
    } else {
        dim3 grid((unsigned)((rows + 15) / 16));
        hipLaunchKernelGGL((attn_combine_kernel<T, 64, false>), grid, dim3(256), 0, st, a);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_vector(const AttnArgs& a, const AttnPlan& p, int dtype, hipStream_t st) {
    return dtype == YGG_F32 ? launch_vector_t<float>(a, p, st) : launch_vector_t<uint16_t>(a, p, st);
}

hipError_t launch_attn_combine(const AttnArgs& a, const AttnPlan& p, int dtype, hipStream_t st) {
    return dtype == YGG_F32 ? launch_combine_t<float>(a, p.use_mfma != 0, st) : launch_combine_t<uint16_t>(a, p.use_mfma != 0, st);
}

}  // namespace ygg
