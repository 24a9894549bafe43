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
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
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

    float* po = a.part_o + ((int64_t)split * rows + r) * DH + lane * EPL;
#pragma unroll
    for (int e = 0; e < EPL; ++e) po[e] = acc[e];
    if (lane == 0) {
        float* pml = a.part_ml + ((int64_t)split * rows + r) * 2;
        pml[0] = m;
        pml[1] = l;
    }
}

// Merge of the per-split partials: m* = max_s m_s, l* = sum_s l_s e^{m_s - m*},
// O = sum_s O~_s e^{m_s - m*} / l*, lse = m* + ln l*.
// A group of DH/4 lanes owns one row, each lane four output elements.  The (m, l) records are read once per
// row -- lane t of the group takes splits t and t + DH/4 -- and the maximum, the weights e^{m_s - m*} and l* are
// formed inside the group with shuffles; the partial outputs are then fetched for the live splits only (m = -inf
// marks an empty split, whose row of the workspace was never written), eight loads in flight at a time.  Balanced
// batches: a sequence's splits are the runs its keys fell into, seq_splits[b] of them (a table the main kernel
// fills); 0 means one run held the whole sequence and the main kernel wrote its final rows itself.
//
// HALF: the partial outputs are the matrix-core kernels' (fp16, each row divided by its scale c, which is kept beside
// m and l): split s then enters with weight w_s c_s instead of w_s; the normaliser is the same.
template <typename T, int DH, bool HALF>
__global__ __launch_bounds__(256) void attn_combine_kernel(AttnArgs a) {
    constexpr int TPR = DH / 4;  // lanes per row: 32 or 16, a power of two that divides the wavefront
    constexpr int GS = 8;        // partial outputs in flight per lane
    const int64_t rows = (int64_t)a.B * a.N * a.Hq;
    const int64_t r_raw = (int64_t)blockIdx.x * (256 / TPR) + threadIdx.x / TPR;
    const bool in_range = r_raw < rows;   // lanes beyond the last row keep their group's shuffles company
    const int64_t r = in_range ? r_raw : rows - 1;
    const int t = threadIdx.x % TPR, c = 4 * t;
    constexpr int NH = 64 / TPR;          // records per lane: the host never plans more than 64 splits
    int nsp = a.nsplit;
    if (a.seq_splits) {  // balanced batches: the sequence's own number of runs; 0 = its rows are final already
        nsp = a.seq_splits[r / ((int64_t)a.N * a.Hq)];
        if (nsp == 0) return;  // (the whole group agrees: same row)
    }

    float m[NH], l[NH], cs[NH];
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        const int sp = t + h * TPR;
        m[h] = -INFINITY;
        l[h] = 0.f;
        cs[h] = 1.f;
        if (sp < nsp) {
            const float2 ml = *reinterpret_cast<const float2*>(a.part_ml + ((int64_t)sp * rows + r) * 2);
            if constexpr (HALF) cs[h] = a.part_c[(int64_t)sp * rows + r];  // (never written for an absent split: unused then)
            m[h] = ml.x;
            l[h] = ml.y;
        }
    }
    float mstar = m[0];
#pragma unroll
    for (int h = 1; h < NH; ++h) mstar = fmaxf(mstar, m[h]);
#pragma unroll
    for (int o = TPR / 2; o > 0; o >>= 1) mstar = fmaxf(mstar, __shfl_xor(mstar, o, TPR));
    // a row always has a visible key (itself), so some split is live and mstar is finite
    float w[NH], lstar = 0.f;
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        w[h] = m[h] == -INFINITY ? 0.f : expf(m[h] - mstar);
        lstar = fmaf(l[h], w[h], lstar);
        if constexpr (HALF) w[h] = w[h] == 0.f ? 0.f : w[h] * cs[h];  // from here on w weighs the stored partial output
    }
#pragma unroll
    for (int o = TPR / 2; o > 0; o >>= 1) lstar += __shfl_xor(lstar, o, TPR);

    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < nsp; s0 += GS) {
        float ws[GS];
        float4 v[GS];   // HALF: the first two words hold the four fp16 values until every load of the batch is out
#pragma unroll
        for (int u = 0; u < GS; ++u) {
            const int sp = s0 + u;   // its weight sits in lane sp % TPR of the group, slot sp / TPR
            float wsel = 0.f;
#pragma unroll
            for (int h = 0; h < NH; ++h) {
                const float wh = __shfl(w[h], sp % TPR, TPR);
                if (sp / TPR == h) wsel = wh;
            }
            ws[u] = sp >= nsp ? 0.f : wsel;
            v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (ws[u] != 0.f) {
                if constexpr (HALF) {
                    const float2 raw = *reinterpret_cast<const float2*>(reinterpret_cast<const _Float16*>(a.part_o) + ((int64_t)sp * rows + r) * DH + c);
                    v[u].x = raw.x;
                    v[u].y = raw.y;
                } else {
                    v[u] = *reinterpret_cast<const float4*>(a.part_o + ((int64_t)sp * rows + r) * DH + c);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < GS; ++u) {
            float4 x = v[u];
            if constexpr (HALF) {
                const f16x4 hv = __builtin_bit_cast(f16x4, make_float2(v[u].x, v[u].y));
                x = make_float4((float)hv[0], (float)hv[1], (float)hv[2], (float)hv[3]);
            }
            acc[0] = fmaf(x.x, ws[u], acc[0]); acc[1] = fmaf(x.y, ws[u], acc[1]);
            acc[2] = fmaf(x.z, ws[u], acc[2]); acc[3] = fmaf(x.w, ws[u], acc[3]);
        }
    }
    if (!in_range) return;
    const float inv = 1.f / lstar;
    if constexpr (sizeof(T) == 4) {
        *reinterpret_cast<float4*>(static_cast<float*>(a.out) + r * DH + c) =
            make_float4(acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv);
    } else {
        __hip_bfloat16 h[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) h[e] = __float2bfloat16(acc[e] * inv);  // round to nearest even
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
hipError_t launch_combine_t(const AttnArgs& a, hipStream_t st) {
    const int64_t rows = (int64_t)a.B * a.N * a.Hq;
    if (a.Dh == 128) {
        dim3 grid((unsigned)((rows + 7) / 8));
        if (a.part_half) hipLaunchKernelGGL((attn_combine_kernel<T, 128, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((attn_combine_kernel<T, 128, false>), grid, dim3(256), 0, st, a);
    } else {
        dim3 grid((unsigned)((rows + 15) / 16));
        if (a.part_half) hipLaunchKernelGGL((attn_combine_kernel<T, 64, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((attn_combine_kernel<T, 64, false>), grid, dim3(256), 0, st, a);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_vector(const AttnArgs& a, const AttnPlan& p, int dtype, hipStream_t st) {
    return dtype == YGG_F32 ? launch_vector_t<float>(a, p, st) : launch_vector_t<uint16_t>(a, p, st);
}

hipError_t launch_attn_combine(const AttnArgs& a, const AttnPlan& p, int dtype, hipStream_t st) {
    (void)p;
    return dtype == YGG_F32 ? launch_combine_t<float>(a, st) : launch_combine_t<uint16_t>(a, st);
}

}  // namespace ygg
