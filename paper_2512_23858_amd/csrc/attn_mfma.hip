// Tree-masked verify attention on the gfx950 matrix cores (bf16 storage, head_dim 128).
//
// Operation (paper Sec. 2 "Source of Improvements", Sec. 4.2 last paragraph): every tree node
// attends to the confirmed prefix, to its ancestors and to itself, all nodes in one pass.
//
// Decomposition.  For one sequence b and kv head g the N tree nodes and the Hq/Hkv query heads
// of the group form R = N*(Hq/Hkv) query rows that all read the same K/V stream.  A workgroup
// owns (b, g, one tile of query rows, one split of the key range); its NW wavefronts own RB
// blocks of 32 rows each and share every K/V tile through LDS, so a K/V byte is fetched from
// L2/HBM once per 32*RB*NW rows.  Workgroup ids are laid out so that all row tiles of one
// (b, g, split) land on the same XCD and hit in its L2.
//
// Per 32-key block and 32-row block (all MFMA are v_mfma_f32_32x32x16_bf16):
//   S^T = K . Q^T      A = K rows from LDS (16-byte reads), B = Q held in registers
//   online softmax     a lane owns one query row: 16 scores in registers, one cross-half
//                      exchange for the row maximum; base-2 exponentials
//   O^T += V^T . P^T   A = V^T through the LDS transpose read (ds_read_b64_tr_b16), B = P^T,
//                      which is exactly the accumulator layout of S^T packed to bf16
// The tree's own keys are the tail of the key range; their ancestor mask comes from per-node
// bitmasks built in LDS from parent_idx.
#include "ygg_internal.h"

namespace ygg {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short i16x4;
typedef __attribute__((ext_vector_type(8))) short i16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int DH = 128;
constexpr int KS = 272;  // bytes between K rows in LDS (256 + 16: conflict-free 16-byte column reads)
constexpr int VS = 288;  // bytes between V rows in LDS (256 + 32: transpose reads of 4 rows x 32 bytes)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ i16x4 lds_read_tr16(const unsigned char* p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)(p));
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    // round-to-nearest-even on both halves
    uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
    a += 0x7fffu + ((a >> 16) & 1u);
    b += 0x7fffu + ((b >> 16) & 1u);
    return (a >> 16) | (b & 0xffff0000u);
}

template <int NW, int RB, int KT>
__global__ __launch_bounds__(NW * 64) void attn_mfma_kernel(AttnArgs a, int RT, int S) {
    constexpr int THREADS = NW * 64;
    constexpr int RW = NW * RB * 32;                             // query rows per workgroup
    constexpr int PIECES = (KT * 16 + THREADS - 1) / THREADS;    // 16-byte pieces per thread per tile
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* k_s = smem;                                   // [2][KT][KS]
    unsigned char* v_s = smem + 2 * KT * KS;                     // [2][KT][VS]
    uint32_t* anc_s = reinterpret_cast<uint32_t*>(smem + 2 * KT * (KS + VS));  // [local node][aw]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, g2 = lane >> 5;

    // workgroup id -> (stream sigma = (b, kv head, split), row tile); sigma % 8 picks the XCD
    const int wg = blockIdx.x;
    const int xcd = wg & 7;
    const int rt = (wg >> 3) % RT;
    const int sigma = (wg / (8 * RT)) * 8 + xcd;
    if (sigma >= S) return;
    const int split = sigma % a.nsplit;
    const int hk = (sigma / a.nsplit) % a.Hkv;
    const int b = sigma / (a.nsplit * a.Hkv);

    const int R = a.N * a.G;
    const int row_base = rt * RW;
    int L = a.seq_lens[b];
    L = L < 0 ? 0 : (L > a.max_seq_len ? a.max_seq_len : L);
    const int Tk = L + a.N;
    int chunk = (Tk + a.nsplit - 1) / a.nsplit;
    chunk = (chunk + kKeyTile - 1) / kKeyTile * kKeyTile;
    const int k0 = split * chunk;
    const int k1 = min(Tk, k0 + chunk);
    const int64_t rows_total = (int64_t)a.B * a.N * a.Hq;

    // rows of this lane: block rb of this wave -> row_base + (wave*RB + rb)*32 + n
    int64_t rg_of[RB];   // global row index (b, node, q head) or -1
    int node_of[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int row = row_base + (wave * RB + rb) * 32 + n;
        const int i = min(row, R - 1) / a.G;
        const int g = min(row, R - 1) % a.G;
        node_of[rb] = i;
        rg_of[rb] = row < R ? ((int64_t)b * a.N + i) * a.Hq + hk * a.G + g : -1;
    }

    if (k0 >= k1) {  // empty split (uniform over the workgroup): mark the partials as absent
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
            if (rg_of[rb] >= 0 && g2 == 0) {
                float* pml = a.part_ml + ((int64_t)split * rows_total + rg_of[rb]) * 2;
                pml[0] = -INFINITY;
                pml[1] = 0.f;
            }
        return;
    }

    // Q as the B operand of S^T = K.Q^T: lane (n, g2) holds Q[row n][16 s + 8 g2 .. +8) for s = 0..7
    bf16x8 qreg[RB][8];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        if (rg_of[rb] >= 0) {
            const bf16x8* qp = reinterpret_cast<const bf16x8*>(static_cast<const uint16_t*>(a.q) + rg_of[rb] * DH + 8 * g2);
#pragma unroll
            for (int s = 0; s < 8; ++s) qreg[rb][s] = qp[2 * s];
        } else {
#pragma unroll
            for (int s = 0; s < 8; ++s) qreg[rb][s] = bf16x8{};
        }
    }

    // ancestor bitmasks of the nodes this workgroup's rows belong to
    const int aw = (a.N + 31) >> 5;
    const int i_first = row_base / a.G;
    const int i_last = min(R - 1, row_base + RW - 1) / a.G;
    if (k1 > L) {
        const int32_t* parent = a.parent_idx + (int64_t)b * a.N;
        for (int t = tid; t <= i_last - i_first; t += THREADS) {
            uint32_t* w = anc_s + t * aw;
            for (int x = 0; x < aw; ++x) w[x] = 0;
            int guard = 0;
            for (int c = i_first + t; c >= 0 && c < a.N && guard < a.N; c = parent[c], ++guard) w[c >> 5] |= 1u << (c & 31);
        }
    }

    const int64_t tok_stride = (int64_t)a.Hkv * DH;  // elements between consecutive tokens
    const uint16_t* kc = static_cast<const uint16_t*>(a.k_cache) + ((int64_t)b * a.cap * a.Hkv + hk) * DH;
    const uint16_t* vc = static_cast<const uint16_t*>(a.v_cache) + ((int64_t)b * a.cap * a.Hkv + hk) * DH;
    const uint16_t* kt = static_cast<const uint16_t*>(a.k_tree) + ((int64_t)b * a.N * a.Hkv + hk) * DH;
    const uint16_t* vt = static_cast<const uint16_t*>(a.v_tree) + ((int64_t)b * a.N * a.Hkv + hk) * DH;

    uint4 kst[PIECES], vst[PIECES];
    auto load_tile = [&](int tile_base) {
#pragma unroll
        for (int it = 0; it < PIECES; ++it) {
            const int pid = tid + it * THREADS;
            const int row = pid >> 4, col = pid & 15;
            const int j = tile_base + row;
            kst[it] = make_uint4(0, 0, 0, 0);
            vst[it] = make_uint4(0, 0, 0, 0);
            if (pid < KT * 16 && j < k1) {
                const int64_t off = (j < L ? (int64_t)j : (int64_t)(j - L)) * tok_stride + col * 8;
                kst[it] = *reinterpret_cast<const uint4*>((j < L ? kc : kt) + off);
                vst[it] = *reinterpret_cast<const uint4*>((j < L ? vc : vt) + off);
            }
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int it = 0; it < PIECES; ++it) {
            const int pid = tid + it * THREADS;
            const int row = pid >> 4, col = pid & 15;
            if (pid < KT * 16) {
                *reinterpret_cast<uint4*>(k_s + (buf * KT + row) * KS + col * 16) = kst[it];
                *reinterpret_cast<uint4*>(v_s + (buf * KT + row) * VS + col * 16) = vst[it];
            }
        }
    };

    f32x16 o[RB][4];
    float m_run[RB], l_run[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        m_run[rb] = -INFINITY;
        l_run[rb] = 0.f;
#pragma unroll
        for (int db = 0; db < 4; ++db) o[rb][db] = f32x16{};
    }
    const float c_scale = a.scale * kLog2e;

    const int ntiles = (k1 - k0 + KT - 1) / KT;
    load_tile(k0);
    store_tile(0);
    __syncthreads();  // also publishes anc_s

    for (int t = 0; t < ntiles; ++t) {
        const int tile_base = k0 + t * KT;
        const int buf = t & 1;
        if (t + 1 < ntiles) load_tile(tile_base + KT);
        const bool clean = tile_base + KT <= min(L, k1);  // whole tile inside the prefix

#pragma unroll 1
        for (int kb = 0; kb < KT / 32; ++kb) {
            const unsigned char* kbuf = k_s + (buf * KT + kb * 32 + n) * KS + 16 * g2;
            f32x16 st[RB];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) st[rb] = f32x16{};
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const bf16x8 ka = *reinterpret_cast<const bf16x8*>(kbuf + 32 * s);
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
                    st[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[rb][s], st[rb], 0, 0, 0);
            }

            i16x8 pb[RB][2];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                uint32_t okmask = 0xffffffffu;  // bit u: key u of this 32-key block is visible to this lane's row
                if (!clean) {
                    const int blk0 = tile_base + kb * 32;   // first key of the block
                    const int bt = blk0 - L;                // its tree-node index (negative inside the prefix)
                    const uint32_t* w = anc_s + (node_of[rb] - i_first) * aw;
                    if (bt >= 0) {
                        const int wi = bt >> 5;
                        const uint64_t w0 = wi < aw ? w[wi] : 0u;
                        const uint64_t w1 = wi + 1 < aw ? w[wi + 1] : 0u;
                        okmask = (uint32_t)(((w1 << 32) | w0) >> (bt & 31));
                    } else if (bt > -32) {                  // block straddles the end of the prefix
                        okmask = (0xffffffffu >> (32 + bt)) | (w[0] << (-bt));
                    }
                    const int left = k1 - blk0;             // keys of this block inside the split
                    if (left < 32) okmask &= left <= 0 ? 0u : (0xffffffffu >> (32 - left));
                }
                float x[16];
                float mt = -INFINITY;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = 8 * (v >> 2) + 4 * g2 + (v & 3);
                    x[v] = ((okmask >> key) & 1u) ? st[rb][v] * c_scale : -INFINITY;
                    mt = fmaxf(mt, x[v]);
                }
                mt = fmaxf(mt, __shfl_xor(mt, 32));
                const float mn = fmaxf(m_run[rb], mt);
                const float ms = mn == -INFINITY ? 0.f : mn;
                const float alpha = __builtin_amdgcn_exp2f(m_run[rb] - ms);
                float ps = 0.f;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    x[v] = __builtin_amdgcn_exp2f(x[v] - ms);
                    ps += x[v];
                }
                l_run[rb] = l_run[rb] * alpha + ps;
                m_run[rb] = mn;
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int v = 0; v < 16; ++v) o[rb][db][v] *= alpha;
#pragma unroll
                for (int m2 = 0; m2 < 2; ++m2) {
                    union { uint32_t u[4]; i16x8 v; } pk;
#pragma unroll
                    for (int e = 0; e < 4; ++e) pk.u[e] = pack_bf16x2(x[8 * m2 + 2 * e], x[8 * m2 + 2 * e + 1]);
                    pb[rb][m2] = pk.v;
                }
            }

            // O^T += V^T . P^T ; lane j of a 16-lane group addresses key row (j/4), dh 4*(j%4)
            const int j16 = lane & 15, blk = (lane >> 4) & 1;
            const unsigned char* vbuf = v_s + (buf * KT + kb * 32 + 4 * g2 + (j16 >> 2)) * VS + (16 * blk + 4 * (j16 & 3)) * 2;
#pragma unroll
            for (int db = 0; db < 4; ++db) {
#pragma unroll
                for (int m2 = 0; m2 < 2; ++m2) {
                    const unsigned char* p = vbuf + (16 * m2) * VS + db * 64;
                    const i16x4 lo = lds_read_tr16(p);
                    const i16x4 hi = lds_read_tr16(p + 8 * VS);
                    const i16x8 va = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
                        o[rb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, va), __builtin_bit_cast(bf16x8, pb[rb][m2]), o[rb][db], 0, 0, 0);
                }
            }
        }

        if (t + 1 < ntiles) store_tile(buf ^ 1);
        __syncthreads();
    }

    // epilogue: lane (n, g2) holds, for its row, dh = 32 db + 8 (v/4) + 4 g2 + (v%4)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const float l_tot = l_run[rb] + __shfl_xor(l_run[rb], 32);
        if (rg_of[rb] < 0) continue;
        if (a.nsplit == 1) {
            const float inv = 1.f / l_tot;
            uint16_t* op = static_cast<uint16_t*>(a.out) + rg_of[rb] * DH + 4 * g2;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    uint2 w;
                    w.x = pack_bf16x2(o[rb][db][4 * vq] * inv, o[rb][db][4 * vq + 1] * inv);
                    w.y = pack_bf16x2(o[rb][db][4 * vq + 2] * inv, o[rb][db][4 * vq + 3] * inv);
                    *reinterpret_cast<uint2*>(op + 32 * db + 8 * vq) = w;
                }
            if (a.lse && g2 == 0) a.lse[rg_of[rb]] = m_run[rb] * kLn2 + logf(l_tot);
        } else {
            float* po = a.part_o + ((int64_t)split * rows_total + rg_of[rb]) * DH + 4 * g2;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int vq = 0; vq < 4; ++vq)
                    *reinterpret_cast<float4*>(po + 32 * db + 8 * vq) =
                        make_float4(o[rb][db][4 * vq], o[rb][db][4 * vq + 1], o[rb][db][4 * vq + 2], o[rb][db][4 * vq + 3]);
            if (g2 == 0) {
                float* pml = a.part_ml + ((int64_t)split * rows_total + rg_of[rb]) * 2;
                pml[0] = m_run[rb] * kLn2;  // natural-log units of the scaled scores
                pml[1] = l_tot;
            }
        }
    }
}

template <int NW, int RB, int KT>
hipError_t launch_cfg(const AttnArgs& a, const AttnPlan& p, hipStream_t st) {
    const int S = a.B * a.Hkv * a.nsplit;
    const int RT = p.row_tiles;
    const int S8 = (S + 7) / 8 * 8;
    const int RW = NW * RB * 32;
    const int nodes_local = (RW + a.G - 1) / a.G + 1;
    const size_t smem = (size_t)2 * KT * (KS + VS) + (size_t)nodes_local * ((a.N + 31) / 32) * 4;
    auto kern = attn_mfma_kernel<NW, RB, KT>;
    static size_t smem_allowed = 0;  // per instantiation; raising the limit again is harmless
    if (smem > smem_allowed) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        smem_allowed = smem;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(S8 * RT)), dim3(NW * 64), smem, st, a, RT, S);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_mfma(const AttnArgs& a, const AttnPlan& p, hipStream_t st) {
    const int key = p.waves * 10 + p.rblocks;
    switch (key) {
        case 11: return launch_cfg<1, 1, 64>(a, p, st);
        case 12: return launch_cfg<1, 2, 64>(a, p, st);
        case 21: return launch_cfg<2, 1, 64>(a, p, st);
        case 22: return launch_cfg<2, 2, 64>(a, p, st);
        case 32: return launch_cfg<3, 2, 64>(a, p, st);
        case 41: return launch_cfg<4, 1, 64>(a, p, st);
        case 42: return launch_cfg<4, 2, 64>(a, p, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ygg
