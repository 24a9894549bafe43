// Greedy acceptance and K/V compaction, entirely on the device (paper Sec. 5: the "accept
// speculation management" stage that idles the GPU when it runs on the host; Sec. 4.1 under
// Eq. 2: bonus token; Sec. 6: the TokenTree's K/V bookkeeping).
//
// Two kernels:
//   argmax_partial  grid (tree node, vocab chunk): coalesced 16-byte streaming of the verifier's
//                   fp32 logits, first maximum per chunk; it also snapshots seq_lens into the
//                   workspace (with the caller's own argmax tokens a one-workgroup kernel does that).
//   match_compact   grid (path slot, sequence, layer group).  Every workgroup works the match of its
//                   sequence out for itself -- finishes the argmax, marks every node whose whole root
//                   path matches, picks the deepest (lowest index on ties) -- which costs less than a
//                   kernel boundary would; the workgroup of slot 0 and layer group 0 writes the path,
//                   the accepted length and the bonus token and advances seq_lens; then each workgroup
//                   copies its slot's K and V rows behind the old end of the cache (read from the
//                   snapshot: seq_lens itself may already have moved), for its share of the layers.
#include "ygg_internal.h"

namespace ygg {
namespace {

struct ArgPart {
    float val;
    int32_t idx;
};

__device__ __forceinline__ void take_first_max(float& v, int& i, float v2, int i2) {
    if (v2 > v || (v2 == v && i2 < i)) { v = v2; i = i2; }
}

// The sequence's length before this call, clamped like everywhere else; the second kernel reads only this copy.
__device__ __forceinline__ void snapshot_len(const AcceptArgs& a, int b) {
    const int L = a.seq_lens[b];
    a.old_len[b] = L < 0 ? 0 : (L > a.max_seq_len ? a.max_seq_len : L);
}

__global__ __launch_bounds__(256) void snapshot_kernel(AcceptArgs a) {
    for (int b = threadIdx.x; b < a.B; b += 256) snapshot_len(a, b);
}

__global__ __launch_bounds__(256) void argmax_partial_kernel(AcceptArgs a) {
    __shared__ float sv[4];
    __shared__ int si[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = blockIdx.x;  // b*N + i
    const int c = blockIdx.y;
    const int c0 = c * a.chunk;
    const int c1 = min(a.V, c0 + a.chunk);
    const float* x = a.target_logits + row * a.V;
    if (c == 0 && tid == 0 && row % a.N == 0) snapshot_len(a, (int)(row / a.N));

    float bv = -INFINITY;
    int bi = 0x7fffffff;
    // 16-byte loads need the row start and the chunk start 16-byte aligned: V % 4 == 0 (chunk is)
    if ((a.V & 3) == 0) {
        const float4* x4 = reinterpret_cast<const float4*>(x);
        for (int j = c0 / 4 + tid; j < c1 / 4; j += 256) {
            const float4 v = x4[j];
            // ascending index order inside the thread, strict > keeps the first maximum
            if (v.x > bv || bi == 0x7fffffff) { bv = v.x; bi = 4 * j; }
            if (v.y > bv) { bv = v.y; bi = 4 * j + 1; }
            if (v.z > bv) { bv = v.z; bi = 4 * j + 2; }
            if (v.w > bv) { bv = v.w; bi = 4 * j + 3; }
        }
    } else {
        for (int j = c0 + tid; j < c1; j += 256) {
            const float v = x[j];
            if (v > bv || bi == 0x7fffffff) { bv = v; bi = j; }
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) take_first_max(bv, bi, __shfl_xor(bv, o), __shfl_xor(bi, o));
    if (lane == 0) { sv[wave] = bv; si[wave] = bi; }
    __syncthreads();
    if (tid == 0) {
#pragma unroll
        for (int w = 1; w < 4; ++w) take_first_max(bv, bi, sv[w], si[w]);
        ArgPart p;
        p.val = bv;
        p.idx = bi;
        static_cast<ArgPart*>(a.part)[row * a.nchunk + c] = p;
    }
}

__global__ __launch_bounds__(256) void match_compact_kernel(AcceptArgs a) {
    __shared__ int parent_s[kMaxNodes];
    __shared__ int tstar_s[kMaxNodes];
    __shared__ int token_s[kMaxNodes];
    __shared__ unsigned long long best_s[4];
    __shared__ int slot_node_s, len_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int k_slot = blockIdx.x, b = blockIdx.y;
    const int N = a.N;
    const int old_len = a.old_len[b];

    for (int i = tid; i < N; i += 256) {
        const int64_t node = (int64_t)b * N + i;
        int p = a.parent_idx[node];
        parent_s[i] = (i == 0 || p < 0 || p >= i) ? -1 : p;  // keeps every walk finite and in range
        token_s[i] = a.token_ids[node];
        int t;
        if (a.target_tokens) {
            t = a.target_tokens[node];
        } else {
            // chunk maxima of this node, eight loads in flight at a time (ascending chunks: first maximum wins)
            const ArgPart* pp = static_cast<const ArgPart*>(a.part) + node * a.nchunk;
            float bv = -INFINITY;
            t = 0x7fffffff;
            for (int c0 = 0; c0 < a.nchunk; c0 += 8) {
                ArgPart pc[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) pc[u] = pp[min(c0 + u, a.nchunk - 1)];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (c0 + u < a.nchunk && (t == 0x7fffffff || pc[u].val > bv || (pc[u].val == bv && pc[u].idx < t))) {
                        bv = pc[u].val;
                        t = pc[u].idx;
                    }
            }
        }
        tstar_s[i] = t;
    }
    __syncthreads();

    // key = (depth+1) << 32 | (0xffffffff - index) for matched nodes no deeper than D, else 0
    unsigned long long key = 0;
    for (int i = tid; i < N; i += 256) {
        bool ok = true;
        int dep = 0;
        for (int n = i; parent_s[n] >= 0; n = parent_s[n]) {
            ok = ok && token_s[n] == tstar_s[parent_s[n]];
            ++dep;
        }
        if (ok && dep <= a.D) {
            const unsigned long long k = ((unsigned long long)(dep + 1) << 32) | (unsigned long long)(0xffffffffu - (unsigned)i);
            key = k > key ? k : key;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const unsigned long long k2 = __shfl_xor(key, o);
        key = k2 > key ? k2 : key;
    }
    if (lane == 0) best_s[wave] = key;
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; ++w) key = best_s[w] > key ? best_s[w] : key;
        const int len = (int)(key >> 32);  // >= 1: the root always matches
        const int best = (int)(0xffffffffu - (unsigned)(key & 0xffffffffu));
        const bool writer = k_slot == 0 && blockIdx.z == 0;
        int32_t* path = a.accept_path + (int64_t)b * (a.D + 1);
        if (writer)
            for (int k = len; k <= a.D; ++k) path[k] = -1;
        int n = best, mine = -1;
        for (int k = len - 1; k >= 0; --k) {
            if (writer) path[k] = n;
            if (k == k_slot) mine = n;
            n = parent_s[n];
        }
        slot_node_s = mine;
        len_s = len;
        if (writer) {
            a.accept_len[b] = len;
            a.bonus_token[b] = tstar_s[best];
            a.seq_lens[b] = old_len + len;
        }
    }
    __syncthreads();

    // this workgroup's slot of the path: the node's K and V rows of every layer of its group go behind the old end
    const int node = slot_node_s;
    const int64_t dst_tok = (int64_t)old_len + k_slot;
    if (k_slot >= len_s || node < 0 || node >= N || dst_tok >= a.cap) return;  // contract violations stay inside the buffers
    const int64_t row16 = (int64_t)a.Hkv * a.Dh * a.elem_bytes / 16;  // 16-byte units per token row
    for (int layer = blockIdx.z; layer < a.n_layers; layer += gridDim.z) {
        const int64_t src = (((int64_t)layer * a.B + b) * N + node) * row16;
        const int64_t dst = (((int64_t)layer * a.B + b) * a.cap + dst_tok) * row16;
        const uint4* ks = static_cast<const uint4*>(a.k_tree) + src;
        const uint4* vs = static_cast<const uint4*>(a.v_tree) + src;
        uint4* kd = static_cast<uint4*>(a.k_cache) + dst;
        uint4* vd = static_cast<uint4*>(a.v_cache) + dst;
        for (int64_t j = tid; j < row16; j += 256) {
            kd[j] = ks[j];
            vd[j] = vs[j];
        }
    }
}

}  // namespace

AcceptPlan plan_accept(const ygg_shape& s) {
    AcceptPlan p;
    // aim for about 2048 workgroups; chunks are multiples of 1024 logits (one float4 per thread)
    const int64_t rows = (int64_t)s.batch * s.n_nodes;
    int64_t chunk = ((int64_t)s.vocab * rows / 2048 + 1023) / 1024 * 1024;
    if (chunk < 4096) chunk = 4096;
    if (chunk > 32768) chunk = 32768;
    p.chunk = (int32_t)chunk;
    p.nchunk = (int32_t)((s.vocab + chunk - 1) / chunk);
    p.part_bytes = ((size_t)rows * (size_t)p.nchunk * sizeof(ArgPart) + 255) / 256 * 256;
    p.oldlen_bytes = ((size_t)s.batch * sizeof(int32_t) + 255) / 256 * 256;
    return p;
}

hipError_t launch_accept(const AcceptArgs& a, hipStream_t st) {
    hipError_t e;
    if (a.target_logits) {
        hipLaunchKernelGGL(argmax_partial_kernel, dim3((unsigned)(a.B * a.N), (unsigned)a.nchunk), dim3(256), 0, st, a);
    } else {
        hipLaunchKernelGGL(snapshot_kernel, dim3(1), dim3(256), 0, st, a);
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;
    // without layers only slot 0 runs (it writes the results); else a slot's layers are dealt out over as many
    // workgroups as keep the grid near a thousand (each redoes the match; a workgroup's layers are copied one after another)
    const unsigned slots = a.n_layers > 0 ? (unsigned)(a.D + 1) : 1u;
    int64_t groups64 = 1024 / ((int64_t)slots * a.B);
    if (groups64 > a.n_layers) groups64 = a.n_layers;
    if (groups64 < 1) groups64 = 1;
    const unsigned groups = (unsigned)groups64;
    hipLaunchKernelGGL(match_compact_kernel, dim3(slots, (unsigned)a.B, groups), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace ygg
