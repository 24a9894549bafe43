// Equal-growth expansion: one draft step keeps exactly W new nodes, the candidates (frontier
// node p, token v) with the largest cumulative draft log-probability (paper Sec. 4.2, "Draft
// Width Selection").
//
// Two kernels:
//   expand_scan   grid (frontier row, vocab chunk): streams the fp32 logits once, coalesced, and
//                 leaves per chunk {max, sum exp(x - max) in fp64, the chunk's W largest logits}.
//                 Inside one row the candidate order is the order of the raw logits, so the
//                 chunk lists are exact whatever the row's normaliser turns out to be.
//   expand_merge  one workgroup per sequence: per-row log-sum-exp from the chunk statistics,
//                 then a W-round tournament over the heads of all chunk lists on the fp64 score
//                 cum[p] + (x - lse_p); ties go to the lower flat index p*V + v.
#include "ygg_internal.h"

namespace ygg {
namespace {

constexpr int kScanThreads = 256;
constexpr int kScanElems = 16;  // logits per thread; chunk = 4096
constexpr long long kNoIndex = 0x7fffffffffffffffLL;

struct ChunkStat {
    double sumexp;
    float maxv;
    int32_t count;
};
struct Cand {
    float val;
    int32_t idx;
};

__device__ __forceinline__ bool beats(double v2, long long i2, double v, long long i) {
    return v2 > v || (v2 == v && i2 < i);
}

// Workgroup-wide argmax of (value, index): larger value first, lower index on equal values.
// `slots` holds 2 x 4 entries (double-buffered by round parity); one barrier per call.
__device__ __forceinline__ void block_argmax(double& v, long long& i, double* slot_v, long long* slot_i, int parity) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const double v2 = __shfl_xor(v, o);
        const long long i2 = __shfl_xor(i, o);
        if (beats(v2, i2, v, i)) { v = v2; i = i2; }
    }
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { slot_v[parity * 4 + wave] = v; slot_i[parity * 4 + wave] = i; }
    __syncthreads();
    v = slot_v[parity * 4];
    i = slot_i[parity * 4];
#pragma unroll
    for (int w = 1; w < 4; ++w) {
        const double v2 = slot_v[parity * 4 + w];
        const long long i2 = slot_i[parity * 4 + w];
        if (beats(v2, i2, v, i)) { v = v2; i = i2; }
    }
}

__global__ __launch_bounds__(kScanThreads) void expand_scan_kernel(ExpandArgs a) {
    __shared__ double slot_v[8];
    __shared__ long long slot_i[8];
    __shared__ double red_d[4];
    __shared__ float red_f[4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = blockIdx.x;  // b*F + p
    const int c = blockIdx.y;
    const int c0 = c * a.chunk;
    const int c1 = min(a.V, c0 + a.chunk);
    const float* x = a.logits + row * a.V;

    float xv[kScanElems];
    uint32_t taken = 0;  // bit k set: element k is absent or already emitted
    float tmax = -INFINITY;
#pragma unroll
    for (int k = 0; k < kScanElems; ++k) {
        const int idx = c0 + k * kScanThreads + tid;
        if (idx < c1) {
            xv[k] = x[idx];
            tmax = fmaxf(tmax, xv[k]);
        } else {
            xv[k] = -INFINITY;
            taken |= 1u << k;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) tmax = fmaxf(tmax, __shfl_xor(tmax, o));
    if (lane == 0) red_f[wave] = tmax;
    __syncthreads();
    const float cmax = fmaxf(fmaxf(red_f[0], red_f[1]), fmaxf(red_f[2], red_f[3]));

    double sum = 0.0;
    if (cmax > -INFINITY) {
#pragma unroll
        for (int k = 0; k < kScanElems; ++k)
            if (!((taken >> k) & 1u)) sum += exp((double)xv[k] - (double)cmax);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    if (lane == 0) red_d[wave] = sum;
    __syncthreads();

    const int rounds = min(a.W, c1 - c0);
    if (tid == 0) {
        ChunkStat st;
        st.sumexp = (red_d[0] + red_d[1]) + (red_d[2] + red_d[3]);
        st.maxv = cmax;
        st.count = rounds;
        static_cast<ChunkStat*>(a.stats)[row * a.nchunk + c] = st;
    }

    // thread-local best among the elements not yet emitted (lowest k wins ties = lowest index)
    auto local_best = [&](double& bv, long long& bi) {
        bv = -INFINITY;
        bi = kNoIndex;
#pragma unroll
        for (int k = 0; k < kScanElems; ++k) {
            if (!((taken >> k) & 1u) && (bi == kNoIndex || (double)xv[k] > bv)) {
                bv = (double)xv[k];
                bi = c0 + k * kScanThreads + tid;
            }
        }
    };
    double bv;
    long long bi;
    local_best(bv, bi);
    Cand* out = static_cast<Cand*>(a.cands) + (row * a.nchunk + c) * a.W;
    for (int r = 0; r < rounds; ++r) {
        double wv = bv;
        long long wi = bi;
        block_argmax(wv, wi, slot_v, slot_i, r & 1);
        if (tid == 0) {
            Cand cd;
            cd.val = (float)wv;
            cd.idx = (int32_t)wi;
            out[r] = cd;
        }
        if (wi == bi && bi != kNoIndex) {
            taken |= 1u << (int)((bi - c0 - tid) / kScanThreads);
            local_best(bv, bi);
        }
    }
}

constexpr int kMaxListsPerThread = 16;  // 256 threads x 16 = 4096 chunk lists at most

__global__ __launch_bounds__(256) void expand_merge_kernel(ExpandArgs a) {
    __shared__ double slot_v[8];
    __shared__ long long slot_i[8];
    __shared__ double lse_s[kMaxWidth];
    __shared__ double cum_s[kMaxWidth];

    const int tid = threadIdx.x;
    const int b = blockIdx.x;
    const int base_prev = a.d == 1 ? 0 : 1 + (a.d - 2) * a.W;
    const int base_new = 1 + (a.d - 1) * a.W;
    const ChunkStat* stats = static_cast<const ChunkStat*>(a.stats) + (int64_t)b * a.F * a.nchunk;
    const Cand* cands = static_cast<const Cand*>(a.cands) + (int64_t)b * a.F * a.nchunk * a.W;

    if (tid < a.F) {
        const ChunkStat* st = stats + (int64_t)tid * a.nchunk;
        float mx = -INFINITY;
        for (int c = 0; c < a.nchunk; ++c) mx = fmaxf(mx, st[c].maxv);
        double s = 0.0;
        for (int c = 0; c < a.nchunk; ++c)
            if (st[c].maxv > -INFINITY) s += st[c].sumexp * exp((double)st[c].maxv - (double)mx);
        lse_s[tid] = (double)mx + log(s);
        cum_s[tid] = (double)a.cum_logprob[(int64_t)b * a.N + base_prev + tid];
    }
    __syncthreads();

    const int K = a.F * a.nchunk;  // number of chunk lists, list q = p*nchunk + c
    // per list: current head (entry pos) and the one after it, prefetched
    double hs[kMaxListsPerThread], ns[kMaxListsPerThread];
    int hv[kMaxListsPerThread], nv[kMaxListsPerThread];
    int pos[kMaxListsPerThread], cnt[kMaxListsPerThread];
    auto score_of = [&](int q, Cand cd) { return cum_s[q / a.nchunk] + ((double)cd.val - lse_s[q / a.nchunk]); };
#pragma unroll
    for (int u = 0; u < kMaxListsPerThread; ++u) {
        const int q = tid + u * 256;
        hs[u] = ns[u] = -INFINITY;
        hv[u] = nv[u] = -1;
        pos[u] = 0;
        cnt[u] = 0;
        if (q < K) {
            cnt[u] = stats[q].count;
            if (cnt[u] > 0) { const Cand cd = cands[(int64_t)q * a.W]; hs[u] = score_of(q, cd); hv[u] = cd.idx; }
            if (cnt[u] > 1) { const Cand cd = cands[(int64_t)q * a.W + 1]; ns[u] = score_of(q, cd); nv[u] = cd.idx; }
        }
    }
    auto flat_of = [&](int u) { return (long long)((tid + u * 256) / a.nchunk) * a.V + hv[u]; };
    int bu = -1;
    auto local_best = [&](double& bv, long long& bi) {
        bv = -INFINITY;
        bi = kNoIndex;
        bu = -1;
#pragma unroll
        for (int u = 0; u < kMaxListsPerThread; ++u) {
            if (pos[u] < cnt[u]) {
                const long long f = flat_of(u);
                if (bu < 0 || beats(hs[u], f, bv, bi)) { bv = hs[u]; bi = f; bu = u; }
            }
        }
    };
    double bv;
    long long bi;
    local_best(bv, bi);
    for (int r = 0; r < a.W; ++r) {
        double wv = bv;
        long long wi = bi;
        block_argmax(wv, wi, slot_v, slot_i, r & 1);
        if (tid == 0) {
            const int64_t node = (int64_t)b * a.N + base_new + r;
            a.parent_idx[node] = base_prev + (int)(wi / a.V);
            a.token_ids[node] = (int)(wi % a.V);
            a.cum_logprob[node] = (float)wv;
        }
        if (bu >= 0 && wi == bi) {  // this thread's list won: advance it
#pragma unroll
            for (int u = 0; u < kMaxListsPerThread; ++u) {
                if (u == bu) {
                    const int q = tid + u * 256;
                    pos[u] += 1;
                    hs[u] = ns[u];
                    hv[u] = nv[u];
                    if (pos[u] + 1 < cnt[u]) {
                        const Cand cd = cands[(int64_t)q * a.W + pos[u] + 1];
                        ns[u] = score_of(q, cd);
                        nv[u] = cd.idx;
                    }
                }
            }
            local_best(bv, bi);
        }
    }
}

}  // namespace

ExpandPlan plan_expand(const ygg_shape& s, int32_t d) {
    ExpandPlan p;
    p.F = d == 1 ? 1 : s.width;
    p.chunk = kScanThreads * kScanElems;
    p.nchunk = (s.vocab + p.chunk - 1) / p.chunk;
    const size_t lists = (size_t)s.batch * (size_t)p.F * (size_t)p.nchunk;
    p.stat_bytes = (lists * sizeof(ChunkStat) + 255) / 256 * 256;
    p.cand_bytes = (lists * (size_t)s.width * sizeof(Cand) + 255) / 256 * 256;
    return p;
}

hipError_t launch_expand(const ExpandArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(expand_scan_kernel, dim3((unsigned)(a.B * a.F), (unsigned)a.nchunk), dim3(kScanThreads), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(expand_merge_kernel, dim3((unsigned)a.B), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace ygg
