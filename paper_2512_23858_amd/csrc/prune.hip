// Verification-width pruning: keep the W_verify nodes of the drafted tree that form the
// maximum-value subtree (paper Sec. 4.2, "Verification Width Pruning"), renumber them, and report
// the width that maximises the speedup objective (Eq. 3) with every other term fixed.
//
// The paper solves the subtree problem with a bottom-up dynamic programme.  With the value of a
// node being the probability that its whole path is accepted, exp(cum_logprob), a child is never
// worth more than its parent, so the k most valuable nodes (equal values: lower index, i.e. the
// parent, first) are already a connected set that contains the root, and they are optimal for
// every k at once: the programme collapses to one sort, and the optimal sets for all widths are
// nested prefixes of that order.  One workgroup per sequence orders the N <= 1024 keys in LDS: by
// counting, for each key, the larger ones (N <= 512), else with a bitonic sort.
#include <type_traits>

#include "ygg_device.h"
#include "ygg_internal.h"

namespace ygg {
namespace {

constexpr int kThreads = 256;

__global__ __launch_bounds__(kThreads) void prune_kernel(PruneArgs a, int n2) {
    __shared__ uint64_t key[kMaxNodes];      // (order key of cum) << 32 | ~index : larger sorts first
    __shared__ double pre[kMaxNodes];        // prefix sums of the sorted values
    __shared__ int32_t newidx[kMaxNodes];    // kept flag, then the node's number in the pruned tree
    __shared__ double wsum[kThreads / 64];
    __shared__ int32_t wcnt[kThreads / 64];
    __shared__ double red_v[kThreads / 64];
    __shared__ int32_t red_n[kThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.x;
    const int N = a.N, w = a.w;
    const float* cum = a.cum_logprob + (int64_t)b * N;
    const int32_t* parent = a.parent_idx + (int64_t)b * N;

    for (int i = tid; i < max(n2, 8); i += kThreads)
        key[i] = i < N ? ((uint64_t)key_of(cum[i]) << 32) | (uint32_t)(0xffffffffu - (uint32_t)i) : 0ull;
    __syncthreads();
    if (N <= 2 * kThreads) {
        // One or two keys per thread: a key's place in the order is the number of larger keys (the keys are distinct: the
        // index sits in their low bits; the padding zeros are smaller than any key).  N broadcast reads from LDS, eight in
        // flight, instead of the sort's log^2 rounds of dependent exchanges.
        auto count_sort = [&](auto kptc) __attribute__((always_inline)) {
            constexpr int KPT = decltype(kptc)::value;
            uint64_t mine[KPT];
            int rank[KPT];
#pragma unroll
            for (int q = 0; q < KPT; ++q) {
                const int i = tid + q * kThreads;
                mine[q] = i < N ? key[i] : 0ull;
                rank[q] = 0;
            }
            for (int j = 0; j < n2; j += 8) {
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const uint64_t x = key[j + u];
#pragma unroll
                    for (int q = 0; q < KPT; ++q) rank[q] += x > mine[q];
                }
            }
            __syncthreads();  // every thread has read the unsorted keys
#pragma unroll
            for (int q = 0; q < KPT; ++q)
                if (tid + q * kThreads < N) key[rank[q]] = mine[q];
        };
        if (N <= kThreads) count_sort(std::integral_constant<int, 1>{});
        else count_sort(std::integral_constant<int, 2>{});
    } else {
    for (int k = 2; k <= n2; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = tid; i < (n2 >> 1); i += kThreads) {
                const int lo = ((i & ~(j - 1)) << 1) | (i & (j - 1));
                const int hi = lo | j;
                const uint64_t x = key[lo], y = key[hi];
                const bool down = (lo & k) == 0;
                if (down ? y > x : x > y) { key[lo] = y; key[hi] = x; }
            }
            // Pairs at distance <= 64 stay inside one 128-element block, and a block belongs to the same wavefront
            // in every stage: two such stages in a row need no workgroup barrier (LDS accesses of one wavefront
            // complete in order; the fence keeps the compiler from moving them).
            const int j_next = j > 1 ? j >> 1 : k;   // first distance of the next k is k
            if (j <= 64 && j_next <= 64) {
                __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
                __builtin_amdgcn_wave_barrier();
            } else {
                __syncthreads();
            }
        }
    }

    __syncthreads();  // the sorted order is read by every wavefront
    // kept flags by original index; sorted values for the prefix sums
    constexpr int PER = kMaxNodes / kThreads;  // 4 consecutive positions per thread
    double v[PER];
    double local = 0.0;
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int r = tid * PER + u;
        v[u] = 0.0;
        if (r < N) {
            const uint64_t kk = key[r];
            const int orig = (int)(0xffffffffu - (uint32_t)kk);
            newidx[orig] = r < w ? 1 : 0;
            v[u] = exp_nonpos((double)float_of((uint32_t)(kk >> 32)));
        }
        local += v[u];
    }
    // inclusive prefix over positions: within the thread, then across lanes, then across wavefronts
    double incl = local;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const double t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    double base = incl - local;
    for (int q = 0; q < wave; ++q) base += wsum[q];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        base += v[u];
        const int r = tid * PER + u;
        if (r < N) pre[r] = base;
    }
    __syncthreads();

    // renumber: exclusive count of kept nodes over the original order
    int flags[PER], cnt = 0;
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int i = tid * PER + u;
        flags[u] = i < N ? newidx[i] : 0;
        cnt += flags[u];
    }
    int cincl = cnt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(cincl, o);
        if (lane >= o) cincl += t;
    }
    if (lane == 63) wcnt[wave] = cincl;
    __syncthreads();
    int cbase = cincl - cnt;
    for (int q = 0; q < wave; ++q) cbase += wcnt[q];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int i = tid * PER + u;
        if (i < N) newidx[i] = flags[u] ? cbase : -1;
        cbase += flags[u];
    }
    __syncthreads();
    for (int i = tid; i < N; i += kThreads) {
        const int k = newidx[i];
        if (k >= 0) {
            const int64_t dst = (int64_t)b * w + k;
            a.kept_nodes[dst] = i;
            const int p = parent[i];
            a.new_parent[dst] = (i == 0 || p < 0 || p >= N) ? -1 : newidx[p];
            a.new_token[dst] = a.token_ids[(int64_t)b * N + i];
        }
    }
    if (tid == 0 && a.expected_len) a.expected_len[b] = (float)pre[w - 1];

    if (a.best_width) {  // first maximum of pre[n-1] / (t_draft + t_verifier[n]) over n = 1..N
        double top = -INFINITY;
        int arg = 0x7fffffff;
        for (int n = 1 + tid; n <= N; n += kThreads) {
            const double obj = pre[n - 1] / ((double)a.t_draft + (double)a.t_verifier[n]);
            if (obj > top) { top = obj; arg = n; }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const double ot = __shfl_xor(top, o);
            const int oa = __shfl_xor(arg, o);
            if (ot > top || (ot == top && oa < arg)) { top = ot; arg = oa; }
        }
        if (lane == 0) { red_v[wave] = top; red_n[wave] = arg; }
        __syncthreads();
        if (tid == 0) {
            for (int q = 1; q < kThreads / 64; ++q)
                if (red_v[q] > top || (red_v[q] == top && red_n[q] < arg)) { top = red_v[q]; arg = red_n[q]; }
            a.best_width[b] = arg;
        }
    }
}

}  // namespace

hipError_t launch_prune(const PruneArgs& a, hipStream_t st) {
    int n2 = 2;
    while (n2 < a.N) n2 <<= 1;
    hipLaunchKernelGGL(prune_kernel, dim3((unsigned)a.B), dim3(kThreads), 0, st, a, n2);
    return hipGetLastError();
}

}  // namespace ygg
