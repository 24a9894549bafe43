// Debug validator for the data-dependent part of the calling contract.  The verification calls
// treat non-topological parents, out-of-range lengths or tokens and NaN logits as undefined
// behaviour (they only promise to stay inside the buffers); this call reports them, per sequence,
// as a bit mask in device memory.  Not on the verification path.
#include "ygg_internal.h"

namespace ygg {
namespace {

__global__ __launch_bounds__(256) void validate_tree_kernel(ValidateArgs a) {
    __shared__ int32_t parent_s[kMaxNodes];
    __shared__ int32_t bad_s;
    const int tid = threadIdx.x, b = blockIdx.x, N = a.N;
    if (tid == 0) bad_s = 0;
    __syncthreads();
    int f = 0;
    if (a.parent_idx) {
        for (int i = tid; i < N; i += 256) {
            const int p = a.parent_idx[(int64_t)b * N + i];
            parent_s[i] = p;
            if (i == 0 ? p != -1 : (p < 0 || p >= i)) f |= YGG_BAD_PARENT;
        }
    }
    if (a.seq_lens && tid == 0) {
        const int L = a.seq_lens[b];
        if (L < 0 || L > a.max_seq_len) f |= YGG_BAD_SEQ_LEN;
    }
    if (a.token_ids) {
        for (int i = tid; i < N; i += 256) {
            const int t = a.token_ids[(int64_t)b * N + i];
            if (t < 0 || t >= a.V) f |= YGG_BAD_TOKEN;
        }
    }
    if (f) atomicOr(&bad_s, f);
    __syncthreads();
    if (a.parent_idx && !(bad_s & YGG_BAD_PARENT)) {   // depths are only defined for a valid tree; walks end at the root
        int deep = 0;
        for (int i = tid; i < N; i += 256) {
            int d = 0;
            for (int n = i; n > 0 && d <= a.D; n = parent_s[n]) ++d;
            deep |= d > a.D;
        }
        if (deep) atomicOr(&bad_s, (int)YGG_BAD_DEPTH);
    }
    __syncthreads();
    if (tid == 0) a.flags[b] = bad_s;
}

// grid (chunks, B): ORs YGG_BAD_LOGIT into flags[b] (written by the kernel above, same stream) if a NaN is seen
__global__ __launch_bounds__(256) void validate_logits_kernel(ValidateArgs a, int64_t per_seq) {
    const int b = blockIdx.y;
    const float* x = a.logits + (int64_t)b * per_seq;
    bool bad = false;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < per_seq; e += (int64_t)gridDim.x * 256) bad |= x[e] != x[e];
    if (__any(bad) && (threadIdx.x & 63) == 0) atomicOr(&a.flags[b], (int)YGG_BAD_LOGIT);
}

}  // namespace

hipError_t launch_validate(const ValidateArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(validate_tree_kernel, dim3((unsigned)a.B), dim3(256), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !a.logits) return e;
    const int64_t per_seq = (int64_t)a.logit_rows * a.V;
    int64_t chunks = (per_seq + 256 * 16 - 1) / (256 * 16);
    chunks = chunks < 1 ? 1 : (chunks > 1024 ? 1024 : chunks);
    hipLaunchKernelGGL(validate_logits_kernel, dim3((unsigned)chunks, (unsigned)a.B), dim3(256), 0, st, a, per_seq);
    return hipGetLastError();
}

}  // namespace ygg
