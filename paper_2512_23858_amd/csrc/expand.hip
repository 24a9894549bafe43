// Equal-growth expansion: one draft step keeps exactly W new nodes, the candidates (frontier
// node p, token v) with the largest cumulative draft log-probability (paper Sec. 4.2, "Draft
// Width Selection").
//
// Two kernels:
//   expand_scan   grid (frontier row, vocab chunk of 4096): streams the fp32 logits once,
//                 coalesced, and leaves per chunk {max, sum exp(x - max) in fp64, the chunk's W
//                 largest logits, best first}.  Inside one row the candidate order is the order
//                 of the raw logits, so the chunk lists are exact whatever the row's normaliser
//                 turns out to be.
//   expand_merge  one workgroup per sequence: per-row log-sum-exp from the chunk statistics, the
//                 fp64 score cum[p] + (x - lse_p) of every list head, the W lists with the best
//                 heads (no entry of any other list can be among the W best), and finally the W
//                 best of those lists' W*W entries; ties go to the lower flat index p*V + v.
//
// Selection of "the W best of a workgroup's candidates" (used three times) never sorts and has no
// serial per-element rounds on its main path: each wavefront bisects, with ballots, for the W-th
// largest of its lanes' maxima (a lower bound of its W-th best candidate), pools the few candidates
// at or above that threshold in LDS, ranks them against each other, and the four sorted wavefront
// lists are merged by rank (binary search).  Candidates are ordered by an order-preserving integer
// key of the value, then by the lower index.
#include "ygg_internal.h"
#include "ygg_device.h"

namespace ygg {
namespace {

constexpr int kScanThreads = 256;
constexpr int kScanElems = 16;  // logits per thread; chunk = 4096, 1024 consecutive logits per wavefront
constexpr uint32_t kNone = 0xffffffffu;

struct ChunkStat {
    double sumexp;
    float maxv;
    int32_t count;
};
struct Cand {
    float val;
    int32_t idx;
};

// ---- the W best of a workgroup's candidates ---------------------------------------------------------
// A candidate: larger key first, then lower tie; key == 0 means "no candidate" (real keys are > 0).
struct __align__(16) Entry {
    uint64_t key;
    uint32_t tie;
    uint32_t tag;
};
__device__ __forceinline__ bool beats(const Entry& a, const Entry& b) {
    return a.key > b.key || (a.key == b.key && a.tie < b.tie);
}

constexpr int kPoolCap = 256;  // pooled candidates per wavefront on the fast path

struct TopWShared {
    Entry pool[4][kPoolCap];
    Entry list[4][kMaxWidth];  // per-wavefront result, best first
    int count[4];
};

// Wave-wide best candidate; lanes without one pass key 0.
__device__ __forceinline__ Entry wave_best(const Entry& e) {
    const uint32_t hi = (uint32_t)(e.key >> 32);
    const uint32_t mh = wave_max_u32(hi);
    const bool in1 = e.key != 0 && hi == mh;
    const uint32_t ml = wave_max_u32(in1 ? (uint32_t)e.key : 0u);
    const bool in2 = in1 && (uint32_t)e.key == ml;
    const uint32_t mt = wave_min_u32(in2 ? e.tie : kNone);
    const bool win = in2 && e.tie == mt;
    const int src = __ffsll((unsigned long long)__ballot(win)) - 1;
    Entry r;
    r.key = ((uint64_t)mh << 32) | ml;
    r.tie = mt;
    r.tag = src >= 0 ? (uint32_t)__builtin_amdgcn_readlane((int)e.tag, src) : 0u;
    return r;
}

// Every lane holds N candidate slots, read through get(k) (key 0 = empty).  Leaves the wavefront's best
// min(W, #candidates) in sh.list[wave], best first, and their number in sh.count[wave].
template <int N, typename Get>
__device__ __forceinline__ void wave_top_w(Get get, int W, int wave, int lane, TopWShared& sh) {
    uint32_t cmax = 0;   // largest coarse key (top 32 bits) of this lane
    int tot = 0;         // candidates of the wavefront
#pragma unroll
    for (int k = 0; k < N; ++k) {
        const Entry e = get(k);
        cmax = max(cmax, (uint32_t)(e.key >> 32));
        tot += (int)__popcll(__ballot(e.key != 0));
    }
    const int want = min(W, tot);
    const int wn = min(W, (int)__popcll(__ballot(cmax != 0)));
    // threshold: at most the wn-th largest lane maximum, so at least wn candidates lie at or above it.  Its low
    // twelve bits stay zero: a slightly lower threshold only pools a few more candidates.
    uint32_t t = 0;
    if (wn > 0) {
        for (int bit = 31; bit >= 12; --bit) {
            const uint32_t c = t | (1u << bit);
            if ((int)__popcll(__ballot(cmax >= c)) >= wn) t = c;
        }
    }
    // pool the candidates at or above the threshold
    int base = 0;
    const unsigned long long below = __lanemask_lt();
    bool fits = true;
#pragma unroll
    for (int k = 0; k < N; ++k) {
        const Entry e = get(k);
        const bool sel = wn > 0 && e.key != 0 && (uint32_t)(e.key >> 32) >= t;
        const unsigned long long m = __ballot(sel);
        const int pos = base + (int)__popcll(m & below);
        if (sel && pos < kPoolCap) sh.pool[wave][pos] = e;
        base += (int)__popcll(m);
    }
    fits = base <= kPoolCap && base >= want;
    // the ranking below reads pool entries written by other lanes of this wavefront
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (fits) {
        // rank the pooled candidates against each other; the best `want` go out in order
        const int C = base;
        for (int j0 = 0; j0 < C; j0 += 64) {
            const int j = j0 + lane;
            const Entry mine = sh.pool[wave][min(j, C - 1)];
            int rank = 0;
            const int C8 = C & ~7;
            for (int i = 0; i < C8; i += 8) {  // eight independent LDS reads in flight
#pragma unroll
                for (int u = 0; u < 8; ++u) rank += beats(sh.pool[wave][i + u], mine);
            }
            for (int i = C8; i < C; ++i) rank += beats(sh.pool[wave][i], mine);
            if (j < C && rank < want) sh.list[wave][rank] = mine;
        }
    } else {
        // Rare (more ties than the pool holds, or too few lanes hold candidates): one candidate per round.
        uint64_t gone = 0;  // bit k: slot k already emitted
        for (int r = 0; r < want; ++r) {
            Entry best = {0, kNone, 0};
            int bk = -1;
#pragma unroll
            for (int k = 0; k < N; ++k) {
                const Entry e = get(k);
                if (e.key != 0 && !((gone >> k) & 1ull) && (bk < 0 || beats(e, best))) { best = e; bk = k; }
            }
            const Entry w = wave_best(best);
            if (bk >= 0 && best.key == w.key && best.tie == w.tie) gone |= 1ull << bk;
            if (lane == 0) sh.list[wave][r] = w;
        }
    }
    if (lane == 0) sh.count[wave] = want;
}

// After wave_top_w in all four wavefronts and a barrier: rank of entry `lane` of this wavefront's list among
// the four lists (-1 if this lane holds none); ranks below W are the workgroup's best W, in order.
__device__ __forceinline__ int merged_rank(const TopWShared& sh, int wave, int lane, Entry& mine) {
    if (lane >= sh.count[wave]) return -1;
    mine = sh.list[wave][lane];
    // first position of each other list whose entry does not beat `mine`: three binary searches in step, so the
    // three LDS reads of a round are in flight together
    int lo[3], hi[3], cnt[3];
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const int w = i + (i >= wave);
        lo[i] = 0;
        hi[i] = cnt[i] = sh.count[w];
    }
    for (int span = max(cnt[0], max(cnt[1], cnt[2])); span > 0; span >>= 1) {  // enough rounds for the longest list
        Entry e[3];
        int mid[3];
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const int w = i + (i >= wave);
            mid[i] = (lo[i] + hi[i]) >> 1;
            e[i] = sh.list[w][min(mid[i], kMaxWidth - 1)];
        }
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const bool open = lo[i] < hi[i];
            const bool b = beats(e[i], mine);
            lo[i] = open && b ? mid[i] + 1 : lo[i];
            hi[i] = open && !b ? mid[i] : hi[i];
        }
    }
    return lane + lo[0] + lo[1] + lo[2];
}

// ---- scan ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kScanThreads) void expand_scan_kernel(ExpandArgs a) {
    __shared__ double red_d[4];
    __shared__ float red_f[4];
    __shared__ TopWShared sh;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t row = blockIdx.x;  // b*F + p
    const int c = blockIdx.y;
    const int c0 = c * a.chunk;
    const int c1 = min(a.V, c0 + a.chunk);
    const float* x = a.logits + row * a.V;
    const int w0 = c0 + wave * (kScanElems * 64);  // this wavefront's 1024 consecutive logits

    float xv[kScanElems];
    float tmax = -INFINITY;
#pragma unroll
    for (int k = 0; k < kScanElems; ++k) {
        const int idx = w0 + k * 64 + lane;
        xv[k] = idx < c1 ? x[idx] : -INFINITY;
        tmax = fmaxf(tmax, xv[k]);
    }
    // chunk maximum and sum of exponentials (fp64)
    const float wmax = float_of(wave_max_u32(key_of(tmax)));
    if (lane == 0) red_f[wave] = wmax;
    __syncthreads();
    const float cmax = fmaxf(fmaxf(red_f[0], red_f[1]), fmaxf(red_f[2], red_f[3]));
    double sum = 0.0;
    if (cmax > -INFINITY) {
        // logits past the end of the chunk are -inf and add exactly 0; no branch, so the sixteen series interleave
#pragma unroll
        for (int k = 0; k < kScanElems; ++k) sum += exp_nonpos((double)xv[k] - (double)cmax);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    if (lane == 0) red_d[wave] = sum;

    // the chunk's W largest logits: value key in the upper half of the key, vocabulary index as the tie-break
    auto get = [&](int k) {
        const int idx = w0 + k * 64 + lane;
        Entry e;
        e.key = idx < c1 ? (uint64_t)key_of(xv[k]) << 32 : 0ull;
        e.tie = (uint32_t)idx;
        e.tag = 0;
        return e;
    };
    wave_top_w<kScanElems>(get, a.W, wave, lane, sh);
    __syncthreads();
    if (tid == 0) {
        ChunkStat st;
        st.sumexp = (red_d[0] + red_d[1]) + (red_d[2] + red_d[3]);
        st.maxv = cmax;
        st.count = min(a.W, c1 - c0);
        static_cast<ChunkStat*>(a.stats)[row * a.nchunk + c] = st;
    }
    Entry mine;
    const int rank = merged_rank(sh, wave, lane, mine);
    if (rank >= 0 && rank < a.W) {
        Cand cd;
        cd.val = float_of((uint32_t)(mine.key >> 32));
        cd.idx = (int32_t)mine.tie;
        static_cast<Cand*>(a.cands)[(row * a.nchunk + c) * a.W + rank] = cd;
    }
}

// ---- merge --------------------------------------------------------------------------------------
constexpr size_t merge_scratch_bytes(int lpt) { return (size_t)256 * lpt * 12; }

template <int LPT, int EPT>  // chunk lists per thread; entries of the selected lists per thread (W*W <= 256*EPT)
__global__ __launch_bounds__(256) void expand_merge_kernel(ExpandArgs a) {
    constexpr int KMAX = 256 * LPT;
    // scratch for the chunk statistics
    extern __shared__ __align__(16) unsigned char raw[];  // merge_scratch_bytes(LPT)
    double* ssum = reinterpret_cast<double*>(raw);               // [KMAX]
    float* smax = reinterpret_cast<float*>(raw + KMAX * 8);      // [KMAX]
    __shared__ TopWShared sh;
    __shared__ double lse_s[kMaxWidth];
    __shared__ double cum_s[kMaxWidth];
    __shared__ uint32_t sel[kMaxWidth];       // the lists with the W best heads

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int b = blockIdx.x;
    const int base_prev = a.d == 1 ? 0 : 1 + (a.d - 2) * a.W;
    const int base_new = 1 + (a.d - 1) * a.W;
    const int K = a.F * a.nchunk;  // number of chunk lists, list q = p*nchunk + c
    const ChunkStat* stats = static_cast<const ChunkStat*>(a.stats) + (int64_t)b * K;
    const Cand* cands = static_cast<const Cand*>(a.cands) + (int64_t)b * K * a.W;

    // entries of chunk list q = p*nchunk + c: min(W, size of chunk c), known without touching memory
    auto list_len = [&](int q) {
        const int c = q % a.nchunk;
        return min(a.W, min(a.V, (c + 1) * a.chunk) - c * a.chunk);
    };
    // 1. chunk statistics -> per-row log-sum-exp (fixed summation order: deterministic)
    int cnt[LPT];
    Cand head[LPT];
#pragma unroll
    for (int u = 0; u < LPT; ++u) {
        const int q = tid + u * 256;
        cnt[u] = 0;
        head[u].val = -INFINITY;
        head[u].idx = 0;
        if (q < K) {
            // a chunk is never empty, so its list has a head: both loads go out together
            const ChunkStat st = stats[q];
            head[u] = cands[(int64_t)q * a.W];
            smax[q] = st.maxv;
            ssum[q] = st.sumexp;
            cnt[u] = list_len(q);
        }
    }
    if (tid < a.F) cum_s[tid] = (double)a.cum_logprob[(int64_t)b * a.N + base_prev + tid];
    __syncthreads();
    // a row's chunks go to a group of g lanes (g a power of two, small enough that all rows are in work at once
    // where possible), 64/g rows per wavefront at a time; the summation order is fixed
    {
        int f2 = 1;
        while (f2 < a.F) f2 <<= 1;
        int g = 1;
        while (g < a.nchunk && g < 64 && g * f2 < 256) g <<= 1;
        const int rpw = 64 / g;
        for (int p0 = wave * rpw; p0 < a.F; p0 += 4 * rpw) {
            const int p = p0 + lane / g, cf = lane % g;
            const int q0 = p * a.nchunk;
            float mx = -INFINITY;
            if (p < a.F)
                for (int c = cf; c < a.nchunk; c += g) mx = fmaxf(mx, smax[q0 + c]);
            for (int o = g >> 1; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
            double s = 0.0;
            if (p < a.F)
                for (int c = cf; c < a.nchunk; c += g) {
                    const float m = smax[q0 + c];
                    if (m > -INFINITY) s += ssum[q0 + c] * exp_nonpos((double)m - (double)mx);
                }
            for (int o = g >> 1; o > 0; o >>= 1) s += __shfl_xor(s, o);
            if (p < a.F && cf == 0) lse_s[p] = (double)mx + log(s);
        }
    }
    __syncthreads();
    auto entry_of = [&](uint32_t q, Cand cd) {  // fp64 score of candidate cd of list q
        const int p = (int)q / a.nchunk;
        Entry e;
        e.key = key_of(cum_s[p] + ((double)cd.val - lse_s[p]));
        e.tie = (uint32_t)(p * a.V + cd.idx);   // flat index p*V + v
        e.tag = q;
        return e;
    };

    // 2. the lists with the W best heads: no entry of any other list can be among the W best candidates
    Entry hd[LPT];
#pragma unroll
    for (int u = 0; u < LPT; ++u) {
        const int q = tid + u * 256;
        hd[u] = Entry{0, kNone, 0};
        if (q < K && cnt[u] > 0) hd[u] = entry_of((uint32_t)q, head[u]);
    }
    if (tid < kMaxWidth) sel[tid] = 0;  // every slot names a real list even if the ranks below were not a permutation
    wave_top_w<LPT>([&](int u) { return hd[u]; }, a.W, wave, lane, sh);
    __syncthreads();
    {
        Entry mine;
        const int rank = merged_rank(sh, wave, lane, mine);
        if (rank >= 0 && rank < a.W) sel[rank] = mine.tag;
    }
    const int nsel = min(a.W, sh.count[0] + sh.count[1] + sh.count[2] + sh.count[3]);
    __syncthreads();  // sel complete; sh and the statistics scratch may be reused

    // 3. the W best entries of the selected lists are the new nodes.  The lists are sorted, so their
    //    entries are dealt out position-major (slot = pos * nsel + list, thread = slot mod 256): the
    //    strongest entries then sit in different lanes and the per-wavefront thresholds are tight.
    //    Every thread fetches its (at most EPT) entries in one batch of loads.
    __shared__ int sel_cnt[kMaxWidth];
    if (tid < nsel) sel_cnt[tid] = list_len((int)sel[tid]);
    __syncthreads();
    auto get = [&](int u) {
        const int slot = tid + u * 256;
        Entry r = {0, kNone, 0};
        if (slot < nsel * a.W) {
            const int pos = slot / nsel, s = slot % nsel;
            if (pos < sel_cnt[s]) r = entry_of(sel[s], cands[(int64_t)sel[s] * a.W + pos]);
        }
        return r;
    };
    Entry pe[EPT];
#pragma unroll
    for (int u = 0; u < EPT; ++u) pe[u] = get(u);
    wave_top_w<EPT>([&](int u) { return pe[u]; }, a.W, wave, lane, sh);
    __syncthreads();
    {
        Entry mine;
        const int rank = merged_rank(sh, wave, lane, mine);
        if (rank >= 0 && rank < a.W) {
            const int64_t node = (int64_t)b * a.N + base_new + rank;
            a.parent_idx[node] = base_prev + (int)(mine.tie / (uint32_t)a.V);
            a.token_ids[node] = (int)(mine.tie % (uint32_t)a.V);
            a.cum_logprob[node] = (float)double_of(mine.key);
        }
    }
}

// ---- equal growth with free attachment -----------------------------------------------------------
// Every node, once the drafter has run on it, offers its W most probable tokens; the pool holds the
// offers not yet taken; a step takes the W best of the pool (paper Sec. 4.2: the W new leaves of a
// step may hang anywhere in the partial tree).  Three kernels per step: expand_scan (above) leaves
// per-chunk statistics and top-W lists of the new rows, attach_rows turns them into each row's W
// offers, attach_pool sorts pool + offers, emits the W new nodes and keeps the best W*(D-t) of the
// rest: an entry of rank r needs r / W more steps before it can be taken and later offers only push
// it down, so nothing beyond the slots still to be filled can ever be chosen.
struct __align__(16) Offer {
    double score;
    int32_t node;
    int32_t token;
};
constexpr int kPoolHeader = 16;  // bytes: int32 count, padding

template <int EPT>  // list entries per thread: nchunk * W <= 256 * EPT
__global__ __launch_bounds__(256) void attach_rows_kernel(ExpandArgs a) {
    __shared__ TopWShared sh;
    __shared__ double lse_sh;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t row = blockIdx.x;  // b*F + p
    const int b = (int)(row / a.F), p = (int)(row % a.F);
    const int node = (a.d == 1 ? 0 : 1 + (a.d - 2) * a.W) + p;
    const ChunkStat* stats = static_cast<const ChunkStat*>(a.stats) + row * a.nchunk;
    const Cand* cands = static_cast<const Cand*>(a.cands) + row * a.nchunk * a.W;

    // this thread's list entries, position-major (slot = pos * nchunk + chunk): all loads issued at once
    Entry pe[EPT];
#pragma unroll
    for (int u = 0; u < EPT; ++u) {
        const int slot = tid + u * 256;
        pe[u] = Entry{0, kNone, 0};
        if (slot < a.nchunk * a.W) {
            const int pos = slot / a.nchunk, c = slot % a.nchunk;
            const int cnt = min(a.W, min(a.V, (c + 1) * a.chunk) - c * a.chunk);
            if (pos < cnt) {
                const Cand cd = cands[c * a.W + pos];
                pe[u].key = (uint64_t)key_of(cd.val) << 32;  // inside a row the order of the raw logits
                pe[u].tie = (uint32_t)cd.idx;
            }
        }
    }
    // log-sum-exp of the row from the chunk statistics: wavefront 0, fixed summation order
    if (wave == 0) {
        float mx = -INFINITY;
        for (int c = lane; c < a.nchunk; c += 64) mx = fmaxf(mx, stats[c].maxv);
        mx = float_of(wave_max_u32(key_of(mx)));
        double sum = 0.0;
        for (int c = lane; c < a.nchunk; c += 64) {
            const ChunkStat st = stats[c];
            if (st.maxv > -INFINITY) sum += st.sumexp * exp_nonpos((double)st.maxv - (double)mx);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
        if (lane == 0) lse_sh = (double)mx + log(sum);
    }
    wave_top_w<EPT>([&](int u) { return pe[u]; }, a.W, wave, lane, sh);
    __syncthreads();
    Entry mine;
    const int rank = merged_rank(sh, wave, lane, mine);
    if (rank >= 0 && rank < a.W) {
        Offer o;
        const double cum = (double)a.cum_logprob[(int64_t)b * a.N + node];
        o.score = cum + ((double)float_of((uint32_t)(mine.key >> 32)) - lse_sh);
        o.node = node;
        o.token = (int32_t)mine.tie;
        static_cast<Offer*>(a.offers)[row * a.W + rank] = o;
    }
}

// One workgroup per sequence (256 to 1024 threads: one compare-exchange per thread and stage where possible, the sort
// is a chain of barriers); dynamic LDS holds n2 (a power of two) entries.
__global__ __launch_bounds__(1024) void attach_pool_kernel(ExpandArgs a, int n2) {
    extern __shared__ __align__(16) unsigned char raw_sort[];
    Entry* e = reinterpret_cast<Entry*>(raw_sort);
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int b = blockIdx.x;
    unsigned char* pool_b = static_cast<unsigned char*>(a.pool) + (size_t)b * (kPoolHeader + (size_t)a.pool_cap * sizeof(Offer));
    int32_t* pool_count = reinterpret_cast<int32_t*>(pool_b);
    Offer* pool = reinterpret_cast<Offer*>(pool_b + kPoolHeader);
    const Offer* offers = static_cast<const Offer*>(a.offers) + (int64_t)b * a.F * a.W;
    int n_old = a.d == 1 ? 0 : *pool_count;
    n_old = n_old < 0 ? 0 : min(n_old, min(a.pool_cap, a.W * (a.D - a.d + 1)));  // what the previous step may have left
    const int n_new = a.F * a.W;
    // Only W*(D-t+1) entries are ever needed: the W new nodes and the pool kept for later.  When the carried pool
    // alone already holds that many, an offer scoring below the pool's last entry cannot be among them, so it is
    // dropped before the sort (exact: equal scores are kept), and the sort runs over what is left.
    __shared__ int n_live;
    const int need = a.W * (a.D - a.d + 1);
    const uint64_t floor_key = (n_old >= need && n_old > 0) ? key_of(pool[n_old - 1].score) : 0ull;
    if (tid == 0) n_live = n_old;
    __syncthreads();
    for (int i = tid; i < n_old + n_new; i += nthr) {
        const Offer o = i < n_old ? pool[i] : offers[i - n_old];
        Entry x;
        x.key = key_of(o.score);
        x.tie = (uint32_t)o.node * (uint32_t)a.V + (uint32_t)o.token;
        x.tag = 0;
        if (i < n_old) e[i] = x;
        else if (x.key >= floor_key) e[atomicAdd(&n_live, 1)] = x;   // order before the sort does not matter
    }
    __syncthreads();
    const int n_sort = n_live;
    int m2 = 2;
    while (m2 < n_sort) m2 <<= 1;   // <= n2: the launch sized the buffer for every offer surviving
    n2 = m2;
    for (int i = n_sort + tid; i < n2; i += nthr) e[i] = Entry{0, kNone, 0};
    __syncthreads();
    // bitonic sort, best first (larger key, then lower node*V + token); empty slots sink to the end
    for (int k = 2; k <= n2; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = tid; i < (n2 >> 1); i += nthr) {
                const int lo = ((i & ~(j - 1)) << 1) | (i & (j - 1));
                const int hi = lo | j;
                const Entry x = e[lo], y = e[hi];
                const bool down = (lo & k) == 0;
                if (down ? beats(y, x) : beats(x, y)) { e[lo] = y; e[hi] = x; }
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
    __syncthreads();  // the sorted order is read by every wavefront
    const int base_new = 1 + (a.d - 1) * a.W;
    const int keep = min(a.W * (a.D - a.d), n_sort - a.W);
    for (int i = tid; i < a.W + keep; i += nthr) {
        const Entry x = e[i];
        const int node = (int)(x.tie / (uint32_t)a.V), token = (int)(x.tie % (uint32_t)a.V);
        const double score = double_of(x.key);
        if (i < a.W) {
            const int64_t dst = (int64_t)b * a.N + base_new + i;
            a.parent_idx[dst] = node;
            a.token_ids[dst] = token;
            a.cum_logprob[dst] = (float)score;
        } else {
            Offer o;
            o.score = score; o.node = node; o.token = token;
            pool[i - a.W] = o;
        }
    }
    if (tid == 0) *pool_count = keep;
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

// Static plus dynamic LDS of these exceeds the 64 KiB default.
hipError_t raise_limits_expand() {
    const void* big[] = {reinterpret_cast<const void*>(expand_merge_kernel<16, 1>),
                         reinterpret_cast<const void*>(expand_merge_kernel<16, 4>),
                         reinterpret_cast<const void*>(expand_merge_kernel<16, 16>)};
    for (const void* f : big) {
        hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)merge_scratch_bytes(16));
        if (e != hipSuccess) return e;
    }
    return hipFuncSetAttribute(reinterpret_cast<const void*>(attach_pool_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)(4096 * sizeof(Entry)));
}

template <int LPT>
static void launch_merge(const ExpandArgs& a, hipStream_t st) {
    const dim3 grid((unsigned)a.B), block(256);
    const size_t lds = merge_scratch_bytes(LPT);
    if (a.W <= 16) hipLaunchKernelGGL((expand_merge_kernel<LPT, 1>), grid, block, lds, st, a);
    else if (a.W <= 32) hipLaunchKernelGGL((expand_merge_kernel<LPT, 4>), grid, block, lds, st, a);
    else hipLaunchKernelGGL((expand_merge_kernel<LPT, 16>), grid, block, lds, st, a);
}

hipError_t launch_expand(const ExpandArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(expand_scan_kernel, dim3((unsigned)(a.B * a.F), (unsigned)a.nchunk), dim3(kScanThreads), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int K = a.F * a.nchunk;
    if (K <= 256) launch_merge<1>(a, st);
    else if (K <= 1024) launch_merge<4>(a, st);
    else launch_merge<16>(a, st);
    return hipGetLastError();
}

size_t attach_offer_bytes(const ygg_shape& s) {
    return ((size_t)s.batch * (size_t)s.width * (size_t)s.width * sizeof(Offer) + 255) / 256 * 256;
}
int64_t attach_pool_capacity(const ygg_shape& s) { return (int64_t)s.width * (s.depth > 1 ? s.depth - 1 : 1); }
size_t attach_pool_bytes(const ygg_shape& s) {
    return ((size_t)s.batch * (kPoolHeader + (size_t)attach_pool_capacity(s) * sizeof(Offer)) + 255) / 256 * 256;
}

hipError_t launch_attach(const ExpandArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(expand_scan_kernel, dim3((unsigned)(a.B * a.F), (unsigned)a.nchunk), dim3(kScanThreads), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int per_row = a.nchunk * a.W;
    const dim3 rows((unsigned)(a.B * a.F)), block(256);
    if (per_row <= 256) hipLaunchKernelGGL(attach_rows_kernel<1>, rows, block, 0, st, a);
    else if (per_row <= 1024) hipLaunchKernelGGL(attach_rows_kernel<4>, rows, block, 0, st, a);
    else hipLaunchKernelGGL(attach_rows_kernel<16>, rows, block, 0, st, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int n = a.F * a.W + (a.d == 1 ? 0 : a.W * (a.D - a.d + 1));
    int n2 = 2;
    while (n2 < n) n2 <<= 1;
    const int pool_threads = n2 / 2 < 256 ? 256 : (n2 / 2 > 1024 ? 1024 : n2 / 2);
    hipLaunchKernelGGL(attach_pool_kernel, dim3((unsigned)a.B), dim3(pool_threads), (size_t)n2 * sizeof(Entry), st, a, n2);
    return hipGetLastError();
}

}  // namespace ygg
