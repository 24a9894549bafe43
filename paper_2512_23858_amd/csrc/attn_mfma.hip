// Tree-masked verify attention on the gfx950 matrix cores (bf16 storage, head_dim 128 or 64).
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
//   online softmax     a lane owns one query row: 16 scores in registers; base-2 exponentials
//                      against a per-row reference that moves rarely (no row maximum on the
//                      common path)
//   O^T += V^T . P^T   A = V^T through the LDS transpose read (ds_read_b64_tr_b16), B = P^T,
//                      which is exactly the accumulator layout of S^T packed to bf16
// The tree's own keys are the tail of the key range; their ancestor mask comes from per-node
// bitmasks built in LDS from parent_idx.
//
// The same kernel also serves K/V stored as 8-bit E4M3 codes (template flag KV8): extra loading
// wavefronts widen the codes to bf16 while filling the LDS tiles, everything else is shared.
#include "attn_common.h"

#include <cstdlib>
#include <type_traits>

namespace ygg {
namespace {

using namespace attn;

// 16-byte load from global memory proper (a pointer chosen between two arrays would otherwise be
// loaded through the generic path, whose completion also counts as an LDS event).
// Streaming hint: the codes are used once (a plain streaming read of the same size measures 6.9 TB/s with it, 6.1 without).
__device__ __forceinline__ u32x4 global_load16(uint64_t gaddr) {
    return __builtin_nontemporal_load(reinterpret_cast<const __attribute__((address_space(1))) u32x4*>(gaddr));
}

// Sixteen E4M3 codes (memory order) -> sixteen bf16; exact, the format has 3 mantissa bits.  One
// conversion instruction per pair of codes (scale operand 1.0).
__device__ __forceinline__ void e4m3x16_to_bf16(const u32x4& raw, uint4& first8, uint4& last8) {
    const uint32_t w[4] = {raw[0], raw[1], raw[2], raw[3]};
    uint32_t o[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        o[2 * i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[i], 1.0f, false));     // bytes 0, 1
        o[2 * i + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[i], 1.0f, true));  // bytes 2, 3
    }
    first8 = make_uint4(o[0], o[1], o[2], o[3]);
    last8 = make_uint4(o[4], o[5], o[6], o[7]);
}

// NW wavefronts, RB 32-row blocks per wavefront, KT keys per tile, KS key shares: with KS = 2 the
// wavefronts pair up on the same rows and each takes one of the two 32-key blocks of every tile (a
// tree of few nodes has too few rows to occupy a workgroup otherwise); the pair's (m, l, O~) are
// merged through LDS before the result is written.
//
// KV8: K and V are stored as 8-bit E4M3 codes with one scale per kv head.  The codes are widened
// to bf16 on their way into LDS (exactly), so tiles, operand reads and matrix work are those of
// the bf16 kernel; the scales fold into the softmax scale and into the final normalisation.  The
// direct-to-LDS path cannot convert, so the workgroup gets four extra wavefronts that do nothing but
// load codes into registers (four tiles ahead; eight measured no faster), widen them and store the
// rows into the tile buffers; the NW computing wavefronts never touch global K/V.  Both kinds meet
// at the same one barrier per tile.
//
// NT: the direct-to-LDS tile fills carry the streaming hint (the host sets it when a K/V stream has one
// row tile, i.e. is read by a single workgroup; with several row tiles the re-reads are meant to hit in L2).
//
// BAL: balanced batches (see the segment loop below); a separate instantiation, so that the single-segment variants
// carry none of its loop state.
//
// DHT: head_dim, 128 or 64 (bf16 K/V only for 64).  Everything below counts in k-steps of 16 and output blocks of 32
// head_dim positions, and a direct-to-LDS instruction brings 1024 / ROWB rows.
template <int NW, int RB, int KT, int KS, bool KV8, bool NT, bool BAL = false, int DHT = 128>
__global__ __launch_bounds__((NW + (KV8 ? 4 : 0)) * 64, (RB == 1 && !KV8 ? 2 : 1)) void attn_mfma_kernel(AttnArgs a, int RT, int S) {
    static_assert(!BAL || KS == 1, "balanced batches: plain 32-row wavefronts only");
    static_assert(DHT == 128 || (DHT == 64 && !KV8), "head_dim 64: bf16 K/V only");
    constexpr int DH = DHT;
    constexpr int ROWB = 2 * DH;                                 // bytes of one K or V row in LDS
    constexpr int NS = DH / 16;                                  // k-steps of S^T = K.Q^T
    constexpr int NDB = DH / 32;                                 // 32-wide blocks of head_dim in O^T
    constexpr int SLOTS = ROWB / 16;                             // 16-byte slots per row = lanes that fill one row
    constexpr int RPI = 1024 / ROWB;                             // rows one direct-to-LDS wave-instruction brings
    static_assert(KS == 1 || (KS == 2 && NW % 2 == 0 && KT == 64), "key shares: one block of the tile each");
    constexpr int NLD = KV8 ? 4 : 0;                             // loading wavefronts (KV8 only)
    constexpr int NSET = 4;                                      // register sets (tiles in flight) per loader
    constexpr int THREADS = (NW + NLD) * 64;
    static_assert(!KV8 || NW <= 4, "loading wavefronts share the SIMDs with at most one computing wavefront each");
    constexpr int NRW = NW / KS;                                 // wavefronts along the rows
    constexpr int RW = NRW * RB * 32;                            // query rows per workgroup
    constexpr int TILEB = KT * ROWB;                             // bytes of one K (or V) tile
    constexpr int NBUF = 3;  // tiles are prefetched two ahead
    // wavefronts that issue tile fills (a power of two, so that each issues the same number per tile)
    constexpr int FILLERS = NW >= 8 ? 8 : NW >= 4 ? 4 : NW >= 2 ? 2 : 1;
    constexpr int PT = 2 * (KT / RPI) / FILLERS;  // direct-to-LDS loads per filling wavefront and tile
    static_assert((KT / RPI) % FILLERS == 0, "every filling wavefront issues the same number of loads");
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* k_s = smem;                                   // [NBUF][KT][ROWB]
    unsigned char* v_s = smem + NBUF * TILEB;                    // [NBUF][KT][ROWB]
    uint32_t* anc_s = reinterpret_cast<uint32_t*>(smem + 2 * NBUF * TILEB);  // [local node][aw], then parent[N]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform by construction
    const int n = lane & 31, g2 = lane >> 5;
    const bool is_loader = KV8 && wave >= NW;      // wave-uniform
    const int wrow = KS == 1 ? wave : wave % NRW;  // position along the rows (computing wavefronts)
    const int kh = KS == 1 ? 0 : wave / NRW;       // which block of every tile (KS = 2)

    // workgroup id -> (stream sigma = (b, kv head, split), row tile); sigma % 8 picks the XCD
    const int wg = blockIdx.x;
    const int xcd = wg & 7;
    const int rt = (wg >> 3) % RT;
    const int sigma = (wg / (8 * RT)) * 8 + xcd;
    if (sigma >= S) return;
    const int R = a.N * a.G;
    const int row_base = rt * RW;
    const int64_t rows_total = (int64_t)a.B * a.N * a.Hq;

    // Which (sequence, key range) segments does this workgroup serve?
    //   classic   one segment: sigma = (sequence, kv head, split); the split is one of nsplit equal chunks of that
    //             sequence's own key range.
    //   balanced  (a.slots > 0, batches) sigma = (kv head, slot).  The sequences' 64-key tiles are laid end to end and
    //             cut into a.slots runs of equal length; the workgroup serves its run, i.e. the tail of one sequence,
    //             whole short sequences, the head of another, one segment after the other.  Every workgroup then has the
    //             same number of tiles whatever the mix of lengths (a ragged batch otherwise takes as long as its longest
    //             sequence).  Segment number (slot - first slot of the sequence) is the split index of its partials;
    //             nsplit = a.slots bounds it.  A sequence that lies inside one slot is written out directly.
    constexpr bool balanced = BAL;
    int hk, b_first, b_last, slot = 0, run_lo = 0, run_hi = 0, tiles_all = 0, tiles_before = 0, nruns = 1;
    if constexpr (!balanced) {
        hk = (sigma / a.nsplit) % a.Hkv;
        b_first = b_last = sigma / (a.nsplit * a.Hkv);
    } else {
        hk = sigma / a.slots;
        slot = sigma % a.slots;
        auto tiles_of = [&](int bb) {
            int Lb = a.seq_lens[bb];
            Lb = Lb < 0 ? 0 : (Lb > a.max_seq_len ? a.max_seq_len : Lb);
            return (Lb + a.N + kKeyTile - 1) / kKeyTile;
        };
        for (int bb = 0; bb < a.B; ++bb) tiles_all += tiles_of(bb);
        // never more runs than tiles (the host sized the grid for the longest lengths the shape allows): every run then
        // holds a tile, so the runs a sequence falls into are consecutive and its split indices have no gaps
        nruns = min(a.slots, tiles_all);
        run_lo = slot < nruns ? (int)((int64_t)slot * tiles_all / nruns) : 0;
        run_hi = slot < nruns ? (int)((int64_t)(slot + 1) * tiles_all / nruns) : 0;
        // first and last sequence with tiles inside [run_lo, run_hi)
        b_first = 0;
        int acc = 0;
        while (b_first < a.B - 1 && acc + tiles_of(b_first) <= run_lo) acc += tiles_of(b_first++);
        tiles_before = acc;  // tiles of the sequences before b_first
        b_last = b_first;
        acc += tiles_of(b_first);
        while (b_last < a.B - 1 && acc < run_hi) acc += tiles_of(++b_last);
        if (run_lo >= run_hi) b_last = b_first - 1;  // a workgroup beyond the last run: nothing to do
    }
    // the run that holds tile x of the concatenation: the largest s with floor(s * tiles_all / nruns) <= x
    auto slot_of_tile = [&](int x) { return (int)((((int64_t)x + 1) * nruns - 1) / tiles_all); };
    // all of this is the same in every lane: keep it in scalar registers (the vector registers are all spoken for)
    auto uni = [](int v) { return __builtin_amdgcn_readfirstlane(v); };
    if constexpr (balanced) {
        hk = uni(hk); b_first = uni(b_first); b_last = uni(b_last); run_lo = uni(run_lo); run_hi = uni(run_hi);
        tiles_before = uni(tiles_before); tiles_all = uni(tiles_all); nruns = uni(nruns);
    } else {
        b_last = b_first;
    }

    for (int b = b_first; b <= b_last; ++b) {
    if (balanced && b != b_first) __syncthreads();   // the previous segment's tile buffers and masks are free again
    // rows of this lane: block rb of this wave -> row_base + (wrow*RB + rb)*32 + n
    int rg_of[RB];       // global row index (b, node, q head) or -1; fits 31 bits (checked on the host)
    int node_of[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int row = row_base + (wrow * RB + rb) * 32 + n;
        const int i = min(row, R - 1) / a.G;
        const int g = min(row, R - 1) % a.G;
        node_of[rb] = i;
        rg_of[rb] = row < R && !is_loader ? (b * a.N + i) * a.Hq + hk * a.G + g : -1;
    }

    // (issued before the sequence length is first needed: the rows do not depend on it, and the length is a
    // dependent load from device memory at the head of every workgroup's critical path)
    // Q as the B operand of S^T = K.Q^T: lane (n, g2) holds Q[row n][16 s + 8 g2 .. +8) for s = 0..NS-1
    bf16x8 qreg[RB][NS];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        if (rg_of[rb] >= 0) {
            const bf16x8* qp = reinterpret_cast<const bf16x8*>(static_cast<const uint16_t*>(a.q) + (int64_t)rg_of[rb] * DH + 8 * g2);
#pragma unroll
            for (int s = 0; s < NS; ++s) qreg[rb][s] = qp[2 * s];
        } else {
#pragma unroll
            for (int s = 0; s < NS; ++s) qreg[rb][s] = bf16x8{};
        }
    }

    int L = a.seq_lens[b];
    L = L < 0 ? 0 : (L > a.max_seq_len ? a.max_seq_len : L);
    const int Tk = L + a.N;
    int k0, k1, split;
    bool direct = a.nsplit == 1;   // this segment is the whole sequence: final rows are written here
    if constexpr (!balanced) {
        // the sequence's own 64-key tiles, dealt out as evenly as whole tiles allow (splits differ by at most one tile)
        split = sigma % a.nsplit;
        const int nt = (Tk + kKeyTile - 1) / kKeyTile;
        k0 = (int)((int64_t)split * nt / a.nsplit) * kKeyTile;
        k1 = min(Tk, (int)((int64_t)(split + 1) * nt / a.nsplit) * kKeyTile);
    } else {
        const int nt = (Tk + kKeyTile - 1) / kKeyTile;
        const int t0 = max(run_lo, tiles_before) - tiles_before, t1 = min(run_hi, tiles_before + nt) - tiles_before;
        const int s_first = slot_of_tile(tiles_before), s_last = slot_of_tile(tiles_before + nt - 1);
        tiles_before += nt;
        k0 = t0 * kKeyTile;
        k1 = min(Tk, t1 * kKeyTile);
        if (t0 >= t1) continue;   // (cannot happen for b_first .. b_last; keeps a wrong split index out of the workspace)
        split = slot - s_first;
        direct = s_first == s_last;
        // the workgroup of kv head 0 and row tile 0 that holds the sequence's first tile tells the merge how many runs the
        // sequence fell into (the run boundaries are the same for every kv head and row tile)
        if (slot == s_first && hk == 0 && rt == 0 && tid == 0) a.seq_splits[b] = direct ? 0 : s_last - s_first + 1;
    }
    if constexpr (balanced) {
        k0 = uni(k0); k1 = uni(k1); split = uni(split); L = uni(L);
        direct = uni(direct) != 0;
    }
    [&]() {   // one segment; wavefronts that have nothing more to do leave through `return`

    if (k0 >= k1) {  // empty split (uniform over the workgroup): mark the partials as absent
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
            if (rg_of[rb] >= 0 && g2 == 0 && kh == 0) {
                float* pml = a.part_ml + ((int64_t)split * rows_total + rg_of[rb]) * 2;
                pml[0] = -INFINITY;
                pml[1] = 0.f;
            }
        return;
    }

    // ancestor bitmasks of the nodes this workgroup's rows belong to
    const int aw = (a.N + 31) >> 5;
    const int i_first = row_base / a.G;
    const int i_last = min(R - 1, row_base + RW - 1) / a.G;
    const bool has_tree_keys = k1 > L;  // uniform over the workgroup
    int32_t* parent_s = reinterpret_cast<int32_t*>(anc_s + (i_last - i_first + 1) * aw);

    // slab bases of this (sequence, kv head): wave-uniform, pinned to scalar registers
    constexpr int EB = KV8 ? 1 : 2;  // bytes of a stored K/V element
    auto uniform_ptr = [](const unsigned char* p) {
        const uint64_t v = (uint64_t)p;
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
        return reinterpret_cast<const unsigned char*>(((uint64_t)hi << 32) | lo);
    };
    const unsigned char* kc = uniform_ptr(static_cast<const unsigned char*>(a.k_cache) + ((int64_t)b * a.cap * a.Hkv + hk) * (DH * EB));
    const unsigned char* vc = uniform_ptr(static_cast<const unsigned char*>(a.v_cache) + ((int64_t)b * a.cap * a.Hkv + hk) * (DH * EB));
    const unsigned char* kt = uniform_ptr(static_cast<const unsigned char*>(a.k_tree) + ((int64_t)b * a.N * a.Hkv + hk) * (DH * EB));
    const unsigned char* vt = uniform_ptr(static_cast<const unsigned char*>(a.v_tree) + ((int64_t)b * a.N * a.Hkv + hk) * (DH * EB));

    // Direct-to-LDS tile fill: wave-instruction `inst` brings rows RPI*inst .. RPI*inst+RPI-1 of the tile;
    // lane l lands at byte 1024*inst + 16*l, i.e. row RPI*inst + l/SLOTS, slot' = l%SLOTS, and therefore
    // fetches the slot that the row's permutation maps there.  Rows past the end of the split fetch
    // the split's last key again: their scores are masked, and their V rows are finite, so that a
    // zero weight times them stays zero.  Every filling wavefront issues exactly PT loads per tile.
    const uint32_t k_lds = (uint32_t)(size_t)(__attribute__((address_space(3))) void*)k_s;  // LDS byte addresses
    const uint32_t v_lds = (uint32_t)(size_t)(__attribute__((address_space(3))) void*)v_s;
    // Addresses are a wave-uniform 64-bit base (one sequence's K or V slab) plus a 32-bit byte offset;
    // the host checks that a slab stays below 4 GiB.
    const uint32_t tok_bytes = (uint32_t)a.Hkv * DH * EB;
    // per-lane byte offsets of this wavefront's loads inside a tile of cache rows (fast path below)
    constexpr int FPW = (KT / RPI) / FILLERS;  // wave-instructions per filling wavefront, tile and tensor
    uint32_t fill_k[FPW], fill_v[FPW];
#pragma unroll
    for (int it = 0; it < FPW; ++it) {
        const int row = RPI * (wave + it * FILLERS) + lane / SLOTS;
        const int slotp = lane % SLOTS;
        fill_k[it] = (uint32_t)row * tok_bytes + 16 * (slotp ^ (row & (SLOTS - 1)));
        fill_v[it] = (uint32_t)row * tok_bytes + 16 * (slotp ^ ((row & (NDB - 1)) << 2));
    }
    auto fill_tile = [&](int buf, int tile_base) {
        if (wave >= FILLERS) return;
        const uint32_t kdst0 = k_lds + buf * TILEB + wave * 1024, vdst0 = v_lds + buf * TILEB + wave * 1024;
        if (tile_base + KT <= min(L, k1)) {  // a whole tile of cache rows: the tile's base joins the scalar pointer,
            // the per-lane offsets are constants of the kernel (no vector arithmetic per load)
            const unsigned char* kc_t = uniform_ptr(kc + (size_t)((uint32_t)tile_base * tok_bytes));
            const unsigned char* vc_t = uniform_ptr(vc + (size_t)((uint32_t)tile_base * tok_bytes));
#pragma unroll
            for (int it = 0; it < FPW; ++it) {
                dma_load16<NT>(kc_t, fill_k[it], __builtin_amdgcn_readfirstlane(kdst0 + it * FILLERS * 1024));
                dma_load16<NT>(vc_t, fill_v[it], __builtin_amdgcn_readfirstlane(vdst0 + it * FILLERS * 1024));
            }
            return;
        }
#pragma unroll
        for (int it = 0; it < FPW; ++it) {
            const int inst = wave + it * FILLERS;
            const int row = RPI * inst + lane / SLOTS;
            const int slotp = lane % SLOTS;
            const int j0 = tile_base + RPI * inst;   // wave-uniform first key of these RPI rows
            const int j = min(tile_base + row, k1 - 1);
            const uint32_t kcol = 16 * (slotp ^ (row & (SLOTS - 1)));
            const uint32_t vcol = 16 * (slotp ^ ((row & (NDB - 1)) << 2));
            const uint32_t kdst = __builtin_amdgcn_readfirstlane(kdst0 + it * FILLERS * 1024);
            const uint32_t vdst = __builtin_amdgcn_readfirstlane(vdst0 + it * FILLERS * 1024);
            if (j0 + RPI <= L) {                     // cache rows only (uniform branch)
                const uint32_t off = (uint32_t)j * tok_bytes;
                dma_load16<NT>(kc, off + kcol, kdst);
                dma_load16<NT>(vc, off + vcol, vdst);
            } else if (j0 >= L) {                    // tree rows only
                const uint32_t off = (uint32_t)(j - L) * tok_bytes;
                dma_load16<NT>(kt, off + kcol, kdst);
                dma_load16<NT>(vt, off + vcol, vdst);
            } else {                                 // the rows straddle the end of the prefix
                const bool in_cache = j < L;
                const uint32_t off = (uint32_t)(in_cache ? j : j - L) * tok_bytes;
                const void* kb = in_cache ? (const void*)kc : (const void*)kt;
                const void* vb = in_cache ? (const void*)vc : (const void*)vt;
                dma_load16_flat<NT>(static_cast<const unsigned char*>(kb) + off + kcol, kdst);
                dma_load16_flat<NT>(static_cast<const unsigned char*>(vb) + off + vcol, vdst);
            }
        }
    };

    // KV8 loaders.  A tile is 16 wave-instructions of 16-byte loads: instruction g < 8 covers rows
    // 8g .. 8g+7 of K, instruction 8 + g the same rows of V, eight lanes per row and sixteen codes per
    // lane.  Loader lw takes instructions lw, lw + NLD, ... (NLD divides 8, so whether a load is K's or
    // V's is known at compile time).  Rows past the end of the split repeat
    // its last key, as above; every address is a cache row below L or a tree row below N whatever
    // tile_base is, so a load may be issued for a tile that does not exist.
    constexpr int LPT = 16 / (NLD > 0 ? NLD : 16);  // loads per loader and tile
    struct Stage {
        u32x4 d[LPT];
    };
    const int lw = wave - NW;
    // per-lane constants of this loader's LPT loads: byte offset inside a tile of cache rows, and the
    // two LDS byte offsets (relative to buffer 0) its sixteen widened values go to
    uint32_t ld_off[LPT], st_off0[LPT], st_off1[LPT];
#pragma unroll
    for (int it = 0; it < LPT; ++it) {
        const bool is_v = it * NLD >= 8;  // known once the loop is unrolled
        const int row = 8 * ((lw + it * NLD) & 7) + (lane >> 3);
        const int c2 = 2 * (lane & 7);    // this lane's two 16-byte slots: c2, c2 + 1
        const int x = is_v ? ((row & 3) << 2) : (row & 15);
        ld_off[it] = (uint32_t)row * tok_bytes + 16 * (lane & 7);
        st_off0[it] = (is_v ? NBUF * TILEB : 0) + row * ROWB + 16 * (c2 ^ x);
        st_off1[it] = (is_v ? NBUF * TILEB : 0) + row * ROWB + 16 * ((c2 + 1) ^ x);
    }
    const int cache_end = min(L, k1);
    auto stage_issue = [&](Stage& sg, int tile_base) {
        if (tile_base + KT <= cache_end) {  // a whole tile of cache rows: uniform base + constant per-lane offsets
            const uint64_t kb = (uint64_t)kc + (uint64_t)((uint32_t)tile_base * tok_bytes);
            const uint64_t vb = (uint64_t)vc + (uint64_t)((uint32_t)tile_base * tok_bytes);
#pragma unroll
            for (int it = 0; it < LPT; ++it) sg.d[it] = global_load16((it * NLD >= 8 ? vb : kb) + ld_off[it]);
            return;
        }
#pragma unroll
        for (int it = 0; it < LPT; ++it) {
            const bool is_v = it * NLD >= 8;
            const int row = 8 * ((lw + it * NLD) & 7) + (lane >> 3);
            const int j = min(tile_base + row, k1 - 1);
            const bool in_cache = j < L;
            const uint32_t off = (uint32_t)(in_cache ? j : j - L) * tok_bytes + 16 * (lane & 7);
            const uint64_t base = is_v ? (in_cache ? (uint64_t)vc : (uint64_t)vt) : (in_cache ? (uint64_t)kc : (uint64_t)kt);
            sg.d[it] = global_load16(base + off);
        }
    };
    // widens the staged codes and stores them where the direct-to-LDS path would have put the bf16 row
    auto stage_write = [&](const Stage& sg, int buf) {
        unsigned char* base = smem + buf * TILEB;
#pragma unroll
        for (int it = 0; it < LPT; ++it) {
            uint4 w0, w1;
            e4m3x16_to_bf16(sg.d[it], w0, w1);
            *reinterpret_cast<uint4*>(base + st_off0[it]) = w0;
            *reinterpret_cast<uint4*>(base + st_off1[it]) = w1;
        }
    };

    f32x16 o[RB][NDB];
    float m_ref[RB], l_run[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        m_ref[rb] = -INFINITY;
        l_run[rb] = 0.f;
#pragma unroll
        for (int db = 0; db < NDB; ++db) o[rb][db] = f32x16{};
    }
    // KV8: K = k_scale * code value, so the scale (positive) joins the softmax scale
    const float c_scale = a.scale * kLog2e * (KV8 ? a.k_scale[hk] : 1.f);

    // ---- the pipeline over 32-key blocks ---------------------------------------------------------
    // Each wavefront alternates between a vector phase (LDS operand reads issued, then the softmax
    // of block j) and a matrix phase (O^T += V^T.P^T of block j, then S^T of block j+1), so that the
    // two wavefronts resident on a SIMD keep its matrix pipe and its vector pipe busy in turn.
    //
    // Softmax uses a per-row reference m_ref, set at the first block in which the row sees a key and
    // raised only when a block's weights p = 2^(x - m_ref) sum to more than kWeightSumLimit: floating
    // point keeps the relative precision of the weights (bf16) and of the sums (fp32) whatever their
    // magnitude, so the common path takes no row maximum at all, and O and l -- which carry the same
    // reference -- are rescaled only in that rare, wave-uniform branch.  Scores far below the
    // reference underflow to weight 0, which is what they are worth next to the key that set it.  The
    // result O / l and lse = m_ref ln 2 + ln l do not depend on the reference.
    const int j16 = lane & 15;
    // K operand of step s: row n, slot 2s+g2 -> slot' = (2s+g2) ^ (n % SLOTS) = 2*(s ^ (n % SLOTS)>>1) + (g2 ^ (n&1))
    const int k_lane_off = n * ROWB + 16 * (g2 ^ (n & 1));
    const int k_pair_xor = ((n & (SLOTS - 1)) >> 1) << 5;
    // V operand: row z = 4*g2 + j16/4 (+ multiples of 8), 32-byte pair 2*db + (lane/16)%2 -> pair' = pair ^ 2*(z % NDB)
    const int v_z = 4 * g2 + (j16 >> 2);
    const int v_lane_off = v_z * ROWB + 8 * (j16 & 3);
    const int v_pair = (lane >> 4) & 1;
    const int v_px = (v_z & (NDB - 1)) << 1;

    auto read_k = [&](int buf, int kb, bf16x8 (&ka)[NS]) {
        const unsigned char* kbuf = k_s + buf * TILEB + kb * 32 * ROWB + k_lane_off;
#pragma unroll
        for (int s = 0; s < NS; ++s) ka[s] = *reinterpret_cast<const bf16x8*>(kbuf + ((32 * s) ^ k_pair_xor));
    };
    // lane j of a 16-lane group addresses key row (j/4), dh 4*(j%4); the transpose read hands each
    // lane four keys of one dh, i.e. the A operand of O^T += V^T.P^T
    auto read_v = [&](int buf, int kb, i16x8 (&va)[NDB][2]) {
        const unsigned char* vbuf = v_s + buf * TILEB + kb * 32 * ROWB + v_lane_off;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int m2 = 0; m2 < 2; ++m2) {
                const unsigned char* p = vbuf + (16 * m2) * ROWB + 32 * ((2 * db + v_pair) ^ v_px);
                const i16x4 lo = lds_read_tr16(p);
                const i16x4 hi = lds_read_tr16(p + 8 * ROWB);
                va[db][m2] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
    };
    auto qk = [&](const bf16x8 (&ka)[NS], f32x16 (&st)[RB]) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) st[rb] = f32x16{};
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
                st[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[s], qreg[rb][s], st[rb], 0, 0, 0);
    };
    auto pv = [&](const i16x8 (&va)[NDB][2], const i16x8 (&pb)[RB][2]) {
#pragma unroll
        for (int m2 = 0; m2 < 2; ++m2)
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int rb = 0; rb < RB; ++rb)
                    o[rb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8, va[db][m2]), __builtin_bit_cast(bf16x8, pb[rb][m2]), o[rb][db], 0, 0, 0);
    };
    // blk0 = first key of the 32-key block; clean = the block's tile lies wholly inside the prefix
    auto softmax = [&](f32x16 (&st)[RB], i16x8 (&pb)[RB][2], int blk0, bool clean) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            if (!clean) {
                uint32_t okmask = 0xffffffffu;  // bit u: key u of this block is visible to this lane's row
                const int bt = blk0 - L;        // tree-node index of the block's first key (negative inside the prefix)
                const uint32_t* w = anc_s + (node_of[rb] - i_first) * aw;
                if (bt >= 0) {
                    const int wi = bt >> 5;
                    const uint64_t w0 = wi < aw ? w[wi] : 0u;
                    const uint64_t w1 = wi + 1 < aw ? w[wi + 1] : 0u;
                    okmask = (uint32_t)(((w1 << 32) | w0) >> (bt & 31));
                } else if (bt > -32) {          // block straddles the end of the prefix
                    okmask = (0xffffffffu >> (32 + bt)) | (w[0] << (-bt));
                }
                const int left = k1 - blk0;     // keys of this block inside the split
                if (left < 32) okmask &= left <= 0 ? 0u : (0xffffffffu >> (32 - left));
                okmask >>= 4 * g2;  // this half-lane's keys are now bits 8*(v/4) + v%4
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    if (!((okmask >> (8 * (v >> 2) + (v & 3))) & 1u)) st[rb][v] = -INFINITY;
            }
            // weights of this lane's 16 keys relative to the reference ms, packed for the P.V product; returns their sum
            auto weights = [&](float ms) __attribute__((always_inline)) {
                float ps = 0.f;
#pragma unroll
                for (int m2 = 0; m2 < 2; ++m2) {
                    union { bf16x2 h[4]; i16x8 v; } pk;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float p0 = __builtin_amdgcn_exp2f(fmaf(st[rb][8 * m2 + 2 * e], c_scale, -ms));
                        const float p1 = __builtin_amdgcn_exp2f(fmaf(st[rb][8 * m2 + 2 * e + 1], c_scale, -ms));
                        ps += p0;
                        ps += p1;
                        const f32x2 pr = {p0, p1};
                        pk.h[e] = __builtin_convertvector(pr, bf16x2);  // v_cvt_pk_bf16_f32, round to nearest even
                    }
                    pb[rb][m2] = pk.v;
                }
                return ps;
            };
            // Common case: the row has a reference and no weight comes out large -- no maximum is taken at all.
            bool move = __any(m_ref[rb] == -INFINITY);  // a row without a reference yet (nothing visible so far)
            float ps = 0.f;
            if (!move) {
                ps = weights(m_ref[rb]);
                move = __any(!(ps <= kWeightSumLimit));  // scores that outgrew the reference
            }
            if (move) {
                // Rare, wave-uniform: set or raise the reference from the block's row maxima, rescale what has been summed.
                float mt = st[rb][0];
#pragma unroll
                for (int v = 1; v < 16; ++v) mt = fmaxf(mt, st[rb][v]);
                mt *= c_scale;  // c_scale > 0: the maximum commutes with the scaling
                const float row_max = fmaxf(mt, __shfl_xor(mt, 32));
                const bool raise = row_max > m_ref[rb] + kRescaleGap;  // same answer in both half-lanes of a row
                const float alpha = raise ? __builtin_amdgcn_exp2f(m_ref[rb] - row_max) : 1.f;
                if (raise) m_ref[rb] = row_max;
                l_run[rb] *= alpha;
#pragma unroll
                for (int db = 0; db < NDB; ++db)
#pragma unroll
                    for (int v = 0; v < 16; ++v) o[rb][db][v] *= alpha;
                ps = weights(m_ref[rb] == -INFINITY ? 0.f : m_ref[rb]);  // the scores are still in st
            }
            l_run[rb] += ps;
        }
    };

    static_assert(KT == 64, "the block pipeline below is written for two 32-key blocks per tile");
    const int ntiles = (k1 - k0 + KT - 1) / KT;
    const int clean_end = min(L, k1);
    auto build_masks = [&]() {  // every wavefront of the workgroup takes part
        if (!has_tree_keys) return;
        // one coalesced read of parent_idx; the walks up the tree then stay in LDS
        const int32_t* parent = a.parent_idx + (int64_t)b * a.N;
        for (int t = tid; t < a.N; t += THREADS) parent_s[t] = parent[t];
        if constexpr (KV8) lds_barrier(); else __syncthreads();
        for (int t = tid; t <= i_last - i_first; t += THREADS) {
            uint32_t* w = anc_s + t * aw;
            for (int x = 0; x < aw; ++x) w[x] = 0;
            int guard = 0;
            for (int c = i_first + t; c >= 0 && c < a.N && guard < a.N; c = parent_s[c], ++guard) w[c >> 5] |= 1u << (c & 31);
        }
    };

    // KV8, loading wavefronts.  Tile tau travels in register set tau % NSET; iteration t (after the
    // barrier that retires tile t) stores tile t+3 into tile t's buffer and reuses the set for the
    // loads of tile t+3+NSET.  Every staged load is issued whether or not its tile exists: the
    // number of loads in flight at each point is then the same on every path, and the compiler's
    // wait for one register set leaves the NSET-1 younger sets in flight.  The barriers match those
    // of the computing wavefronts one for one.
    if constexpr (KV8) {
        if (is_loader) {
            Stage stage[NSET];
            static_for<0, NSET>([&](auto i) { stage_issue(stage[i.value], k0 + i.value * KT); });
            build_masks();
            static_for<0, 3>([&](auto i) {
                stage_write(stage[i.value], i.value);
                stage_issue(stage[i.value], k0 + (NSET + i.value) * KT);
            });
            lds_barrier();  // tiles 0..2 are in LDS for everybody; anc_s published
            int lbuf = 0;
            auto lstep = [&](int t, Stage& sg) {
                lds_barrier();
                if (t + 3 < ntiles) stage_write(sg, lbuf);
                stage_issue(sg, k0 + (t + 3 + NSET) * KT);
                lbuf = lbuf + 1 == NBUF ? 0 : lbuf + 1;
            };
            int t = 0;
            for (; t + NSET - 1 < ntiles; t += NSET)
                static_for<0, NSET>([&](auto i) { lstep(t + i.value, stage[(i.value + 3) % NSET]); });
            static_for<0, NSET - 1>([&](auto i) {
                if (t + i.value < ntiles) lstep(t + i.value, stage[(i.value + 3) % NSET]);
            });
            if constexpr (KS == 2) {  // the merge of the key shares has two more workgroup barriers
                __syncthreads();
                __syncthreads();
            }
            return;
        }
    }

    // prologue of the computing wavefronts: up to three tiles go into flight at once (direct-to-LDS
    // path); the ancestor masks are built meanwhile
    if constexpr (!KV8) {
#pragma unroll
        for (int i = 0; i < 3; ++i)
            if (i < ntiles) fill_tile(i, k0 + i * KT);
    }
    build_masks();
    constexpr int PT2 = 2 * PT > 63 ? 63 : 2 * PT;  // a single filling wavefront has 64 loads in flight: wait for one more
    if constexpr (KV8) {
        lds_barrier();
    } else {
        if (ntiles >= 3) dma_wait_keep<PT2>(); else if (ntiles == 2) dma_wait_keep<PT>(); else dma_wait_keep<0>();
        __syncthreads();  // tile 0 has landed for everybody; anc_s published
    }

    // After the barrier of iteration t every wavefront is done with tile t, whose buffer then receives
    // tile t+3: by direct-to-LDS loads that the barrier of iteration t+2 awaits, or (KV8) from the loaders.
    auto turn = [&](int t, int buf, int tile_base) {
        if constexpr (KV8) {
            lds_barrier();
        } else {
            if (t + 2 < ntiles) dma_wait_keep<PT>(); else dma_wait_keep<0>();  // tile t+1 landed, t+2 may be in flight
            __syncthreads();
            if (t + 3 < ntiles) fill_tile(buf, tile_base + 3 * KT);  // tile t's buffer: every wavefront has read it
        }
    };

    // One barrier per tile (inside turn).
    bf16x8 ka[NS];
    i16x8 va[NDB][2];
    f32x16 st[RB];
    i16x8 pb[RB][2];
    // Tile t lives in buffer t % NBUF.  The loop is unrolled NBUF-fold with the buffer index a compile-time constant, so
    // that every LDS operand address is a loop-invariant per-lane register plus an immediate (no address arithmetic
    // per block).
    // A wavefront whose 32 rows all lie beyond the last query row (the padding of the last row tile) only keeps the
    // barriers and its share of the tile fills company: its matrix and vector work would be spent on zeros, and what it
    // does not burn the others get back as clock (config 5: 3 of 16 wavefronts per K/V stream, call 172.4 -> 165.9 us).
    // Wavefronts 0 to 4 always work, so that one SIMD keeps its pair and the workgroup keeps the pace of the other row
    // tiles of its K/V stream: a workgroup that runs ahead of them fetches every tile from HBM a second time (config 4
    // with all seven idle wavefronts of its last row tile skipping: 221 MB fetched per launch instead of 149).  Only the
    // 256-row shape takes the branch: the six-wavefront shape measured 1.5 % slower with it.
    constexpr bool kSkipIdle = NW == 8 && KS == 1;
    const bool has_rows = !kSkipIdle || wave <= 4 || __builtin_amdgcn_readfirstlane((int)(row_base + wrow * RB * 32 < R)) != 0;
    auto body = [&](int t, auto bufc) __attribute__((always_inline)) {
        constexpr int buf = decltype(bufc)::value;
        constexpr int buf_next = buf + 1 == NBUF ? 0 : buf + 1;
        const int tile_base = k0 + t * KT;
        const bool clean = tile_base + KT <= clean_end;
        if (!has_rows) {
            turn(t, buf, tile_base);
            return;
        }
        if constexpr (KS == 1) {
            // block 0 of the tile
            read_v(buf, 0, va);
            __builtin_amdgcn_sched_barrier(0);
            softmax(st, pb, tile_base, clean);
            read_k(buf, 1, ka);
            __builtin_amdgcn_sched_barrier(0);
            pv(va, pb);
            qk(ka, st);
            __builtin_amdgcn_sched_barrier(0);
            // block 1 of the tile; the next tile becomes visible before its first K operand is read
            read_v(buf, 1, va);
            __builtin_amdgcn_sched_barrier(0);
            softmax(st, pb, tile_base + 32, clean);
        } else {
            read_v(buf, kh, va);
            __builtin_amdgcn_sched_barrier(0);
            softmax(st, pb, tile_base + 32 * kh, clean);
        }
        turn(t, buf, tile_base);
        if (t + 1 < ntiles) read_k(buf_next, kh, ka);
        __builtin_amdgcn_sched_barrier(0);
        pv(va, pb);
        if (t + 1 < ntiles) qk(ka, st);
        __builtin_amdgcn_sched_barrier(0);
    };
    if (has_rows) {
        read_k(0, kh, ka);
        qk(ka, st);
    }
    static_assert(NBUF == 3, "the unrolling below names the three buffers");
    int t = 0;
    for (; t + 3 <= ntiles; t += 3) {
        body(t, IntC<0>{});
        body(t + 1, IntC<1>{});
        body(t + 2, IntC<2>{});
    }
    if (t < ntiles) {
        body(t, IntC<0>{});
        if (t + 1 < ntiles) body(t + 1, IntC<1>{});
    }
    if constexpr (KS == 2) {
        // Merge of the two key shares of a row block.  Both carry O~ and l relative to their own
        // reference m_ref; the share of block 1 hands its state over through the (now idle) tile
        // buffers, lane for lane, and the share of block 0 rescales both to the larger reference.
        constexpr int XR = 16 * NDB + 2;  // a lane's accumulators, then m and l
        float* xch = reinterpret_cast<float*>(smem) + wrow * (RB * XR * 64) + lane;  // [wrow][rb][XR][64 lanes]
        __syncthreads();  // every wavefront is done with the tiles
        if (kh == 1) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                float* x = xch + rb * XR * 64;
#pragma unroll
                for (int db = 0; db < NDB; ++db)
#pragma unroll
                    for (int v = 0; v < 16; ++v) x[(16 * db + v) * 64] = o[rb][db][v];
                x[(XR - 2) * 64] = m_ref[rb];
                x[(XR - 1) * 64] = l_run[rb];
            }
        }
        __syncthreads();
        if (kh == 1) return;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const float* x = xch + rb * XR * 64;
            const float m1 = x[(XR - 2) * 64], l1 = x[(XR - 1) * 64];
            const float mm = fmaxf(m_ref[rb], m1);
            // a share that saw no visible key has m = -inf, l = 0, O~ = 0: weight 0 keeps it out
            const float w0 = m_ref[rb] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_ref[rb] - mm);
            const float w1 = m1 == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m1 - mm);
            m_ref[rb] = mm;
            l_run[rb] = l_run[rb] * w0 + l1 * w1;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[rb][db][v] = o[rb][db][v] * w0 + x[(16 * db + v) * 64] * w1;
        }
    }

    // epilogue: lane (n, g2) holds, for its row, dh = 32 db + 8 (v/4) + 4 g2 + (v%4)
    const float v_unit = KV8 ? a.v_scale[hk] : 1.f;  // KV8: V = v_scale * code value
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const float l_tot = l_run[rb] + __shfl_xor(l_run[rb], 32);
        if (rg_of[rb] < 0) continue;
        if (direct) {
            const float inv = v_unit / l_tot;
            uint16_t* op = static_cast<uint16_t*>(a.out) + (int64_t)rg_of[rb] * DH + 4 * g2;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    uint2 w;
                    w.x = pack_bf16x2(o[rb][db][4 * vq] * inv, o[rb][db][4 * vq + 1] * inv);
                    w.y = pack_bf16x2(o[rb][db][4 * vq + 2] * inv, o[rb][db][4 * vq + 3] * inv);
                    *reinterpret_cast<uint2*>(op + 32 * db + 8 * vq) = w;
                }
            if (a.lse && g2 == 0) a.lse[rg_of[rb]] = m_ref[rb] * kLn2 + logf(l_tot);
        } else {
            // Partial outputs travel as fp16 relative to the row's largest magnitude c (kept in fp32 beside m and l):
            // half the traffic of fp32 here and in the merge, an error of at most 2^-12 c per element whatever the
            // range of V (bf16 partials would cost up to a whole bf16 ulp of the merged row, which outputs of
            // magnitude 4 cannot afford inside 2e-2).  Streaming stores: the partials are read once, by the merge,
            // and leaving them dirty in L2 only lengthens the write-back at the end of this kernel.
            float rmax = 0.f;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) rmax = fmaxf(rmax, fabsf(o[rb][db][v]));
            rmax = fmaxf(rmax, __shfl_xor(rmax, 32));
            const float c = fmaxf(rmax, 1e-30f);
            const float inv_c = 1.f / c;
            // The two lanes of a row hold alternating groups of four head_dim positions; swapping halves between them
            // (v_permlane32_swap) leaves each with eight consecutive ones, so a store covers 32 contiguous bytes of a row.
            _Float16* po = reinterpret_cast<_Float16*>(a.part_o) + ((int64_t)split * rows_total + rg_of[rb]) * DH + 8 * g2;
            u32x4 w[NDB][2];
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int vp = 0; vp < 2; ++vp) {
                    const f32x4 ve = {o[rb][db][8 * vp] * inv_c, o[rb][db][8 * vp + 1] * inv_c,
                                      o[rb][db][8 * vp + 2] * inv_c, o[rb][db][8 * vp + 3] * inv_c};
                    const f32x4 vo = {o[rb][db][8 * vp + 4] * inv_c, o[rb][db][8 * vp + 5] * inv_c,
                                      o[rb][db][8 * vp + 6] * inv_c, o[rb][db][8 * vp + 7] * inv_c};
                    const u32x2 he = __builtin_bit_cast(u32x2, __builtin_convertvector(ve, f16x4));
                    const u32x2 ho = __builtin_bit_cast(u32x2, __builtin_convertvector(vo, f16x4));
                    const auto s0 = __builtin_amdgcn_permlane32_swap(he[0], ho[0], false, false);
                    const auto s1 = __builtin_amdgcn_permlane32_swap(he[1], ho[1], false, false);
                    w[db][vp] = u32x4{s0[0], s1[0], s0[1], s1[1]};
                }
            // the stores of a row leave back to back: neighbouring 32-byte pieces then combine into whole lines
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int vp = 0; vp < 2; ++vp)
                    __builtin_nontemporal_store(w[db][vp], reinterpret_cast<u32x4*>(po + 32 * db + 16 * vp));
            __builtin_amdgcn_sched_barrier(0);
            if (g2 == 0) a.part_c[(int64_t)split * rows_total + rg_of[rb]] = c * v_unit;  // KV8: V = v_scale * code value
            if (g2 == 0) {
                float* pml = a.part_ml + ((int64_t)split * rows_total + rg_of[rb]) * 2;
                pml[0] = m_ref[rb] * kLn2;  // natural-log units of the scaled scores
                pml[1] = l_tot;
            }
        }
    }
    }();   // one segment
    }      // segments of this workgroup
}

// Largest dynamic shared memory any shape asks for: six 16 KiB tiles (head_dim 128), ancestor masks of up to 257 nodes x
// 32 words, and the parent table of 1024 nodes.  Every variant's limit is raised to it once per device.
constexpr size_t kMaxSmem = (size_t)2 * 3 * 64 * 256 + (size_t)257 * 32 * 4 + 1024 * 4;

template <int NW, int RB, int KT, int KS, bool KV8, bool NT, bool BAL = false, int DHT = 128>
hipError_t raise_variant() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(attn_mfma_kernel<NW, RB, KT, KS, KV8, NT, BAL, DHT>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxSmem);
}

template <int NW, int RB, int KT, int KS, bool KV8, bool NT, bool BAL = false, int DHT = 128>
hipError_t launch_variant(const AttnArgs& a, const AttnPlan& p, hipStream_t st) {
    const int S = a.slots > 0 ? a.Hkv * a.slots : a.B * a.Hkv * a.nsplit;   // K/V streams, each read by RT workgroups
    const int RT = p.row_tiles;
    const int S8 = (S + 7) / 8 * 8;
    const int RW = NW / KS * RB * 32;
    const int nodes_local = (RW + a.G - 1) / a.G + 1;
    // three K and three V tile buffers, the ancestor bitmasks and the parent table
    const size_t smem = (size_t)2 * 3 * KT * (2 * DHT) + (size_t)nodes_local * ((a.N + 31) / 32) * 4 + (size_t)a.N * 4;
    auto kern = attn_mfma_kernel<NW, RB, KT, KS, KV8, NT, BAL, DHT>;
    const unsigned threads = (NW + (KV8 ? 4 : 0)) * 64;  // KV8: plus the four loading wavefronts
    if (a.Dh != DHT) return hipErrorInvalidValue;
    if (smem > kMaxSmem) return hipErrorInvalidValue;  // cannot happen for N <= 1024: checked again for the sake of the launch
    hipLaunchKernelGGL(kern, dim3((unsigned)(S8 * RT)), dim3(threads), smem, st, a, RT, S);
    return hipGetLastError();
}

template <int NW, int RB, int KT, int KS, bool KV8 = false, int DHT = 128>
hipError_t launch_cfg(const AttnArgs& a, const AttnPlan& p, hipStream_t st) {
    if constexpr (KV8) {
        if constexpr (KS == 1) {
            if (a.slots > 0) return launch_variant<NW, RB, KT, KS, true, false, true>(a, p, st);
        }
        if (a.slots > 0) return hipErrorInvalidValue;
        return launch_variant<NW, RB, KT, KS, true, false>(a, p, st);  // the loaders' register loads always stream
    } else {
        if constexpr (KS == 1) {
            if (a.slots > 0)
                return p.row_tiles == 1 ? launch_variant<NW, RB, KT, KS, false, true, true, DHT>(a, p, st)
                                        : launch_variant<NW, RB, KT, KS, false, false, true, DHT>(a, p, st);
        }
        if (a.slots > 0) return hipErrorInvalidValue;
        return p.row_tiles == 1 ? launch_variant<NW, RB, KT, KS, false, true, false, DHT>(a, p, st)
                                : launch_variant<NW, RB, KT, KS, false, false, false, DHT>(a, p, st);
    }
}

// the six workgroup shapes of the bf16 kernel for one head_dim
template <int DHT>
hipError_t launch_shape(const AttnArgs& a, const AttnPlan& p, hipStream_t st) {
    switch (p.waves * 10 + p.kshares) {
        case 41: return launch_cfg<4, 1, 64, 1, false, DHT>(a, p, st);
        case 61: return launch_cfg<6, 1, 64, 1, false, DHT>(a, p, st);
        case 81: return launch_cfg<8, 1, 64, 1, false, DHT>(a, p, st);
        case 22: return launch_cfg<2, 1, 64, 2, false, DHT>(a, p, st);
        case 42: return launch_cfg<4, 1, 64, 2, false, DHT>(a, p, st);
        case 82: return launch_cfg<8, 1, 64, 2, false, DHT>(a, p, st);
        default: return hipErrorInvalidValue;
    }
}

template <int DHT>
hipError_t raise_shapes() {
    hipError_t e = hipSuccess;
    auto both = [&](auto nw, auto ks) {
        if (e == hipSuccess) e = raise_variant<decltype(nw)::value, 1, 64, decltype(ks)::value, false, false, false, DHT>();
        if (e == hipSuccess) e = raise_variant<decltype(nw)::value, 1, 64, decltype(ks)::value, false, true, false, DHT>();
        if constexpr (decltype(ks)::value == 1) {
            if (e == hipSuccess) e = raise_variant<decltype(nw)::value, 1, 64, 1, false, false, true, DHT>();
            if (e == hipSuccess) e = raise_variant<decltype(nw)::value, 1, 64, 1, false, true, true, DHT>();
        }
    };
    both(IntC<4>{}, IntC<1>{}); both(IntC<6>{}, IntC<1>{}); both(IntC<8>{}, IntC<1>{});
    both(IntC<2>{}, IntC<2>{}); both(IntC<4>{}, IntC<2>{}); both(IntC<8>{}, IntC<2>{});
    return e;
}

}  // namespace

hipError_t raise_limits_attn_mfma() {
    hipError_t e = raise_shapes<128>();
    if (e == hipSuccess) e = raise_shapes<64>();
    if (e == hipSuccess) e = raise_variant<2, 1, 64, 2, true, false>();
    if (e == hipSuccess) e = raise_variant<4, 1, 64, 2, true, false>();
    if (e == hipSuccess) e = raise_variant<4, 1, 64, 1, true, false>();
    if (e == hipSuccess) e = raise_variant<4, 1, 64, 1, true, false, true>();
    return e;
}

hipError_t launch_attn_mfma(const AttnArgs& a, const AttnPlan& p, hipStream_t st) {
    if (p.rblocks != 1) return hipErrorInvalidValue;
    if (a.k_scale || a.v_scale) {  // K/V held as E4M3 codes (head_dim 128)
        if (!a.k_scale || !a.v_scale || a.Dh != 128) return hipErrorInvalidValue;
        switch (p.waves * 10 + p.kshares) {  // computing wavefronts; four loaders on top
            case 22: return launch_cfg<2, 1, 64, 2, true>(a, p, st);
            case 42: return launch_cfg<4, 1, 64, 2, true>(a, p, st);
            case 41: return launch_cfg<4, 1, 64, 1, true>(a, p, st);
            default: return hipErrorInvalidValue;
        }
    }
    if (a.Dh == 128) return launch_shape<128>(a, p, st);
    if (a.Dh == 64) return launch_shape<64>(a, p, st);
    return hipErrorInvalidValue;
}

}  // namespace ygg
