// Internal declarations shared by the host API and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ygg.h"

namespace ygg {

constexpr int kMaxNodes = 1024;      // N limit (ancestor bitmasks and per-tree tables live in LDS)
constexpr int kMaxWidth = 64;        // W limit (one wavefront holds a candidate list)
constexpr int kKeyTile = 64;         // split boundaries of the key range are multiples of this

// ---- tree attention ---------------------------------------------------------------------------
// Key index space of sequence b: [0, L_b) are cache rows, [L_b, L_b + N) are the tree's own rows.
// Vector kernel: split s of nsplit covers [s*chunk, min((s+1)*chunk, L_b+N)), chunk = ceil((L_b+N)/nsplit)
// rounded up to kKeyTile.  Matrix-core kernel: split s covers the 64-key tiles floor(s*nt/nsplit) ..
// floor((s+1)*nt/nsplit) - 1 of the sequence's nt tiles.  Every split writes an un-normalised partial
// (m, l, O~) per query row.
struct AttnArgs {
    const void* q;
    const void* k_cache;
    const void* v_cache;
    const void* k_tree;
    const void* v_tree;
    const int32_t* seq_lens;
    const int32_t* parent_idx;
    const float* k_scale;  // [Hkv], both set: K and V hold 8-bit E4M3 codes; both null: plain elements
    const float* v_scale;
    float* part_o;    // [nsplit][B*N*Hq][Dh]  fp32 O~, or (part_half) fp16 O~ / part_c: same indexing, half the bytes
    float* part_ml;   // [nsplit][B*N*Hq][2]   (running max m in scaled-score units, sum l)
    float* part_c;    // [nsplit][B*N*Hq]      part_half only: the row's scale, max |O~| over head_dim
    int32_t* seq_splits;  // [B], balanced batches only: how many runs a sequence's keys fell into (its partials carry split
                          // indices 0 .. n-1), or 0 if one run held it all and its rows are final already
    int32_t part_half;  // 1: the matrix-core kernels' partial outputs (fp16, scaled per row); 0: the vector kernel's fp32 ones
    void* out;
    float* lse;
    int32_t B, N, Hq, Hkv, G, Dh;
    int32_t nsplit, max_seq_len;
    int32_t slots;    // matrix-core kernel, batches: > 0 = workgroups take equal runs of the concatenated key tiles (nsplit = slots)
    int64_t cap;
    float scale;
};

struct AttnPlan {
    int32_t nsplit;
    int32_t use_mfma;       // 1: bf16 matrix-core kernel, 0: fp32 vector kernel
    int32_t waves;          // MFMA kernel: wavefronts per workgroup
    int32_t rblocks;        // MFMA kernel: 32-row blocks per wavefront
    int32_t kshares;        // MFMA kernel: 1, or 2 = pairs of wavefronts split every key tile
    int32_t row_tiles;      // MFMA kernel: workgroups along the N*G query rows of one kv head
    int32_t slots;          // MFMA kernel, batches: equal runs of key tiles per (kv head, row tile); 0 = one sequence per workgroup
    size_t part_o_bytes, part_ml_bytes, part_c_bytes, seq_splits_bytes;
};

AttnPlan plan_attention(const ygg_shape& s);
hipError_t launch_attn_vector(const AttnArgs& a, const AttnPlan& p, int dtype, hipStream_t st);
hipError_t launch_attn_mfma(const AttnArgs& a, const AttnPlan& p, hipStream_t st);
hipError_t launch_attn_combine(const AttnArgs& a, const AttnPlan& p, int dtype, hipStream_t st);

// One-time raising of the dynamic shared-memory limits of every kernel variant of a translation unit (current device).
hipError_t raise_limits_attn_mfma();
hipError_t raise_limits_expand();
int32_t ensure_device_ready();

// ---- equal-growth expansion -------------------------------------------------------------------
struct ExpandPlan {
    int32_t F;            // frontier rows
    int32_t chunk;        // vocab entries per scan workgroup
    int32_t nchunk;
    size_t stat_bytes;    // [B*F][nchunk] {double sumexp; float max; int32 count}
    size_t cand_bytes;    // [B*F][nchunk][W] {float val; int32 idx}
};
struct ExpandArgs {
    const float* logits;
    int32_t* parent_idx;
    int32_t* token_ids;
    float* cum_logprob;
    void* stats;
    void* cands;
    void* offers;      // free attachment only: [B*F][W] {double score; int32 node; int32 token}
    void* pool;        // free attachment only: per sequence {int32 count, pad to 16 B, pool_cap offers}
    int32_t pool_cap;
    int32_t B, D, W, V, N, d, F, chunk, nchunk;
};
ExpandPlan plan_expand(const ygg_shape& s, int32_t d);
hipError_t launch_expand(const ExpandArgs& a, hipStream_t st);
// free attachment: d is the draft step; rows belong to the nodes added at step d-1
size_t attach_offer_bytes(const ygg_shape& s);
int64_t attach_pool_capacity(const ygg_shape& s);
size_t attach_pool_bytes(const ygg_shape& s);
hipError_t launch_attach(const ExpandArgs& a, hipStream_t st);

// ---- verification-width pruning ------------------------------------------------------------------
struct PruneArgs {
    const int32_t* parent_idx;
    const int32_t* token_ids;
    const float* cum_logprob;
    const float* t_verifier;   // [N+1] or null
    int32_t* kept_nodes;
    int32_t* new_parent;
    int32_t* new_token;
    float* expected_len;       // or null
    int32_t* best_width;       // or null
    float t_draft;
    int32_t B, N, w;
};
hipError_t launch_prune(const PruneArgs& a, hipStream_t st);

// ---- debug validator ------------------------------------------------------------------------------
struct ValidateArgs {
    const int32_t* parent_idx;
    const int32_t* seq_lens;
    const int32_t* token_ids;
    const float* logits;
    int32_t* flags;
    int32_t B, N, D, V, max_seq_len, logit_rows;
};
hipError_t launch_validate(const ValidateArgs& a, hipStream_t st);

// ---- acceptance + compaction ------------------------------------------------------------------
struct AcceptPlan {
    int32_t chunk, nchunk;
    size_t part_bytes;    // [B*N][nchunk] {float val; int32 idx}
    size_t oldlen_bytes;  // [B] int32: sequence lengths before the update
};
struct AcceptArgs {
    const float* target_logits;
    const int32_t* target_tokens;
    const int32_t* parent_idx;
    const int32_t* token_ids;
    const void* k_tree;
    const void* v_tree;
    void* k_cache;
    void* v_cache;
    int32_t* seq_lens;
    int32_t* accept_len;
    int32_t* accept_path;
    int32_t* bonus_token;
    void* part;
    int32_t* old_len;
    int32_t B, N, D, V, Hkv, Dh, n_layers, chunk, nchunk, max_seq_len;
    int32_t elem_bytes;
    int64_t cap;
};
AcceptPlan plan_accept(const ygg_shape& s);
hipError_t launch_accept(const AcceptArgs& a, hipStream_t st);

}  // namespace ygg
