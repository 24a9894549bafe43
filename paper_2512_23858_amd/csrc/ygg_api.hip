// Host side of the C ABI: argument validation, launch plans, workspace carving.  No device work
// is done here other than enqueuing kernels on the caller's stream; nothing synchronises.
#include "ygg_internal.h"

#include <atomic>
#include <cmath>
#include <mutex>

namespace ygg {
namespace {

// Launch-plan override for tuning runs (ygg_debug_set_attention_plan): waves << 24 | rblocks << 16 | kshares << 8 in the
// upper word, the forced split count in the lower; 0 = no override.
std::atomic<uint64_t> g_plan_override{0};

// One-time set-up per device: every kernel variant that needs more dynamic shared memory than the default gets its limit
// raised, so that no later call (possibly under stream capture) has to.
constexpr int kMaxDevices = 64;
std::atomic<bool> g_device_ready[kMaxDevices];
std::mutex g_init_mutex;

// Library-owned workspace of ygg_equal_growth_expand_static, for callers that cannot provide one.  Every device
// holds its own copy at its own address (looked up once per device, below); host code only ever uses that
// address.  Nothing in it has to start at zero: every call writes what it reads.
constexpr size_t kStaticScratchBytes = YGG_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
unsigned char* g_scratch_ptr[kMaxDevices];

inline size_t align256(size_t x) { return (x + 255) / 256 * 256; }

bool common_shape_ok(const ygg_shape& s) {
    if (s.batch < 1 || s.batch > 65535) return false;
    if (s.n_q_heads < 1 || s.n_kv_heads < 1 || s.n_q_heads % s.n_kv_heads != 0) return false;
    if (s.depth < 0 || s.width < 1 || s.n_nodes < 1) return false;
    if (s.max_seq_len < 0 || s.kv_capacity < (int64_t)s.max_seq_len + s.depth + 1) return false;
    return true;
}

int32_t check_shape(const ygg_shape* s, bool need_kv, bool need_vocab) {
    if (!s) return YGG_ERR_NULL;
    if (!common_shape_ok(*s)) return YGG_ERR_SHAPE;
    if (s->n_nodes > kMaxNodes || s->width > kMaxWidth) return YGG_ERR_UNSUPPORTED;
    if (need_kv) {
        if (s->kv_dtype != YGG_F32 && s->kv_dtype != YGG_BF16 && s->kv_dtype != YGG_FP8_E4M3) return YGG_ERR_UNSUPPORTED;
        if (s->head_dim != 64 && s->head_dim != 128) return YGG_ERR_UNSUPPORTED;
        if (s->kv_dtype == YGG_FP8_E4M3 && s->head_dim != 128) return YGG_ERR_UNSUPPORTED;
        // the matrix-core kernel takes row maxima before scaling, which needs a positive finite scale
        if (!(s->softmax_scale > 0.f) || !std::isfinite(s->softmax_scale)) return YGG_ERR_SHAPE;
    }
    if (need_vocab && s->vocab < 1) return YGG_ERR_SHAPE;
    return YGG_OK;
}

int32_t check_workspace(const void* ws, size_t have, size_t need) {
    if (need == 0) return YGG_OK;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) != 0 || have < need) return YGG_ERR_WORKSPACE;
    return YGG_OK;
}

}  // namespace

AttnPlan plan_attention(const ygg_shape& s) {
    AttnPlan p{};
    const int64_t rows = (int64_t)s.batch * s.n_nodes * s.n_q_heads;
    const int64_t T = (int64_t)s.max_seq_len + s.n_nodes;
    const int64_t tiles = (T + kKeyTile - 1) / kKeyTile;
    int64_t ns;
    const bool kv8 = s.kv_dtype == YGG_FP8_E4M3;  // K/V as 8-bit codes, Q and O bf16 (head_dim 128 only)
    p.use_mfma = (s.kv_dtype == YGG_BF16 && (s.head_dim == 128 || s.head_dim == 64)) || (kv8 && s.head_dim == 128);
    if (p.use_mfma) {
        // query rows that share one K/V stream, and the workgroup shape that wastes the fewest of them
        const int R = s.n_nodes * (s.n_q_heads / s.n_kv_heads);
        p.rblocks = 1;
        p.kshares = 1;
        // Workgroup shapes, by rows per workgroup: 256 (8 wavefronts), 192 (6), 128 (8 wavefronts in
        // pairs that split every key tile), 64 and 32 (4 and 2 wavefronts in pairs).  More rows per
        // workgroup amortise the K/V tile traffic and the per-tile barrier over more matrix work, so
        // a smaller shape is taken only when it saves a good share of padded rows.
        auto padded = [R](int rw) { return (R + rw - 1) / rw * rw; };
        if (R <= 32) { p.waves = 2; p.kshares = 2; }
        else if (R <= 64) { p.waves = 4; p.kshares = 2; }
        else if (kv8) { p.waves = 4; }  // 8-bit K/V: at most four computing wavefronts, the loaders take the other slots
        else if (R <= 128) { p.waves = 8; p.kshares = 2; }
        else {
            p.waves = 8;
            int best = padded(256);
            if (padded(128) * 100 <= best * 85) { best = padded(128); p.kshares = 2; }
            // 192 rows: two of the four SIMDs carry one wavefront only, so against 256-row workgroups it has to save a
            // fifth of the rows (config 4 with 1344 instead of 1536 padded rows: 210 vs 202 us); against the paired
            // 128-row shape, which meets a barrier every 16 matrix instructions, a tenth is enough (config 3 with 576
            // instead of 640 padded rows and 10 instead of 6 key splits: 27.5 vs 28.1 us per call)
            if (padded(192) * 100 <= best * (p.kshares == 2 ? 92 : 80)) { p.waves = 6; p.kshares = 1; }
        }
        int64_t ns_forced = 0;
        if (const uint64_t ov = g_plan_override.load(std::memory_order_relaxed)) {
            const int w = (int)(ov >> 56), r = (int)(ov >> 48) & 0xff, k = (int)(ov >> 40) & 0xff;
            const bool known = r == 1 && (kv8 ? (w == 4 && (k == 1 || k == 2)) || (w == 2 && k == 2)
                                              : k == 2 ? (w == 2 || w == 4 || w == 8) : (k == 1 && (w == 4 || w == 6 || w == 8)));
            if (known) { p.waves = w; p.rblocks = r; p.kshares = k; }
            ns_forced = (int64_t)(ov & 0xffffffffu);
        }
        const int rw = p.waves / p.kshares * p.rblocks * 32;
        p.row_tiles = (R + rw - 1) / rw;
        // fill the 256 CUs once -- the tile buffers leave room for one workgroup per CU, and a second round of
        // workgroups pays the start-up latency again while more splits add partial-result traffic --
        // with about three key tiles per split at least (config 2's 17 tiles: 5 / 6 / 8 splits measured 16.4 / 15.7 / 16.4 us
        // per layer)
        const int64_t per_split = (int64_t)s.batch * s.n_kv_heads * p.row_tiles;
        ns = 256 / per_split;
        if (ns > (tiles + 2) / 3) ns = (tiles + 2) / 3;
        if (ns_forced) ns = ns_forced < tiles ? ns_forced : tiles;
        // Batches: sequence lengths live on the device and may be ragged, so instead of giving every sequence the same
        // number of splits the key tiles of all sequences are laid end to end and cut into equal runs, one per workgroup
        // of a (kv head, row tile): 256 workgroups in all, each with the same number of tiles whatever the lengths.
        const int64_t streams = (int64_t)s.n_kv_heads * p.row_tiles;
        if (p.kshares == 1 && s.batch >= 2 && s.batch <= 256 && streams <= 128 && !ns_forced) {
            int64_t slots = 256 / streams;
            const int64_t most = (int64_t)s.batch * tiles;   // never more runs than tiles
            if (slots > most) slots = most;
            if (slots > 64) slots = 64;                      // the merge takes at most 64 splits per row
            if (slots >= 2) p.slots = (int32_t)slots;
        }
    } else {
        // vector path: one wavefront per (row, split); aim for ~4096 wavefronts
        ns = (4096 + rows - 1) / rows;
        if (ns > tiles) ns = tiles;
    }
    if (ns < 1) ns = 1;
    if (ns > 64) ns = 64;
    if (!p.use_mfma) {
        // vector kernel: equal chunks rounded up to whole key tiles; drop the splits that rounding leaves empty
        // (the matrix-core kernel deals whole tiles out evenly instead, and no split of at most `tiles` is empty)
        const int64_t chunk = ((T + ns - 1) / ns + kKeyTile - 1) / kKeyTile * kKeyTile;
        ns = (T + chunk - 1) / chunk;
    }
    p.nsplit = p.slots > 0 ? p.slots : (int32_t)ns;   // balanced batches: a sequence may span every run
    // matrix-core kernels: fp16 partial outputs with one fp32 scale per row; vector kernel: fp32 partial outputs
    p.part_o_bytes = align256((size_t)p.nsplit * (size_t)rows * (size_t)s.head_dim * (p.use_mfma ? 2 : 4));
    p.part_ml_bytes = align256((size_t)p.nsplit * (size_t)rows * 2 * sizeof(float));
    p.part_c_bytes = p.use_mfma ? align256((size_t)p.nsplit * (size_t)rows * sizeof(float)) : 0;
    p.seq_splits_bytes = p.slots > 0 ? align256((size_t)s.batch * sizeof(int32_t)) : 0;
    return p;
}

// Raises the shared-memory limits of the current device's kernels once; later calls cost one atomic load.
int32_t ensure_device_ready() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return YGG_ERR_LAUNCH;
    if (g_device_ready[dev].load(std::memory_order_acquire)) return YGG_OK;
    std::lock_guard<std::mutex> lock(g_init_mutex);
    if (g_device_ready[dev].load(std::memory_order_relaxed)) return YGG_OK;
    if (raise_limits_attn_mfma() != hipSuccess || raise_limits_expand() != hipSuccess) return YGG_ERR_LAUNCH;
    void* sp = nullptr;
    if (hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch)) != hipSuccess || !sp) return YGG_ERR_LAUNCH;
    g_scratch_ptr[dev] = static_cast<unsigned char*>(sp);
    g_device_ready[dev].store(true, std::memory_order_release);
    return YGG_OK;
}

}  // namespace ygg

using namespace ygg;

extern "C" {

int32_t ygg_init(void) { return ensure_device_ready(); }

int32_t ygg_debug_set_attention_plan(int32_t waves, int32_t rblocks, int32_t nsplit, int32_t kshares) {
    if (waves < 0 || waves > 255 || rblocks < 0 || rblocks > 255 || kshares < 0 || kshares > 255 || nsplit < 0) return YGG_ERR_SHAPE;
    g_plan_override.store(((uint64_t)waves << 56) | ((uint64_t)rblocks << 48) | ((uint64_t)kshares << 40) | (uint32_t)nsplit,
                          std::memory_order_relaxed);
    return YGG_OK;
}

int32_t ygg_debug_attention_plan(const ygg_shape* s, int32_t* plan) {
    if (int32_t rc = check_shape(s, true, false)) return rc;
    if (!plan) return YGG_ERR_NULL;
    const AttnPlan p = plan_attention(*s);
    plan[0] = p.use_mfma; plan[1] = p.waves; plan[2] = p.kshares; plan[3] = p.row_tiles; plan[4] = p.nsplit;
    return YGG_OK;
}

const char* ygg_status_string(int32_t status) {
    switch (status) {
        case YGG_OK: return "ok";
        case YGG_ERR_NULL: return "null pointer";
        case YGG_ERR_SHAPE: return "inconsistent shape";
        case YGG_ERR_UNSUPPORTED: return "unsupported dtype, head_dim or size";
        case YGG_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case YGG_ERR_LAUNCH: return "kernel launch failed";
        default: return "unknown status";
    }
}

size_t ygg_workspace_bytes(const ygg_shape* s, int32_t op, int32_t n_layers) {
    (void)n_layers;
    if (!s) return 0;
    switch (op) {
        case YGG_OP_ATTENTION: {
            if (check_shape(s, true, false) != YGG_OK) return 0;
            const AttnPlan p = plan_attention(*s);
            return p.part_o_bytes + p.part_ml_bytes + p.part_c_bytes + p.seq_splits_bytes;
        }
        case YGG_OP_EXPAND: {
            if (check_shape(s, false, true) != YGG_OK) return 0;
            const ExpandPlan p = plan_expand(*s, 2);  // the widest frontier
            return p.stat_bytes + p.cand_bytes;
        }
        case YGG_OP_ATTACH: {
            if (check_shape(s, false, true) != YGG_OK) return 0;
            const ExpandPlan p = plan_expand(*s, 2);
            return p.stat_bytes + p.cand_bytes + attach_offer_bytes(*s);
        }
        case YGG_OP_ACCEPT: {
            if (check_shape(s, false, true) != YGG_OK) return 0;
            const AcceptPlan p = plan_accept(*s);
            return p.part_bytes + p.oldlen_bytes;
        }
        default: return 0;
    }
}

static int32_t tree_attention_impl(const ygg_shape* s, const void* q, const void* k_cache, const void* v_cache,
                                   const int32_t* seq_lens, const void* k_tree, const void* v_tree,
                                   const float* k_scale, const float* v_scale,
                                   const int32_t* parent_idx, void* out, float* lse, void* workspace,
                                   size_t workspace_bytes, void* hip_stream, bool main_only = false) {
    if (!q || !k_tree || !v_tree || !seq_lens || !parent_idx || !out) return YGG_ERR_NULL;
    if (s->max_seq_len > 0 && (!k_cache || !v_cache)) return YGG_ERR_NULL;
    // the kernels index query rows with 31 bits and address one sequence's K/V slab with 32-bit byte offsets
    const int64_t elem = s->kv_dtype == YGG_F32 ? 4 : s->kv_dtype == YGG_BF16 ? 2 : 1;
    if ((int64_t)s->batch * s->n_nodes * s->n_q_heads > 0x7fffffffLL) return YGG_ERR_UNSUPPORTED;
    if (s->kv_capacity * s->n_kv_heads * s->head_dim * elem > 0xffffffffLL) return YGG_ERR_UNSUPPORTED;
    const AttnPlan p = plan_attention(*s);
    if (int32_t rc = check_workspace(workspace, workspace_bytes, p.part_o_bytes + p.part_ml_bytes + p.part_c_bytes + p.seq_splits_bytes)) return rc;
    if (int32_t rc = ensure_device_ready()) return rc;

    AttnArgs a{};
    a.q = q; a.k_cache = k_cache; a.v_cache = v_cache; a.k_tree = k_tree; a.v_tree = v_tree;
    a.seq_lens = seq_lens; a.parent_idx = parent_idx; a.k_scale = k_scale; a.v_scale = v_scale;
    a.part_o = static_cast<float*>(workspace);
    a.part_ml = reinterpret_cast<float*>(static_cast<char*>(workspace) + p.part_o_bytes);
    a.part_c = reinterpret_cast<float*>(static_cast<char*>(workspace) + p.part_o_bytes + p.part_ml_bytes);
    a.seq_splits = p.slots > 0 ? reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + p.part_o_bytes + p.part_ml_bytes + p.part_c_bytes) : nullptr;
    a.part_half = p.use_mfma;
    a.out = out; a.lse = lse;
    a.B = s->batch; a.N = s->n_nodes; a.Hq = s->n_q_heads; a.Hkv = s->n_kv_heads;
    a.G = s->n_q_heads / s->n_kv_heads; a.Dh = s->head_dim;
    a.nsplit = p.nsplit; a.max_seq_len = s->max_seq_len; a.cap = s->kv_capacity; a.scale = s->softmax_scale;
    a.slots = p.slots;

    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int out_dtype = s->kv_dtype == YGG_F32 ? YGG_F32 : YGG_BF16;  // element type of Q and O
    hipError_t e = p.use_mfma ? launch_attn_mfma(a, p, st) : launch_attn_vector(a, p, s->kv_dtype, st);
    if (e != hipSuccess) return YGG_ERR_LAUNCH;
    if (main_only) return YGG_OK;
    if (p.use_mfma && p.nsplit == 1) return YGG_OK;  // the kernel wrote the final rows itself
    e = launch_attn_combine(a, p, out_dtype, st);
    return e == hipSuccess ? YGG_OK : YGG_ERR_LAUNCH;
}

int32_t ygg_tree_attention(const ygg_shape* s, const void* q, const void* k_cache, const void* v_cache,
                           const int32_t* seq_lens, const void* k_tree, const void* v_tree,
                           const int32_t* parent_idx, void* out, float* lse, void* workspace,
                           size_t workspace_bytes, void* hip_stream) {
    if (int32_t rc = check_shape(s, true, false)) return rc;
    if (s->kv_dtype == YGG_FP8_E4M3) return YGG_ERR_UNSUPPORTED;  // codes need their scales: ygg_tree_attention_fp8kv
    return tree_attention_impl(s, q, k_cache, v_cache, seq_lens, k_tree, v_tree, nullptr, nullptr, parent_idx, out, lse,
                               workspace, workspace_bytes, hip_stream);
}

int32_t ygg_debug_tree_attention_main(const ygg_shape* s, const void* q, const void* k_cache, const void* v_cache,
                                      const int32_t* seq_lens, const void* k_tree, const void* v_tree,
                                      const int32_t* parent_idx, void* out, float* lse, void* workspace,
                                      size_t workspace_bytes, void* hip_stream) {
    if (int32_t rc = check_shape(s, true, false)) return rc;
    if (s->kv_dtype == YGG_FP8_E4M3) return YGG_ERR_UNSUPPORTED;
    return tree_attention_impl(s, q, k_cache, v_cache, seq_lens, k_tree, v_tree, nullptr, nullptr, parent_idx, out, lse,
                               workspace, workspace_bytes, hip_stream, /*main_only=*/true);
}

int32_t ygg_tree_attention_fp8kv(const ygg_shape* s, const void* q, const void* k_cache, const void* v_cache,
                                 const int32_t* seq_lens, const void* k_tree, const void* v_tree,
                                 const float* k_scale, const float* v_scale, const int32_t* parent_idx, void* out,
                                 float* lse, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (int32_t rc = check_shape(s, true, false)) return rc;
    if (s->kv_dtype != YGG_FP8_E4M3) return YGG_ERR_UNSUPPORTED;
    if (!k_scale || !v_scale) return YGG_ERR_NULL;
    return tree_attention_impl(s, q, k_cache, v_cache, seq_lens, k_tree, v_tree, k_scale, v_scale, parent_idx, out, lse,
                               workspace, workspace_bytes, hip_stream);
}

int32_t ygg_equal_growth_expand(const ygg_shape* s, int32_t d, const float* draft_logits, int32_t* parent_idx,
                                int32_t* token_ids, float* cum_logprob, void* workspace, size_t workspace_bytes,
                                void* hip_stream) {
    if (int32_t rc = check_shape(s, false, true)) return rc;
    if (!draft_logits || !parent_idx || !token_ids || !cum_logprob) return YGG_ERR_NULL;
    if (s->depth < 1 || d < 1 || d > s->depth) return YGG_ERR_SHAPE;
    if ((int64_t)s->n_nodes != 1 + (int64_t)s->depth * s->width) return YGG_ERR_SHAPE;
    const ExpandPlan p = plan_expand(*s, d);
    if ((int64_t)p.F * s->vocab < s->width) return YGG_ERR_SHAPE;
    if ((int64_t)p.F * p.nchunk > 4096) return YGG_ERR_UNSUPPORTED;  // merge holds <= 16 lists per thread
    if ((int64_t)p.F * s->vocab >= 0x7fffffffLL) return YGG_ERR_UNSUPPORTED;  // flat candidate index is 32 bits
    if ((int64_t)s->batch * p.F > 0x7fffffffLL || p.nchunk > 65535) return YGG_ERR_UNSUPPORTED;
    if (int32_t rc = check_workspace(workspace, workspace_bytes, p.stat_bytes + p.cand_bytes)) return rc;
    if (int32_t rc = ensure_device_ready()) return rc;

    ExpandArgs a{};
    a.logits = draft_logits; a.parent_idx = parent_idx; a.token_ids = token_ids; a.cum_logprob = cum_logprob;
    a.stats = workspace;
    a.cands = static_cast<char*>(workspace) + p.stat_bytes;
    a.B = s->batch; a.D = s->depth; a.W = s->width; a.V = s->vocab; a.N = s->n_nodes; a.d = d;
    a.F = p.F; a.chunk = p.chunk; a.nchunk = p.nchunk;
    return launch_expand(a, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? YGG_OK : YGG_ERR_LAUNCH;
}

int32_t ygg_equal_growth_expand_static(const ygg_shape* s, int32_t d, const float* draft_logits, int32_t* parent_idx,
                                       int32_t* token_ids, float* cum_logprob, void* hip_stream) {
    const size_t need = ygg_workspace_bytes(s, YGG_OP_EXPAND, 0);
    if (need > kStaticScratchBytes) return YGG_ERR_WORKSPACE;   // shape too large for the built-in scratch (0: invalid shape, reported below)
    if (int32_t rc = ensure_device_ready()) return rc;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices || !g_scratch_ptr[dev]) return YGG_ERR_LAUNCH;
    return ygg_equal_growth_expand(s, d, draft_logits, parent_idx, token_ids, cum_logprob, g_scratch_ptr[dev],
                                   kStaticScratchBytes, hip_stream);
}

size_t ygg_attach_pool_bytes(const ygg_shape* s) {
    if (!s || check_shape(s, false, true) != YGG_OK || s->depth < 1) return 0;
    return attach_pool_bytes(*s);
}

int32_t ygg_equal_growth_attach(const ygg_shape* s, int32_t t, const float* draft_logits, int32_t* parent_idx,
                                int32_t* token_ids, float* cum_logprob, void* pool, size_t pool_bytes,
                                void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (int32_t rc = check_shape(s, false, true)) return rc;
    if (!draft_logits || !parent_idx || !token_ids || !cum_logprob || !pool) return YGG_ERR_NULL;
    if (s->depth < 1 || t < 1 || t > s->depth) return YGG_ERR_SHAPE;
    if ((int64_t)s->n_nodes != 1 + (int64_t)s->depth * s->width) return YGG_ERR_SHAPE;
    if (s->vocab < s->width) return YGG_ERR_SHAPE;  // every row must be able to offer W tokens
    const ExpandPlan p = plan_expand(*s, t);
    if ((int64_t)p.nchunk * s->width > 4096) return YGG_ERR_UNSUPPORTED;   // a row's chunk lists: <= 16 entries per thread
    if ((int64_t)s->n_nodes * s->vocab > 0xffffffffLL) return YGG_ERR_UNSUPPORTED;  // node*V + token is 32 bits
    if ((int64_t)s->batch * p.F > 0x7fffffffLL || p.nchunk > 65535) return YGG_ERR_UNSUPPORTED;
    // pool + offers are sorted in one workgroup's LDS: at most 4096 entries
    if ((int64_t)p.F * s->width + (int64_t)s->width * (s->depth - t + 1) > 4096) return YGG_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(pool) & 15u) != 0 || pool_bytes < attach_pool_bytes(*s)) return YGG_ERR_WORKSPACE;
    const size_t offer_bytes = attach_offer_bytes(*s);
    if (int32_t rc = check_workspace(workspace, workspace_bytes, p.stat_bytes + p.cand_bytes + offer_bytes)) return rc;
    if (int32_t rc = ensure_device_ready()) return rc;

    ExpandArgs a{};
    a.logits = draft_logits; a.parent_idx = parent_idx; a.token_ids = token_ids; a.cum_logprob = cum_logprob;
    a.stats = workspace;
    a.cands = static_cast<char*>(workspace) + p.stat_bytes;
    a.offers = static_cast<char*>(workspace) + p.stat_bytes + p.cand_bytes;
    a.pool = pool; a.pool_cap = (int32_t)attach_pool_capacity(*s);
    a.B = s->batch; a.D = s->depth; a.W = s->width; a.V = s->vocab; a.N = s->n_nodes; a.d = t;
    a.F = p.F; a.chunk = p.chunk; a.nchunk = p.nchunk;
    return launch_attach(a, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? YGG_OK : YGG_ERR_LAUNCH;
}

int32_t ygg_prune_for_verification(const ygg_shape* s, int32_t w_verify, const int32_t* parent_idx,
                                   const int32_t* token_ids, const float* cum_logprob, const float* t_verifier,
                                   float t_draft, int32_t* kept_nodes, int32_t* new_parent, int32_t* new_token,
                                   float* expected_len, int32_t* best_width, void* hip_stream) {
    if (int32_t rc = check_shape(s, false, false)) return rc;
    if (!parent_idx || !token_ids || !cum_logprob || !kept_nodes || !new_parent || !new_token) return YGG_ERR_NULL;
    if (best_width && !t_verifier) return YGG_ERR_NULL;
    if (w_verify < 1 || w_verify > s->n_nodes) return YGG_ERR_SHAPE;
    if (!(t_draft >= 0.f)) return YGG_ERR_SHAPE;
    PruneArgs a{};
    a.parent_idx = parent_idx; a.token_ids = token_ids; a.cum_logprob = cum_logprob; a.t_verifier = t_verifier;
    a.kept_nodes = kept_nodes; a.new_parent = new_parent; a.new_token = new_token;
    a.expected_len = expected_len; a.best_width = best_width; a.t_draft = t_draft;
    a.B = s->batch; a.N = s->n_nodes; a.w = w_verify;
    return launch_prune(a, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? YGG_OK : YGG_ERR_LAUNCH;
}

int32_t ygg_debug_validate(const ygg_shape* s, const int32_t* parent_idx, const int32_t* seq_lens,
                           const int32_t* token_ids, const float* logits, int32_t logit_rows, int32_t* flags,
                           void* hip_stream) {
    if (int32_t rc = check_shape(s, false, token_ids != nullptr || logits != nullptr)) return rc;
    if (!flags) return YGG_ERR_NULL;
    if (logits && logit_rows < 1) return YGG_ERR_SHAPE;
    if (s->batch > 65535) return YGG_ERR_UNSUPPORTED;
    ValidateArgs a{};
    a.parent_idx = parent_idx; a.seq_lens = seq_lens; a.token_ids = token_ids; a.logits = logits; a.flags = flags;
    a.B = s->batch; a.N = s->n_nodes; a.D = s->depth; a.V = s->vocab; a.max_seq_len = s->max_seq_len;
    a.logit_rows = logit_rows;
    return launch_validate(a, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? YGG_OK : YGG_ERR_LAUNCH;
}

int32_t ygg_accept_and_compact(const ygg_shape* s, int32_t n_layers, const float* target_logits,
                               const int32_t* target_tokens, const int32_t* parent_idx, const int32_t* token_ids,
                               const void* k_tree, const void* v_tree, void* k_cache, void* v_cache,
                               int32_t* seq_lens, int32_t* accept_len, int32_t* accept_path, int32_t* bonus_token,
                               void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (int32_t rc = check_shape(s, n_layers > 0, target_logits != nullptr)) return rc;
    if (n_layers < 0 || n_layers > 65535) return YGG_ERR_SHAPE;
    if ((target_logits == nullptr) == (target_tokens == nullptr)) return YGG_ERR_NULL;
    if (!parent_idx || !token_ids || !seq_lens || !accept_len || !accept_path || !bonus_token) return YGG_ERR_NULL;
    if (n_layers > 0 && (!k_tree || !v_tree || !k_cache || !v_cache)) return YGG_ERR_NULL;
    const AcceptPlan p = plan_accept(*s);
    if ((int64_t)s->batch * s->n_nodes > 0x7fffffffLL || p.nchunk > 65535) return YGG_ERR_UNSUPPORTED;
    if (int32_t rc = check_workspace(workspace, workspace_bytes, p.part_bytes + p.oldlen_bytes)) return rc;

    AcceptArgs a{};
    a.target_logits = target_logits; a.target_tokens = target_tokens;
    a.parent_idx = parent_idx; a.token_ids = token_ids;
    a.k_tree = k_tree; a.v_tree = v_tree; a.k_cache = k_cache; a.v_cache = v_cache;
    a.seq_lens = seq_lens; a.accept_len = accept_len; a.accept_path = accept_path; a.bonus_token = bonus_token;
    a.part = workspace;
    a.old_len = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + p.part_bytes);
    a.B = s->batch; a.N = s->n_nodes; a.D = s->depth; a.V = s->vocab; a.Hkv = s->n_kv_heads; a.Dh = s->head_dim;
    a.n_layers = n_layers; a.chunk = p.chunk; a.nchunk = p.nchunk; a.max_seq_len = s->max_seq_len;
    a.elem_bytes = s->kv_dtype == YGG_F32 ? 4 : s->kv_dtype == YGG_BF16 ? 2 : 1; a.cap = s->kv_capacity;
    return launch_accept(a, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? YGG_OK : YGG_ERR_LAUNCH;
}

}  // extern "C"
