/*
 * ygg.h -- C ABI of the MI355X (gfx950) tree-verification library.
 *
 * Three operations make up one verification step of a static-shape, equal-growth
 * draft token tree (Yggdrasil, arXiv 2512.23858):
 *
 *   ygg_equal_growth_expand   one draft step of the Equal-Growth Tree (Sec. 4.2)
 *   ygg_tree_attention        tree-masked attention of the verifier pass (Sec. 2, Sec. 4.2)
 *   ygg_accept_and_compact    acceptance of the matching draft path (Sec. 1, Sec. 5) and the
 *                             TokenTree's K/V bookkeeping (Sec. 6), done on the device
 *
 * Around them: ygg_equal_growth_attach (the same draft step with free attachment, Sec. 4.2),
 * ygg_prune_for_verification (verification-width pruning, Sec. 4.2), and ygg_debug_validate, which
 * reports the data-dependent contract violations that the three calls above do not check.
 *
 * Conventions shared by every call
 *   - All tensor pointers are DEVICE pointers owned by the caller; the ygg_shape struct is HOST
 *     memory and is only read during the call.  The library never allocates, frees or keeps
 *     device memory; scratch space is the caller's `workspace` (size from ygg_workspace_bytes,
 *     256-byte aligned, contents undefined on entry and on return).  Calls that may run
 *     concurrently need workspaces of their own.
 *   - Calls only enqueue kernels on `hip_stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and never synchronise, so a sequence of calls can be captured in a HIP
 *     graph.  All shapes are static: nothing on the host depends on device data.  This is the
 *     static-runtime property the paper asks of the drafting algorithm (Sec. 3, Sec. 4.2).
 *     The first launching call on a device (or ygg_init) raises the dynamic shared-memory limits
 *     of the library's kernels, once, under a lock; call ygg_init before capturing if the first
 *     call of a process would otherwise be made under stream capture.  That per-device flag is
 *     the library's only state.
 *   - The return code reports host-checkable errors only (null pointers, inconsistent shape,
 *     unsupported type, workspace too small, launch failure).  Data-dependent contract
 *     violations (parent_idx not topological, seq_lens[b] > max_seq_len, NaN logits) are
 *     undefined behaviour, except that no kernel reads or writes outside the buffers as
 *     described by ygg_shape; ygg_debug_validate reports them.
 *   - Tensors are dense, row-major, token-major: [.., token, head, head_dim].
 *   - Tree layout: node 0 is the root (the last confirmed token, whose K/V is not yet in the
 *     cache); parent_idx[b][0] = -1 and 0 <= parent_idx[b][i] < i.  For the expansion call the
 *     tree is level structured: depth d (1..D) occupies nodes 1+(d-1)W .. dW, N = 1 + D*W.
 *     Attention and acceptance accept any topologically ordered tree of N nodes whose depth
 *     does not exceed `depth`.
 */
#ifndef YGG_H
#define YGG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    YGG_OK = 0,
    YGG_ERR_NULL = 1,        /* a required pointer is NULL */
    YGG_ERR_SHAPE = 2,       /* inconsistent or out-of-range shape field / argument */
    YGG_ERR_UNSUPPORTED = 3, /* dtype / head_dim / size outside what the kernels implement */
    YGG_ERR_WORKSPACE = 4,   /* workspace missing, misaligned or too small */
    YGG_ERR_LAUNCH = 5       /* the HIP runtime refused a launch */
} ygg_status;

typedef enum {
    YGG_F32 = 0,
    YGG_BF16 = 1,
    YGG_FP8_E4M3 = 2   /* K and V (cache and tree) as 8-bit E4M3 codes, Q and O bf16; head_dim 128;
                          accepted by ygg_tree_attention_fp8kv and ygg_accept_and_compact only */
} ygg_dtype;

typedef enum { YGG_OP_ATTENTION = 0, YGG_OP_EXPAND = 1, YGG_OP_ACCEPT = 2, YGG_OP_ATTACH = 3 } ygg_op;

typedef struct {
    int32_t batch;         /* B >= 1 sequences, one tree each */
    int32_t n_q_heads;     /* Hq */
    int32_t n_kv_heads;    /* Hkv, Hq % Hkv == 0; query head h uses kv head h / (Hq/Hkv) */
    int32_t head_dim;      /* Dh: 64 or 128 */
    int32_t depth;         /* D >= 0: number of draft steps = maximum node depth */
    int32_t width;         /* W: nodes added per draft step (1..64) */
    int32_t n_nodes;       /* N (1..1024); must equal 1 + D*W for ygg_equal_growth_expand */
    int32_t vocab;         /* V (only used by expand / accept) */
    int32_t kv_dtype;      /* ygg_dtype of Q, K, V and O (see YGG_FP8_E4M3 for the mixed case) */
    float softmax_scale;   /* multiplies q.k; typically 1/sqrt(Dh); must be finite and > 0 where K/V are used */
    int64_t kv_capacity;   /* token slots per sequence in the cache, >= max_seq_len + D + 1 */
    int32_t max_seq_len;   /* host-known upper bound of seq_lens[b] (sizes the launch grids) */
} ygg_shape;

/* Bytes of workspace the given operation needs for this shape (0 if the shape is invalid). */
size_t ygg_workspace_bytes(const ygg_shape *shape, int32_t op /* ygg_op */, int32_t n_layers);

/* Static, human-readable name of a status code. */
const char *ygg_status_string(int32_t status);

/*
 * Optional: prepares the current device (raises the kernels' shared-memory limits).  Every launching
 * call does the same on first use; calling it up front keeps that out of a stream capture.  Thread safe.
 * Returns YGG_ERR_LAUNCH when there is no usable device.
 */
int32_t ygg_init(void);

/*
 * Tree-masked verify attention for one layer (paper Sec. 2 "Source of Improvements": the
 * speculative tokens are verified in one parallel pass under a sequence-level mask; Sec. 4.2,
 * last paragraph: the mask follows the tree's causal dependency).
 *
 * For every sequence b, node i and query head h (kv head g = h / (Hq/Hkv)):
 *     keys   J(i) = cache rows 0 .. seq_lens[b]-1  U  tree rows {i, parent[i], ..., 0}
 *     out[b,i,h,:] = sum_j softmax_j(softmax_scale * q[b,i,h,:] . k_j[g,:]) * v_j[g,:]
 *     lse[b,i,h]   = ln sum_j exp(softmax_scale * q . k_j)            (optional)
 * Scores, softmax and accumulation are fp32; bf16 inputs use bf16 matrix instructions with the
 * softmax weights rounded to bf16 before the value product.
 *
 *   q          [B,N,Hq,Dh]      kv_dtype
 *   k_cache    [B,cap,Hkv,Dh]   kv_dtype, rows [0,seq_lens[b]) valid, others never read
 *   v_cache    [B,cap,Hkv,Dh]
 *   seq_lens   [B] int32        0 <= seq_lens[b] <= max_seq_len
 *   k_tree     [B,N,Hkv,Dh]     K/V of the tree's own tokens; must not overlap the cache
 *   v_tree     [B,N,Hkv,Dh]
 *   parent_idx [B,N] int32
 *   out        [B,N,Hq,Dh]      kv_dtype (written)
 *   lse        [B,N,Hq] fp32    written, or NULL
 * Inputs are read-only; out/lse/workspace must not alias them.
 */
int32_t ygg_tree_attention(const ygg_shape *shape,
                           const void *q, const void *k_cache, const void *v_cache,
                           const int32_t *seq_lens, const void *k_tree, const void *v_tree,
                           const int32_t *parent_idx, void *out, float *lse,
                           void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The same attention with K and V stored in 8 bits (shape->kv_dtype == YGG_FP8_E4M3).  The paper
 * leaves the K/V precision open (Sec. 6: the TokenTree owns the K/V tensors); this variant halves
 * the bytes of the prefix, which is what bounds verification of small trees over long or batched
 * prefixes.  A stored element is an E4M3 code (1 sign, 4 exponent bits with bias 7, 3 mantissa
 * bits, subnormals, no infinities; codes 0x7f and 0xff are NaN and must not occur) and stands for
 *     K = k_scale[g] * value(code),   V = v_scale[g] * value(code)        (g = kv head)
 * The codes are widened to bf16 exactly, so the result is that of ygg_tree_attention on the
 * dequantised K/V with the scales applied in fp32.
 *
 *   q, out     [B,N,Hq,Dh] bf16;  lse [B,N,Hq] fp32 or NULL
 *   k_cache, v_cache [B,cap,Hkv,Dh] uint8;  k_tree, v_tree [B,N,Hkv,Dh] uint8
 *   k_scale, v_scale [Hkv] fp32 device, finite and > 0
 * Everything else as for ygg_tree_attention; workspace size is ygg_workspace_bytes(ATTENTION).
 */
int32_t ygg_tree_attention_fp8kv(const ygg_shape *shape,
                                 const void *q, const void *k_cache, const void *v_cache,
                                 const int32_t *seq_lens, const void *k_tree, const void *v_tree,
                                 const float *k_scale, const float *v_scale,
                                 const int32_t *parent_idx, void *out, float *lse,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * One draft step d (1..D) of the Equal-Growth Tree (paper Sec. 4.2 "Draft Width Selection":
 * exactly W_draft leaves are grown per draft step, at the positions with the largest path-wise
 * gain, using generation probabilities as acceptance surrogates).  Candidates are the
 * (frontier node p, token v) pairs of the previous depth, F = 1 row (the root) for d = 1 and
 * F = W rows otherwise:
 *     score(p,v) = cum_logprob[frontier p] + log_softmax(draft_logits[b,p,:])[v]
 * The W best candidates (higher score first; equal scores: lower p*V+v first) become nodes
 * 1+(d-1)W .. dW in that order: parent_idx <- frontier node, token_ids <- v, cum_logprob <-
 * score rounded to fp32.  Scores are evaluated in fp64.
 *
 *   draft_logits [B,F,V] fp32    row p belongs to node 1+(d-2)W+p (node 0 for d = 1)
 *   parent_idx, token_ids [B,N] int32 and cum_logprob [B,N] fp32: in/out; depth d-1 entries are
 *   read, depth d entries written.  The caller initialises node 0 (parent -1, cum 0).
 * Requires N == 1 + D*W and F*V >= W.
 */
int32_t ygg_equal_growth_expand(const ygg_shape *shape, int32_t d, const float *draft_logits,
                                int32_t *parent_idx, int32_t *token_ids, float *cum_logprob,
                                void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * ygg_equal_growth_expand for callers that cannot allocate or carry a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid allocation.  Same operation, same kernels, same results; the
 * scratch is a fixed array inside the library's device image (YGG_STATIC_SCRATCH_BYTES per GPU, held until the
 * process ends), so the call allocates nothing and takes no workspace argument.  Shapes whose
 * ygg_workspace_bytes(shape, YGG_OP_EXPAND) exceeds YGG_STATIC_SCRATCH_BYTES are rejected with
 * YGG_ERR_WORKSPACE.  All calls on one GPU share that array: calls that may overlap on one GPU (different
 * streams, concurrent graphs) race and must use ygg_equal_growth_expand with workspaces of their own.
 */
#define YGG_STATIC_SCRATCH_BYTES (4u << 20)
int32_t ygg_equal_growth_expand_static(const ygg_shape *shape, int32_t d, const float *draft_logits,
                                       int32_t *parent_idx, int32_t *token_ids, float *cum_logprob,
                                       void *hip_stream);

/*
 * Equal growth with free attachment: draft step t (1..D) of the Equal-Growth Tree as the paper words
 * it (Sec. 4.2 "Draft Width Selection": every step grows exactly W_draft leaves, and they may hang
 * anywhere in the partial tree, at the positions with the largest path-wise gain).  Reading: every
 * node, once the drafter has run on it, offers its W most probable tokens (larger logit first, equal
 * logits: lower token first), each scored cum_logprob[node] + log_softmax(row)[token] in fp64; the
 * pool holds the offers not yet taken.  Step t adds the offers of the nodes grown at step t-1 (the
 * root for t = 1; F = 1 or W rows of draft_logits, in node order), orders the pool by (score
 * descending, node*V + token ascending) and turns the first W entries into nodes 1+(t-1)W .. tW in
 * that order: parent_idx <- offering node, token_ids, cum_logprob <- score rounded to fp32.  Node
 * depth no longer equals the step; it never exceeds t.
 *
 *   draft_logits [B,F,V] fp32; parent_idx, token_ids [B,N] int32 and cum_logprob [B,N] fp32 in/out
 *   pool         device memory owned by the caller and carried from step to step, at least
 *                ygg_attach_pool_bytes(shape) bytes, 16-byte aligned.  Step 1 initialises it.  Per
 *                sequence: int32 count, 12 bytes padding, then W*max(D-1,1) records {double score;
 *                int32 node; int32 token}, the first `count` valid and ordered best first.  After
 *                step t it holds the best W*(D-t) untaken offers: an entry of rank r cannot be
 *                taken before r/W more steps, so nothing else can ever become a node.
 * Requires N == 1 + D*W, V >= W, N*V < 2^32 and W*F + W*(D-t+1) <= 4096.
 */
size_t ygg_attach_pool_bytes(const ygg_shape *shape);
int32_t ygg_equal_growth_attach(const ygg_shape *shape, int32_t t, const float *draft_logits,
                                int32_t *parent_idx, int32_t *token_ids, float *cum_logprob,
                                void *pool, size_t pool_bytes,
                                void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Verification-width pruning (paper Sec. 4.2 "Verification Width Pruning": after drafting, the
 * maximum-value subtree with W_verify nodes is kept for verification; Eq. 3 with every term but
 * W_verify fixed decides the width).  The value of a node is the probability that its whole path is
 * accepted with the drafter's probabilities as surrogates, exp(cum_logprob[i]) (the root counts 1:
 * the bonus token); the sum over a kept set estimates the accepted length.
 *
 *   w_verify     HOST integer 1..N: the static width of the verifier pass that follows
 *   parent_idx, token_ids [B,N] int32, cum_logprob [B,N] fp32: the drafted tree, with
 *                cum_logprob[child] <= cum_logprob[parent] (true of sums of log-probabilities; the
 *                kept set is the w_verify largest values, which is the optimal connected subtree
 *                under exactly that condition)
 *   t_verifier   [N+1] fp32 device, t_verifier[n] > 0 = verifier latency with n tokens; NULL if
 *                best_width is NULL.  t_draft >= 0: total drafting latency, same unit (host scalar)
 *   kept_nodes   [B,w_verify] int32 out: kept original indices, ascending (still topological)
 *   new_parent   [B,w_verify] int32 out: parent in the renumbered tree (-1 for the root)
 *   new_token    [B,w_verify] int32 out
 *   expected_len [B] fp32 out or NULL: sum of the kept values
 *   best_width   [B] int32 out or NULL: the n in 1..N maximising (sum of the n largest values) /
 *                (t_draft + t_verifier[n]), first maximum -- a hint for the next step's width; it
 *                stays on the device
 * The renumbered tree feeds ygg_tree_attention / ygg_accept_and_compact with n_nodes = w_verify.
 * Needs no workspace.
 */
int32_t ygg_prune_for_verification(const ygg_shape *shape, int32_t w_verify,
                                   const int32_t *parent_idx, const int32_t *token_ids,
                                   const float *cum_logprob, const float *t_verifier, float t_draft,
                                   int32_t *kept_nodes, int32_t *new_parent, int32_t *new_token,
                                   float *expected_len, int32_t *best_width, void *hip_stream);

/*
 * Greedy acceptance and K/V compaction (paper Sec. 1: draft tokens that match the verifier's
 * own output are accepted; Sec. 5: the "accept speculation management" stage; Sec. 4.1 under
 * Eq. 2: the verifier's token after the last accepted one is the bonus token; Sec. 6: the
 * TokenTree owns the K/V tensors).  Everything stays on the device:
 *     t*[i]    = argmax_v target_logits[b,i,v]          (first maximum)
 *     match[0] = 1;  match[i] = match[parent[i]] and token_ids[i] == t*[parent[i]]
 *     best     = matched node of greatest depth (lowest index among equals)
 *     accept_path[b,:] = root .. best, padded with -1;  accept_len[b] = depth(best)+1
 *     bonus_token[b]   = t*[best]
 *     for every layer: cache[layer,b,seq_lens[b]+k] = tree[layer,b,accept_path[b,k]], K and V
 *     seq_lens[b] += accept_len[b]
 *
 *   target_logits [B,N,V] fp32, or NULL when target_tokens [B,N] int32 (the argmax) is given;
 *                 exactly one of the two must be non-NULL
 *   parent_idx, token_ids [B,N] int32
 *   k_tree, v_tree   [n_layers,B,N,Hkv,Dh]    kv_dtype (may be NULL when n_layers == 0)
 *   k_cache, v_cache [n_layers,B,cap,Hkv,Dh]  kv_dtype, updated in place
 *                    (with YGG_FP8_E4M3 the four K/V arrays hold one-byte codes; rows are copied as bytes)
 *   seq_lens [B] int32 in/out; accept_len [B], accept_path [B,D+1], bonus_token [B] int32 out
 */
int32_t ygg_accept_and_compact(const ygg_shape *shape, int32_t n_layers,
                               const float *target_logits, const int32_t *target_tokens,
                               const int32_t *parent_idx, const int32_t *token_ids,
                               const void *k_tree, const void *v_tree,
                               void *k_cache, void *v_cache, int32_t *seq_lens,
                               int32_t *accept_len, int32_t *accept_path, int32_t *bonus_token,
                               void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Debug validator for the data-dependent part of the contract above (the paper's runtime keeps the
 * tree-structure array, the KV lengths and the token ids in a TokenTree object, Sec. 6; the calls
 * here trust them).  Writes one bit mask per sequence to flags[b] (device memory, [B] int32); every
 * input may be NULL, its checks are then skipped.  Not on the verification path: call it while
 * bringing a caller up, read the flags after synchronising.
 *   parent_idx [B,N]: YGG_BAD_PARENT if parent_idx[b][0] != -1 or some parent_idx[b][i] not in
 *                     [0, i); otherwise YGG_BAD_DEPTH if some node is deeper than `depth`
 *   seq_lens   [B]:   YGG_BAD_SEQ_LEN if outside [0, max_seq_len]
 *   token_ids  [B,N]: YGG_BAD_TOKEN if outside [0, vocab)
 *   logits     [B,logit_rows,V] fp32: YGG_BAD_LOGIT if any entry is NaN
 */
typedef enum {
    YGG_BAD_PARENT = 1, YGG_BAD_SEQ_LEN = 2, YGG_BAD_DEPTH = 4, YGG_BAD_TOKEN = 8, YGG_BAD_LOGIT = 16
} ygg_violation;
int32_t ygg_debug_validate(const ygg_shape *shape, const int32_t *parent_idx, const int32_t *seq_lens,
                           const int32_t *token_ids, const float *logits, int32_t logit_rows,
                           int32_t *flags, void *hip_stream);

/*
 * The launch plan ygg_tree_attention uses for a shape, for tests and tuning (host only, no GPU needed):
 * plan[0] = 1 matrix-core kernel / 0 vector kernel, plan[1] = wavefronts per workgroup, plan[2] = 2 if
 * wavefront pairs split every key tile else 1, plan[3] = workgroups along the query rows of one kv head,
 * plan[4] = key splits (the last three are 0 / meaningless for the vector kernel except plan[4]).
 */
int32_t ygg_debug_attention_plan(const ygg_shape *shape, int32_t *plan /* [5], host */);

/*
 * Tuning hook: forces the workgroup shape (wavefronts, 32-row blocks per wavefront, key shares) and/or the number
 * of key splits of every later ygg_tree_attention call of this process; a field left 0 keeps the library's own
 * choice, an unknown shape is ignored, and (0, 0, 0, 0) removes the override.  The workspace must be sized
 * (ygg_workspace_bytes) while the same override is in force.  Process-wide; meant for sweeps, not for production.
 */
int32_t ygg_debug_set_attention_plan(int32_t waves, int32_t rblocks, int32_t nsplit, int32_t kshares);

/*
 * Measurement hook for benchmarks (not part of the verification path): ygg_tree_attention without the launch that
 * merges the key splits, i.e. the main kernel alone, enqueued like any other call.  `out` and `lse` are only
 * complete for shapes with a single key split.  Timing a captured sequence of such calls gives the main kernel's
 * duration without event pairs, host gaps or library state.  Same arguments and errors as ygg_tree_attention.
 */
int32_t ygg_debug_tree_attention_main(const ygg_shape *shape,
                                      const void *q, const void *k_cache, const void *v_cache,
                                      const int32_t *seq_lens, const void *k_tree, const void *v_tree,
                                      const int32_t *parent_idx, void *out, float *lse,
                                      void *workspace, size_t workspace_bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* YGG_H */
