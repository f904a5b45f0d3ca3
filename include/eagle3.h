/*
 * eagle3.h — C ABI of the MI355X (gfx950) library for one EAGLE-3 speculative-decoding step
 * (arXiv 2503.01840): multi-layer feature fusion, draft-tree expansion, tree-masked verification
 * and the acceptance walk, plus what closes the loop around a step (prefill, commit, batched chain
 * drafting) and the training-time-test attention forward.
 *
 * General conventions
 *   - Unless marked HOST, every tensor pointer is a DEVICE pointer allocated and owned by the caller.
 *     The library allocates no device memory: scratch lives in the workspace the caller hands over
 *     with eagle3_set_workspace (size from eagle3_workspace_bytes).
 *   - All tensors are dense, row-major, innermost dimension contiguous.  Weights are [out, in]
 *     (y = W x).  Weights, norm gains, the embedding table and KV caches have the storage type
 *     `eagle3_config.dtype` (bf16 or fp32); activations exchanged across this boundary (features,
 *     logits, scores, uniforms) are fp32; indices are int32.
 *   - Every call outside the life-cycle section enqueues kernels on the given stream and returns without synchronising.
 *     Two calls using the same context must not overlap in time (they share the workspace).
 *   - Return value: EAGLE3_OK or a negative error code; nothing is enqueued when an argument check
 *     fails.  Device-side contents (e.g. parent[i] < i, token ids inside the vocabulary) are NOT
 *     validated; out-of-range values there are clamped by the kernels, never dereferenced.
 *   - Outputs are fully overwritten.
 */
#ifndef EAGLE3_H
#define EAGLE3_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct eagle3_ctx eagle3_ctx;
typedef void* eagle3_stream;              /* a hipStream_t; NULL = the default stream */

enum { EAGLE3_FP32 = 0, EAGLE3_BF16 = 1 };

enum {
  EAGLE3_OK = 0,
  EAGLE3_E_NULL = -1,       /* a required pointer is NULL                                           */
  EAGLE3_E_SHAPE = -2,      /* a size is outside what the configuration / the kernels support        */
  EAGLE3_E_STATE = -3,      /* weights or workspace not set, or workspace too small                  */
  EAGLE3_E_HIP = -4         /* a HIP call failed; eagle3_last_error() has the runtime's text         */
};

/* Model and limits; copied at eagle3_create.
 * bf16 configurations require head_dim == 128 and hidden, intermediate multiples of 128; vocab and
 * draft_vocab may be any size as long as no call runs more than 64 rows (max_batch * max_nodes <= 64
 * and max_batch * max_new <= 64), otherwise they must be multiples of 4 (the many-row GEMM stores
 * four outputs at a time); fp32 configurations accept any even head_dim <= 256 (slow,
 * exact-arithmetic kernels meant for small models). */
typedef struct {
  int32_t hidden, n_heads, n_kv_heads, head_dim, intermediate, vocab, draft_vocab, n_layers;
  int32_t tap_layers[3];    /* 0-based; the low/mid/high feature is the residual-stream OUTPUT of that layer */
  int32_t dtype;            /* EAGLE3_BF16 or EAGLE3_FP32 */
  float rope_theta, rms_eps;
  int32_t max_batch;        /* sequences per eagle3_tree_verify / eagle3_accept call */
  int32_t max_nodes;        /* tree nodes per sequence including the root, <= 64 */
  int32_t max_depth;        /* draft forwards D */
  int32_t max_topk;         /* K; (max_depth-1)*max_topk <= 128 */
  int32_t max_new;          /* rows of draft forward 1 / of eagle3_fuse_features, <= 64 */
} eagle3_config;

/* One decoder layer (LLaMA style, no biases).  For the draft layer wq/wk/wv have 2*hidden inputs and
 * norm_attn is unused (may be NULL). */
typedef struct {
  const void *wq, *wk, *wv, *wo;          /* [H*d, in], [Hkv*d, in], [Hkv*d, in], [hidden, H*d] */
  const void *w_gate, *w_up, *w_down;     /* [I, hidden], [I, hidden], [hidden, I]               */
  const void *norm_attn, *norm_mlp;       /* [hidden] gains                                      */
} eagle3_layer_weights;

typedef struct {
  const eagle3_layer_weights* layers;     /* HOST array [n_layers] (copied by eagle3_set_weights) */
  const void *embed, *final_norm, *lm_head;   /* [vocab, hidden], [hidden], [vocab, hidden]       */
} eagle3_target_weights;

typedef struct {
  const void* w_fc;                       /* [hidden, 3*hidden]: fusion of (low | mid | high)       */
  eagle3_layer_weights layer;             /* the single draft decoder layer                          */
  const void *norm_embed, *norm_feat;     /* [hidden] gains of the two halves of the layer's input  */
  const void *final_norm, *lm_head;       /* [hidden], [draft_vocab, hidden]                         */
  const int32_t* d2t;                     /* [draft_vocab] draft id -> target id                     */
} eagle3_draft_weights;

/* A (possibly ragged, batched) KV cache.  Sequence b owns token slots [kv_indptr[b], kv_indptr[b+1])
 * of every layer's arrays; its first prefix_len[b] slots hold the context, the following slots are
 * written by the call (tree nodes / draft rows) and must exist. */
typedef struct {
  void* const* k;                         /* HOST array [layers] of device pointers [slots, Hkv, d] (rotated keys) */
  void* const* v;                         /* HOST array [layers] of device pointers [slots, Hkv, d]                */
  const int32_t* kv_indptr;               /* DEVICE [B+1] */
  const int32_t* prefix_len;              /* DEVICE [B]   */
  int32_t max_prefix_len;                 /* HOST upper bound of prefix_len[b]; only sizes the launch     */
} eagle3_kv;

/* Optional device outputs of eagle3_draft_expand that expose every selection it made, so that a
 * checker can tell an admissible near-tie from an error.  Any pointer may be NULL.
 * Pool ids: 0 = root; level 1 -> 1..K in rank order; level l >= 2 -> 1 + K + (l-2)*K*K + r*K + c
 * for the c-th best token of the r-th frontier node. */
typedef struct {
  int32_t* pool_tok;        /* [1 + K + (D-1)*K*K] draft-vocabulary ids                        */
  int32_t* pool_parent;     /* same length, pool id of the parent                               */
  float* pool_score;        /* same length, cumulative log-probability                          */
  int32_t* frontier;        /* [D-1, K] row j: pool ids run by draft forward j+2, in rank order   */
  int32_t* chosen;          /* [N-1] pool ids kept by the final rerank, ascending               */
} eagle3_draft_debug;

/* ---- life cycle (host only; these may synchronise) ---------------------------------------------- */
int eagle3_create(const eagle3_config* cfg, eagle3_ctx** out);
int eagle3_destroy(eagle3_ctx* ctx);
int eagle3_workspace_bytes(const eagle3_ctx* ctx, size_t* out);
int eagle3_set_workspace(eagle3_ctx* ctx, void* dev, size_t bytes);      /* 256-byte aligned device memory */
int eagle3_set_weights(eagle3_ctx* ctx, const eagle3_target_weights* target /* may be NULL */,
                       const eagle3_draft_weights* draft /* may be NULL */);
const char* eagle3_strerror(int code);
const char* eagle3_last_error(void);      /* text of the last HIP failure seen by this thread */

/* ---- the speculative step ---------------------------------------------------------------------- */

/* Section 3.1 ("Inference Pipeline"): the k-dimensional low, mid and high features of a position are
 * concatenated to 3k and passed through one FC layer back to k:  g = W_fc [low; mid; high].
 * low/mid/high: fp32 [M, hidden] each, 1 <= M <= max_new.  g_out: fp32 [M, hidden]. */
int eagle3_fuse_features(eagle3_ctx* ctx, const float* low, const float* mid, const float* high,
                         int32_t M, float* g_out, eagle3_stream stream);

/* Section 3.1 (draft steps 1, 2, 3, ...: the draft layer reads [feature; embedding of the sampled
 * token], its output a replaces the unavailable feature in later steps, the LM head scores the next
 * token) combined with Section 2.2 / Appendix A (EAGLE-2's dynamic draft tree: expand the `topk`
 * most confident nodes per level for `depth` levels, then keep the n_nodes-1 best candidates by
 * cumulative log-probability).
 *   g_new    fp32 [n_new, hidden]   fused features of the positions accepted by the previous step
 *   tok_new  int32 [n_new]          target ids; tok_new[j] FOLLOWS the position that produced g_new[j];
 *                                   tok_new[n_new-1] is the root of the tree
 *   draft_kv one layer, one sequence; the call appends n_new + (depth-1)*topk slots after the prefix
 *   outputs  tree_tok [n_nodes] target ids ([0] = root), parent [n_nodes] ([0] = -1, parent[i] < i),
 *            node_depth [n_nodes], cum_logprob [n_nodes] ([0] = 0); nodes are in ascending pool id.
 * Ordering rule everywhere: larger score first, ties -> smaller id.
 * Requires 1 <= n_new <= max_new, 1 <= depth <= max_depth, 1 <= topk <= max_topk,
 * 2 <= n_nodes <= min(max_nodes, 1 + pool size). */
int eagle3_draft_expand(eagle3_ctx* ctx, const float* g_new, const int32_t* tok_new, int32_t n_new,
                        const eagle3_kv* draft_kv, int32_t depth, int32_t topk, int32_t n_nodes,
                        int32_t* tree_tok, int32_t* parent, int32_t* node_depth, float* cum_logprob,
                        const eagle3_draft_debug* dbg /* HOST struct, may be NULL */, eagle3_stream stream);

/* Section 2.2 (tree attention: the whole draft tree is verified in one target forward) and Section 3.1
 * (the low/mid/high features are recorded during verification).  Runs every target layer over the
 * B*N node rows; node i of sequence b sits at position prefix_len[b] + depth(i), its query sees the
 * prefix and exactly its ancestors and itself; node keys/values are written to cache slots
 * prefix_len[b] + i.
 *   tree_tok, parent  int32 [B, N] (parent[b][0] = -1, parent[b][i] < i)
 *   logits            fp32 [B, N, vocab]
 *   taps              fp32 [3, B, N, hidden]  outputs of layers tap_layers[0..2]
 *   dbg_hidden        fp32 [n_layers+1, B, N, hidden] residual stream before layer 0 and after every
 *                     layer, or NULL
 * Requires 1 <= B <= max_batch, 1 <= N <= max_nodes. */
int eagle3_tree_verify(eagle3_ctx* ctx, int32_t B, int32_t N, const int32_t* tree_tok, const int32_t* parent,
                       const eagle3_kv* kv, float* logits, float* taps, float* dbg_hidden,
                       eagle3_stream stream);

/* The same forward restricted to target layers [layer_begin, layer_end): the building block of a
 * layer-sharded (pipelined) deployment, and the way to check single layers at full size.
 *   x_in   fp32 [B, N, hidden] residual stream entering layer_begin; NULL = token embeddings
 *          (then layer_begin must be 0)
 *   x_out  fp32 [B, N, hidden] residual stream after layer_end - 1, or NULL
 *   logits fp32 [B, N, vocab] or NULL; non-NULL requires layer_end == n_layers (final norm + LM head)
 * kv->k / kv->v are indexed by absolute layer number; only entries of the range are read.  At least one
 * of x_out, logits must be given.  Feature taps are not produced by this call. */
int eagle3_tree_verify_layers(eagle3_ctx* ctx, int32_t B, int32_t N, const int32_t* tree_tok, const int32_t* parent,
                              const eagle3_kv* kv, const float* x_in, int32_t layer_begin, int32_t layer_end,
                              float* x_out, float* logits, eagle3_stream stream);

/* Section 2.1 (accept draft tokens front to back; on the first rejection emit one token from the
 * residual distribution and discard the rest), applied along the tree.  temperature == 0: follow the
 * child equal to the target argmax (ties -> smaller id).  temperature > 0: p = softmax(logits/T);
 * children of the current node are tested in ascending node id, child c is accepted iff
 * uniforms[2c] < p[tok_c] / (1 - rejected mass); otherwise its token is struck from the residual; when
 * no child is accepted the bonus token is the inverse CDF (vocabulary order) of the renormalised
 * residual at uniforms[2*cur+1].
 *   logits [B, N, vocab] fp32; tree_tok, parent [B, N]; uniforms fp32 [B, 2N] (NULL iff temperature == 0)
 *   accept_len [B] drafted tokens accepted; path [B, N] node ids from the root, -1 padded;
 *   bonus_tok [B]. */
int eagle3_accept(eagle3_ctx* ctx, int32_t B, int32_t N, const float* logits, const int32_t* tree_tok,
                  const int32_t* parent, float temperature, const float* uniforms,
                  int32_t* accept_len, int32_t* path, int32_t* bonus_tok, eagle3_stream stream);

/* Chain drafting for a batch (Section 4.3 / 4.4: at large batch sizes the serving experiments draft a chain of 2-3
 * tokens per sequence instead of a tree).  The draft steps of Section 3.1 with one proposal per step: forward 1 runs,
 * for every sequence b, the rows (g_new[b][j], tok_new[b][j]), j < n_new[b] (the positions accepted by the previous
 * step, causal among themselves); its last row gives the first drafted token (arg-max of the draft distribution,
 * ties -> smaller id); every further forward runs one row per sequence, (previous output a, previous token).
 *   g_new      fp32 [B, rows1, hidden], tok_new int32 [B, rows1] (target ids), n_new DEVICE int32 [B] with
 *              1 <= n_new[b] <= rows1; rows j >= n_new[b] are padding (read, never used)
 *   draft_kv   one layer, B sequences (ragged): forward 1 appends rows1 slots per sequence of which the first
 *              n_new[b] stay valid, the later forwards overwrite the slots after those; prefix_len is not changed
 *   chain_tok  int32 [B, length + 1]: [b][0] = the root tok_new[b][n_new[b]-1], [b][l] = the l-th drafted token
 *              (target id); with parent[l] = l - 1 this is the tree eagle3_tree_verify takes
 *   chain_logp fp32 [B, length + 1]: cumulative log-probability ([b][0] = 0)
 * Requires 1 <= B <= max_batch, 1 <= rows1 <= min(max_new, max_nodes), 1 <= length <= max_depth. */
int eagle3_draft_chain(eagle3_ctx* ctx, int32_t B, const float* g_new, const int32_t* tok_new, const int32_t* n_new,
                       int32_t rows1, const eagle3_kv* draft_kv, int32_t length, int32_t* chain_tok, float* chain_logp,
                       eagle3_stream stream);

/* Section 3.1, first paragraph of the pipeline: during the prefill phase the target model runs over the prompt, the
 * low / mid / high feature sequences of its positions are recorded and fused, and the draft model's context is built
 * from them.  One sequence.  The T prompt tokens are run through every target layer in chunks of
 * min(max_nodes, max_new) positions (each chunk a chain on top of everything cached before it), their keys and
 * values are appended to the target cache at slots prefix_len .. prefix_len + T - 1, and for every position i whose
 * following token is known (all but the last) the draft layer's key / value of the row (g_i, tokens[i+1]) is appended
 * to the draft cache (a draft row's key and value depend only on that row, so no draft attention runs here).
 *   tokens       DEVICE int32 [T]
 *   kv, draft_kv  target cache (all layers) and draft cache (one layer), one sequence each; BOTH prefix_len arrays
 *                 are read and then ADVANCED by the call (by T and by T - 1); max_prefix_len bounds the values on
 *                 entry; the caches need T (T - 1) free slots after their prefixes
 *   g_last       fp32 [hidden]  fused feature of the last prompt position: with the first sampled token it is the
 *                               n_new = 1 input of the first eagle3_draft_expand
 *   logits_last  fp32 [vocab]   next-token logits after the prompt
 * Requires T >= 1 and both weight sets. */
int eagle3_prefill(eagle3_ctx* ctx, const int32_t* tokens, int32_t T, const eagle3_kv* kv, const eagle3_kv* draft_kv,
                   float* g_last, float* logits_last, eagle3_stream stream);

/* Between two steps.  Section 2.1: the accepted draft tokens are kept and everything after the first rejection is
 * discarded; Section 3.1: the features recorded during this verification are the next draft's input.  For every
 * sequence b with path[b][0..a] (a = accept_len[b]) the call
 *   - moves, in every target layer and in place, the cache rows of the accepted nodes from slots
 *     prefix_len[b] + path[b][j] to slots prefix_len[b] + j (keys and values);
 *   - writes taps_new[t][b][j] = taps[t][b][path[b][j]] (j <= a): the low / mid / high features of the accepted
 *     positions, ready for eagle3_fuse_features;
 *   - writes tok_new[b][j] = the token FOLLOWING accepted position j: tree_tok[b][path[b][j+1]] for j < a and
 *     bonus_tok[b] for j = a (the next tree's root), and n_new[b] = a + 1;
 *   - adds a + 1 to prefix_len[b] and, if draft_prefix_len is given, draft_rows to draft_prefix_len[b] (the rows that
 *     this step's draft forward 1 appended to the draft cache stay valid whatever was accepted).
 *   tree_tok, path [B, N]; accept_len, bonus_tok [B] (as written by eagle3_accept); kv: the target cache of the
 *   verification (kv->prefix_len is NOT used: prefix_len, DEVICE [B], is read and then updated; it may be the same
 *   array); taps [3, B, N, hidden] from eagle3_tree_verify; rows: row capacity of the outputs per sequence
 *   (a + 1 is clamped to it); taps_new fp32 [3, B, rows, hidden] or NULL; tok_new int32 [B, rows]; n_new int32 [B].
 * The caller keeps kv->max_prefix_len (a host bound) ahead of the device lengths, e.g. by adding rows per step. */
int eagle3_commit(eagle3_ctx* ctx, int32_t B, int32_t N, const int32_t* tree_tok, const int32_t* path,
                  const int32_t* accept_len, const int32_t* bonus_tok, const eagle3_kv* kv, int32_t* prefix_len,
                  const float* taps, int32_t rows, float* taps_new, int32_t* tok_new, int32_t* n_new,
                  int32_t* draft_prefix_len, int32_t draft_rows, eagle3_stream stream);

/* Section 3.2 ("Draft Model Training", Figure 6), forward only: the draft layer's self-attention during a
 * training-time-test step.  At simulated step `step` (0 = the native step) query i attends to the ORIGINAL
 * training positions 0..i (a lower-triangular mask) and, of every simulated step t = 1..step, to position i alone
 * (diagonal masks; those scores are per-position vector dot products, not a matrix product).  No context needed.
 *   dtype    EAGLE3_BF16 (head_dim must be 128) or EAGLE3_FP32 (exact kernels, (T + step) * 4 bytes <= 60 KiB)
 *   q        [T, n_heads, head_dim]                 queries of this step (already rotated)
 *   k_steps  [step + 1, T, n_kv_heads, head_dim]    keys of the original inputs (index 0) and of steps 1..step
 *   v_steps  [step + 1, T, n_kv_heads, head_dim]    values, same order
 *   out      fp32 [T, n_heads, head_dim]
 * Softmax scale 1/sqrt(head_dim); query head h reads KV head h * n_kv_heads / n_heads. */
int eagle3_ttt_attention(int32_t dtype, int32_t T, int32_t n_heads, int32_t n_kv_heads, int32_t head_dim, int32_t step,
                         const void* q, const void* k_steps, const void* v_steps, float* out, eagle3_stream stream);

/* For callers that cannot allocate device memory and hold no context: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  The same acceptance walk as eagle3_accept (same kernels, same
 * results) with its per-(row, 2048-logit chunk) statistics kept in a fixed 1 MiB device array inside the library
 * instead of a workspace: no eagle3_ctx, no workspace, no allocation of any kind.
 *   Limits: 1 <= N <= 64 and B*N * ceil(vocab / 2048) <= 65536 (e.g. 1040 rows at vocab 128256); beyond that the
 *   call returns EAGLE3_E_SHAPE and enqueues nothing.
 *   The array is per GPU (the device current at the call must be the stream's device) and is shared by every call
 *   on that GPU: calls that overlap in time on one GPU race on it; calls on one stream are safe back to back.
 *   Nothing in it needs clearing between calls (every entry a call reads it has written itself). */
int eagle3_accept_static(int32_t B, int32_t N, int32_t vocab, const float* logits, const int32_t* tree_tok,
                         const int32_t* parent, float temperature, const float* uniforms,
                         int32_t* accept_len, int32_t* path, int32_t* bonus_tok, eagle3_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* EAGLE3_H */
