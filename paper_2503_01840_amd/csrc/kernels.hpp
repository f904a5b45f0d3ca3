// Host-side launch interface of the gfx950 kernels (one definition per .hip file).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint16_t bf16_t;

// ---------------------------------------------------------------- GEMM (gemm_skinny.hip, gemm_f32.hip)
// Weight operand: up to three [rows_i, K] row-major matrices.
//   mode 0: their rows are concatenated (q|k|v projections run as one GEMM);
//   mode 1: tiles interleave 32 rows of w[0] (gate) with the same 32 rows of w[1] (up) so that the
//           SwiGLU product can be formed in the epilogue.
struct GemmWeights {
  const void* w[3];
  int rows[3];
  int nmat;
  int mode;
};
enum { GEMM_EPI_PARTIAL = 0, GEMM_EPI_SWIGLU = 1 };

// Y = X W^T for few rows (M <= a few hundred) streaming the weights once: bf16 inputs, fp32 accumulate.
//   x      fragment-major bf16 [ceil64(M), K] (see xf_offset)
//   out    epi PARTIAL: fp32 [S, M, N] (split-K partial sums, S = splits); the consumer adds them
//          epi SWIGLU : fragment-major bf16 [ceil64(M), N/2] = silu(gate) * up   (requires S == 1)
// Requires K % (128*S) == 0.  N = total weight rows.  ev_start / ev_stop (optional): events attached to the dispatch.
hipError_t launch_gemm_skinny(const bf16_t* x, const GemmWeights& W, int M, int N, int K, int S, int epi,
                              void* out, hipStream_t st, hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);
// Whether launch_gemm_skinny takes the 128-weight-row workgroups for this shape.
bool gemm_skinny_uses_tile128(const GemmWeights& W, int M, int N, int S);
// Chooses the split-K factor for a [N, K] weight so that about two workgroups per CU are resident.
int gemm_skinny_pick_splits(int N, int K, int M);

// The same product for many rows (M > 64): MFMA-bound tiling, see gemm_wide.hip.  Chooses tile shape and split-K
// itself (S <= what fits into out_capacity_floats; 0 forces S = 1) and reports S.
hipError_t launch_gemm_wide(const bf16_t* x, const GemmWeights& W, int M, int N, int K, int epi, void* out,
                            size_t out_capacity_floats, int* S_out, hipStream_t st, hipEvent_t ev_start = nullptr,
                            hipEvent_t ev_stop = nullptr);

// fp32 reference-quality GEMM: out[m, col0 + n] = sum_k x[m,k] w[n,k]; x [M,K], w [N,K], out row stride ld.
hipError_t launch_gemm_f32(const float* x, const float* w, int M, int N, int K, float* out, int ld, int col0,
                           hipStream_t st);

// ---------------------------------------------------------------- elementwise (elementwise.hip)
struct SeqInfo {           // one per sequence, device resident
  int32_t kv_base;         // first cache slot of the sequence
  int32_t n_prefix;        // slots visible to every row
  int32_t n_tail;          // following slots, visible according to the per-row bit mask
  int32_t order;           // entry i: the sequence that attention workgroup group i works on (longest first)
};

hipError_t launch_embed_rows(bool bf16, const void* embed, const int32_t* tok, int R, int k, int vocab, float* x,
                             hipStream_t st);
// x += sum_s partial[s]; copies x to each non-null copy_out; act = RMSNorm(x; gain) in the activation layout.
hipError_t launch_add_norm(bool bf16, float* x, const float* partial, int S, int R, int k, const void* gain, float eps,
                           void* act, float* const copy_out[4], hipStream_t st);
// Tree bookkeeping for verification: depth, 128-bit ancestor masks, cache slot and rotary tables per row.
hipError_t launch_tree_prep(const int32_t* parent, const int32_t* kv_indptr, const int32_t* prefix_len, int B, int N,
                            int head_dim, float theta, int32_t* depth, uint32_t* mask, int32_t* slot, float* cs,
                            SeqInfo* seq, hipStream_t st);
// Sums the q|k|v split-K partials, rotates q and k, writes q (activation type, [R,H,d]) and the cache rows.
hipError_t launch_rope_kv_write(bool bf16, const float* qkv_partial, int S, int R, int H, int Hkv, int d, const float* cs,
                                const int32_t* slot, void* q, void* kcache, void* vcache, hipStream_t st);
hipError_t launch_swiglu_f32(const float* gu, int R, int I, float* h, hipStream_t st);
hipError_t launch_pack3(bool bf16, const float* a, const float* b, const float* c, int M, int k, void* act, hipStream_t st);
hipError_t launch_reduce_partials(const float* partial, int S, int M, int N, float* out, hipStream_t st);
// Draft layer input: act[r] = [RMSNorm(E[tok[r]]; g_embed) ; RMSNorm(f_r; g_feat)], y[r] = f_r,
// with f_r = feat[src_row ? src_row[r] : r]; also the rotary table cs[r] of position pos[r] (positions already on
// the device).
hipError_t launch_draft_input(bool bf16, const void* embed, int vocab, const int32_t* tok, const float* feat,
                              const int32_t* src_row, int M, int k, const void* g_embed, const void* g_feat, float eps,
                              void* act, float* y, const int32_t* pos, int head_dim, float theta, float* cs, hipStream_t st);
// Rows of draft forward 1: positions, slots, causal masks, sequence info.
hipError_t launch_draft_prep1(const int32_t* kv_indptr, const int32_t* prefix_len, int n_new, int32_t* pos, int32_t* slot,
                              uint32_t* mask, SeqInfo* seq, hipStream_t st);

hipError_t launch_chain_parent(int32_t* parent, int n, hipStream_t st);                 // parent[i] = i - 1
hipError_t launch_advance_lengths(int32_t* len, int B, int by, hipStream_t st);          // len[b] += by

// ---------------------------------------------------------------- attention (attention.hip)
// Tree-masked attention of rows [B * rows_per_seq] against a (ragged) cache.
//   bf16: q [R,H,d] bf16, cache bf16, out = fragment-major bf16 [R, H*d]; d must be 128.
//   fp32: q fp32, cache fp32, out row-major fp32.
// scratch: fp32 workspace of attention_scratch_floats(...) elements.
size_t attention_scratch_floats(int R, int H, int d, int max_splits);
int attention_pick_splits(int B, int rows_per_seq, int H, int Hkv, int max_len);
hipError_t launch_tree_attention(bool bf16, const void* q, const void* kcache, const void* vcache, const SeqInfo* seq,
                                 const uint32_t* mask, int B, int rows_per_seq, int H, int Hkv, int d, int max_len,
                                 int n_splits, float* scratch, void* out, hipStream_t st);

// ---------------------------------------------------------------- draft tree (select.hip)
#define DRAFT_MAX_POOL 2048   /* candidates the final rerank can hold: 1 + K + (D-1) K^2 must not exceed it */
struct DraftState {          // device arrays owned by the workspace
  int32_t* pool_tok;         // [pool] draft ids
  int32_t* pool_parent;      // [pool]
  int32_t* pool_depth;       // [pool]
  float* pool_score;         // [pool]
  uint32_t* pool_mask;       // [pool][4] tail-slot mask of a candidate once it is put on a frontier
  int32_t* frontier;         // [D][K] pool ids expanded by forward l+1 (row 0 = level-1 candidates)
  float* top_val;            // [max_rows][K] log-probabilities of the per-row top-K
  int32_t* top_idx;          // [max_rows][K]
  // inputs of the next forward
  int32_t* row_tok;          // [K] target ids
  int32_t* row_src;          // [K] row of the feature buffer holding the parent's output
  int32_t* row_pos;          // [K]
  int32_t* row_slot;         // [K]
  uint32_t* row_mask;        // [K][4]
  SeqInfo* seq;              // [1]
};
// Per-row log-softmax normaliser and top-K (value desc, id asc) over z[row, 0..V).
// scratch: topk_scratch_floats(n_rows, V, K) floats.
size_t topk_scratch_floats(int n_rows, int V, int K);
hipError_t launch_topk_rows(const float* z, int ld, int row0, int n_rows, int V, int K, float* scratch, float* top_val,
                            int32_t* top_idx, hipStream_t st);
// Level bookkeeping after forward `level` (1-based): writes the new pool entries and, when level < depth,
// picks the next frontier and the next forward's row inputs.
hipError_t launch_draft_select(const DraftState& s, const int32_t* d2t, const int32_t* kv_indptr, const int32_t* prefix_len,
                               int level, int depth, int K, int n_new, int feat_row0, hipStream_t st);
hipError_t launch_draft_rerank(const DraftState& s, const int32_t* d2t, const int32_t* tok_new, int n_new, int depth, int K,
                               int n_nodes, int32_t* tree_tok, int32_t* parent, int32_t* node_depth, float* cum_logprob,
                               int32_t* chosen_dbg, hipStream_t st);

// Batched chain drafting: per-sequence state of the next forward (one row per sequence), device arrays.
struct ChainState {
  float* top_val;            // [B] log-probability of the top-1 token of every sequence's last row
  int32_t* top_idx;          // [B] its draft id
  int32_t* row_tok;          // [B] target ids
  int32_t* row_src;          // [B]
  int32_t* row_pos;          // [B]
  int32_t* row_slot;         // [B]
  uint32_t* row_mask;        // [B][4]
  SeqInfo* seq;              // [B]
};
hipError_t launch_chain_prep1(const int32_t* kv_indptr, const int32_t* prefix_len, int B, int rows1, int32_t* pos,
                              int32_t* slot, uint32_t* mask, SeqInfo* seq, hipStream_t st);
hipError_t launch_chain_select(const ChainState& s, const int32_t* d2t, const int32_t* kv_indptr, const int32_t* prefix_len,
                               const int32_t* n_new, const int32_t* tok_new, int B, int rows1, int level, int length,
                               int32_t* chain_tok, float* chain_logp, hipStream_t st);
hipError_t launch_chain_gather(const float* x, const int32_t* n_new, int B, int rows1, int k, float* x_out, hipStream_t st);

// ---------------------------------------------------------------- acceptance (accept.hip)
#define ACCEPT_CHUNK 2048
size_t accept_scratch_floats(int R, int V);
hipError_t launch_accept(const float* logits, const int32_t* tree_tok, const int32_t* parent, int B, int N, int V,
                         float temperature, const float* uniforms, float* scratch, int32_t* accept_len, int32_t* path,
                         int32_t* bonus, hipStream_t st);

// ---------------------------------------------------------------- commit (commit.hip)
// Moves the accepted nodes' cache rows to the front of the tree slots (every layer, in place), gathers their
// features and following tokens, advances the prefix lengths.  k_layers / v_layers: host arrays of device pointers.
hipError_t launch_commit(void* const* k_layers, void* const* v_layers, int n_layers, const int32_t* kv_indptr,
                         int32_t* prefix_len, const int32_t* tree_tok, const int32_t* path, const int32_t* accept_len,
                         const int32_t* bonus, const float* taps, int B, int N, int hidden, int row_bytes, int rows,
                         float* taps_new, int32_t* tok_new, int32_t* n_new, int32_t* draft_prefix_len, int draft_rows,
                         hipStream_t st);

// ---------------------------------------------------------------- training-time-test attention (ttt_attention.hip)
// q [T,H,d], k / v [s+1,T,Hkv,d] (bf16 with d == 128, or fp32), out fp32 [T,H,d].
hipError_t launch_ttt_attention(bool bf16, const void* q, const void* k, const void* v, int T, int H, int Hkv, int d, int s,
                                float* out, hipStream_t st);
