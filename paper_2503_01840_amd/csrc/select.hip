// Draft-tree bookkeeping on the device: per-row log-softmax + top-K over the draft vocabulary, the
// per-level frontier choice by cumulative log-probability, and the final global rerank.  Ordering rule
// everywhere: larger score first, ties -> smaller id.  Everything here is latency-bound integer/compare
// work on a few hundred candidates, done with wavefront shuffles and LDS reductions; no host round trip.
#include <limits.h>

#include "common.hpp"
#include "kernels.hpp"

namespace {

struct ValIdx { float v; int i; };

__device__ __forceinline__ bool better(float va, int ia, float vb, int ib) { return va > vb || (va == vb && ia < ib); }

__device__ __forceinline__ ValIdx wave_best(ValIdx x) {
  wave_best_pair(x.v, x.i);
  return x;
}

// `red` : __shared__ ValIdx[17]
__device__ __forceinline__ ValIdx block_best(ValIdx x, ValIdx* red) {
  x = wave_best(x);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = x;
  __syncthreads();
  if (threadIdx.x == 0) {
    ValIdx b = red[0];
    for (int i = 1; i < nw; ++i)
      if (better(red[i].v, red[i].i, b.v, b.i)) b = red[i];
    red[16] = b;
  }
  __syncthreads();
  return red[16];
}

// Row top-K in two levels, no workgroup barrier anywhere.
// Level 1: one wavefront per 512 consecutive logits (8 per lane, held in registers) finds its own top K by K
// rounds of a wavefront arg-max, and the (max, sum of exp) of its span.
constexpr int TOPK_SPAN = 512;
__global__ __launch_bounds__(256) void topk_spans_kernel(const float* __restrict__ z, int ld, int row0, int V, int K,
                                                        int n_spans, float* __restrict__ cand_val,
                                                        int32_t* __restrict__ cand_idx, float* __restrict__ span_stat) {
  const int lane = threadIdx.x & 63, span = blockIdx.x * 4 + (threadIdx.x >> 6), row = blockIdx.y;
  if (span >= n_spans) return;
  const float* zr = z + (size_t)(row0 + row) * ld;
  const int base = span * TOPK_SPAN;
  float v[8];
  float mx = -INFINITY;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int c = base + j * 64 + lane;
    v[j] = c < V ? zr[c] : -INFINITY;
    mx = fmaxf(mx, v[j]);
  }
  mx = wave_max(mx);                                   // base < V, so at least one entry is finite
  float sum = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j) sum += expf(v[j] - mx);  // exp(-inf) = 0 for the padding
  sum = wave_sum_butterfly(sum);
  const size_t o = (size_t)row * n_spans + span;
  if (lane == 0) { span_stat[2 * o] = mx; span_stat[2 * o + 1] = sum; }
  for (int r = 0; r < K; ++r) {
    ValIdx b = {-INFINITY, INT_MAX};
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (v[j] > b.v) { b.v = v[j]; b.i = base + j * 64 + lane; }   // ascending index per lane: first maximum kept
    b = wave_best(b);
    if (lane == 0) { cand_val[o * K + r] = b.v; cand_idx[o * K + r] = b.i; }
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (b.i == base + j * 64 + lane) v[j] = -INFINITY;
  }
}

// Level 2: one wavefront per row merges the spans' candidates and statistics, without sequential selection rounds.
// In the order (value desc, index asc) the K-th best of the spans' BEST candidates bounds the answer from below:
// at least K candidates are not worse than it, so only candidates not worse than it can be among the top K, and
// those come from exactly K spans (at most K * K survivors).  The survivors are ranked by counting, and rank r < K
// is output r.
constexpr int TOPK_MAX_SPANS = 1024, TOPK_MAX_K = 16;
__global__ __launch_bounds__(64) void topk_merge_kernel(const float* __restrict__ cand_val, const int32_t* __restrict__ cand_idx,
                                                       const float* __restrict__ span_stat, int n_spans, int K,
                                                       float* __restrict__ top_val, int32_t* __restrict__ top_idx) {
  __shared__ float head_v[TOPK_MAX_SPANS];
  __shared__ int head_i[TOPK_MAX_SPANS];
  __shared__ float surv_v[TOPK_MAX_K * TOPK_MAX_K];
  __shared__ int surv_i[TOPK_MAX_K * TOPK_MAX_K];
  __shared__ float bound_v;
  __shared__ int bound_i, n_surv;
  const int lane = threadIdx.x, row = blockIdx.x;
  const float* st = span_stat + (size_t)row * n_spans * 2;
  float mx = -INFINITY;
  for (int i = lane; i < n_spans; i += 64) mx = fmaxf(mx, st[2 * i]);
  mx = wave_max(mx);
  float sum = 0.f;
  for (int i = lane; i < n_spans; i += 64) sum += st[2 * i + 1] * expf(st[2 * i] - mx);
  sum = wave_sum_butterfly(sum);
  const float lse = logf(sum);
  const int C = n_spans * K;
  const float* cv = cand_val + (size_t)row * C;
  const int32_t* ci = cand_idx + (size_t)row * C;
  for (int i = lane; i < n_spans; i += 64) { head_v[i] = cv[i * K]; head_i[i] = ci[i * K]; }
  if (lane == 0) { n_surv = 0; bound_v = -INFINITY; bound_i = INT_MAX; }      // fewer than K spans: everything survives
  __syncthreads();
  const int kth = K - 1;
  for (int i = lane; i < n_spans; i += 64) {
    const float v = head_v[i];
    const int id = head_i[i];
    int rank = 0;
    for (int j = 0; j < n_spans; ++j) rank += better(head_v[j], head_i[j], v, id) ? 1 : 0;
    if (rank == kth) { bound_v = v; bound_i = id; }
  }
  __syncthreads();
  const float bv = bound_v;
  const int bi = bound_i;
  for (int i = lane; i < n_spans; i += 64) {
    if (better(bv, bi, head_v[i], head_i[i])) continue;                        // the whole span is worse than the bound
    for (int r = 0; r < K; ++r) {
      const float v = cv[i * K + r];
      const int id = ci[i * K + r];
      if (better(bv, bi, v, id)) break;                                        // a span's candidates are in order
      const int pos = atomicAdd(&n_surv, 1);
      surv_v[pos] = v;
      surv_i[pos] = id;
    }
  }
  __syncthreads();
  const int T = n_surv;
  for (int t = lane; t < T; t += 64) {
    const float v = surv_v[t];
    const int id = surv_i[t];
    int rank = 0;
    for (int j = 0; j < T; ++j) rank += better(surv_v[j], surv_i[j], v, id) ? 1 : 0;
    if (rank < K) {
      top_val[row * K + rank] = v - mx - lse;
      top_idx[row * K + rank] = id;
    }
  }
}

__device__ __forceinline__ int level_base(int level, int K) { return level <= 1 ? 1 : 1 + K + (level - 2) * K * K; }

__global__ __launch_bounds__(256) void draft_select_kernel(DraftState s, const int32_t* __restrict__ d2t,
                                                          const int32_t* __restrict__ kv_indptr,
                                                          const int32_t* __restrict__ prefix_len, int level, int depth,
                                                          int K, int n_new) {
  __shared__ float sc[256];
  const int tid = threadIdx.x;
  const int base = level_base(level, K);
  const int n_cand = level == 1 ? K : K * K;
  if (level == 1 && tid == 0) {
    s.pool_tok[0] = 0; s.pool_parent[0] = -1; s.pool_depth[0] = 0; s.pool_score[0] = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) s.pool_mask[w] = 0u;
  }
  __syncthreads();
  for (int e = tid; e < n_cand; e += 256) {
    const int par = level == 1 ? 0 : s.frontier[(level - 2) * K + e / K];
    const float score = (level == 1 ? 0.f : s.pool_score[par]) + s.top_val[e];
    s.pool_tok[base + e] = s.top_idx[e];
    s.pool_parent[base + e] = par;
    s.pool_depth[base + e] = level;
    s.pool_score[base + e] = score;
    sc[e] = score;
  }
  __syncthreads();
  if (level >= depth) return;
  // next frontier: level 1 -> all K candidates in rank order; later levels -> top-K of the K*K
  int32_t* fr = s.frontier + (level - 1) * K;
  for (int e = tid; e < n_cand; e += 256) {
    int rank = 0;
    for (int j = 0; j < n_cand; ++j) rank += better(sc[j], j, sc[e], e) ? 1 : 0;
    if (rank < K) fr[rank] = base + e;
  }
  __threadfence_block();
  __syncthreads();
  // rows of the next forward (level + 1)
  if (tid < K) {
    const int r = tid, pid = fr[r], par = s.pool_parent[pid];
    const int P = prefix_len[0];
    const int tail_slot = (level - 1) * K + r;
    s.row_tok[r] = d2t[s.pool_tok[pid]];
    s.row_src[r] = level == 1 ? n_new - 1 : n_new + (level - 2) * K + (pid - base) / K;
    s.row_pos[r] = P + n_new - 1 + level;
    s.row_slot[r] = kv_indptr[0] + P + n_new + tail_slot;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      uint32_t m = s.pool_mask[par * 4 + w];
      if ((tail_slot >> 5) == w) m |= 1u << (tail_slot & 31);
      s.pool_mask[pid * 4 + w] = m;
      s.row_mask[r * 4 + w] = m;
    }
    if (r == 0) {
      s.seq[0].kv_base = kv_indptr[0];
      s.seq[0].n_prefix = P + n_new;
      s.seq[0].n_tail = level * K;
      s.seq[0].order = 0;
    }
  }
}

constexpr int MAX_POOL = DRAFT_MAX_POOL;

__global__ __launch_bounds__(1024) void draft_rerank_kernel(DraftState s, const int32_t* __restrict__ d2t,
                                                           const int32_t* __restrict__ tok_new, int n_new, int pool,
                                                           int n_nodes, int32_t* __restrict__ tree_tok,
                                                           int32_t* __restrict__ parent, int32_t* __restrict__ node_depth,
                                                           float* __restrict__ cum_logprob,
                                                           int32_t* __restrict__ chosen_dbg) {
  __shared__ float sc[MAX_POOL];
  __shared__ int16_t node_of[MAX_POOL];       // node id of a kept pool entry, -1 otherwise
  __shared__ int16_t surv[MAX_POOL];          // pool ids that can still be among the best `keep`
  __shared__ int16_t kept[64];                // the kept pool ids, in no particular order
  __shared__ float bound_v;
  __shared__ int bound_i, n_surv, n_kept;
  const int tid = threadIdx.x, keep = n_nodes - 1;
  for (int e = tid; e < pool; e += 1024) { sc[e] = s.pool_score[e]; node_of[e] = -1; }
  if (tid == 0) { bound_v = -INFINITY; bound_i = INT_MAX; n_surv = 0; n_kept = 0; }
  __syncthreads();
  // In the order (score desc, pool id asc) the keep-th best of ANY subset bounds the answer from below: at least
  // `keep` entries are not worse than it, so an entry worse than it cannot be kept.  The subset is the first 2 keep
  // (at least 64) drafted entries: the early levels, whose cumulative scores are the highest.  Ranking by counting
  // then only runs over the survivors.
  const int m = min(pool - 1, max(2 * keep, 64));
  if (m >= keep && tid >= 1 && tid <= m) {
    const float se = sc[tid];
    int rank = 0;
    for (int j = 1; j <= m; ++j) rank += better(sc[j], j, se, tid) ? 1 : 0;
    if (rank == keep - 1) { bound_v = se; bound_i = tid; }
  }
  __syncthreads();
  const float bv = bound_v;
  const int bi = bound_i;
  for (int e = tid; e < pool; e += 1024)
    if (e > 0 && !better(bv, bi, sc[e], e)) surv[atomicAdd(&n_surv, 1)] = (int16_t)e;
  __syncthreads();
  const int T = n_surv;
  for (int t = tid; t < T; t += 1024) {
    const int e = surv[t];
    const float se = sc[e];
    int rank = 0;
    for (int j = 0; j < T; ++j) {
      const int o = surv[j];
      rank += better(sc[o], o, se, e) ? 1 : 0;
    }
    if (rank < keep) kept[atomicAdd(&n_kept, 1)] = (int16_t)e;
  }
  __syncthreads();
  // node ids: the kept entries in ascending pool id (the order they were drafted in), after the root
  if (tid < n_kept) {
    const int e = kept[tid];
    int before = 0;
    for (int j = 0; j < n_kept; ++j) before += kept[j] < e ? 1 : 0;
    node_of[e] = (int16_t)(1 + before);
  }
  if (tid == 0) node_of[0] = 0;
  __syncthreads();
  if (tid == 0) {
    tree_tok[0] = tok_new[n_new - 1];
    parent[0] = -1;
    node_depth[0] = 0;
    cum_logprob[0] = 0.f;
  }
  for (int e = tid; e < pool; e += 1024) {
    const int nid = node_of[e];
    if (e == 0 || nid < 0) continue;
    tree_tok[nid] = d2t[s.pool_tok[e]];
    parent[nid] = node_of[s.pool_parent[e]];
    node_depth[nid] = s.pool_depth[e];
    cum_logprob[nid] = sc[e];
    if (chosen_dbg) chosen_dbg[nid - 1] = e;
  }
}

// ---------------------------------------------------------------------------------------------- batched chains
// Chain drafting for a batch (top-1 per level, no tree): forward 1 runs rows1 rows per sequence (the n_new[b] <= rows1
// positions accepted by the previous step, the rest padding), every later forward one row per sequence.

// Rows of forward 1: row (b, j) sits at position P_b + j, cache slot base_b + P_b + j, and sees the draft context plus
// rows 0..j of its own sequence.  Padding rows (j >= n_new[b]) see the same (their results are never used; their
// cache rows land in slots that later forwards overwrite or that stay invisible).
__global__ __launch_bounds__(64) void chain_prep1_kernel(const int32_t* __restrict__ kv_indptr,
                                                        const int32_t* __restrict__ prefix_len, int B, int rows1,
                                                        int32_t* __restrict__ pos, int32_t* __restrict__ slot,
                                                        uint32_t* __restrict__ mask, SeqInfo* __restrict__ seq) {
  const int b = blockIdx.x, j = threadIdx.x;
  const int P = prefix_len[b], base = kv_indptr[b];
  if (j < rows1) {
    const int r = b * rows1 + j;
    pos[r] = P + j;
    slot[r] = base + P + j;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const int lo = 32 * w;
      mask[r * 4 + w] = j < lo ? 0u : (j - lo >= 31 ? 0xFFFFFFFFu : ((2u << (j - lo)) - 1u));
    }
  }
  if (j == 0) { seq[b].kv_base = base; seq[b].n_prefix = P; seq[b].n_tail = rows1; seq[b].order = b; }
}

// After forward `level` (1-based) of a chain batch: the top-1 token of every sequence's last row extends its chain;
// when level < length, the inputs of the next forward (one row per sequence) are written.
__global__ __launch_bounds__(64) void chain_select_kernel(ChainState s, const int32_t* __restrict__ d2t,
                                                         const int32_t* __restrict__ kv_indptr,
                                                         const int32_t* __restrict__ prefix_len,
                                                         const int32_t* __restrict__ n_new,
                                                         const int32_t* __restrict__ tok_new, int B, int rows1, int level,
                                                         int length, int32_t* __restrict__ chain_tok,
                                                         float* __restrict__ chain_logp) {
  const int b = blockIdx.x * 64 + threadIdx.x;
  if (b >= B) return;
  const int n = min(max(n_new[b], 1), rows1);
  if (level == 1) {                                  // entry 0 of a chain: its root, the last sampled token
    chain_tok[b * (length + 1)] = tok_new[b * rows1 + n - 1];
    chain_logp[b * (length + 1)] = 0.f;
  }
  const int tok = d2t[s.top_idx[b]];
  const float cum = (level == 1 ? 0.f : chain_logp[b * (length + 1) + level - 1]) + s.top_val[b];
  chain_tok[b * (length + 1) + level] = tok;
  chain_logp[b * (length + 1) + level] = cum;
  if (level >= length) return;
  const int P = prefix_len[b], base = kv_indptr[b];
  s.row_tok[b] = tok;
  s.row_src[b] = b;                                  // the gathered / previous output row of this sequence
  s.row_pos[b] = P + n - 1 + level;
  s.row_slot[b] = base + P + n + (level - 1);
  const int tail = level;                            // chain rows visible to the new row, itself included
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const int lo = 32 * w;
    s.row_mask[b * 4 + w] = tail <= lo ? 0u : (tail - lo >= 32 ? 0xFFFFFFFFu : ((1u << (tail - lo)) - 1u));
  }
  s.seq[b].kv_base = base;
  s.seq[b].n_prefix = P + n;
  s.seq[b].n_tail = level;
  s.seq[b].order = b;
}

// x_out[b] = x[b * rows1 + n_new[b] - 1]: the output row of every sequence's last real position.
__global__ __launch_bounds__(256) void chain_gather_kernel(const float* __restrict__ x, const int32_t* __restrict__ n_new,
                                                          int rows1, int k, float* __restrict__ x_out) {
  const int b = blockIdx.x;
  const int n = min(max(n_new[b], 1), rows1);
  const float4* src = (const float4*)(x + ((size_t)b * rows1 + n - 1) * k);
  float4* dst = (float4*)(x_out + (size_t)b * k);
  for (int c = threadIdx.x; c < k / 4; c += 256) dst[c] = src[c];
}

}  // namespace

hipError_t launch_chain_prep1(const int32_t* kv_indptr, const int32_t* prefix_len, int B, int rows1, int32_t* pos,
                              int32_t* slot, uint32_t* mask, SeqInfo* seq, hipStream_t st) {
  if (rows1 < 1 || rows1 > 64) return hipErrorInvalidValue;
  hipLaunchKernelGGL(chain_prep1_kernel, dim3(B), dim3(64), 0, st, kv_indptr, prefix_len, B, rows1, pos, slot, mask, seq);
  return hipGetLastError();
}
hipError_t launch_chain_select(const ChainState& s, const int32_t* d2t, const int32_t* kv_indptr, const int32_t* prefix_len,
                               const int32_t* n_new, const int32_t* tok_new, int B, int rows1, int level, int length,
                               int32_t* chain_tok, float* chain_logp, hipStream_t st) {
  if (length > 120) return hipErrorInvalidValue;
  hipLaunchKernelGGL(chain_select_kernel, dim3((B + 63) / 64), dim3(64), 0, st, s, d2t, kv_indptr, prefix_len, n_new, tok_new, B,
                     rows1, level, length, chain_tok, chain_logp);
  return hipGetLastError();
}
hipError_t launch_chain_gather(const float* x, const int32_t* n_new, int B, int rows1, int k, float* x_out, hipStream_t st) {
  hipLaunchKernelGGL(chain_gather_kernel, dim3(B), dim3(256), 0, st, x, n_new, rows1, k, x_out);
  return hipGetLastError();
}

size_t topk_scratch_floats(int n_rows, int V, int K) {
  const size_t n_spans = (size_t)(V + TOPK_SPAN - 1) / TOPK_SPAN;
  return (size_t)n_rows * n_spans * (2 * (size_t)K + 2);
}

hipError_t launch_topk_rows(const float* z, int ld, int row0, int n_rows, int V, int K, float* scratch, float* top_val,
                            int32_t* top_idx, hipStream_t st) {
  if (n_rows <= 0 || V <= 0 || K <= 0 || K > TOPK_MAX_K) return hipErrorInvalidValue;
  const int n_spans = (V + TOPK_SPAN - 1) / TOPK_SPAN;
  if (n_spans > TOPK_MAX_SPANS) return hipErrorInvalidValue;
  float* cand_val = scratch;
  int32_t* cand_idx = (int32_t*)(scratch + (size_t)n_rows * n_spans * K);
  float* span_stat = scratch + 2 * (size_t)n_rows * n_spans * K;
  hipLaunchKernelGGL(topk_spans_kernel, dim3((n_spans + 3) / 4, n_rows), dim3(256), 0, st, z, ld, row0, V, K, n_spans,
                     cand_val, cand_idx, span_stat);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(topk_merge_kernel, dim3(n_rows), dim3(64), 0, st, cand_val, cand_idx, span_stat, n_spans, K, top_val,
                     top_idx);
  return hipGetLastError();
}

hipError_t launch_draft_select(const DraftState& s, const int32_t* d2t, const int32_t* kv_indptr, const int32_t* prefix_len,
                               int level, int depth, int K, int n_new, int /*feat_row0*/, hipStream_t st) {
  if (K * K > 256) return hipErrorInvalidValue;
  hipLaunchKernelGGL(draft_select_kernel, dim3(1), dim3(256), 0, st, s, d2t, kv_indptr, prefix_len, level, depth, K, n_new);
  return hipGetLastError();
}

hipError_t launch_draft_rerank(const DraftState& s, const int32_t* d2t, const int32_t* tok_new, int n_new, int depth, int K,
                               int n_nodes, int32_t* tree_tok, int32_t* parent, int32_t* node_depth, float* cum_logprob,
                               int32_t* chosen_dbg, hipStream_t st) {
  const int pool = 1 + K + (depth - 1) * K * K;
  if (pool > MAX_POOL || n_nodes - 1 > pool - 1 || n_nodes - 1 > 64) return hipErrorInvalidValue;   // the kept list holds 64
  hipLaunchKernelGGL(draft_rerank_kernel, dim3(1), dim3(1024), 0, st, s, d2t, tok_new, n_new, pool, n_nodes, tree_tok,
                     parent, node_depth, cum_logprob, chosen_dbg);
  return hipGetLastError();
}
