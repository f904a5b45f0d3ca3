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
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float v = __shfl_xor(x.v, o, 64);
    const int i = __shfl_xor(x.i, o, 64);
    if (better(v, i, x.v, x.i)) { x.v = v; x.i = i; }
  }
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

// Row top-K with the row held in registers (V <= 1024 * EPT): every thread keeps the best of its own
// entries; each of the K rounds is one block-wide arg-max, after which only the winning thread rescans.
template <int EPT>
__global__ __launch_bounds__(1024) void topk_rows_kernel(const float* __restrict__ z, int ld, int row0, int V, int K,
                                                        float* __restrict__ top_val, int32_t* __restrict__ top_idx) {
  __shared__ float red[17];
  __shared__ ValIdx redv[17];
  const float* zr = z + (size_t)(row0 + blockIdx.x) * ld;
  const int tid = threadIdx.x;
  float v[EPT];
  float mx = -INFINITY;
#pragma unroll
  for (int j = 0; j < EPT; ++j) {
    const int c = tid + j * 1024;
    v[j] = c < V ? zr[c] : -INFINITY;
    mx = fmaxf(mx, v[j]);
  }
  mx = block_max(mx, red);
  float sum = 0.f;
#pragma unroll
  for (int j = 0; j < EPT; ++j) sum += expf(v[j] - mx);          // exp(-inf) = 0 for the padding
  sum = block_sum(sum, red);
  const float lse = logf(sum);
  for (int r = 0; r < K; ++r) {
    ValIdx b = {-INFINITY, INT_MAX};
#pragma unroll
    for (int j = 0; j < EPT; ++j)
      if (v[j] > b.v) { b.v = v[j]; b.i = tid + j * 1024; }      // ascending index per thread: first maximum kept
    b = block_best(b, redv);
    if (tid == 0) {
      top_val[blockIdx.x * K + r] = b.v - mx - lse;
      top_idx[blockIdx.x * K + r] = b.i;
    }
    if ((b.i & 1023) == tid) {
#pragma unroll
      for (int j = 0; j < EPT; ++j)
        if (j == (b.i >> 10)) v[j] = -INFINITY;
    }
  }
}

// Any V: K passes over the row in global memory.
__global__ __launch_bounds__(1024) void topk_rows_big_kernel(const float* __restrict__ z, int ld, int row0, int V, int K,
                                                            float* __restrict__ top_val, int32_t* __restrict__ top_idx) {
  __shared__ float red[17];
  __shared__ ValIdx redv[17];
  const float* zr = z + (size_t)(row0 + blockIdx.x) * ld;
  const int tid = threadIdx.x;
  float mx = -INFINITY;
  for (int c = tid; c < V; c += 1024) mx = fmaxf(mx, zr[c]);
  mx = block_max(mx, red);
  float sum = 0.f;
  for (int c = tid; c < V; c += 1024) sum += expf(zr[c] - mx);
  sum = block_sum(sum, red);
  const float lse = logf(sum);
  float pv = INFINITY;
  int pi = -1;
  for (int r = 0; r < K; ++r) {
    ValIdx b = {-INFINITY, INT_MAX};
    for (int c = tid; c < V; c += 1024) {
      const float v = zr[c];
      if ((v < pv || (v == pv && c > pi)) && better(v, c, b.v, b.i)) { b.v = v; b.i = c; }
    }
    b = block_best(b, redv);
    if (tid == 0) {
      top_val[blockIdx.x * K + r] = b.v - mx - lse;
      top_idx[blockIdx.x * K + r] = b.i;
    }
    pv = b.v;
    pi = b.i;
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
      s.seq[0].pad = 0;
    }
  }
}

constexpr int MAX_POOL = 2048;

__global__ __launch_bounds__(1024) void draft_rerank_kernel(DraftState s, const int32_t* __restrict__ d2t,
                                                           const int32_t* __restrict__ tok_new, int n_new, int pool,
                                                           int n_nodes, int32_t* __restrict__ tree_tok,
                                                           int32_t* __restrict__ parent, int32_t* __restrict__ node_depth,
                                                           float* __restrict__ cum_logprob,
                                                           int32_t* __restrict__ chosen_dbg) {
  __shared__ float sc[MAX_POOL];
  __shared__ int16_t node_of[MAX_POOL];       // node id of a kept pool entry, -1 otherwise
  const int tid = threadIdx.x, keep = n_nodes - 1;
  for (int e = tid; e < pool; e += 1024) sc[e] = s.pool_score[e];
  __syncthreads();
  for (int e = tid; e < pool; e += 1024) {
    int rank = 0;
    if (e > 0)
      for (int j = 1; j < pool; ++j) rank += better(sc[j], j, sc[e], e) ? 1 : 0;
    node_of[e] = (e > 0 && rank < keep) ? 1 : 0;
  }
  __syncthreads();
  int my_node[(MAX_POOL + 1023) / 1024];
#pragma unroll
  for (int it = 0; it < (MAX_POOL + 1023) / 1024; ++it) {
    const int e = tid + it * 1024;
    my_node[it] = -1;
    if (e < pool && e > 0 && node_of[e]) {
      int before = 0;
      for (int j = 1; j < e; ++j) before += node_of[j];
      my_node[it] = 1 + before;                  // kept entries in ascending pool id
    }
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < (MAX_POOL + 1023) / 1024; ++it) {
    const int e = tid + it * 1024;
    if (e < pool) node_of[e] = e == 0 ? 0 : (int16_t)my_node[it];
  }
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

}  // namespace

hipError_t launch_topk_rows(const float* z, int ld, int row0, int n_rows, int V, int K, float* top_val, int32_t* top_idx,
                            hipStream_t st) {
  if (V <= 8 * 1024)
    hipLaunchKernelGGL(topk_rows_kernel<8>, dim3(n_rows), dim3(1024), 0, st, z, ld, row0, V, K, top_val, top_idx);
  else if (V <= 32 * 1024)
    hipLaunchKernelGGL(topk_rows_kernel<32>, dim3(n_rows), dim3(1024), 0, st, z, ld, row0, V, K, top_val, top_idx);
  else
    hipLaunchKernelGGL(topk_rows_big_kernel, dim3(n_rows), dim3(1024), 0, st, z, ld, row0, V, K, top_val, top_idx);
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
  if (pool > MAX_POOL || n_nodes - 1 > pool - 1) return hipErrorInvalidValue;
  hipLaunchKernelGGL(draft_rerank_kernel, dim3(1), dim3(1024), 0, st, s, d2t, tok_new, n_new, pool, n_nodes, tree_tok,
                     parent, node_depth, cum_logprob, chosen_dbg);
  return hipGetLastError();
}
