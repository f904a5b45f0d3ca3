// Commit of an accepted path: what one speculative step hands to the next.
//   * the cache rows of the accepted nodes (written by the verification at slots prefix + node id) are moved to
//     slots prefix + 0, 1, 2, ... in path order, in every layer, in place;
//   * the low / mid / high features of the accepted nodes are gathered in path order (the next step's fusion input);
//   * the token FOLLOWING each accepted position is written (the next node on the path, the bonus token after the
//     last one), the prefix lengths grow by accept_len + 1.
// Moving rows in place: destination j reads source path[j] >= j.  A thread owns one 16-byte column of a row and
// moves it for EIGHT consecutive path positions at a time, reading all eight sources before it writes; windows go
// in ascending order.  A destination of window w (slots <= 8w + 8) is never the source of a later window (their
// sources are > 8w + 8), and inside a window every read precedes every write, so no row is overwritten before it
// has been read.
#include "common.hpp"
#include "kernels.hpp"

namespace {

constexpr int LAYERS_PER_LAUNCH = 16;
struct CachePtrs { void* k[LAYERS_PER_LAUNCH]; void* v[LAYERS_PER_LAUNCH]; };

__global__ __launch_bounds__(256) void commit_kv_kernel(CachePtrs cp, const int32_t* __restrict__ kv_indptr,
                                                       const int32_t* __restrict__ prefix_len,
                                                       const int32_t* __restrict__ path,
                                                       const int32_t* __restrict__ accept_len, int N, int rows,
                                                       int row_bytes) {
  const int b = blockIdx.y, which = blockIdx.z;                   // which = 2 * layer + (0: keys, 1: values)
  unsigned char* base = (unsigned char*)((which & 1) ? cp.v[which >> 1] : cp.k[which >> 1]);
  const int a = min(max(accept_len[b], 0), min(N, rows) - 1);
  const size_t first = ((size_t)kv_indptr[b] + prefix_len[b]) * row_bytes;       // the root's row
  const int col = (blockIdx.x * 256 + threadIdx.x) * 16;
  if (col >= row_bytes) return;
  for (int j0 = 1; j0 <= a; j0 += 8) {
    uint4 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int j = min(j0 + i, a);
      const int src = min(max(path[b * N + j], 0), N - 1);
      v[i] = *(const uint4*)(base + first + (size_t)src * row_bytes + col);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (j0 + i <= a) *(uint4*)(base + first + (size_t)(j0 + i) * row_bytes + col) = v[i];
  }
}

// One workgroup per (sequence, path position j <= accept_len): the three feature rows and the following token.
__global__ __launch_bounds__(256) void commit_rows_kernel(const int32_t* __restrict__ tree_tok, const int32_t* __restrict__ path,
                                                         const int32_t* __restrict__ accept_len,
                                                         const int32_t* __restrict__ bonus, const float* __restrict__ taps,
                                                         int B, int N, int k, int rows, float* __restrict__ taps_new,
                                                         int32_t* __restrict__ tok_new) {
  const int j = blockIdx.x, b = blockIdx.y;
  const int a = min(max(accept_len[b], 0), min(N, rows) - 1);
  if (j > a) return;
  const int node = min(max(path[b * N + j], 0), N - 1);
  if (taps_new)
    for (int t = 0; t < 3; ++t) {
      const float4* src = (const float4*)(taps + (((size_t)t * B + b) * N + node) * k);
      float4* dst = (float4*)(taps_new + (((size_t)t * B + b) * rows + j) * k);
      for (int c = threadIdx.x; c < k / 4; c += 256) dst[c] = src[c];
    }
  if (threadIdx.x == 0)
    tok_new[b * rows + j] = j < a ? tree_tok[b * N + min(max(path[b * N + j + 1], 0), N - 1)] : bonus[b];
}

// Runs after every reader of the old prefix lengths.
__global__ __launch_bounds__(64) void commit_lengths_kernel(const int32_t* __restrict__ accept_len, int B, int N, int rows,
                                                           int32_t* __restrict__ prefix_len, int32_t* __restrict__ n_new,
                                                           int32_t* __restrict__ draft_prefix_len, int draft_rows) {
  const int b = blockIdx.x * 64 + threadIdx.x;
  if (b >= B) return;
  const int n = min(max(accept_len[b], 0), min(N, rows) - 1) + 1;
  prefix_len[b] += n;
  n_new[b] = n;
  if (draft_prefix_len) draft_prefix_len[b] += draft_rows;
}

}  // namespace

hipError_t launch_commit(void* const* k_layers, void* const* v_layers, int n_layers, const int32_t* kv_indptr,
                         int32_t* prefix_len, const int32_t* tree_tok, const int32_t* path, const int32_t* accept_len,
                         const int32_t* bonus, const float* taps, int B, int N, int hidden, int row_bytes, int rows,
                         float* taps_new, int32_t* tok_new, int32_t* n_new, int32_t* draft_prefix_len, int draft_rows,
                         hipStream_t st) {
  if (row_bytes % 16 || hidden % 4 || rows < 1 || N < 1) return hipErrorInvalidValue;
  for (int l0 = 0; l0 < n_layers; l0 += LAYERS_PER_LAUNCH) {
    CachePtrs cp;
    const int nl = n_layers - l0 < LAYERS_PER_LAUNCH ? n_layers - l0 : LAYERS_PER_LAUNCH;
    for (int i = 0; i < LAYERS_PER_LAUNCH; ++i) {
      cp.k[i] = i < nl ? k_layers[l0 + i] : nullptr;
      cp.v[i] = i < nl ? v_layers[l0 + i] : nullptr;
    }
    hipLaunchKernelGGL(commit_kv_kernel, dim3((row_bytes / 16 + 255) / 256, B, 2 * nl), dim3(256), 0, st, cp, kv_indptr,
                       prefix_len, path, accept_len, N, rows, row_bytes);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(commit_rows_kernel, dim3(N < rows ? N : rows, B), dim3(256), 0, st, tree_tok, path, accept_len, bonus,
                     taps, B, N, hidden, rows, taps_new, tok_new);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(commit_lengths_kernel, dim3((B + 63) / 64), dim3(64), 0, st, accept_len, B, N, rows, prefix_len, n_new,
                     draft_prefix_len, draft_rows);
  return hipGetLastError();
}
