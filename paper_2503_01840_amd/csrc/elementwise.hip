// Row-wise kernels between the GEMMs: embedding gather, residual add + RMSNorm, rotary embedding and
// cache write, tree bookkeeping, SwiGLU (fp32 path), feature packing.  All are tiny next to the weight
// streams; they exist to hand the next GEMM its operand in the layout it reads.
#include <algorithm>

#include "common.hpp"
#include "kernels.hpp"

namespace {

template <typename TW>
__global__ __launch_bounds__(256) void embed_rows_kernel(const TW* __restrict__ embed, const int32_t* __restrict__ tok,
                                                        int k, int vocab, float* __restrict__ x) {
  const int r = blockIdx.x;
  const int t = min(max(tok[r], 0), vocab - 1);
  for (int c = threadIdx.x; c < k; c += 256) x[(size_t)r * k + c] = load_f32(embed, (size_t)t * k + c);
}

struct CopyOut { float* p[4]; };

// One workgroup per row, four consecutive columns per thread (two such groups when k > 4096): the row stays
// in registers between the partial-sum reduction and the normalised store.
template <bool BF16>
__global__ __launch_bounds__(1024) void add_norm_kernel(float* __restrict__ x, const float* __restrict__ partial, int S,
                                                       int R, int k, const typename Act<BF16>::type* __restrict__ gain,
                                                       float eps, typename Act<BF16>::type* __restrict__ act, CopyOut co) {
  __shared__ float red[17];
  const int r = blockIdx.x, nvec = k >> 2, bd = blockDim.x;
  constexpr int VPT = 2;
  float4 val[VPT];
  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < VPT; ++j) {
    const int v = threadIdx.x + j * bd;
    if (v < nvec) {
      float4 a = *(const float4*)(x + (size_t)r * k + 4 * v);
      // four partial sums per round, all requested before the first is added (one memory round trip per round
      // instead of one per partial sum); the order of the additions stays s = 0, 1, 2, ...
      for (int s0 = 0; s0 < S; s0 += 4) {
        float4 p[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) p[i] = *(const float4*)(partial + ((size_t)min(s0 + i, S - 1) * R + r) * k + 4 * v);
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (s0 + i < S) { a.x += p[i].x; a.y += p[i].y; a.z += p[i].z; a.w += p[i].w; }
      }
      *(float4*)(x + (size_t)r * k + 4 * v) = a;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (co.p[i]) *(float4*)(co.p[i] + (size_t)r * k + 4 * v) = a;
      ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
      val[j] = a;
    }
  }
  float4 g[VPT];                                      // requested before the reduction, used after it
  if (act != nullptr) {
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
      const int v = threadIdx.x + j * bd;
      if (v < nvec) g[j] = load4_f32(gain, 4 * v);
    }
  }
  ss = block_sum(ss, red);
  if (act == nullptr) return;
  const float inv = 1.0f / sqrtf(ss / (float)k + eps);
#pragma unroll
  for (int j = 0; j < VPT; ++j) {
    const int v = threadIdx.x + j * bd;
    if (v < nvec)
      Act<BF16>::store4(act, r, 4 * v, k, val[j].x * inv * g[j].x, val[j].y * inv * g[j].y, val[j].z * inv * g[j].z,
                        val[j].w * inv * g[j].w);
  }
}

// cos/sin of pos * theta^(-2i/d) in fp64, stored fp32: cs[r][i] = cos, cs[r][d/2 + i] = sin
__device__ __forceinline__ void rope_entry(float* cs, int r, int i, int d, int pos, float theta) {
  const double inv = pow((double)theta, -2.0 * (double)i / (double)d);
  double s, c;
  sincos((double)pos * inv, &s, &c);
  cs[(size_t)r * d + i] = (float)c;
  cs[(size_t)r * d + d / 2 + i] = (float)s;
}

__global__ __launch_bounds__(256) void tree_prep_kernel(const int32_t* __restrict__ parent,
                                                       const int32_t* __restrict__ kv_indptr,
                                                       const int32_t* __restrict__ prefix_len, int N, int d, float theta,
                                                       int32_t* __restrict__ depth, uint32_t* __restrict__ mask,
                                                       int32_t* __restrict__ slot, float* __restrict__ cs,
                                                       SeqInfo* __restrict__ seq) {
  // Workgroup (b, y): every y walks sequence b's tree (parents staged in LDS: one memory round trip, then the walks
  // stay on chip) and fills its share of the rotary table, whose sines and cosines are the bulk of the work; y = 0
  // also writes the masks, depths, slots and the sequence record.
  __shared__ int sdepth[64], spar[64];
  __shared__ int rank;
  const int b = blockIdx.x, y = blockIdx.y, i = threadIdx.x, B = gridDim.x;
  const int P = prefix_len[b], base = kv_indptr[b];
  if (i < N) spar[i] = parent[b * N + i];
  if (i == 0) rank = 0;
  __syncthreads();
  if (y == 0) {
    // rank of this sequence by prefix length, longest first (ties: smaller index first): attention hands out its
    // workgroups in that order, so that the long sequences start first and the short ones fill the tail
    int longer = 0;
    for (int o = i; o < B; o += 256) {
      const int Po = prefix_len[o];
      longer += (Po > P || (Po == P && o < b)) ? 1 : 0;
    }
    if (longer) atomicAdd(&rank, longer);
  }
  if (i < N) {
    uint32_t m[4] = {0u, 0u, 0u, 0u};
    int cur = i, dep = 0;
    for (int it = 0; it < N; ++it) {                     // bounded walk: malformed parents cannot loop
      m[cur >> 5] |= 1u << (cur & 31);
      const int p = spar[cur];
      if (p < 0 || p >= cur) break;
      cur = p;
      ++dep;
    }
    sdepth[i] = dep;
    if (y == 0) {
      const int r = b * N + i;
      depth[r] = dep;
      slot[r] = base + P + i;
#pragma unroll
      for (int w = 0; w < 4; ++w) mask[r * 4 + w] = m[w];
    }
  }
  __syncthreads();
  if (y == 0 && i == 0) {
    seq[rank].order = b;
    seq[b].kv_base = base; seq[b].n_prefix = P; seq[b].n_tail = N;
  }
  const int half = d / 2;
  for (int e = y * 256 + i; e < N * half; e += 256 * gridDim.y) {
    const int row = e / half, f = e % half;
    rope_entry(cs, b * N + row, f, d, P + sdepth[row], theta);
  }
}

// One workgroup per row; a thread handles four consecutive rotary pairs (i..i+3, i+d/2..i+d/2+3) of one head.
template <bool BF16>
__global__ __launch_bounds__(1024) void rope_kv_write_kernel(const float* __restrict__ qkv, int S, int R, int H, int Hkv,
                                                            int d, const float* __restrict__ cs,
                                                            const int32_t* __restrict__ slot,
                                                            typename Act<BF16>::type* __restrict__ q,
                                                            typename Act<BF16>::type* __restrict__ kc,
                                                            typename Act<BF16>::type* __restrict__ vc) {
  typedef typename Act<BF16>::type T;
  const int r = blockIdx.x, half = d / 2, NT = (H + 2 * Hkv) * d, q4 = half / 4;
  const size_t sl = (size_t)slot[r];
  for (int e = threadIdx.x; e < (H + 2 * Hkv) * q4; e += blockDim.x) {
    const int h = e / q4, i = (e % q4) * 4;
    float4 x1 = make_float4(0.f, 0.f, 0.f, 0.f), x2 = x1;
    for (int s0 = 0; s0 < S; s0 += 4) {                 // four partial sums per memory round trip, added in order
      float4 a[4], b[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float* row = qkv + ((size_t)min(s0 + j, S - 1) * R + r) * NT + h * d;
        a[j] = *(const float4*)(row + i);
        b[j] = *(const float4*)(row + i + half);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (s0 + j < S) {
          x1.x += a[j].x; x1.y += a[j].y; x1.z += a[j].z; x1.w += a[j].w;
          x2.x += b[j].x; x2.y += b[j].y; x2.z += b[j].z; x2.w += b[j].w;
        }
    }
    T* dst;
    if (h < H + Hkv) {
      const float4 c = *(const float4*)(cs + (size_t)r * d + i), sn = *(const float4*)(cs + (size_t)r * d + half + i);
      const float4 o1 = make_float4(x1.x * c.x - x2.x * sn.x, x1.y * c.y - x2.y * sn.y, x1.z * c.z - x2.z * sn.z,
                                    x1.w * c.w - x2.w * sn.w);
      const float4 o2 = make_float4(x2.x * c.x + x1.x * sn.x, x2.y * c.y + x1.y * sn.y, x2.z * c.z + x1.z * sn.z,
                                    x2.w * c.w + x1.w * sn.w);
      x1 = o1; x2 = o2;
      dst = h < H ? q + ((size_t)r * H + h) * d : kc + (sl * Hkv + (h - H)) * d;
    } else {
      dst = vc + (sl * Hkv + (h - H - Hkv)) * d;
    }
    store4_plain(dst, i, x1.x, x1.y, x1.z, x1.w);
    store4_plain(dst, i + half, x2.x, x2.y, x2.z, x2.w);
  }
}

__global__ __launch_bounds__(256) void swiglu_f32_kernel(const float* __restrict__ gu, int I, float* __restrict__ h) {
  const int r = blockIdx.x;
  for (int c = threadIdx.x; c < I; c += 256) {
    const float g = gu[(size_t)r * 2 * I + c], u = gu[(size_t)r * 2 * I + I + c];
    h[(size_t)r * I + c] = g / (1.f + expf(-g)) * u;
  }
}

template <bool BF16>
__global__ __launch_bounds__(256) void pack3_kernel(const float* __restrict__ a, const float* __restrict__ b,
                                                   const float* __restrict__ c, int k,
                                                   typename Act<BF16>::type* __restrict__ act) {
  const int r = blockIdx.x;
  for (int j = blockIdx.y * 256 + threadIdx.x; j < k; j += 256 * gridDim.y) {
    Act<BF16>::store(act, r, j, 3 * k, a[(size_t)r * k + j]);
    Act<BF16>::store(act, r, k + j, 3 * k, b[(size_t)r * k + j]);
    Act<BF16>::store(act, r, 2 * k + j, 3 * k, c[(size_t)r * k + j]);
  }
}

__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ partial, int S, size_t MN,
                                                             float* __restrict__ out) {
  for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < MN; e += (size_t)gridDim.x * 256) {
    float v = 0.f;
    for (int s = 0; s < S; ++s) v += partial[(size_t)s * MN + e];
    out[e] = v;
  }
}

// One workgroup per row, four consecutive columns per thread and pass, the row kept in registers between the
// sum-of-squares pass and the normalising pass (k <= 4 * 4 * blockDim.x).
template <bool BF16>
__global__ __launch_bounds__(1024) void draft_input_kernel(const typename Act<BF16>::type* __restrict__ embed, int vocab,
                                                          const int32_t* __restrict__ tok, const float* __restrict__ feat,
                                                          const int32_t* __restrict__ src_row, int k,
                                                          const typename Act<BF16>::type* __restrict__ g_embed,
                                                          const typename Act<BF16>::type* __restrict__ g_feat, float eps,
                                                          typename Act<BF16>::type* __restrict__ act,
                                                          float* __restrict__ y, const int32_t* __restrict__ pos,
                                                          int head_dim, float theta, float* __restrict__ cs) {
  __shared__ float red_e[17], red_f[17];
  const int r = blockIdx.x;
  const int t = min(max(tok[r], 0), vocab - 1);
  const float* f = feat + (size_t)(src_row ? src_row[r] : r) * k;
  float4 e[4], v[4];
  float se = 0.f, sf = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int c = 4 * (threadIdx.x + j * blockDim.x);
    if (c < k) {
      e[j] = load4_f32(embed, (size_t)t * k + c);
      v[j] = *(const float4*)(f + c);
      *(float4*)(y + (size_t)r * k + c) = v[j];
      se += e[j].x * e[j].x + e[j].y * e[j].y + e[j].z * e[j].z + e[j].w * e[j].w;
      sf += v[j].x * v[j].x + v[j].y * v[j].y + v[j].z * v[j].z + v[j].w * v[j].w;
    }
  }
  se = block_sum(se, red_e);
  sf = block_sum(sf, red_f);
  const float ie = 1.0f / sqrtf(se / (float)k + eps), iv = 1.0f / sqrtf(sf / (float)k + eps);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int c = 4 * (threadIdx.x + j * blockDim.x);
    if (c < k) {
      const float4 ge = load4_f32(g_embed, c), gf = load4_f32(g_feat, c);
      Act<BF16>::store4(act, r, c, 2 * k, e[j].x * ie * ge.x, e[j].y * ie * ge.y, e[j].z * ie * ge.z, e[j].w * ie * ge.w);
      Act<BF16>::store4(act, r, k + c, 2 * k, v[j].x * iv * gf.x, v[j].y * iv * gf.y, v[j].z * iv * gf.z, v[j].w * iv * gf.w);
    }
  }
  // the row's rotary table, for the q/k rotation that follows the projection
  for (int i = threadIdx.x; i < head_dim / 2; i += blockDim.x) rope_entry(cs, r, i, head_dim, pos[r], theta);
}

__global__ __launch_bounds__(64) void draft_prep1_kernel(const int32_t* __restrict__ kv_indptr,
                                                        const int32_t* __restrict__ prefix_len, int n_new,
                                                        int32_t* __restrict__ pos, int32_t* __restrict__ slot,
                                                        uint32_t* __restrict__ mask, SeqInfo* __restrict__ seq) {
  const int j = threadIdx.x, P = prefix_len[0], base = kv_indptr[0];
  if (j < n_new) {
    pos[j] = P + j;
    slot[j] = base + P + j;
#pragma unroll
    for (int w = 0; w < 4; ++w) {                        // causal among the new rows: bits 0..j
      const int lo = 32 * w;
      mask[j * 4 + w] = j < lo ? 0u : (j - lo >= 31 ? 0xFFFFFFFFu : ((2u << (j - lo)) - 1u));
    }
  }
  if (j == 0) { seq[0].kv_base = base; seq[0].n_prefix = P; seq[0].n_tail = n_new; seq[0].order = 0; }
}

// parent[i] = i - 1: a chain (ordinary causal decoding as a tree)
__global__ __launch_bounds__(64) void chain_parent_kernel(int32_t* __restrict__ parent, int n) {
  if ((int)threadIdx.x < n) parent[threadIdx.x] = (int)threadIdx.x - 1;
}
__global__ __launch_bounds__(64) void advance_lengths_kernel(int32_t* __restrict__ len, int B, int by) {
  const int b = blockIdx.x * 64 + threadIdx.x;
  if (b < B) len[b] += by;
}

}  // namespace

hipError_t launch_chain_parent(int32_t* parent, int n, hipStream_t st) {
  if (n > 64) return hipErrorInvalidValue;
  hipLaunchKernelGGL(chain_parent_kernel, dim3(1), dim3(64), 0, st, parent, n);
  return hipGetLastError();
}
hipError_t launch_advance_lengths(int32_t* len, int B, int by, hipStream_t st) {
  hipLaunchKernelGGL(advance_lengths_kernel, dim3((B + 63) / 64), dim3(64), 0, st, len, B, by);
  return hipGetLastError();
}

#define DISPATCH_BF16(flag, KERNEL, grid, block, st, ...)                                       \
  do {                                                                                          \
    if (flag) hipLaunchKernelGGL(KERNEL<true>, grid, block, 0, st, __VA_ARGS__);               \
    else hipLaunchKernelGGL(KERNEL<false>, grid, block, 0, st, __VA_ARGS__);                   \
  } while (0)

hipError_t launch_embed_rows(bool bf16, const void* embed, const int32_t* tok, int R, int k, int vocab, float* x,
                             hipStream_t st) {
  if (bf16) hipLaunchKernelGGL(embed_rows_kernel<bf16_t>, dim3(R), dim3(256), 0, st, (const bf16_t*)embed, tok, k, vocab, x);
  else hipLaunchKernelGGL(embed_rows_kernel<float>, dim3(R), dim3(256), 0, st, (const float*)embed, tok, k, vocab, x);
  return hipGetLastError();
}

hipError_t launch_add_norm(bool bf16, float* x, const float* partial, int S, int R, int k, const void* gain, float eps,
                           void* act, float* const copy_out[4], hipStream_t st) {
  CopyOut co;
  for (int i = 0; i < 4; ++i) co.p[i] = copy_out ? copy_out[i] : nullptr;
  if (k % 4 || k > 8192) return hipErrorInvalidValue;
  const int bd = std::min(1024, (k / 4 + 63) / 64 * 64);
  if (bf16)
    hipLaunchKernelGGL(add_norm_kernel<true>, dim3(R), dim3(bd), 0, st, x, partial, S, R, k, (const bf16_t*)gain, eps,
                       (bf16_t*)act, co);
  else
    hipLaunchKernelGGL(add_norm_kernel<false>, dim3(R), dim3(bd), 0, st, x, partial, S, R, k, (const float*)gain, eps,
                       (float*)act, co);
  return hipGetLastError();
}

hipError_t launch_tree_prep(const int32_t* parent, const int32_t* kv_indptr, const int32_t* prefix_len, int B, int N,
                            int head_dim, float theta, int32_t* depth, uint32_t* mask, int32_t* slot, float* cs,
                            SeqInfo* seq, hipStream_t st) {
  if (N > 64) return hipErrorInvalidValue;
  // enough workgroups that each thread computes one or two table entries, no more than ~1024 workgroups in all
  const int per_seq = std::max(1, std::min((N * (head_dim / 2) + 511) / 512, std::max(1, 1024 / B)));
  hipLaunchKernelGGL(tree_prep_kernel, dim3(B, per_seq), dim3(256), 0, st, parent, kv_indptr, prefix_len, N, head_dim, theta, depth,
                     mask, slot, cs, seq);
  return hipGetLastError();
}

hipError_t launch_rope_kv_write(bool bf16, const float* qkv_partial, int S, int R, int H, int Hkv, int d, const float* cs,
                                const int32_t* slot, void* q, void* kcache, void* vcache, hipStream_t st) {
  if (d % 8) return hipErrorInvalidValue;
  const int bd = std::min(1024, ((H + 2 * Hkv) * d / 8 + 63) / 64 * 64);
  if (bf16)
    hipLaunchKernelGGL(rope_kv_write_kernel<true>, dim3(R), dim3(bd), 0, st, qkv_partial, S, R, H, Hkv, d, cs, slot,
                       (bf16_t*)q, (bf16_t*)kcache, (bf16_t*)vcache);
  else
    hipLaunchKernelGGL(rope_kv_write_kernel<false>, dim3(R), dim3(bd), 0, st, qkv_partial, S, R, H, Hkv, d, cs, slot,
                       (float*)q, (float*)kcache, (float*)vcache);
  return hipGetLastError();
}

hipError_t launch_swiglu_f32(const float* gu, int R, int I, float* h, hipStream_t st) {
  hipLaunchKernelGGL(swiglu_f32_kernel, dim3(R), dim3(256), 0, st, gu, I, h);
  return hipGetLastError();
}

hipError_t launch_pack3(bool bf16, const float* a, const float* b, const float* c, int M, int k, void* act, hipStream_t st) {
  const dim3 grid(M, std::max(1, std::min(k / 512, 64 / std::max(M, 1))));   // few rows: several workgroups per row
  if (bf16) hipLaunchKernelGGL(pack3_kernel<true>, grid, dim3(256), 0, st, a, b, c, k, (bf16_t*)act);
  else hipLaunchKernelGGL(pack3_kernel<false>, grid, dim3(256), 0, st, a, b, c, k, (float*)act);
  return hipGetLastError();
}

hipError_t launch_reduce_partials(const float* partial, int S, int M, int N, float* out, hipStream_t st) {
  const size_t MN = (size_t)M * N;
  const int blocks = (int)((MN + 255) / 256 < 1024 ? (MN + 255) / 256 : 1024);
  hipLaunchKernelGGL(reduce_partials_kernel, dim3(blocks), dim3(256), 0, st, partial, S, MN, out);
  return hipGetLastError();
}

hipError_t launch_draft_input(bool bf16, const void* embed, int vocab, const int32_t* tok, const float* feat,
                              const int32_t* src_row, int M, int k, const void* g_embed, const void* g_feat, float eps,
                              void* act, float* y, const int32_t* pos, int head_dim, float theta, float* cs, hipStream_t st) {
  if (k % 4 || k > 16384) return hipErrorInvalidValue;
  const int threads = std::min(1024, ((k / 4 + 63) / 64) * 64);
  if (bf16)
    hipLaunchKernelGGL(draft_input_kernel<true>, dim3(M), dim3(threads), 0, st, (const bf16_t*)embed, vocab, tok, feat,
                       src_row, k, (const bf16_t*)g_embed, (const bf16_t*)g_feat, eps, (bf16_t*)act, y, pos, head_dim, theta, cs);
  else
    hipLaunchKernelGGL(draft_input_kernel<false>, dim3(M), dim3(threads), 0, st, (const float*)embed, vocab, tok, feat,
                       src_row, k, (const float*)g_embed, (const float*)g_feat, eps, (float*)act, y, pos, head_dim, theta, cs);
  return hipGetLastError();
}

hipError_t launch_draft_prep1(const int32_t* kv_indptr, const int32_t* prefix_len, int n_new, int32_t* pos, int32_t* slot,
                              uint32_t* mask, SeqInfo* seq, hipStream_t st) {
  if (n_new > 64) return hipErrorInvalidValue;
  hipLaunchKernelGGL(draft_prep1_kernel, dim3(1), dim3(64), 0, st, kv_indptr, prefix_len, n_new, pos, slot, mask, seq);
  return hipGetLastError();
}
