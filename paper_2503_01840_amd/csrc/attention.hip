// Tree-masked attention against a (ragged) KV cache.
//
// Every query row sees the first n_prefix slots of its sequence unconditionally and the following
// n_tail slots (tree nodes / draft rows, just written to the cache) according to a 128-bit mask that
// was derived from the parent array: no dense rows x keys mask exists anywhere.
//
// bf16 kernel (head_dim 128): flash-style, split over the key range.
//   * workgroup = (sequence, KV head, block of 128 query rows of that KV head's group, key split);
//     the rows of one KV head's group are (query head in group, node) pairs, so all of them share
//     the K/V tiles staged in LDS;
//   * each wavefront owns 32 query rows.  Scores are produced transposed, S^T = K Q^T, with
//     v_mfma_f32_32x32x16_bf16, so a lane holds 16 keys of ONE query: the running max / sum need a
//     single cross-lane exchange and exp(S^T) is already in B-operand position for O^T += V^T P^T;
//   * V tiles are transposed on their way into LDS (keys permuted to match that operand order);
//   * partial (max, sum, O) per split go to scratch; a second kernel merges the splits and writes the
//     result in the fragment-major layout the output projection reads.
// fp32 kernel: one workgroup per (row, head), scores in LDS; exact arithmetic for the tiny model.
#include "common.hpp"
#include "kernels.hpp"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int D = 128;
constexpr int KT = 64;                       // keys per tile = two 32-key score blocks worked on together
constexpr int KROW = D * 2 + 16;             // LDS bytes per staged key row
constexpr int VROW = KT * 2 + 16;            // LDS bytes per transposed value row (one head-dim index)
constexpr int TILE_BYTES = KT * KROW + D * VROW;
constexpr float NEG = -1e30f;
constexpr int PFA = 2;                       // K/V tiles in flight per workgroup (register ring)

struct AttnParams {
  const bf16_t* q;
  const bf16_t* kc;
  const bf16_t* vc;
  const SeqInfo* seq;
  const uint32_t* mask;
  int B, N, H, Hkv, n_splits, n_qblocks;
  float scale_log2;
  float* o_part;     // [B][H][n_splits][N][D]
  float* ml_part;    // [B][H][n_splits][N][2]
};

// value of lane l and of lane l^32, in some order (v_permlane32_swap: no LDS crossbar round trip)
__device__ __forceinline__ void pair_values(float x, float& a, float& b) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  a = __uint_as_float(r[0]);
  b = __uint_as_float(r[1]);
}

// 8 wavefronts.  Wavefront w works on query rows 32 (w & 3) .. +31 and on key block sb = w >> 2 (32 of the 64
// keys) of every tile, with its own running max / sum / output: the serial chain per tile (8 score MFMAs,
// softmax, 16 value MFMAs) is what bounds this kernel, so it is cut in two and the halves are merged through
// LDS at the end.  All 512 threads stage the K/V tiles.
__global__ __launch_bounds__(512, 1) void attn_tree_bf16_kernel(AttnParams p) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * TILE_BYTES];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int cw = wave & 3, sb = wave >> 2;
  int idx = blockIdx.x;
  const int g = idx % p.Hkv; idx /= p.Hkv;
  const int split = idx % p.n_splits; idx /= p.n_splits;
  const int qb = idx % p.n_qblocks;
  const int b = idx / p.n_qblocks;
  const int G = p.H / p.Hkv, N = p.N;
  const SeqInfo si = p.seq[b];
  const int L = si.n_prefix + si.n_tail;

  // this lane's query: row rho of the KV head's group
  const int rho = qb * 128 + cw * 32 + (lane & 31);
  const bool q_valid = rho < G * N;
  const int head = g * G + (q_valid ? rho / N : 0), node = q_valid ? rho % N : 0;
  const int row = b * N + node;
  const bool wave_active = qb * 128 + cw * 32 < G * N;
  const int kg = lane >> 5;

  u32x4 qf[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    if (q_valid) qf[ks] = *(const u32x4*)(p.q + ((size_t)row * p.H + head) * D + ks * 16 + kg * 8);
    else qf[ks] = (u32x4){0u, 0u, 0u, 0u};
  }
  uint32_t mw[4];
#pragma unroll
  for (int w = 0; w < 4; ++w) mw[w] = p.mask[(size_t)row * 4 + w];

  const int n_tiles = (L + KT - 1) / KT;
  const int tps = (n_tiles + p.n_splits - 1) / p.n_splits;
  const int t_begin = split * tps, t_end = min(n_tiles, t_begin + tps);
  const int t_last = max(t_end - 1, 0);

  // Staging roles.  K: 16-byte chunks c = tid + 512 i (key = c >> 4, column = c & 15).
  // V: head-dim chunk vc8 = tid & 15 and the key pair pp = tid >> 4 at permuted positions 2pp, 2pp+1, where
  // position pi = 32 sb + 16 m + 8 kg + 4 g + e holds key 32 sb + 16 m + 8 g + 4 kg + e: the order in which the
  // P^T operand of the second MFMA carries the keys of score block sb.
  const int vc8 = tid & 15, pp = tid >> 4;
  int vkey[2];
#pragma unroll
  for (int w = 0; w < 2; ++w) {
    const int pi = 2 * pp + w;
    vkey[w] = (pi & 48) + 8 * ((pi >> 2) & 1) + 4 * ((pi >> 3) & 1) + (pi & 3);
  }
  // Register prefetch ring, PFA tiles deep.  Tile indices past the end of the split are clamped to its last
  // tile (a redundant, harmless load), so the loop body has no branch and the loads stay in flight.
  u32x4 kreg[PFA][2], vreg[PFA][2];
  auto load_tile = [&](int t, int slot) {
    t = min(t, t_last);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int c = tid + 512 * i;
      const int kk = min(t * KT + (c >> 4), L - 1);
      kreg[slot][i] = *(const u32x4*)(p.kc + ((size_t)(si.kv_base + kk) * p.Hkv + g) * D + (c & 15) * 8);
    }
#pragma unroll
    for (int w = 0; w < 2; ++w) {
      const int kk = min(t * KT + vkey[w], L - 1);
      vreg[slot][w] = *(const u32x4*)(p.vc + ((size_t)(si.kv_base + kk) * p.Hkv + g) * D + vc8 * 8);
    }
  };
  auto store_tile = [&](unsigned char* buf, int slot) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int c = tid + 512 * i;
      *(u32x4*)(buf + (c >> 4) * KROW + (c & 15) * 16) = kreg[slot][i];
    }
    unsigned char* vt = buf + KT * KROW;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t a = vreg[slot][0][j], c2 = vreg[slot][1][j];
      *(uint32_t*)(vt + (vc8 * 8 + 2 * j) * VROW + 4 * pp) = (a & 0xFFFFu) | (c2 << 16);
      *(uint32_t*)(vt + (vc8 * 8 + 2 * j + 1) * VROW + 4 * pp) = (a >> 16) | (c2 & 0xFFFF0000u);
    }
  };

  floatx16 o[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
  float m_run = NEG, l_run = 0.f;

  auto tile_step = [&](int t, int slot) {
    unsigned char* buf = smem + ((t - t_begin) & 1) * TILE_BYTES;
#ifndef ATTN_NO_STAGE
    store_tile(buf, slot);
    load_tile(t + PFA, slot);
#endif
    __syncthreads();
#ifdef ATTN_NO_COMPUTE
    return;
#endif
    if (!wave_active) return;
    // S^T = K Q^T for this wavefront's 32-key block, as two interleaved chains over the head dimension
    floatx16 s, s2;
#pragma unroll
    for (int r = 0; r < 16; ++r) { s[r] = 0.f; s2[r] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < 8; ks += 2) {
      const u32x4 a0 = *(const u32x4*)(buf + (sb * 32 + (lane & 31)) * KROW + (ks * 16 + kg * 8) * 2);
      const u32x4 a1 = *(const u32x4*)(buf + (sb * 32 + (lane & 31)) * KROW + ((ks + 1) * 16 + kg * 8) * 2);
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a0), __builtin_bit_cast(bf16x8, qf[ks]), s, 0, 0, 0);
      s2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a1), __builtin_bit_cast(bf16x8, qf[ks + 1]), s2, 0, 0, 0);
    }
    const int kb = t * KT + 32 * sb;
    float mx = NEG;
    if (kb + 32 > si.n_prefix) {                       // uniform per wavefront: the block touches the masked tail or the end
      // visibility of the block's 32 keys as one word per lane: bit i <-> key kb + i
      const int off0 = kb - si.n_prefix, w0 = off0 >> 5, sh = off0 & 31;
      auto word = [&](int i) -> uint32_t {             // i is uniform; keys before the tail are all visible
        return i < 0 ? 0xFFFFFFFFu : i == 0 ? mw[0] : i == 1 ? mw[1] : i == 2 ? mw[2] : i == 3 ? mw[3] : 0u;
      };
      const uint64_t both = ((uint64_t)word(w0 + 1) << 32) | word(w0);
      uint32_t vis = (uint32_t)(both >> sh);
      if (L - kb < 32) vis &= L > kb ? (1u << (L - kb)) - 1u : 0u;       // keys past the end of the sequence
      vis >>= 4 * kg;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float v = ((vis >> (8 * (r >> 2) + (r & 3))) & 1u) ? (s[r] + s2[r]) * p.scale_log2 : NEG;
        s[r] = v;
        mx = fmaxf(mx, v);
      }
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        s[r] = (s[r] + s2[r]) * p.scale_log2;
        mx = fmaxf(mx, s[r]);
      }
    }
    float xa, xb;
    pair_values(mx, xa, xb);
    const float m_new = fmaxf(m_run, fmaxf(xa, xb));
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    float ls = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      s[r] = __builtin_amdgcn_exp2f(s[r] - m_new);
      ls += s[r];
    }
    pair_values(ls, xa, xb);
    l_run = l_run * alpha + (xa + xb);
    m_run = m_new;
    if (__any(alpha != 1.0f)) {
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
    }
    // O^T += V^T P^T.  Operand m of P^T holds keys 32 sb + 16 m + {4kg..4kg+3, 8+4kg..8+4kg+3} = registers 8m..8m+7.
    // exp(S) is split into a bf16 head and a bf16 tail (p = hi + lo, 16 significant bits) and both are
    // multiplied with V: rounding P to a single bf16 would put a 2^-9 relative error on the attention output,
    // which the following RMSNorm can magnify when the residual stream is small.
    const unsigned char* vt = buf + KT * KROW;
#pragma unroll
    for (int m = 0; m < 2; ++m) {
      u32x4 ph, pl;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float p0 = s[8 * m + 2 * j], p1 = s[8 * m + 2 * j + 1];
        const uint32_t h = pack_bf16x2(p0, p1);
        ph[j] = h;
        pl[j] = pack_bf16x2(p0 - __uint_as_float(h << 16), p1 - __uint_as_float(h & 0xFFFF0000u));
      }
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const u32x4 a = *(const u32x4*)(vt + (db * 32 + (lane & 31)) * VROW + (sb * 32 + m * 16 + kg * 8) * 2);
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, ph),
                                                       o[db], 0, 0, 0);
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, pl),
                                                       o[db], 0, 0, 0);
      }
    }
  };
#pragma unroll
  for (int sl = 0; sl < PFA; ++sl) {
    load_tile(t_begin + sl, sl);
    __builtin_amdgcn_sched_barrier(0);
  }
  int t = t_begin;
  for (; t + PFA <= t_end; t += PFA) {
#pragma unroll
    for (int sl = 0; sl < PFA; ++sl) tile_step(t + sl, sl);
  }
#pragma unroll
  for (int sl = 0; sl < PFA; ++sl)
    if (t + sl < t_end) tile_step(t + sl, sl);

  // merge the two key-block halves: wavefronts 4-7 hand their state to wavefronts 0-3 through LDS
  __syncthreads();
  float* xo = (float*)smem + (size_t)cw * (66 * 64);           // [64 output registers + m + l][64 lanes]
  if (sb == 1) {
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) xo[(db * 16 + r) * 64 + lane] = o[db][r];
    xo[64 * 64 + lane] = m_run;
    xo[65 * 64 + lane] = l_run;
  }
  __syncthreads();
  if (sb == 1 || !q_valid) return;
  {
    const float m2 = xo[64 * 64 + lane], l2 = xo[65 * 64 + lane];
    const float m_new = fmaxf(m_run, m2);
    const float w1 = __builtin_amdgcn_exp2f(m_run - m_new), w2 = __builtin_amdgcn_exp2f(m2 - m_new);
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[db][r] = o[db][r] * w1 + xo[(db * 16 + r) * 64 + lane] * w2;
    l_run = l_run * w1 + l2 * w2;
    m_run = m_new;
  }
  const size_t pr = (((size_t)b * p.H + head) * p.n_splits + split) * N + node;
  float* op = p.o_part + pr * D;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
      floatx4 v = {o[db][4 * gq], o[db][4 * gq + 1], o[db][4 * gq + 2], o[db][4 * gq + 3]};
      *(floatx4*)(op + db * 32 + 8 * gq + 4 * kg) = v;
    }
  if (kg == 0) {
    p.ml_part[pr * 2] = m_run;
    p.ml_part[pr * 2 + 1] = l_run;
  }
}

// one thread per (row, head, 4 consecutive head-dim entries); one pass over the splits in chunks of 8 whose
// loads are all independent (online rescaling between chunks)
__global__ __launch_bounds__(256) void attn_merge_kernel(const float* __restrict__ o_part, const float* __restrict__ ml_part,
                                                        int R, int N, int H, int n_splits, bf16_t* __restrict__ out) {
  const int gid = blockIdx.x * 256 + threadIdx.x;
  const int d4 = gid & 31, rh = gid >> 5;
  if (rh >= R * H) return;
  const int h = rh % H, r = rh / H, b = r / N, node = r % N;
  const size_t base = (((size_t)b * H + h) * n_splits) * N + node;
  float M = NEG, den = 0.f;
  float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s0 = 0; s0 < n_splits; s0 += 8) {
    float2 ml[8];
    float4 o[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const size_t pr = base + (size_t)min(s0 + j, n_splits - 1) * N;
      ml[j] = *(const float2*)(ml_part + pr * 2);
      o[j] = *(const float4*)(o_part + pr * D + 4 * d4);
    }
    float cm = M;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (s0 + j < n_splits) cm = fmaxf(cm, ml[j].x);
    const float a = __builtin_amdgcn_exp2f(M - cm);
    num.x *= a; num.y *= a; num.z *= a; num.w *= a; den *= a;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (s0 + j < n_splits) {
        const float w = __builtin_amdgcn_exp2f(ml[j].x - cm);
        num.x += w * o[j].x; num.y += w * o[j].y; num.z += w * o[j].z; num.w += w * o[j].w;
        den += w * ml[j].y;
      }
    M = cm;
  }
  const float inv = 1.0f / den;
  Act<true>::store4(out, r, h * D + 4 * d4, H * D, num.x * inv, num.y * inv, num.z * inv, num.w * inv);
}

// ---------------------------------------------------------------------------------------------- fp32
__global__ __launch_bounds__(256) void attn_tree_f32_kernel(const float* __restrict__ q, const float* __restrict__ kc,
                                                           const float* __restrict__ vc, const SeqInfo* __restrict__ seq,
                                                           const uint32_t* __restrict__ mask, int N, int H, int Hkv, int d,
                                                           float scale, float* __restrict__ out) {
  extern __shared__ float sc[];
  __shared__ float red[17];
  const int r = blockIdx.x, h = blockIdx.y, b = r / N, g = h * Hkv / H, tid = threadIdx.x;
  const SeqInfo si = seq[b];
  const int L = si.n_prefix + si.n_tail;
  const float* qr = q + ((size_t)r * H + h) * d;
  float mx = -INFINITY;
  for (int kk = tid; kk < L; kk += 256) {
    const int off = kk - si.n_prefix;
    bool vis = true;
    if (off >= 0) vis = (mask[(size_t)r * 4 + ((off >> 5) & 3)] >> (off & 31)) & 1u;
    float s = -INFINITY;
    if (vis) {
      const float* kr = kc + ((size_t)(si.kv_base + kk) * Hkv + g) * d;
      float acc = 0.f;
      for (int i = 0; i < d; ++i) acc = fmaf(qr[i], kr[i], acc);
      s = acc * scale;
    }
    sc[kk] = s;
    mx = fmaxf(mx, s);
  }
  mx = block_max(mx, red);
  float sum = 0.f;
  for (int kk = tid; kk < L; kk += 256) {
    const float e = expf(sc[kk] - mx);      // exp(-inf) = 0 for masked slots
    sc[kk] = e;
    sum += e;
  }
  sum = block_sum(sum, red);
  for (int i = tid; i < d; i += 256) {
    float acc = 0.f;
    for (int kk = 0; kk < L; ++kk) acc = fmaf(sc[kk], vc[((size_t)(si.kv_base + kk) * Hkv + g) * d + i], acc);
    out[(size_t)r * H * d + h * d + i] = acc / sum;
  }
}

}  // namespace

int attention_pick_splits(int B, int rows_per_seq, int H, int Hkv, int max_len) {
  const int G = H / Hkv;
  const int qblocks = (G * rows_per_seq + 127) / 128;
  const int base = B * Hkv * qblocks;
  const int tiles = (max_len + KT - 1) / KT;
  int s = (256 + base - 1) / base;               // aim at one workgroup per CU
  s = s < 1 ? 1 : s;
  const int cap = (tiles + 3) / 4;               // at least 4 key tiles per split
  if (s > cap) s = cap < 1 ? 1 : cap;
  return s;
}

size_t attention_scratch_floats(int R, int H, int d, int max_splits) {
  return (size_t)R * H * max_splits * (d + 2);
}

hipError_t launch_tree_attention(bool bf16, const void* q, const void* kcache, const void* vcache, const SeqInfo* seq,
                                 const uint32_t* mask, int B, int rows_per_seq, int H, int Hkv, int d, int max_len,
                                 int n_splits, float* scratch, void* out, hipStream_t st) {
  const int R = B * rows_per_seq;
  if (!bf16) {
    const size_t lds = (size_t)max_len * sizeof(float);
    if (lds > 60 * 1024) return hipErrorInvalidValue;
    hipLaunchKernelGGL(attn_tree_f32_kernel, dim3(R, H), dim3(256), lds, st, (const float*)q, (const float*)kcache,
                       (const float*)vcache, seq, mask, rows_per_seq, H, Hkv, d, 1.0f / sqrtf((float)d), (float*)out);
    return hipGetLastError();
  }
  if (d != D || H % Hkv) return hipErrorInvalidValue;
  AttnParams p;
  p.q = (const bf16_t*)q; p.kc = (const bf16_t*)kcache; p.vc = (const bf16_t*)vcache;
  p.seq = seq; p.mask = mask;
  p.B = B; p.N = rows_per_seq; p.H = H; p.Hkv = Hkv; p.n_splits = n_splits;
  p.n_qblocks = (H / Hkv * rows_per_seq + 127) / 128;
  p.scale_log2 = 1.4426950408889634f / sqrtf((float)d);
  p.o_part = scratch;
  p.ml_part = scratch + (size_t)R * H * n_splits * D;
  hipLaunchKernelGGL(attn_tree_bf16_kernel, dim3(B * p.n_qblocks * n_splits * Hkv), dim3(512), 0, st, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attn_merge_kernel, dim3((R * H * 32 + 255) / 256), dim3(256), 0, st, p.o_part, p.ml_part, R,
                     rows_per_seq, H, n_splits, (bf16_t*)out);
  return hipGetLastError();
}
