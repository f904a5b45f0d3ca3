// Self-attention of the draft layer during a training-time-test step (forward only).
//
// Simulated step s over a training sequence of T positions: query i sees the ORIGINAL positions 0..i (ordinary
// causal context) and, of every simulated step t = 1..s, only position i itself.  The causal part is a flash-style
// pass over the original keys with the matrix cores; the s extra keys of a query are handled as the per-position
// vector dot products they are (one key per query and step: a matrix product would compute T x T scores to keep T).
//
// bf16 kernel (head_dim 128): workgroup = (64 consecutive queries, one query head), 4 wavefronts = 2 blocks of 32
// queries x 2 halves of every 64-key tile.  Tiles of the original keys / values reach LDS by direct global-to-LDS
// loads, one tile ahead, swizzled per key; scores are produced transposed (S^T = K Q^T) so that a lane owns one
// query; the V^T operand comes from the transposing LDS read; exp(S) enters the value product as a bf16 head plus a
// bf16 tail.  Only the last tile of a workgroup (the one on the diagonal) needs a mask.  After the two key halves
// are merged, each query's s own keys are added by dot products straight from global memory.
// fp32 kernel: one workgroup per (query, head), exact arithmetic, for small checks.
#include "common.hpp"
#include "kernels.hpp"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
constexpr int D = 128;
constexpr int KT = 64;
constexpr int ROWB = D * 2;
constexpr int TILE_BYTES = 2 * KT * ROWB;
constexpr int RD = 2;
constexpr float NEG = -1e30f;
constexpr float MAX_SLACK = 8.f;

struct TttParams {
  const bf16_t* q;        // [T, H, D] queries of step s
  const bf16_t* k;        // [s+1, T, Hkv, D]
  const bf16_t* v;        // [s+1, T, Hkv, D]
  int T, H, Hkv, s, n_qblocks;
  float scale_log2;
  float* out;             // [T, H, D] fp32
};

__device__ __forceinline__ void pair_values(float x, float& a, float& b) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  a = __uint_as_float(r[0]);
  b = __uint_as_float(r[1]);
}

// One wavefront-wide direct load: lane l's 16 bytes at `src` land at LDS byte address lds_base + 16 l.  The compiler
// does not see these as memory operations; the kernel counts them itself (s_waitcnt vmcnt).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16(const void* src, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(src) : "memory", "m0");
}
#pragma clang diagnostic pop
#define TTT_WAIT_LOADS(n) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(n) : "memory")

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

__global__ __launch_bounds__(256, 2) void ttt_attn_bf16_kernel(TttParams p) {
  constexpr int IPW = 4;                        // direct loads per wavefront per tile, for K and again for V
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int cw = wave >> 1, sb = wave & 1;
  const int qb = p.n_qblocks - 1 - (int)blockIdx.x;          // the longest workgroups first
  const int head = blockIdx.y, g = head * p.Hkv / p.H;
  const int T = p.T;
  const int row_in_block = cw * 32 + (lane & 31);
  const int row = qb * 64 + row_in_block;
  const bool q_valid = row < T;
  const bool wave_active = qb * 64 + cw * 32 < T;
  const int kg = lane >> 5;
  const int L = min(T, (qb + 1) * 64);                       // original keys this workgroup walks over
  const int n_tiles = qb + 1;

  const size_t row_stride = (size_t)p.Hkv * D;
  const bf16_t* kbase = p.k + (size_t)g * D;
  const bf16_t* vbase = p.v + (size_t)g * D;
  const int lkey = lane >> 4;
  const int vpiece = (lane & 15) ^ ((lkey & 3) << 2);
  auto issue_tile = [&](int t) {
    const uint32_t slot = lds0 + (t % RD) * TILE_BYTES;
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
      const int j = wave * IPW + i;
      const int key = min(t * KT + 4 * j + lkey, L - 1);     // keys past the end repeat the last one (masked later)
      const int kpiece = (lane & 15) ^ (4 * (j & 3) + lkey);
      dma16(kbase + (size_t)key * row_stride + kpiece * 8, slot + j * 1024);
    }
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
      const int j = wave * IPW + i;
      const int key = min(t * KT + 4 * j + lkey, L - 1);
      dma16(vbase + (size_t)key * row_stride + vpiece * 8, slot + KT * ROWB + j * 1024);
    }
  };

  const int kkey = sb * 32 + (lane & 31);
  const int k_off = kkey * ROWB, k_swz = kkey & 15;
  const int vkey0 = sb * 32 + 4 * kg + ((lane & 15) >> 2);
  const int v_swz = (vkey0 & 3) << 2;
  const int vcol = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
  const int v_half = (lane & 1) * 8;

  uint32_t minus_lo = 0x0000BF80u, minus_hi = 0xBF800000u;   // bf16 pairs (-1, 0) and (0, -1), kept in registers
  asm volatile("" : "+v"(minus_lo), "+v"(minus_hi));

  floatx16 o[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
  float m_run = NEG, l_run = 0.f;
  u32x4 qf[8];

  issue_tile(0);
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    if (q_valid) qf[ks] = *(const u32x4*)(p.q + ((size_t)row * p.H + head) * D + ks * 16 + kg * 8);
    else qf[ks] = (u32x4){0u, 0u, 0u, 0u};
  }
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) asm volatile("" ::"v"(qf[ks]));

  for (int t = 0; t < n_tiles; ++t) {
    TTT_WAIT_LOADS(0);
    __syncthreads();
    if (t + 1 < n_tiles) issue_tile(t + 1);
    if (!wave_active) continue;
    const unsigned char* kt = smem + (t % RD) * TILE_BYTES;
    floatx16 s;
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
    {
      floatx16 s2;
#pragma unroll
      for (int r = 0; r < 16; ++r) s2[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ks += 2) {
        const u32x4 a0 = *(const u32x4*)(kt + k_off + (((2 * ks + kg) ^ k_swz) * 16));
        const u32x4 a1 = *(const u32x4*)(kt + k_off + (((2 * ks + 2 + kg) ^ k_swz) * 16));
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a0), __builtin_bit_cast(bf16x8, qf[ks]), s, 0, 0, 0);
        s2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a1), __builtin_bit_cast(bf16x8, qf[ks + 1]), s2, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] += s2[r];
    }
    // the diagonal tile: key 64 qb + 32 sb + i is visible to the lane's query iff 32 sb + i <= row_in_block
    const bool masked_block = t == qb;
    uint32_t vis = 0xFFFFFFFFu;
    float mx = NEG;
    if (masked_block) {
      const int n_vis = row_in_block - 32 * sb + 1;
      vis = n_vis >= 32 ? 0xFFFFFFFFu : n_vis <= 0 ? 0u : ((1u << n_vis) - 1u);
      vis >>= 4 * kg;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float v = ((vis >> (8 * (r >> 2) + (r & 3))) & 1u) ? s[r] : NEG;
        s[r] = v;
        mx = fmaxf(mx, v);
      }
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[r]);
    }
    mx *= p.scale_log2;
    float xa, xb;
    pair_values(mx, xa, xb);
    const float m_cand = fmaxf(m_run, fmaxf(xa, xb));
    const float m_new = __any(m_cand - m_run > MAX_SLACK) ? m_cand : m_run;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    float ls = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], p.scale_log2, -m_new));
      s[r] = (!masked_block || ((vis >> (8 * (r >> 2) + (r & 3))) & 1u)) ? e : 0.f;
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
    u32x4 ph[2], pl[2];
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float p0 = s[8 * m + 2 * j], p1 = s[8 * m + 2 * j + 1];
        const uint32_t h = pack_bf16x2(p0, p1);
        ph[m][j] = h;
        const float t0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, h), __builtin_bit_cast(bf16x2_t, minus_lo), p0, false);
        const float t1 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, h), __builtin_bit_cast(bf16x2_t, minus_hi), p1, false);
        pl[m][j] = pack_bf16x2(t0, t1);
      }
    const unsigned char* vt = kt + KT * ROWB;
#pragma unroll
    for (int m = 0; m < 2; ++m) {
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const unsigned char* a0 = vt + (vkey0 + 16 * m) * ROWB + (((db * 4 + vcol) ^ v_swz) * 16) + v_half;
        const short4v lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)(__attribute__((address_space(3))) unsigned char*)a0);
        const short4v hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)(__attribute__((address_space(3))) unsigned char*)(a0 + 8 * ROWB));
        const short8v a = __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, ph[m]), o[db], 0, 0, 0);
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, pl[m]), o[db], 0, 0, 0);
      }
    }
  }
  TTT_WAIT_LOADS(0);

  // merge the two key halves: the sb = 1 wavefronts hand their state to their sb = 0 partners through LDS
  __syncthreads();
  float* xo = (float*)smem + (size_t)cw * (66 * 64);
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
  // the query's own key of every simulated step: one dot product and one scaled row of values each.  This lane holds
  // the query's entries 16 ks + 8 kg + 0..7 (its partner lane ^ 32 the other half) and the output entries
  // 32 db + 8 gq + 4 kg + 0..3.
  for (int t = 1; t <= p.s; ++t) {
    const bf16_t* kr = p.k + (((size_t)t * T + row) * p.Hkv + g) * D;
    const bf16_t* vr = p.v + (((size_t)t * T + row) * p.Hkv + g) * D;
    float dot = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const u32x4 kk = *(const u32x4*)(kr + ks * 16 + kg * 8);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        dot = fmaf(bf16_lo(qf[ks][e]), bf16_lo(kk[e]), dot);
        dot = fmaf(bf16_hi(qf[ks][e]), bf16_hi(kk[e]), dot);
      }
    }
    float xa, xb;
    pair_values(dot, xa, xb);
    const float sc = (xa + xb) * p.scale_log2;
    const float m_new = fmaxf(m_run, sc);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new), pw = __builtin_amdgcn_exp2f(sc - m_new);
    l_run = l_run * alpha + pw;
    m_run = m_new;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        const uint2 vv = *(const uint2*)(vr + db * 32 + 8 * gq + 4 * kg);
        o[db][4 * gq] = o[db][4 * gq] * alpha + pw * bf16_lo(vv.x);
        o[db][4 * gq + 1] = o[db][4 * gq + 1] * alpha + pw * bf16_hi(vv.x);
        o[db][4 * gq + 2] = o[db][4 * gq + 2] * alpha + pw * bf16_lo(vv.y);
        o[db][4 * gq + 3] = o[db][4 * gq + 3] * alpha + pw * bf16_hi(vv.y);
      }
  }
  const float inv = 1.0f / l_run;
  float* op = p.out + ((size_t)row * p.H + head) * D;
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
      floatx4 v = {o[db][4 * gq] * inv, o[db][4 * gq + 1] * inv, o[db][4 * gq + 2] * inv, o[db][4 * gq + 3] * inv};
      *(floatx4*)(op + db * 32 + 8 * gq + 4 * kg) = v;
    }
}

// fp32: one workgroup per (query, head); scores of the i + 1 + s visible keys in LDS
__global__ __launch_bounds__(256) void ttt_attn_f32_kernel(const float* __restrict__ q, const float* __restrict__ k,
                                                          const float* __restrict__ v, int T, int H, int Hkv, int d, int s,
                                                          float scale, float* __restrict__ out) {
  extern __shared__ float sc[];
  __shared__ float red[17];
  const int i = blockIdx.x, h = blockIdx.y, g = h * Hkv / H, tid = threadIdx.x;
  const int n = i + 1 + s;
  const float* qr = q + ((size_t)i * H + h) * d;
  auto key_row = [&](int j) { return j <= i ? (size_t)j : (size_t)(j - i) * T + i; };      // row of the [s+1, T] arrays
  float mx = -INFINITY;
  for (int j = tid; j < n; j += 256) {
    const float* kr = k + (key_row(j) * Hkv + g) * d;
    float acc = 0.f;
    for (int e = 0; e < d; ++e) acc = fmaf(qr[e], kr[e], acc);
    sc[j] = acc * scale;
    mx = fmaxf(mx, sc[j]);
  }
  mx = block_max(mx, red);
  float sum = 0.f;
  for (int j = tid; j < n; j += 256) {
    const float e = expf(sc[j] - mx);
    sc[j] = e;
    sum += e;
  }
  sum = block_sum(sum, red);
  for (int e = tid; e < d; e += 256) {
    float acc = 0.f;
    for (int j = 0; j < n; ++j) acc = fmaf(sc[j], v[(key_row(j) * Hkv + g) * d + e], acc);
    out[((size_t)i * H + h) * d + e] = acc / sum;
  }
}

}  // namespace

hipError_t launch_ttt_attention(bool bf16, const void* q, const void* k, const void* v, int T, int H, int Hkv, int d, int s,
                                float* out, hipStream_t st) {
  if (T < 1 || H < 1 || Hkv < 1 || H % Hkv || s < 0) return hipErrorInvalidValue;
  if (!bf16) {
    const size_t lds = (size_t)(T + s) * sizeof(float);
    if (lds > 60 * 1024 || d > 1024) return hipErrorInvalidValue;
    hipLaunchKernelGGL(ttt_attn_f32_kernel, dim3(T, H), dim3(256), lds, st, (const float*)q, (const float*)k, (const float*)v,
                       T, H, Hkv, d, s, 1.0f / sqrtf((float)d), out);
    return hipGetLastError();
  }
  if (d != D) return hipErrorInvalidValue;
  constexpr int LDS = RD * TILE_BYTES;
  static DeviceOnce configured;
  hipError_t ce = configured.run([&] {
    return hipFuncSetAttribute((const void*)ttt_attn_bf16_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
  });
  if (ce != hipSuccess) return ce;
  TttParams p;
  p.q = (const bf16_t*)q; p.k = (const bf16_t*)k; p.v = (const bf16_t*)v;
  p.T = T; p.H = H; p.Hkv = Hkv; p.s = s; p.n_qblocks = (T + 63) / 64;
  p.scale_log2 = 1.4426950408889634f / sqrtf((float)d);
  p.out = out;
  hipLaunchKernelGGL(ttt_attn_bf16_kernel, dim3(p.n_qblocks, H), dim3(256), LDS, st, p);
  return hipGetLastError();
}
