// Tree-masked attention against a (ragged) KV cache.
//
// Every query row sees the first n_prefix slots of its sequence unconditionally and the following
// n_tail slots (tree nodes / draft rows, just written to the cache) according to a 128-bit mask that
// was derived from the parent array: no dense rows x keys mask exists anywhere.
//
// bf16 kernel (head_dim 128): flash-style, split over the key range.
//   * workgroup = (sequence, KV head, block of 32 CW query rows of that KV head's group, key split);
//     the rows of one KV head's group are (query head in group, node) pairs, so all of them share
//     the K/V tiles staged in LDS.  CW is 1, 2 or 4 according to how many such rows there are: many
//     short-row workgroups (batched verification) pack two to a CU, a single long one fills it;
//   * K/V tiles of 64 keys reach LDS by direct global-to-LDS loads (1 KiB per wavefront instruction =
//     four 256-byte cache rows) into two tile slots, one tile ahead: no staging registers, no LDS store
//     instructions.  Which 16-byte piece of a row a lane fetches is XOR-swizzled with the key
//     index so that the operand reads below touch every LDS bank once;
//   * each wavefront owns 32 query rows and one 32-key block of every tile.  Scores are produced
//     transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16, so a lane holds 16 keys of ONE query: the
//     running max / sum need a single cross-lane exchange and exp(S^T) is already in B-operand position
//     for O^T += V^T P^T.  The V^T operand (8 keys of one head-dim index per lane) is read from the
//     row-major V tile with the transposing LDS read (ds_read_b64_tr_b16: 16 lanes hand in 4 key rows x
//     16 head-dim values and get back 4 keys of one head-dim value each);
//   * the two key-block halves are merged through LDS at the end; partial (max, sum, O) per split go to
//     scratch; a second kernel merges the splits and writes the result in the fragment-major layout the
//     output projection reads.
// fp32 kernel: one workgroup per (row, head), scores in LDS; exact arithmetic for the tiny model.
#include "common.hpp"
#include "kernels.hpp"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
constexpr int D = 128;
constexpr int KT = 64;                       // keys per tile = two 32-key score blocks
constexpr int ROWB = D * 2;                  // bytes per cache row
constexpr int TILE_BYTES = 2 * KT * ROWB;    // K tile, then V tile
constexpr float NEG = -1e30f;
constexpr float MAX_SLACK = 8.f;

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

// One wavefront-wide direct load: lane l's 16 bytes at `src` land at LDS byte address lds_base + 16 l.
// The compiler does not see these as memory operations; the kernel counts them itself (s_waitcnt vmcnt).
// (m0 carries the LDS address; naming it as clobbered is what is meant, the compiler's remark about reserved
// registers on a clobber list is switched off for this one statement.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16(const void* src, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(src) : "memory", "m0");
}
// Same, with the address given as a wavefront-uniform base plus a 32-bit byte offset per lane.
__device__ __forceinline__ void dma16(const void* base, uint32_t lane_off, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(lane_off), "s"(base)
               : "memory", "m0");
}
#pragma clang diagnostic pop
#define ATTN_WAIT_LOADS(n) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(n) : "memory")

constexpr int RD = 2;                        // tiles in LDS: the one being worked on and the next one arriving

// 2 CW wavefronts.  Wavefront w works on query rows 32 (w >> 1) .. +31 and on key block sb = w & 1 (32 of the 64
// keys) of every tile, with its own running max / sum / output: the serial chain per tile (8 score MFMAs,
// softmax, 16 value MFMAs) is what bounds a wavefront, so it is cut in two and the halves are merged through
// LDS at the end.
template <int CW>
__global__ __launch_bounds__(128 * CW, CW == 1 ? 1 : 2) void attn_tree_bf16_kernel(AttnParams p) {
  constexpr int NW = 2 * CW;
  constexpr int IPW = 16 / NW;                 // direct loads per wavefront per tile, for K and again for V
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int cw = wave >> 1, sb = wave & 1;
  int idx = blockIdx.x;
  const int g = idx % p.Hkv; idx /= p.Hkv;
  const int split = idx % p.n_splits; idx /= p.n_splits;
  const int qb = idx % p.n_qblocks;
  const int b = p.B == 1 ? 0 : p.seq[idx / p.n_qblocks].order;      // longest sequences first (one sequence: no look-up)
  const int G = p.H / p.Hkv, N = p.N;
  const SeqInfo si = p.seq[b];
  const int L = si.n_prefix + si.n_tail;

  // this lane's query: row rho of the KV head's group
  const int rho = (qb * CW + cw) * 32 + (lane & 31);
  const bool q_valid = rho < G * N;
  const int head = g * G + (q_valid ? rho / N : 0), node = q_valid ? rho % N : 0;
  const int row = b * N + node;
  const bool wave_active = (qb * CW + cw) * 32 < G * N;
  const int kg = lane >> 5;

  u32x4 qf[8];                                 // filled after the first K/V tiles are on their way
  uint32_t mw[4];

  const int n_tiles = (L + KT - 1) / KT;
  const int tps = (n_tiles + p.n_splits - 1) / p.n_splits;
  const int t_begin = split * tps, t_end = min(n_tiles, t_begin + tps);

  // Direct loads.  Instruction j (0..15) of a tile brings keys 4j .. 4j+3; lane l fetches, for key 4j + (l >> 4),
  // the piece that belongs at position l & 15 of the swizzled row: K rows hold piece c at position c ^ (key & 15),
  // V rows hold piece c at position c ^ ((key & 3) << 2).  A tile that lies wholly inside the sequence is fetched
  // from a wavefront-uniform tile base plus per-lane byte offsets that never change; in the sequence's last tile
  // keys past the end are clamped to its last key (masked later).
  const size_t row_stride = (size_t)p.Hkv * D;                        // elements between consecutive cache slots
  const bf16_t* kbase = p.kc + ((size_t)si.kv_base * p.Hkv + g) * D;
  const bf16_t* vbase = p.vc + ((size_t)si.kv_base * p.Hkv + g) * D;
  const int lkey = lane >> 4;
  const int vpiece = (lane & 15) ^ ((lkey & 3) << 2);
  uint32_t koff[IPW], voff[IPW];
#pragma unroll
  for (int i = 0; i < IPW; ++i) {
    const int j = wave * IPW + i;
    const uint32_t key_bytes = (uint32_t)(4 * j + lkey) * (uint32_t)(row_stride * 2);
    koff[i] = key_bytes + (uint32_t)(((lane & 15) ^ (4 * (j & 3) + lkey)) * 16);
    voff[i] = key_bytes + (uint32_t)(vpiece * 16);
  }
  auto issue_tile = [&](int t) {
    const uint32_t slot = lds0 + ((t - t_begin) % RD) * TILE_BYTES;
    if ((t + 1) * KT <= L) {
      const bf16_t* kt0 = kbase + (size_t)t * KT * row_stride;
      const bf16_t* vt0 = vbase + (size_t)t * KT * row_stride;
#pragma unroll
      for (int i = 0; i < IPW; ++i) dma16(kt0, koff[i], slot + (wave * IPW + i) * 1024);
#pragma unroll
      for (int i = 0; i < IPW; ++i) dma16(vt0, voff[i], slot + KT * ROWB + (wave * IPW + i) * 1024);
    } else {
#pragma unroll
      for (int i = 0; i < IPW; ++i) {
        const int j = wave * IPW + i;
        const int key = max(min(t * KT + 4 * j + lkey, L - 1), 0);
        const int kpiece = (lane & 15) ^ (4 * (j & 3) + lkey);
        dma16(kbase + (size_t)key * row_stride + kpiece * 8, slot + j * 1024);
      }
#pragma unroll
      for (int i = 0; i < IPW; ++i) {
        const int j = wave * IPW + i;
        const int key = max(min(t * KT + 4 * j + lkey, L - 1), 0);
        dma16(vbase + (size_t)key * row_stride + vpiece * 8, slot + KT * ROWB + j * 1024);
      }
    }
  };

  // LDS read offsets inside a tile.  K operand (32 keys x 16 k): lane (key = l & 31, pieces 2 ks + kg).
  const int kkey = sb * 32 + (lane & 31);
  const int k_off = kkey * ROWB, k_swz = kkey & 15;
  // V^T operand via transposing reads: call c of k-step m returns, for head-dim index db * 32 + (l & 31), keys
  // 16 m + 8 c + 4 kg + 0..3 of the block; the lane hands in the address of 4 head-dim values of ONE of those keys:
  // key + ((l & 15) >> 2), head-dim chunk 16 ((l >> 4) & 1) + 4 (l & 3).
  const int vkey0 = sb * 32 + 4 * kg + ((lane & 15) >> 2);            // + 16 m + 8 c
  const int v_swz = (vkey0 & 3) << 2;                                 // (key & 3) does not depend on m, c
  const int vcol = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);         // piece within the 32-wide head-dim block
  const int v_half = (lane & 1) * 8;

  // bf16 pairs (-1, 0) and (0, -1), kept in registers: written as literals the compiler folds them into an
  // inline constant whose two halves the instruction does not read that way
  uint32_t minus_lo = 0x0000BF80u, minus_hi = 0xBF800000u;
  asm volatile("" : "+v"(minus_lo), "+v"(minus_hi));

  floatx16 o[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
  float m_run = NEG, l_run = 0.f;

  // scores and softmax of tile t: updates the running max / sum, rescales the output, leaves exp(S^T) as bf16
  // head (ph) and tail (pl) operands
  auto score_tile = [&](int t, u32x4 (&ph)[2], u32x4 (&pl)[2]) {
    const unsigned char* kt = smem + ((t - t_begin) % RD) * TILE_BYTES;
    // S^T = K Q^T for this wavefront's 32-key block, as two interleaved chains over the head dimension
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
    const int kb = t * KT + 32 * sb;
    float mx = NEG;
    const bool masked_block = kb + 32 > si.n_prefix;   // uniform per wavefront: the block touches the masked tail or the end
    uint32_t vis = 0xFFFFFFFFu;
    if (masked_block) {
      // visibility of the block's 32 keys as one word per lane: bit i <-> key kb + i
      const int off0 = kb - si.n_prefix, w0 = off0 >> 5, sh = off0 & 31;
      auto word = [&](int i) -> uint32_t {             // i is uniform; keys before the tail are all visible
        return i < 0 ? 0xFFFFFFFFu : i == 0 ? mw[0] : i == 1 ? mw[1] : i == 2 ? mw[2] : i == 3 ? mw[3] : 0u;
      };
      const uint64_t both = ((uint64_t)word(w0 + 1) << 32) | word(w0);
      vis = (uint32_t)(both >> sh);
      if (L - kb < 32) vis &= L > kb ? (1u << (L - kb)) - 1u : 0u;       // keys past the end of the sequence
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
    mx *= p.scale_log2;                                 // the scale is positive: max and scaling commute
    float xa, xb;
    pair_values(mx, xa, xb);
    const float m_cand = fmaxf(m_run, fmaxf(xa, xb));
    // The running max only moves when some row of the wavefront would raise its own by more than MAX_SLACK
    // (log2 units): until then exp2 may exceed 1 by up to 2^MAX_SLACK, which the fp32 sums and the head/tail
    // split carry without loss, and the 64 output registers need no rescaling in most tiles.
    const float m_new = __any(m_cand - m_run > MAX_SLACK) ? m_cand : m_run;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    float ls = 0.f;
    if (masked_block) {
      // invisible keys get weight zero by selection, not by the size of NEG: when a wavefront's first blocks are
      // wholly invisible for a row, m_new itself is NEG-like and the exponent of a masked score is a rounding remainder
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], p.scale_log2, -m_new));
        s[r] = ((vis >> (8 * (r >> 2) + (r & 3))) & 1u) ? e : 0.f;
        ls += s[r];
      }
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        s[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], p.scale_log2, -m_new));
        ls += s[r];
      }
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
    // Operand m of P^T holds keys 32 sb + 16 m + {4kg..4kg+3, 8+4kg..8+4kg+3} = registers 8m..8m+7.
    // exp(S) is split into a bf16 head and a bf16 tail (p = hi + lo, 16 significant bits) and both are
    // multiplied with V: rounding P to a single bf16 would put a 2^-9 relative error on the attention output,
    // which the following RMSNorm can magnify when the residual stream is small.
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float p0 = s[8 * m + 2 * j], p1 = s[8 * m + 2 * j + 1];
        const uint32_t h = pack_bf16x2(p0, p1);
        ph[m][j] = h;
        // tail = p - head, one v_dot2c_f32_bf16 each: p + head.lo * -1 + head.hi * 0 (exact)
        const float t0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, h), __builtin_bit_cast(bf16x2_t, minus_lo), p0, false);
        const float t1 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, h), __builtin_bit_cast(bf16x2_t, minus_hi), p1, false);
        pl[m][j] = pack_bf16x2(t0, t1);
      }
  };
  // O^T += V^T P^T for tile t
  auto value_tile = [&](int t, const u32x4 (&ph)[2], const u32x4 (&pl)[2]) {
    const unsigned char* vt = smem + ((t - t_begin) % RD) * TILE_BYTES + KT * ROWB;
#pragma unroll
    for (int m = 0; m < 2; ++m) {
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        short4v lo4, hi4;
        {
          const unsigned char* a0 = vt + (vkey0 + 16 * m) * ROWB + (((db * 4 + vcol) ^ v_swz) * 16) + v_half;
          lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)(__attribute__((address_space(3))) unsigned char*)a0);
          hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)(__attribute__((address_space(3))) unsigned char*)(a0 + 8 * ROWB));
        }
        typedef short short8v __attribute__((ext_vector_type(8)));
        const short8v a = __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, ph[m]),
                                                       o[db], 0, 0, 0);
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, pl[m]),
                                                       o[db], 0, 0, 0);
      }
    }
  };

  // Two tile slots: tile t + 1 is requested when the barrier of iteration t has freed its slot and arrives while
  // tile t is worked on.  (Deeper rings were slower: the first tile waits behind everything requested before it.)
  if (t_begin < t_end) issue_tile(t_begin);
  // The query fragments and mask words are ordinary loads issued AFTER those tiles, so that both latencies run
  // side by side; the compiler's wait for them (at their first use, just below) also covers every direct load
  // issued so far, and the counted waits in the loop only ever see direct loads younger than that.
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    if (q_valid) qf[ks] = *(const u32x4*)(p.q + ((size_t)row * p.H + head) * D + ks * 16 + kg * 8);
    else qf[ks] = (u32x4){0u, 0u, 0u, 0u};
  }
#pragma unroll
  for (int w = 0; w < 4; ++w) mw[w] = p.mask[(size_t)row * 4 + w];
  // consume them here, once: otherwise the compiler re-waits for them inside the loop, which would drain the ring
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) asm volatile("" ::"v"(qf[ks]));
#pragma unroll
  for (int w = 0; w < 4; ++w) asm volatile("" ::"v"(mw[w]));
  u32x4 ph[2], pl[2];
  for (int t = t_begin; t < t_end; ++t) {
    ATTN_WAIT_LOADS(0);                        // my part of tile t has landed; the barrier extends that to everyone's
    __syncthreads();
    if (t + 1 < t_end) issue_tile(t + 1);
    if (wave_active) {
      score_tile(t, ph, pl);
      value_tile(t, ph, pl);
    }
  }
  ATTN_WAIT_LOADS(0);                          // nothing may still be writing LDS when it is reused or released

  // merge the two key-block halves: the sb = 1 wavefronts hand their state to their sb = 0 partners through LDS
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

// Wavefront pairs per workgroup.  More than 64 rows per KV head can go to 8-wavefront workgroups (two wavefronts
// on every SIMD, which overlap each other's MFMA and softmax phases: ~0.8 us of SIMD time per wavefront-tile
// against 1.3 us for a lone wavefront) or to 4-wavefront ones (half as many key splits for the same number of
// workgroups, so half the partial results to write and merge).  The first pays once every SIMD has more than
// about a dozen wavefront-tiles to work through (measured crossover at 240 rows: between 4096 and 8192 keys).
static int attn_cw(int B, int rows_per_group, int Hkv, int max_len) {
  if (rows_per_group <= 32) return 1;
  if (rows_per_group <= 64) return 2;
  const long wave_tiles = (long)B * Hkv * ((rows_per_group + 31) / 32) * 2 * ((max_len + KT - 1) / KT);
  return wave_tiles <= 12 * 1024 ? 2 : 4;
}

int attention_pick_splits(int B, int rows_per_seq, int H, int Hkv, int max_len) {
  const int G = H / Hkv, cw = attn_cw(B, G * rows_per_seq, Hkv, max_len);
  const int qblocks = (G * rows_per_seq + 32 * cw - 1) / (32 * cw);
  const int base = B * Hkv * qblocks;
  const int tiles = (max_len + KT - 1) / KT;
  const int slots = cw == 1 ? 512 : 256;         // one workgroup per CU, two of the smallest kind
  int s = (slots + base - 1) / base;
  s = s < 1 ? 1 : s;
  // a batch that already fills the chip is still cut in two: its sequences differ in length, workgroups are
  // handed out longest sequence first, and the halves of the short ones fill in behind the long ones
  // (measured on a 64-sequence batch of 512..2048 keys: 89 us against 102 us unsplit)
  if (B > 1 && base >= slots && tiles >= 16) s = 2;
  const int cap = (tiles + 3) / 4;               // at least 4 key tiles per split
  if (s > cap) s = cap < 1 ? 1 : cap;
  return s;
}

size_t attention_scratch_floats(int R, int H, int d, int max_splits) {
  return (size_t)R * H * max_splits * (d + 2);
}

template <int CW>
static hipError_t launch_attn_cw(const AttnParams& p, int grid, hipStream_t st) {
  // the tile ring, reused by the end-of-kernel merge of the two key-block halves
  constexpr int LDS = RD * TILE_BYTES > CW * 66 * 64 * 4 ? RD * TILE_BYTES : CW * 66 * 64 * 4;
  auto kernel = attn_tree_bf16_kernel<CW>;
  static DeviceOnce configured;                  // the attribute belongs to the loaded code object of a device
  hipError_t ce = configured.run([&] { return hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, LDS); });
  if (ce != hipSuccess) return ce;
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(128 * CW), LDS, st, p);
  return hipGetLastError();
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
  const int cw = attn_cw(B, H / Hkv * rows_per_seq, Hkv, max_len);
  AttnParams p;
  p.q = (const bf16_t*)q; p.kc = (const bf16_t*)kcache; p.vc = (const bf16_t*)vcache;
  p.seq = seq; p.mask = mask;
  p.B = B; p.N = rows_per_seq; p.H = H; p.Hkv = Hkv; p.n_splits = n_splits;
  p.n_qblocks = (H / Hkv * rows_per_seq + 32 * cw - 1) / (32 * cw);
  p.scale_log2 = 1.4426950408889634f / sqrtf((float)d);
  p.o_part = scratch;
  p.ml_part = scratch + (size_t)R * H * n_splits * D;
  const int grid = B * p.n_qblocks * n_splits * Hkv;
  hipError_t e = cw == 1 ? launch_attn_cw<1>(p, grid, st) : cw == 2 ? launch_attn_cw<2>(p, grid, st) : launch_attn_cw<4>(p, grid, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attn_merge_kernel, dim3((R * H * 32 + 255) / 256), dim3(256), 0, st, p.o_part, p.ml_part, R,
                     rows_per_seq, H, n_splits, (bf16_t*)out);
  return hipGetLastError();
}
