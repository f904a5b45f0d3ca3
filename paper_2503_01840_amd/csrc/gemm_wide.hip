// bf16 GEMM for MANY activation rows (batched verification: 64 sequences x 8 nodes = 512 rows):
// Y[M, N] = X[M, K] * W[N, K]^T, fp32 accumulate.  At this width the projections sit at the MFMA ridge, so the
// kernel is organised around operand reuse instead of pure weight streaming:
//   * a workgroup owns a (32 FM WGM) x (32 FN WGN) output tile; its WGM x WGN wavefronts each hold FM x FN
//     accumulators of v_mfma_f32_32x32x16_bf16 and there is no cross-wavefront reduction;
//   * both operands go through double-buffered LDS, 64 k per stage.  The activation tile is copied verbatim: its
//     fragment-major global layout already is the MFMA operand order, so LDS reads are linear 16-byte-per-lane
//     reads.  Weight rows arrive row-contiguous (8 lanes cover 128 bytes of one row) and are scattered into the
//     same operand order, with 16 bytes of padding per 32x8 block so that neither side has bank conflicts;
//   * global loads of stage j+1 are issued into registers before the MFMAs of stage j and stored to the other
//     LDS buffer after them: one barrier per stage;
//   * every workgroup starts its walk over K at a different stage, so that the workgroups sharing an activation
//     tile do not all ask the same L2 channel for the same lines at the same moment;
//   * the weights are the MFMA's first operand: a lane then holds, for ONE activation row, runs of four
//     consecutive output columns, which is what both epilogues store: fp32 split-K partials (16-byte stores), or
//     SwiGLU (the tile interleaves gate and up rows so that both values of a pair sit in the same lane) written
//     as fragment-major bf16 (8-byte stores).
#include "common.hpp"
#include "kernels.hpp"

namespace {

constexpr int BK = 64;                  // k per stage
constexpr int KS = BK / 16;             // MFMA k-steps per stage
constexpr int A_TILE = 64 * BK * 2;     // bytes of one 64-row activation tile per stage (8 KiB, contiguous in HBM)
constexpr int B_COL = 32 * 16 + 16;     // bytes of one padded (32 rows x 8 k) weight block
constexpr int B_FRAG = (BK / 8) * B_COL;  // 32 weight rows x 64 k

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct WideParams {
  const bf16_t* x;
  const bf16_t* w[3];
  int rows[3];
  int nmat, mode;
  int M, N, K, S, epi;
  float* out_f32;
  bf16_t* out_xf;
};

// Global weight row behind row `row` of workgroup tile `tile` (TN rows per tile).
template <int TN>
__device__ __forceinline__ const bf16_t* weight_row(const WideParams& p, int tile, int row) {
  if (p.mode == 1) {                                   // TN/2 gate rows | TN/2 up rows
    int r = tile * (TN / 2) + (row % (TN / 2));
    r = min(r, p.rows[0] - 1);
    return p.w[row / (TN / 2)] + (size_t)r * p.K;
  }
  int n = min(tile * TN + row, p.N - 1);
  int m = 0;
  while (m + 1 < p.nmat && n >= p.rows[m]) { n -= p.rows[m]; ++m; }
  return p.w[m] + (size_t)n * p.K;
}

template <int WGM, int WGN, int FM, int FN, int OCC>
__global__ __launch_bounds__(64 * WGM * WGN, OCC) void gemm_wide_kernel(WideParams p) {
  constexpr int TM = 32 * FM * WGM, TN = 32 * FN * WGN, NT = 64 * WGM * WGN;
  constexpr int A_BYTES = (TM / 64) * A_TILE, B_BYTES = (TN / 32) * B_FRAG, STAGE = A_BYTES + B_BYTES;
  constexpr int ACH = A_BYTES / 16 / NT, BCH = TN * (BK / 8) / NT;   // 16-byte chunks per thread per stage
  static_assert(TM % 64 == 0 && A_BYTES % (16 * NT) == 0 && (TN * (BK / 8)) % NT == 0, "tile / thread mismatch");
  static_assert(FN % 2 == 0, "SwiGLU pairs need an even number of weight fragments per wavefront");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int tile = blockIdx.x, split = blockIdx.y, mblock = blockIdx.z;
  const int Kc = p.K / p.S, k_begin = split * Kc, KT = Kc / BK;
  const int MT = (p.M + 63) >> 6;                      // 64-row activation tiles that exist

  // ---- global sources and LDS destinations of this thread's chunks
  const bf16_t* aptr[ACH];
  const bf16_t* bptr[BCH];
  int blds[BCH];
#pragma unroll
  for (int i = 0; i < ACH; ++i) {
    const int c = tid + NT * i, rt = min(mblock * (TM / 64) + c / 512, MT - 1), within = c % 512;
    aptr[i] = p.x + ((size_t)rt * (p.K >> 4) + (k_begin >> 4)) * 1024 + within * 8;
  }
#pragma unroll
  for (int i = 0; i < BCH; ++i) {
    const int c = tid + NT * i, row = c >> 3, col = c & 7;
    bptr[i] = weight_row<TN>(p, tile, row) + k_begin + col * 8;
    blds[i] = A_BYTES + (row >> 5) * B_FRAG + col * B_COL + (row & 31) * 16;
  }
  u32x4 areg[ACH], breg[BCH];
  auto load_regs = [&](int kk) {
#pragma unroll
    for (int i = 0; i < ACH; ++i) areg[i] = *(const u32x4*)(aptr[i] + (size_t)kk * (KS * 1024));
#pragma unroll
    for (int i = 0; i < BCH; ++i) breg[i] = *(const u32x4*)(bptr[i] + (size_t)kk * BK);
  };
  auto store_lds = [&](unsigned char* buf) {
#pragma unroll
    for (int i = 0; i < ACH; ++i) *(u32x4*)(buf + (tid + NT * i) * 16) = areg[i];
#pragma unroll
    for (int i = 0; i < BCH; ++i) *(u32x4*)(buf + blds[i]) = breg[i];
  };

  // ---- operand fragments of this wavefront inside a stage buffer
  int a_off[FM], b_off[FN];
#pragma unroll
  for (int f = 0; f < FM; ++f) {
    const int fa = wm * FM + f;                        // 32-row fragment of the tile
    a_off[f] = (fa >> 1) * A_TILE + (fa & 1) * 1024 + lane * 16;
  }
#pragma unroll
  for (int f = 0; f < FN; ++f) {
    const int nf = p.mode == 1 ? (f / (FN / 2)) * (TN / 64) + wn * (FN / 2) + f % (FN / 2) : wn * FN + f;
    b_off[f] = A_BYTES + nf * B_FRAG + (lane >> 5) * B_COL + (lane & 31) * 16;
  }

  floatx16 acc[FM][FN];
#pragma unroll
  for (int fm = 0; fm < FM; ++fm)
#pragma unroll
    for (int fn = 0; fn < FN; ++fn)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[fm][fn][r] = 0.f;

  auto compute = [&](const unsigned char* buf) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      bf16x8 a[FM], b[FN];
#pragma unroll
      for (int f = 0; f < FM; ++f) a[f] = *(const bf16x8*)(buf + a_off[f] + ks * 2048);
#pragma unroll
      for (int f = 0; f < FN; ++f) b[f] = *(const bf16x8*)(buf + b_off[f] + ks * 2 * B_COL);
#pragma unroll
      for (int fn = 0; fn < FN; ++fn)
#pragma unroll
        for (int fm = 0; fm < FM; ++fm)
          acc[fm][fn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[fn], a[fm], acc[fm][fn], 0, 0, 0);
    }
  };

  // ---- the walk over K starts at a workgroup-dependent stage
  int kk = (tile * 5 + split * 3 + mblock * 7) % KT;
  auto next_stage = [&]() { kk = kk + 1 == KT ? 0 : kk + 1; };
  load_regs(kk);
  store_lds(smem);
  __syncthreads();
  for (int j = 0; j + 1 < KT; ++j) {
    next_stage();
#ifndef WIDE_NO_GLOAD
    load_regs(kk);
#endif
    __builtin_amdgcn_sched_barrier(0);                 // keep the loads ahead of the MFMAs that hide their latency
#ifndef WIDE_NO_COMPUTE
    compute(smem + (j & 1) * STAGE);
#endif
    __builtin_amdgcn_sched_barrier(0);
#ifndef WIDE_NO_STORE
    store_lds(smem + ((j + 1) & 1) * STAGE);
#endif
#ifndef WIDE_NO_BARRIER
    __syncthreads();
#endif
  }
  compute(smem + ((KT - 1) & 1) * STAGE);

  // ---- epilogue.  Accumulator r of lane l: activation row 32 fm + (l & 31) of the wavefront's rows, weight row
  // 8 (r >> 2) + 4 (l >> 5) + (r & 3) of fragment fn.
  const int m0 = mblock * TM + wm * (32 * FM) + (lane & 31);
  const int nsub = 4 * (lane >> 5);
  if (p.epi == GEMM_EPI_PARTIAL) {
    float* out = p.out_f32 + (size_t)split * p.M * p.N;
#pragma unroll
    for (int fm = 0; fm < FM; ++fm) {
      const int m = m0 + 32 * fm;
      if (m >= p.M) continue;
#pragma unroll
      for (int fn = 0; fn < FN; ++fn)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int n = tile * TN + (wn * FN + fn) * 32 + 8 * c + nsub;
          if (n < p.N)
            *(float4*)(out + (size_t)m * p.N + n) =
                make_float4(acc[fm][fn][4 * c], acc[fm][fn][4 * c + 1], acc[fm][fn][4 * c + 2], acc[fm][fn][4 * c + 3]);
        }
    }
  } else {
    const int I = p.N >> 1;
#pragma unroll
    for (int fm = 0; fm < FM; ++fm) {
      const int m = m0 + 32 * fm;
      if (m >= p.M) continue;
#pragma unroll
      for (int fn = 0; fn < FN / 2; ++fn)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int n = tile * (TN / 2) + (wn * (FN / 2) + fn) * 32 + 8 * c + nsub;
          if (n >= I) continue;
          float h[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float g = acc[fm][fn][4 * c + e], u = acc[fm][fn + FN / 2][4 * c + e];
            h[e] = g / (1.f + expf(-g)) * u;
          }
          Act<true>::store4(p.out_xf, m, n, I, h[0], h[1], h[2], h[3]);
        }
    }
  }
}

template <int WGM, int WGN, int FM, int FN, int OCC>
hipError_t launch_cfg(const WideParams& p, int S, hipStream_t st) {
  constexpr int TM = 32 * FM * WGM, TN = 32 * FN * WGN;
  constexpr int LDS = 2 * ((TM / 64) * A_TILE + (TN / 32) * B_FRAG);
  auto kernel = gemm_wide_kernel<WGM, WGN, FM, FN, OCC>;
  static bool configured = false;                      // per process; the attribute belongs to the code object
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int tiles = (p.N + TN - 1) / TN, mblocks = (p.M + TM - 1) / TM;
  hipLaunchKernelGGL(kernel, dim3(tiles, S, mblocks), dim3(64 * WGM * WGN), LDS, st, p);
  return hipGetLastError();
}

}  // namespace

int g_gemm_wide_force_cfg = -1, g_gemm_wide_force_S = -1;   // tuning hooks (benchmarks only)

// Picks the tile shape and the split-K factor, then launches: 256 x 256 tiles (8 wavefronts) for more than 128
// rows, else 128 x 128 tiles (4 wavefronts, two workgroups per CU); split-K until about 192 workgroups exist.
hipError_t launch_gemm_wide(const bf16_t* x, const GemmWeights& W, int M, int N, int K, int epi, void* out,
                            size_t out_capacity_floats, int* S_out, hipStream_t st) {
  if (M <= 0 || N <= 0 || K <= 0 || K % BK || N % 4) return hipErrorInvalidValue;
  if (epi == GEMM_EPI_SWIGLU ? (W.mode != 1 || N % 8) : W.mode != 0) return hipErrorInvalidValue;
  WideParams p;
  p.x = x;
  for (int i = 0; i < 3; ++i) { p.w[i] = (const bf16_t*)W.w[i]; p.rows[i] = W.rows[i]; }
  p.nmat = W.nmat; p.mode = W.mode;
  p.M = M; p.N = N; p.K = K; p.epi = epi;
  p.out_f32 = (float*)out; p.out_xf = (bf16_t*)out;
  const int KT = K / BK;
  int cfg = M > 128 ? 0 : 1;
  if (g_gemm_wide_force_cfg >= 0) cfg = g_gemm_wide_force_cfg;
  const int TM = cfg == 0 ? 256 : 128, TN = cfg == 0 ? 256 : 128;
  const int wgs = ((N + TN - 1) / TN) * ((M + TM - 1) / TM);
  int S = 1;
  if (epi == GEMM_EPI_PARTIAL) {
    for (int s = 1; s <= 8; ++s) {
      if (KT % s) continue;
      if (s > 1 && ((size_t)s * M * N > out_capacity_floats || KT / s < 8)) break;
      S = s;
      if (wgs * s >= (cfg == 0 ? 192 : 384)) break;
    }
    if (g_gemm_wide_force_S > 0 && KT % g_gemm_wide_force_S == 0 && (size_t)g_gemm_wide_force_S * M * N <= out_capacity_floats)
      S = g_gemm_wide_force_S;
  }
  p.S = S;
  if (S_out) *S_out = S;
  return cfg == 0 ? launch_cfg<2, 4, 4, 2, 1>(p, S, st) : launch_cfg<2, 2, 2, 2, 2>(p, S, st);
}
