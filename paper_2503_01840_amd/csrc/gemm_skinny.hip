// Weight-streaming bf16 GEMM for few activation rows:  Y[M, N] = X[M, K] * W[N, K]^T, fp32 accumulate.
//
// Every projection of the speculative step (fusion FC, q/k/v, o, gate/up, down, both LM heads) has at
// most a few dozen rows per sequence, so the kernel is bound by reading W once from HBM.  Two kernels: the
// one described here, and further down a variant with 128 weight rows per workgroup for the largest matrices.
//   * one workgroup (4 wavefronts) owns 64 weight rows and one K range (split-K over blockIdx.y);
//   * W is read with 16-byte loads that are contiguous per row (16 lanes = 256 B of one row), staged
//     through registers into a double-buffered, row-padded LDS tile, and read back as MFMA B operands;
//   * X arrives in the fragment-major layout (one 1 KiB block per MFMA A operand), so it is read straight
//     from L2 with perfectly coalesced 16-byte loads and never touches LDS;
//   * the four wavefronts split the K range of a stage (intra-workgroup split-K), each accumulating the
//     whole 64 x 64 tile with v_mfma_f32_32x32x16_bf16; partial tiles are summed through LDS at the end;
//   * PF stages of global loads are kept in flight per wavefront (register prefetch ring).
#include "common.hpp"
#include "kernels.hpp"

namespace {

constexpr int BK = 128;                 // k per stage: 256-byte pieces of a weight row
constexpr int WCH = BK / 32;            // 16-byte weight chunks per thread per stage
constexpr int KSW = BK / 64;            // MFMA k-steps per wavefront per stage
constexpr int CPR = BK / 8;             // 16-byte chunks per weight row per stage
constexpr int BN = 64;                  // weight rows per workgroup
constexpr int WROW = BK * 2 + 16;       // LDS bytes per staged weight row (padded)
constexpr int PF = 4;                   // stages in flight (5 and more spill the prefetch ring to scratch)
constexpr int ROT_MUL = 5;              // stagger of the starting stage from tile to tile
constexpr int RED_LD = 65;              // floats per row of the reduction buffer
constexpr int SMEM_BYTES = 4 * 64 * RED_LD * 4 > 2 * BN * WROW ? 4 * 64 * RED_LD * 4 : 2 * BN * WROW;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct GemmParams {
  const bf16_t* x;
  const bf16_t* w[3];
  int rows[3];
  int nmat, mode;
  int M, N, K, S, epi;
  float* out_f32;
  bf16_t* out_xf;
};

__device__ __forceinline__ const bf16_t* weight_row(const GemmParams& p, int tile, int row) {
  if (p.mode == 1) {                                   // 32 gate rows | 32 up rows
    int r = tile * 32 + (row & 31);
    r = min(r, p.rows[0] - 1);
    return p.w[row >> 5] + (size_t)r * p.K;
  }
  int n = min(tile * BN + row, p.N - 1);
  int m = 0;
  while (m + 1 < p.nmat && n >= p.rows[m]) { n -= p.rows[m]; ++m; }
  return p.w[m] + (size_t)n * p.K;
}

template <int MH>
__global__ __launch_bounds__(256, 2) void gemm_skinny_kernel(GemmParams p) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM_BYTES];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tile = blockIdx.x, split = blockIdx.y, mtile = blockIdx.z;
  const int Kc = p.K / p.S, k_begin = split * Kc, KT = Kc / BK;

  const bf16_t* wptr[WCH];
  int wlds[WCH];
#pragma unroll
  for (int i = 0; i < WCH; ++i) {
    const int c = tid + 256 * i, row = c / CPR, col = c % CPR;
    wptr[i] = weight_row(p, tile, row) + k_begin + col * 8;
    wlds[i] = row * WROW + col * 16;
  }
  // A-operand blocks of this wavefront: k-steps (k_begin + kt*BK + wave*(BK/4))/16 + {0..KSW-1}, halves 0..MH-1
  const bf16_t* xptr = p.x + (((size_t)mtile * (p.K >> 4) + ((k_begin + wave * (BK / 4)) >> 4)) * 2 * 64 + lane) * 8;

  u32x4 wreg[PF][WCH];
  u32x4 xreg[PF][KSW][MH];
  // Workgroups walk their K range from staggered starting stages: with power-of-two row strides, all
  // workgroups reading the same k offset at the same time would hammer the same few HBM channels.
  const int rot = (tile * ROT_MUL + split) % KT;
  auto load_stage = [&](int kt0_, int slot) {
    int kt = kt0_ + rot;
    kt = kt >= KT ? kt - KT : kt;
#pragma unroll
    for (int i = 0; i < WCH; ++i) {
      wreg[slot][i] = *(const u32x4*)(wptr[i] + (size_t)kt * BK);
    }
#pragma unroll
    for (int ks = 0; ks < KSW; ++ks)
#pragma unroll
      for (int mh = 0; mh < MH; ++mh)
        xreg[slot][ks][mh] = *(const u32x4*)(xptr + ((size_t)(kt * (BK / 16) + ks) * 2 + mh) * 512);
  };
  floatx16 acc[MH][2];
#pragma unroll
  for (int mh = 0; mh < MH; ++mh)
#pragma unroll
    for (int nh = 0; nh < 2; ++nh)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mh][nh][r] = 0.f;

  const int b_off = (lane & 31) * WROW + (wave * (BK / 4) + 8 * (lane >> 5)) * 2;
  // One stage: stage `kt`'s weights go from prefetch slot `s` to LDS, its A operands are set aside, the
  // slot is refilled with stage kt + PF (when `refill`), and after the barrier the tile is multiplied.
  auto do_stage = [&](int kt, int s, bool refill) {
    unsigned char* buf = smem + (kt & 1) * (BN * WROW);
#pragma unroll
    for (int i = 0; i < WCH; ++i) *(u32x4*)(buf + wlds[i]) = wreg[s][i];
    u32x4 xc[KSW][MH];
#pragma unroll
    for (int ks = 0; ks < KSW; ++ks)
#pragma unroll
      for (int mh = 0; mh < MH; ++mh) xc[ks][mh] = xreg[s][ks][mh];
    if (refill) load_stage(kt + PF, s);
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < KSW; ++ks)
#pragma unroll
      for (int nh = 0; nh < 2; ++nh) {
        const u32x4 b = *(const u32x4*)(buf + nh * 32 * WROW + b_off + ks * 32);
#pragma unroll
        for (int mh = 0; mh < MH; ++mh)
          acc[mh][nh] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              __builtin_bit_cast(bf16x8, xc[ks][mh]), __builtin_bit_cast(bf16x8, b), acc[mh][nh], 0, 0, 0);
      }
  };
  // drain: groups whose refills may not all exist (at most the last two groups of a K range)
  auto drain = [&](int kt0) {
    for (; kt0 < KT; kt0 += PF) {
#pragma unroll
      for (int s = 0; s < PF; ++s) {
        const int kt = kt0 + s;
        if (kt < KT) do_stage(kt, s, kt + PF < KT);
      }
    }
  };
  if (KT >= 2 * PF) {
    // Steady state with no branch between the prologue and the loop body, so that the compiler's wait
    // counters stay exact and PF-1 stages of loads remain in flight while one is consumed.
#pragma unroll
    for (int s = 0; s < PF; ++s) {
      load_stage(s, s);
      __builtin_amdgcn_sched_barrier(0);      // keep the issue order: the loop's wait counts depend on it
    }
    int kt0 = 0;
    for (; kt0 + 2 * PF <= KT; kt0 += PF) {
#pragma unroll
      for (int s = 0; s < PF; ++s) do_stage(kt0 + s, s, true);
    }
    drain(kt0);
  } else {
#pragma unroll
    for (int s = 0; s < PF; ++s)
      if (s < KT) load_stage(s, s);
    drain(0);
  }

  // sum the four wavefronts' partial tiles through LDS
  __syncthreads();
  float* red = (float*)smem;
#pragma unroll
  for (int mh = 0; mh < MH; ++mh)
#pragma unroll
    for (int nh = 0; nh < 2; ++nh)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int tok = mh * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        red[(wave * 64 + tok) * RED_LD + nh * 32 + (lane & 31)] = acc[mh][nh][r];
      }
  __syncthreads();
  if (p.epi == GEMM_EPI_PARTIAL) {
#pragma unroll
    for (int e = 0; e < 8 * MH; ++e) {
      const int idx = tid + 256 * e, tok = idx >> 6, f = idx & 63;
      const float v = red[tok * RED_LD + f] + red[(64 + tok) * RED_LD + f] + red[(128 + tok) * RED_LD + f] +
                      red[(192 + tok) * RED_LD + f];
      const int row = mtile * 64 + tok, n = tile * BN + f;
      if (row < p.M && n < p.N) p.out_f32[((size_t)split * p.M + row) * p.N + n] = v;
    }
  } else {
    const int I = p.N >> 1;
#pragma unroll
    for (int e = 0; e < 4 * MH; ++e) {
      const int idx = tid + 256 * e, tok = idx >> 5, f = idx & 31;
      float g = 0.f, u = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        g += red[(w * 64 + tok) * RED_LD + f];
        u += red[(w * 64 + tok) * RED_LD + 32 + f];
      }
      const int row = mtile * 64 + tok, n = tile * 32 + f;
      if (row < p.M && n < I) p.out_xf[xf_offset(row, n, I)] = f32_to_bf16(g / (1.f + expf(-g)) * u);
    }
  }
}

// ---- 128 weight rows per workgroup, for 33..64 activation rows ----
//
// Every 16-byte load a wavefront issues, weight or activation, takes one of the CU's ~200 in-order slots for
// outstanding vector-memory lines, and an activation line that only comes from L2 holds its slot as long as
// the HBM lines queued before it.  With 64 weight rows per workgroup a 64-row activation tile is as many lines
// per stage as the weights (hardware counters: ~95 HBM lines in flight per CU, against ~135 for the 32-row
// kernel and ~185 for a pure weight stream); with 128 weight rows it is half as many.  Eight wavefronts = 2
// halves of the weight rows x 4 quarters of the stage's K; the activation stage (16 KiB, contiguous in the
// fragment-major layout) goes through LDS once instead of being fetched by each half.
namespace wide_tile {
constexpr int BN2 = 128;
constexpr int W_BYTES = BN2 * WROW;                  // one staged weight tile
constexpr int X_BYTES = 64 * BK * 2;                 // one staged activation tile (two 32-row halves x BK/16 k-steps)
constexpr int STAGE_BYTES = W_BYTES + X_BYTES;
constexpr int RED_BYTES = 8 * 64 * RED_LD * 4;
constexpr int SMEM2 = 2 * STAGE_BYTES > RED_BYTES ? 2 * STAGE_BYTES : RED_BYTES;
constexpr int XCH = X_BYTES / 16 / 512;              // 16-byte activation chunks per thread per stage
}  // namespace wide_tile

__device__ __forceinline__ const bf16_t* weight_row128(const GemmParams& p, int tile, int row) {
  if (p.mode == 1) {                                   // 64 gate rows | 64 up rows
    int r = tile * 64 + (row & 63);
    r = min(r, p.rows[0] - 1);
    return p.w[row >> 6] + (size_t)r * p.K;
  }
  int n = min(tile * wide_tile::BN2 + row, p.N - 1);
  int m = 0;
  while (m + 1 < p.nmat && n >= p.rows[m]) { n -= p.rows[m]; ++m; }
  return p.w[m] + (size_t)n * p.K;
}

__global__ __launch_bounds__(512) void gemm_skinny128_kernel(GemmParams p) {
  using namespace wide_tile;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem2[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rh = wave >> 2, kq = wave & 3;
  const int tile = blockIdx.x, split = blockIdx.y, mtile = blockIdx.z;
  const int Kc = p.K / p.S, k_begin = split * Kc, KT = Kc / BK;

  const bf16_t* wptr[WCH];
  int wlds[WCH];
#pragma unroll
  for (int i = 0; i < WCH; ++i) {
    const int c = tid + 512 * i, row = c / CPR, col = c % CPR;
    wptr[i] = weight_row128(p, tile, row) + k_begin + col * 8;
    wlds[i] = row * WROW + col * 16;
  }
  // the activation stage kt: BK/16 k-steps x 2 halves x 1 KiB, contiguous
  const bf16_t* xptr = p.x + ((size_t)mtile * (p.K >> 4) + (k_begin >> 4)) * 2 * 512 + (size_t)tid * 8;

  u32x4 wreg[PF][WCH];
  u32x4 xreg[PF][XCH];
  const int rot = (tile * ROT_MUL + split) % KT;
  auto load_stage = [&](int kt0_, int slot) {
    int kt = kt0_ + rot;
    kt = kt >= KT ? kt - KT : kt;
#pragma unroll
    for (int i = 0; i < WCH; ++i) wreg[slot][i] = *(const u32x4*)(wptr[i] + (size_t)kt * BK);
#pragma unroll
    for (int i = 0; i < XCH; ++i) xreg[slot][i] = *(const u32x4*)(xptr + (size_t)kt * (X_BYTES / 2) + i * 512 * 8);
  };
  floatx16 acc[2][2];                                  // [activation half][32 weight rows]
#pragma unroll
  for (int mh = 0; mh < 2; ++mh)
#pragma unroll
    for (int nh = 0; nh < 2; ++nh)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mh][nh][r] = 0.f;

  const int b_off = (rh * 64 + (lane & 31)) * WROW + (kq * (BK / 4) + 8 * (lane >> 5)) * 2;
  const int a_off = W_BYTES + kq * KSW * 2048 + lane * 16;
  auto do_stage = [&](int kt, int s, bool refill) {
    unsigned char* buf = smem2 + (kt & 1) * STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < WCH; ++i) *(u32x4*)(buf + wlds[i]) = wreg[s][i];
#pragma unroll
    for (int i = 0; i < XCH; ++i) *(u32x4*)(buf + W_BYTES + (tid + 512 * i) * 16) = xreg[s][i];
    if (refill) load_stage(kt + PF, s);
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < KSW; ++ks) {
      u32x4 a[2];
#pragma unroll
      for (int mh = 0; mh < 2; ++mh) a[mh] = *(const u32x4*)(buf + a_off + (ks * 2 + mh) * 1024);
#pragma unroll
      for (int nh = 0; nh < 2; ++nh) {
        const u32x4 b = *(const u32x4*)(buf + nh * 32 * WROW + b_off + ks * 32);
#pragma unroll
        for (int mh = 0; mh < 2; ++mh)
          acc[mh][nh] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              __builtin_bit_cast(bf16x8, a[mh]), __builtin_bit_cast(bf16x8, b), acc[mh][nh], 0, 0, 0);
      }
    }
  };
  auto drain = [&](int kt0) {
    for (; kt0 < KT; kt0 += PF) {
#pragma unroll
      for (int s = 0; s < PF; ++s) {
        const int kt = kt0 + s;
        if (kt < KT) do_stage(kt, s, kt + PF < KT);
      }
    }
  };
  if (KT >= 2 * PF) {
#pragma unroll
    for (int s = 0; s < PF; ++s) {
      load_stage(s, s);
      __builtin_amdgcn_sched_barrier(0);      // keep the issue order: the loop's wait counts depend on it
    }
    int kt0 = 0;
    for (; kt0 + 2 * PF <= KT; kt0 += PF) {
#pragma unroll
      for (int s = 0; s < PF; ++s) do_stage(kt0 + s, s, true);
    }
    drain(kt0);
  } else {
#pragma unroll
    for (int s = 0; s < PF; ++s)
      if (s < KT) load_stage(s, s);
    drain(0);
  }

  // sum the four K-quarter tiles of each weight-row half through LDS: red[wave][activation row][weight row]
  __syncthreads();
  float* red = (float*)smem2;
#pragma unroll
  for (int mh = 0; mh < 2; ++mh)
#pragma unroll
    for (int nh = 0; nh < 2; ++nh)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int tok = mh * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        red[(wave * 64 + tok) * RED_LD + nh * 32 + (lane & 31)] = acc[mh][nh][r];
      }
  __syncthreads();
  auto summed = [&](int half, int tok, int f) {
    const float* r0 = red + ((half * 4) * 64 + tok) * RED_LD + f;
    return r0[0] + r0[64 * RED_LD] + r0[128 * RED_LD] + r0[192 * RED_LD];
  };
  if (p.epi == GEMM_EPI_PARTIAL) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int idx = tid + 512 * e, tok = idx >> 7, f = idx & 127;
      const float v = summed(f >> 6, tok, f & 63);
      const int row = mtile * 64 + tok, n = tile * BN2 + f;
      if (row < p.M && n < p.N) p.out_f32[((size_t)split * p.M + row) * p.N + n] = v;
    }
  } else {
    const int I = p.N >> 1;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int idx = tid + 512 * e, tok = idx >> 6, f = idx & 63;
      const float g = summed(0, tok, f), u = summed(1, tok, f);
      const int row = mtile * 64 + tok, n = tile * 64 + f;
      if (row < p.M && n < I) p.out_xf[xf_offset(row, n, I)] = f32_to_bf16(g / (1.f + expf(-g)) * u);
    }
  }
}

}  // namespace

// Split-K factor, from measurements on MI355X (two of these workgroups fit a CU):
//   * 192-256 workgroups already stream a [4096..6144, 4096] weight at its best rate, and every extra split adds an
//     fp32 partial tile the consumer has to read back: take the smallest divisor of the stage count that reaches 192;
//   * between 256 and ~450 workgroups some CUs get two and the others one, and the launch takes as long as with
//     512 (320 workgroups on a [10240, 8192] weight: 46.7 us, 160 or 640: 43.5 us): skip those;
//   * a K range left longer than 64 stages is cut further (a [8192, 28672] weight streams 22 % faster as 512
//     workgroups of 56 stages than as 256 of 112).
int gemm_skinny_pick_splits(int N, int K, int M) {
  const int tiles = (N + BN - 1) / BN * ((M + 63) / 64);
  const int KT = K / BK;
  int best = 1;
  for (int S = 1; S <= 16; ++S) {
    if (KT % S) continue;
    if (S > 1 && KT / S < 4) break;
    const int wgs = tiles * S;
    if (S > 1 && wgs > 256 && wgs < 450) continue;
    best = S;
    if (wgs >= 192 && (KT / S <= 64 || wgs >= 512)) break;
  }
  return best;
}

bool gemm_skinny_uses_tile128(const GemmWeights& W, int M, int N, int S) {
  const int tiles128 = W.mode == 1 ? (N / 2 + 63) / 64 : (N + wide_tile::BN2 - 1) / wide_tile::BN2;
  return M > 32 && S == 1 && tiles128 >= 192;
}

hipError_t launch_gemm_skinny(const bf16_t* x, const GemmWeights& W, int M, int N, int K, int S, int epi, void* out,
                              hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
  if (M <= 0 || N <= 0 || K <= 0 || S <= 0 || K % (BK * S) != 0) return hipErrorInvalidValue;
  if (epi == GEMM_EPI_SWIGLU && (S != 1 || W.mode != 1)) return hipErrorInvalidValue;
  GemmParams p;
  p.x = x;
  for (int i = 0; i < 3; ++i) { p.w[i] = (const bf16_t*)W.w[i]; p.rows[i] = W.rows[i]; }
  p.nmat = W.nmat; p.mode = W.mode;
  p.M = M; p.N = N; p.K = K; p.S = S; p.epi = epi;
  p.out_f32 = (float*)out; p.out_xf = (bf16_t*)out;
  // 33..64 rows: 128 weight rows per workgroup where that still gives most CUs a tile without split-K (gate/up,
  // LM head: 5 % faster); matrices with few rows need the splits for parallelism and then the smaller
  // workgroup's shorter prologue and reduction win (q/k/v, o, down: 5-15 % slower with the large tile)
  if (gemm_skinny_uses_tile128(W, M, N, S)) {
    const int tiles = W.mode == 1 ? (N / 2 + 63) / 64 : (N + wide_tile::BN2 - 1) / wide_tile::BN2;
    static DeviceOnce configured;                // the attribute belongs to the loaded code object of a device
    hipError_t ce = configured.run([&] {
      return hipFuncSetAttribute((const void*)gemm_skinny128_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, wide_tile::SMEM2);
    });
    if (ce != hipSuccess) return ce;
    launch_with_events(gemm_skinny128_kernel, dim3(tiles, S, (M + 63) / 64), dim3(512), wide_tile::SMEM2, st, ev_start, ev_stop, p);
    return hipGetLastError();
  }
  const int tiles = W.mode == 1 ? (N / 2 + 31) / 32 : (N + BN - 1) / BN;
  dim3 grid(tiles, S, (M + 63) / 64);
  if (M <= 32)
    launch_with_events(gemm_skinny_kernel<1>, grid, dim3(256), 0, st, ev_start, ev_stop, p);
  else
    launch_with_events(gemm_skinny_kernel<2>, grid, dim3(256), 0, st, ev_start, ev_stop, p);
  return hipGetLastError();
}
