// bf16 GEMM for MANY activation rows (batched verification: 64 sequences x 8 nodes = 512 rows):
// Y[M, N] = X[M, K] * W[N, K]^T, fp32 accumulate.  At this width the projections sit at the ridge between weight
// streaming and the MFMA rate, so the kernel is organised around operand reuse and around keeping the loads, the
// LDS reads and the MFMAs of a wavefront all in flight at once:
//   * a workgroup owns a (32 FM WGM) x (32 FN WGN) output tile; its WGM x WGN wavefronts each hold FM x FN
//     accumulators of v_mfma_f32_32x32x16_bf16 and there is no cross-wavefront reduction;
//   * both operands reach LDS by direct global-to-LDS loads (global_load_lds_dwordx4: each wavefront
//     instruction deposits 1 KiB contiguously, no staging registers).  A CU accepts roughly one cache line per
//     four clocks whatever its size, so every request is a whole 128-byte line: activations come in 32-k slots
//     (ring of 4; their fragment-major global layout already is the MFMA operand order, so the copy is verbatim
//     and the LDS reads are linear), weights in 64-k slots (ring of 3; eight lanes per 128-byte row piece, and
//     which 16 bytes a lane fetches is XOR-swizzled with the row index so that the MFMA operand reads, 32 rows x
//     one piece, touch every bank once);
//   * one barrier per 32-k half-stage.  The barrier of half-stage h also publishes the data of half-stage h + 1,
//     so the first operand fragments of h + 1 are read into registers while the MFMAs of h still run and the
//     matrix pipe does not idle after the next barrier; the four loads a wavefront issues per half-stage are
//     spread between groups of MFMAs, so that a full load queue never holds up MFMA issue;
//   * the workgroups that share a weight tile (one per 256 activation rows) are launched next to each other on
//     the same XCD, so the tile leaves HBM once;
//   * the weights are the MFMA's first operand: a lane then holds, for ONE activation row, runs of four
//     consecutive output columns, which is what both epilogues store: fp32 split-K partials (16-byte stores), or
//     SwiGLU (the tile interleaves gate and up rows so that both values of a pair sit in the same lane) written
//     as fragment-major bf16 (8-byte stores).
#include "common.hpp"
#include "kernels.hpp"

namespace {

constexpr int BK = 64;                  // k per weight slot; the activation slots and the barriers are per BK / 2
constexpr int A_SLOTS = 4, B_SLOTS = 3;

struct WideParams {
  const bf16_t* x;
  const bf16_t* w[3];
  int rows[3];
  int nmat, mode;
  int M, N, K, S, epi;
  int tiles, groups, mblocks;           // weight tiles, ceil(tiles / 8), activation-row blocks
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

// One wavefront-wide direct load: lane l's 16 bytes at `src` land at LDS byte address lds_base + 16 l.
// The compiler does not see these as memory operations; the kernel counts them itself (s_waitcnt vmcnt).
// (m0 carries the LDS address; naming it as clobbered is what is meant, the compiler's remark about reserved
// registers on a clobber list is switched off for this one statement.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16(const void* src, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(src) : "memory", "m0");
}
#pragma clang diagnostic pop
#define WIDE_WAIT_LOADS(n) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(n) : "memory")
#define WIDE_PIN() __builtin_amdgcn_sched_barrier(0)

template <int WGM, int WGN, int FM, int FN, int OCC>
__global__ __launch_bounds__(64 * WGM * WGN, OCC) void gemm_wide_kernel(WideParams p) {
  constexpr int TM = 32 * FM * WGM, TN = 32 * FN * WGN, NW = WGM * WGN;
  constexpr int A_SLOT = TM * (BK / 2) * 2, B_SLOT = TN * BK * 2;   // bytes
  constexpr int B_BASE = A_SLOTS * A_SLOT;
  // direct-to-LDS instructions (1 KiB each) per wavefront per activation / weight slot; a weight slot goes out in two halves
  constexpr int A_DMA = A_SLOT / (1024 * NW), B_DMA = B_SLOT / (1024 * NW), BH = B_DMA / 2;
  static_assert(A_DMA == 2 && (B_DMA == 2 || B_DMA == 4) && A_SLOT == A_DMA * 1024 * NW && B_SLOT == B_DMA * 1024 * NW,
                "1 KiB pieces per wavefront");
  static_assert(TM % 64 == 0 && FN == 2, "whole 64-row activation tiles; one SwiGLU pair per wavefront");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;

  // Workgroups go to the XCDs round-robin by their linear id: id % 8 is the XCD.  Consecutive workgroups of one
  // XCD take the activation-row blocks of ONE weight tile, so that the tile is fetched into that L2 once.
  int j = blockIdx.x >> 3;
  const int mblock = j % p.mblocks;  j /= p.mblocks;
  const int tile = (j % p.groups) * 8 + (blockIdx.x & 7), split = j / p.groups;
  if (tile >= p.tiles) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WGN, wn = wave % WGN;
  const int Kc = p.K / p.S, k_begin = split * Kc, KT = Kc / BK;   // KT weight stages = 2 KT half-stages
  const int MT = (p.M + 63) >> 6;                      // 64-row activation tiles that exist

  // ---- this lane's global sources.  Piece q of an activation slot is (row tile q / 4, k-step (q / 2) % 2, row
  // half q % 2); piece q of a weight slot is rows 8 q .. 8 q + 7, eight lanes per row.
  const bf16_t* aptr[A_DMA];
  const bf16_t* bptr[B_DMA];
#pragma unroll
  for (int i = 0; i < A_DMA; ++i) {
    const int q = wave * A_DMA + i;
    const int rt = min(mblock * (TM / 64) + (q >> 2), MT - 1);
    aptr[i] = p.x + (((size_t)rt * (p.K >> 4) + (k_begin >> 4) + ((q >> 1) & 1)) * 2 + (q & 1)) * 512 + lane * 8;
  }
#pragma unroll
  for (int i = 0; i < B_DMA; ++i) {
    const int row = 8 * (wave * B_DMA + i) + (lane >> 3), piece = (lane & 7) ^ ((row >> 1) & 7);
    bptr[i] = weight_row<TN>(p, tile, row) + k_begin + piece * 8;
  }
  // Loads past the end of the walk over K repeat the last (half-)stage into a slot nobody reads any more, which
  // keeps the number of loads in flight, and with it the waits below, the same in every iteration.
  auto issue_a = [&](int h, int i) {                   // piece i of half-stage h
    dma16(aptr[i] + (size_t)min(h, 2 * KT - 1) * 2048, lds0 + (h % A_SLOTS) * A_SLOT + (wave * A_DMA + i) * 1024);
  };
  auto issue_b = [&](int s, int i) {                   // piece i of weight stage s
    dma16(bptr[i] + (size_t)min(s, KT - 1) * BK, lds0 + B_BASE + (s % B_SLOTS) * B_SLOT + (wave * B_DMA + i) * 1024);
  };

  // ---- operand fragments of this wavefront inside their slots
  int a_off[FM], b_off[FN][4];
#pragma unroll
  for (int f = 0; f < FM; ++f) {
    const int fa = wm * FM + f;                        // 32-row fragment of the tile
    a_off[f] = (fa >> 1) * 4096 + (fa & 1) * 1024 + lane * 16;
  }
#pragma unroll
  for (int f = 0; f < FN; ++f) {
    const int nf = p.mode == 1 ? f * (TN / 64) + wn : wn * FN + f;
    const int row = nf * 32 + (lane & 31);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) b_off[f][ks] = B_BASE + row * (BK * 2) + (((2 * ks + (lane >> 5)) ^ ((row >> 1) & 7)) * 16);
  }
  auto a_slot_of = [&](int h) { return smem + (h % A_SLOTS) * A_SLOT; };
  auto b_slot_of = [&](int s) { return smem + (s % B_SLOTS) * B_SLOT; };
  auto load_frags = [&](bf16x8 (&a)[FM], bf16x8 (&b)[FN], const unsigned char* a_slot, const unsigned char* b_slot, int ks) {
#pragma unroll
    for (int f = 0; f < FM; ++f) a[f] = *(const bf16x8*)(a_slot + a_off[f] + (ks & 1) * 2048);
#pragma unroll
    for (int f = 0; f < FN; ++f) b[f] = *(const bf16x8*)(b_slot + b_off[f][ks]);
  };

  floatx16 acc[FM][FN];
#pragma unroll
  for (int fm = 0; fm < FM; ++fm)
#pragma unroll
    for (int fn = 0; fn < FN; ++fn)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[fm][fn][r] = 0.f;
  auto mfma_col = [&](const bf16x8 (&a)[FM], const bf16x8 (&b)[FN], int fn) {
#pragma unroll
    for (int fm = 0; fm < FM; ++fm) acc[fm][fn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[fn], a[fm], acc[fm][fn], 0, 0, 0);
  };

  // Loads complete in issue order.  Per wavefront the order is
  //   B0lo A0 B0hi A1 B1lo A2 B1hi | half-stage h = 2 s: A(h+3) B(s+2)lo | half-stage h = 2 s + 1: A(h+3) B(s+2)hi
  // (A(h) = both pieces of activation half-stage h, B(s)lo / hi = the first / second half of the pieces of weight stage s).
  auto issue_b_half = [&](int s, int half) {
#pragma unroll
    for (int i = 0; i < BH; ++i) issue_b(s, half * BH + i);
  };
  issue_b_half(0, 0); issue_a(0, 0); issue_a(0, 1); issue_b_half(0, 1);
  issue_a(1, 0); issue_a(1, 1); issue_b_half(1, 0); issue_a(2, 0); issue_a(2, 1); issue_b_half(1, 1);
  WIDE_WAIT_LOADS(2 * A_DMA + B_DMA);                  // A0 and B0 are in LDS ...
  __syncthreads();                                     // ... for every wavefront
  bf16x8 a0[FM], b0[FN], a1[FM], b1[FN];
  load_frags(a0, b0, a_slot_of(0), b_slot_of(0), 0);

  // One 32-k half-stage: a0 / b0 hold its first k-step on entry and the first k-step of the next one on exit.
  auto half_stage = [&](int s, int half) {
    const int h = 2 * s + half;
    // everything up to A(h+1) (even h) / up to B(s+1)hi (odd h) has landed when only the loads issued after it
    // are in flight: what the NEXT half-stage reads is in LDS, what THIS one reads was published a barrier ago
    if (half == 0) WIDE_WAIT_LOADS(A_DMA + B_DMA); else WIDE_WAIT_LOADS(A_DMA + B_DMA / 2);
    __syncthreads();                                   // ... for every wavefront; the slots of half-stage h - 1 are free
    WIDE_PIN();
    issue_a(h + 3, 0);
    load_frags(a1, b1, a_slot_of(h), b_slot_of(s), 2 * half + 1);
    mfma_col(a0, b0, 0);
    WIDE_PIN();
    issue_a(h + 3, 1);
    mfma_col(a0, b0, 1);
    WIDE_PIN();
    issue_b(s + 2, BH * half);
    load_frags(a0, b0, a_slot_of(h + 1), b_slot_of(s + half), 2 * (1 - half));
    mfma_col(a1, b1, 0);
    WIDE_PIN();
    if (BH == 2) issue_b(s + 2, BH * half + 1);
    mfma_col(a1, b1, 1);
    WIDE_PIN();
  };
  for (int s = 0; s < KT; ++s) {
    half_stage(s, 0);
    half_stage(s, 1);
  }
  WIDE_WAIT_LOADS(0);                                  // nothing may still be writing LDS when the workgroup ends

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
      for (int c = 0; c < 4; ++c) {
        const int n = tile * (TN / 2) + wn * 32 + 8 * c + nsub;
        if (n >= I) continue;
        float h[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float g = acc[fm][0][4 * c + e], u = acc[fm][1][4 * c + e];
          h[e] = g / (1.f + expf(-g)) * u;
        }
        Act<true>::store4(p.out_xf, m, n, I, h[0], h[1], h[2], h[3]);
      }
    }
  }
}

template <int WGM, int WGN, int FM, int FN, int OCC>
hipError_t launch_cfg(WideParams& p, int S, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
  constexpr int TM = 32 * FM * WGM, TN = 32 * FN * WGN;
  constexpr int LDS = A_SLOTS * TM * (BK / 2) * 2 + B_SLOTS * TN * BK * 2;
  auto kernel = gemm_wide_kernel<WGM, WGN, FM, FN, OCC>;
  static DeviceOnce configured;                        // the attribute belongs to the loaded code object of a device
  hipError_t ce = configured.run([&] { return hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, LDS); });
  if (ce != hipSuccess) return ce;
  p.tiles = (p.N + TN - 1) / TN;
  p.groups = (p.tiles + 7) / 8;
  p.mblocks = (p.M + TM - 1) / TM;
  launch_with_events(kernel, dim3(8 * p.groups * p.mblocks * S), dim3(64 * WGM * WGN), LDS, st, ev_start, ev_stop, p);
  return hipGetLastError();
}

}  // namespace

// Picks the tile shape and the split-K factor, then launches.
hipError_t launch_gemm_wide(const bf16_t* x, const GemmWeights& W, int M, int N, int K, int epi, void* out,
                            size_t out_capacity_floats, int* S_out, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
  if (M <= 0 || N <= 0 || K <= 0 || K % BK || N % 4) return hipErrorInvalidValue;
  if (epi == GEMM_EPI_SWIGLU ? (W.mode != 1 || N % 8) : W.mode != 0) return hipErrorInvalidValue;
  WideParams p;
  p.x = x;
  for (int i = 0; i < 3; ++i) { p.w[i] = (const bf16_t*)W.w[i]; p.rows[i] = W.rows[i]; }
  p.nmat = W.nmat; p.mode = W.mode;
  p.M = M; p.N = N; p.K = K; p.epi = epi;
  p.out_f32 = (float*)out; p.out_xf = (bf16_t*)out;
  const int KT = K / BK;
  // 256 x 256 tiles when there are enough rows and, with at least 16 stages left per workgroup after split-K,
  // enough workgroups; 129..256 rows: ONE 256-row block x 128 weight rows per workgroup (8 wavefronts x 64 x 64), so that
  // every weight line enters exactly one CU and a stage takes in 48 KB instead of the 2 x 32 KB of two 128 x 128
  // workgroups (measured at 256 rows, 8B shapes: q/k/v 33.4 -> 26.6 us, down 54.3 -> 47.6, gate/up 86.0 -> 78.9);
  // else 128 x 128 tiles, two workgroups per CU.
  auto pick = [&](int TM, int TN, int want, int min_stages, int* S_pick) {
    const int wgs = ((N + TN - 1) / TN) * ((M + TM - 1) / TM);
    int S = 1;
    if (epi == GEMM_EPI_PARTIAL)
      for (int s = 1; s <= 8 && wgs * S < want; ++s) {
        if (KT % s) continue;
        if (s > 1 && ((size_t)s * M * N > out_capacity_floats || KT / s < min_stages)) break;
        S = s;
      }
    *S_pick = S;
    return wgs * S;
  };
  int S = 1, cfg = 0;
  if (M > 128 && M <= 256) {
    cfg = 2;
    pick(256, 128, 192, 8, &S);
  } else if (M < 384 || (pick(256, 256, 160, 16, &S) < 160 && epi == GEMM_EPI_PARTIAL)) {
    cfg = 1;
    pick(128, 128, 384, 8, &S);
  }
  p.S = S;
  if (S_out) *S_out = S;
  if (cfg == 2) return launch_cfg<4, 2, 2, 2, 1>(p, S, st, ev_start, ev_stop);
  return cfg == 0 ? launch_cfg<2, 4, 4, 2, 1>(p, S, st, ev_start, ev_stop) : launch_cfg<2, 2, 2, 2, 2>(p, S, st, ev_start, ev_stop);
}
