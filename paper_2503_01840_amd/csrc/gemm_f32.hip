// fp32 GEMM for the exact-arithmetic (tiny model) configuration: out[m, col0+n] = sum_k x[m,k] w[n,k].
// One wavefront per (weight row, group of 8 activation rows); lanes stride over K and the partial sums
// are combined with a butterfly, so the result is deterministic.  Not a performance path.
#include "common.hpp"
#include "kernels.hpp"

namespace {
constexpr int RM = 8;

__global__ __launch_bounds__(64) void gemm_f32_kernel(const float* __restrict__ x, const float* __restrict__ w, int M,
                                                     int N, int K, float* __restrict__ out, int ld, int col0) {
  const int n = blockIdx.x, m0 = blockIdx.y * RM, lane = threadIdx.x;
  float acc[RM];
#pragma unroll
  for (int r = 0; r < RM; ++r) acc[r] = 0.f;
  const float* wr = w + (size_t)n * K;
  for (int k = lane; k < K; k += 64) {
    const float wv = wr[k];
#pragma unroll
    for (int r = 0; r < RM; ++r) {
      const int m = min(m0 + r, M - 1);
      acc[r] = fmaf(x[(size_t)m * K + k], wv, acc[r]);
    }
  }
#pragma unroll
  for (int r = 0; r < RM; ++r) {
    const float s = wave_sum(acc[r]);
    if (lane == 0 && m0 + r < M) out[(size_t)(m0 + r) * ld + col0 + n] = s;
  }
}
}  // namespace

hipError_t launch_gemm_f32(const float* x, const float* w, int M, int N, int K, float* out, int ld, int col0,
                           hipStream_t st) {
  if (M <= 0 || N <= 0 || K <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(gemm_f32_kernel, dim3(N, (M + RM - 1) / RM), dim3(64), 0, st, x, w, M, N, K, out, ld, col0);
  return hipGetLastError();
}
