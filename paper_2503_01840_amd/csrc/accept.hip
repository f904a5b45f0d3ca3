// Acceptance walk over the verified tree.
//
// Pass 1 (whole chip): per (row, chunk of ACCEPT_CHUNK vocabulary entries) the maximum, its first index and
// the sum of exp(z - chunk max) of z = logits / T.  Pass 2: ONE wavefront per sequence walks from the root:
//   greedy     follow the child whose token is the row argmax (ties -> smaller id), else stop with it;
//   stochastic test the children in ascending node id against the running residual distribution, and on
//              failure draw the bonus token by inverse CDF of the residual in vocabulary order.
// The walk touches only the statistics of the visited rows plus, for the bonus draw, one chunk of logits.
#include <limits.h>

#include <mutex>

#include "../../include/eagle3.h"
#include "common.hpp"
#include "kernels.hpp"

namespace {

constexpr int CH = ACCEPT_CHUNK;

// One workgroup per (row, chunk of 2048 logits): the chunk is read once (two 16-byte loads per thread), every
// wavefront reduces its 512 entries to (max, first arg-max, sum of exp relative to that max) with shuffles, and the
// four results are combined after a single barrier.
__global__ __launch_bounds__(256) void accept_stats_kernel(const float* __restrict__ logits, int V, int n_chunks,
                                                          float inv_t, float* __restrict__ stats) {
  __shared__ float redv[4], reds[4];
  __shared__ int redi[4];
  const int c = blockIdx.x, r = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* z = logits + (size_t)r * V;
  const int lo = c * CH + wave * 512;
  float x[8];
  int idx[8];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int v0 = lo + h * 256 + 4 * lane;
    if (v0 + 3 < V && (V & 3) == 0) {
      const float4 q = *(const float4*)(z + v0);
      x[4 * h] = q.x; x[4 * h + 1] = q.y; x[4 * h + 2] = q.z; x[4 * h + 3] = q.w;
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) x[4 * h + j] = v0 + j < V ? z[v0 + j] : -INFINITY;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) { x[4 * h + j] *= inv_t; idx[4 * h + j] = v0 + j; }
  }
  float mx = -INFINITY;
  int am = INT_MAX;
#pragma unroll
  for (int j = 0; j < 8; ++j)
    if (x[j] > mx) { mx = x[j]; am = idx[j]; }   // ascending index per thread: first maximum kept
  wave_best_pair(mx, am);
  float sum = 0.f;
  if (mx > -INFINITY) {
#pragma unroll
    for (int j = 0; j < 8; ++j) sum += expf(x[j] - mx);   // exp(-inf) = 0 for the padding
  }
  sum = wave_sum_butterfly(sum);
  if (lane == 0) { redv[wave] = mx; redi[wave] = am; reds[wave] = sum; }
  __syncthreads();
  if (tid == 0) {
    float M = redv[0];
    int A = redi[0];
#pragma unroll
    for (int w = 1; w < 4; ++w)
      if (redv[w] > M || (redv[w] == M && redi[w] < A)) { M = redv[w]; A = redi[w]; }
    float S = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w)
      if (redv[w] > -INFINITY) S += reds[w] * expf(redv[w] - M);
    float* o = stats + ((size_t)r * n_chunks + c) * 4;
    o[0] = M;
    o[1] = __int_as_float(A);
    o[2] = S;
    o[3] = 0.f;
  }
}

__device__ __forceinline__ float wave_incl_scan(float v, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const float t = __shfl_up(v, o, 64);
    if (lane >= o) v += t;
  }
  return v;
}

__global__ __launch_bounds__(64) void accept_walk_kernel(const float* __restrict__ logits,
                                                        const int32_t* __restrict__ tree_tok,
                                                        const int32_t* __restrict__ parent, int N, int V, int n_chunks,
                                                        float inv_t, bool greedy, const float* __restrict__ uniforms,
                                                        const float* __restrict__ stats, int32_t* __restrict__ accept_len,
                                                        int32_t* __restrict__ path, int32_t* __restrict__ bonus_tok) {
  __shared__ int struck[64];
  const int b = blockIdx.x, lane = threadIdx.x;
  const int my_par = lane < N ? parent[b * N + lane] : INT_MIN;
  const int my_tok = lane < N ? tree_tok[b * N + lane] : -1;
  if (lane < N) path[b * N + lane] = lane == 0 ? 0 : -1;
  // what the child tests of the stochastic walk read, fetched for every node at once: the target's logit of the node's
  // own token at its parent's row, and the node's uniform (one memory round trip instead of one per tested child)
  float my_z = 0.f, my_u = 0.f;
  if (!greedy && lane > 0 && lane < N && my_par >= 0 && my_par < lane) {
    my_z = logits[((size_t)b * N + my_par) * V + min(max(my_tok, 0), V - 1)];
    my_u = uniforms[(size_t)b * 2 * N + 2 * lane];
  }
  int cur = 0, len = 0, bonus = 0;
  for (int step = 0; step < N; ++step) {
    const int row = b * N + cur;
    const float* st = stats + (size_t)row * n_chunks * 4;
    float mx = -INFINITY;
    int am = INT_MAX;
    for (int c = lane; c < n_chunks; c += 64) {
      const float v = st[c * 4];
      const int i = __float_as_int(st[c * 4 + 1]);
      if (v > mx || (v == mx && i < am)) { mx = v; am = i; }
    }
    wave_best_pair(mx, am);
    const unsigned long long kids = __ballot(lane < N && lane > cur && my_par == cur);
    if (greedy) {
      const unsigned long long hit = __ballot(lane < N && lane > cur && my_par == cur && my_tok == am);
      if (hit) {
        cur = __ffsll((long long)hit) - 1;
        ++len;
        if (lane == 0) path[b * N + len] = cur;
        continue;
      }
      bonus = am;
      break;
    }
    // ---- stochastic
    float tot = 0.f;
    for (int c = lane; c < n_chunks; c += 64) tot += st[c * 4 + 2] * expf(st[c * 4] - mx);
    tot = wave_sum_butterfly(tot);
    const float* z = logits + (size_t)row * V;
    float rej = 0.f;
    int n_struck = 0, accepted = -1;
    unsigned long long rest = kids;
    while (rest) {
      const int c = __ffsll((long long)rest) - 1;
      rest &= rest - 1;
      const int t = min(max(__shfl(my_tok, c, 64), 0), V - 1);
      bool is_struck = false;
      for (int j = 0; j < n_struck; ++j) is_struck |= struck[j] == t;
      const float pt = expf(__shfl(my_z, c, 64) * inv_t - mx) / tot;
      const float thr = is_struck ? 0.f : pt / (1.f - rej);
      const float u = __shfl(my_u, c, 64);
      if (u < thr) { accepted = c; break; }
      if (!is_struck) {
        rej += pt;
        if (lane == 0) struck[n_struck] = t;
        ++n_struck;
        __syncthreads();
      }
    }
    if (accepted >= 0) {
      cur = accepted;
      ++len;
      if (lane == 0) path[b * N + len] = cur;
      continue;
    }
    // bonus token: first v (vocabulary order) whose residual CDF reaches u * (1 - rej), in un-normalised units
    const float target = uniforms[(size_t)b * 2 * N + 2 * cur + 1] * (1.f - rej) * tot;
    float carry = 0.f;
    int chunk = -1, last_pos_chunk = -1;
    float before = 0.f;
    for (int c0 = 0; c0 < n_chunks && chunk < 0; c0 += 64) {
      const int c = c0 + lane;
      float sc = 0.f;
      if (c < n_chunks) {
        sc = st[c * 4 + 2] * expf(st[c * 4] - mx);
        for (int j = 0; j < n_struck; ++j)
          if (struck[j] / CH == c) sc -= expf(z[struck[j]] * inv_t - mx);
        sc = fmaxf(sc, 0.f);
      }
      const float incl = wave_incl_scan(sc, lane) + carry;
      const unsigned long long pos = __ballot(sc > 0.f);
      const unsigned long long cross = __ballot(sc > 0.f && incl >= target);
      if (pos) last_pos_chunk = c0 + 63 - __clzll((long long)pos);
      if (cross) {
        const int l = __ffsll((long long)cross) - 1;
        chunk = c0 + l;
        before = __shfl(incl - sc, l, 64);
      }
      carry = __shfl(incl, 63, 64);
    }
    bool take_last = false;
    if (chunk < 0) { chunk = max(last_pos_chunk, 0); take_last = true; }   // rounding left the total short of the target
    // inside the chunk: 32 consecutive entries per lane
    const int v0 = chunk * CH + lane * (CH / 64);
    float e[CH / 64];
    float ltot = 0.f;
#pragma unroll
    for (int i = 0; i < CH / 64; ++i) {
      const int v = v0 + i;
      float x = 0.f;
      if (v < V) {
        x = expf(z[v] * inv_t - mx);
        for (int j = 0; j < n_struck; ++j)
          if (struck[j] == v) x = 0.f;
      }
      e[i] = x;
      ltot += x;
    }
    const float lincl = wave_incl_scan(ltot, lane) + before;
    const unsigned long long lpos = __ballot(ltot > 0.f);
    unsigned long long lcross = take_last ? 0ull : __ballot(ltot > 0.f && lincl >= target);
    int win_lane;
    bool last_in_lane = false;
    if (lcross) win_lane = __ffsll((long long)lcross) - 1;
    else { win_lane = lpos ? 63 - __clzll((long long)lpos) : 0; last_in_lane = true; }
    int found = -1;
    if (lane == win_lane) {
      float run = lincl - ltot;
      int last = -1;
#pragma unroll
      for (int i = 0; i < CH / 64; ++i) {
        if (e[i] > 0.f) {
          run += e[i];
          last = v0 + i;
          if (!last_in_lane && found < 0 && run >= target) found = v0 + i;
        }
      }
      if (found < 0) found = last;
    }
    bonus = __shfl(found, win_lane, 64);
    break;
  }
  if (lane == 0) {
    accept_len[b] = len;
    bonus_tok[b] = bonus;
  }
}

}  // namespace

size_t accept_scratch_floats(int R, int V) { return (size_t)R * ((V + CH - 1) / CH) * 4; }

hipError_t launch_accept(const float* logits, const int32_t* tree_tok, const int32_t* parent, int B, int N, int V,
                         float temperature, const float* uniforms, float* scratch, int32_t* accept_len, int32_t* path,
                         int32_t* bonus, hipStream_t st) {
  const int n_chunks = (V + CH - 1) / CH;
  const bool greedy = temperature <= 0.f;
  const float inv_t = greedy ? 1.f : 1.f / temperature;
  hipLaunchKernelGGL(accept_stats_kernel, dim3(n_chunks, B * N), dim3(256), 0, st, logits, V, n_chunks, inv_t, scratch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(accept_walk_kernel, dim3(B), dim3(64), 0, st, logits, tree_tok, parent, N, V, n_chunks, inv_t, greedy,
                     uniforms, scratch, accept_len, path, bonus);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------------
// The same walk for callers that cannot allocate and hold no context (code under HIP graph capture, tight serving
// loops): the per-(row, chunk) statistics live in a fixed device array of this library instead of a workspace.
// Each GPU holds its own copy of the array at its own address; the address is looked up once per device, with that
// device current, and only that pointer (never the array's name) is handed to the kernels.
#define ACCEPT_STATIC_FLOATS (256 * 1024)                    /* 1 MiB: rows * chunks <= 65536 */
static __device__ __align__(256) float scratch[ACCEPT_STATIC_FLOATS];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_static_mu;
float* g_static_ptr[MAX_DEVICES] = {};

// Device address of `scratch` on the current device (looked up on the first call per device).
hipError_t static_scratch(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_static_mu);
  if (!g_static_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_static_ptr[dev] = (float*)p;
  }
  *out = g_static_ptr[dev];
  return hipSuccess;
}
}  // namespace

extern "C" int eagle3_accept_static(int32_t B, int32_t N, int32_t vocab, const float* logits, const int32_t* tree_tok,
                                    const int32_t* parent, float temperature, const float* uniforms, int32_t* accept_len,
                                    int32_t* path, int32_t* bonus_tok, eagle3_stream stream) {
  if (!logits || !tree_tok || !parent || !accept_len || !path || !bonus_tok) return EAGLE3_E_NULL;
  if (temperature > 0.f && !uniforms) return EAGLE3_E_NULL;
  if (B < 1 || N < 1 || N > 64 || vocab < 1 || !(temperature >= 0.f)) return EAGLE3_E_SHAPE;
  if ((size_t)B * N > (size_t)ACCEPT_STATIC_FLOATS) return EAGLE3_E_SHAPE;
  if (accept_scratch_floats(B * N, vocab) > (size_t)ACCEPT_STATIC_FLOATS) return EAGLE3_E_SHAPE;
  float* ptr = nullptr;
  if (static_scratch(&ptr) != hipSuccess) return EAGLE3_E_HIP;
  // every (row, chunk) entry the walk reads is written by the statistics pass of the same call: nothing to clear
  if (launch_accept(logits, tree_tok, parent, B, N, vocab, temperature, uniforms, ptr, accept_len, path, bonus_tok,
                    (hipStream_t)stream) != hipSuccess)
    return EAGLE3_E_HIP;
  return EAGLE3_OK;
}
