// Shared device helpers for the gfx950 kernels: bf16 conversion, the fragment-major activation
// layout read by the MFMA GEMMs, and small reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint16_t bf16_t;          // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));

// two fp32 -> two bf16 (round to nearest even) packed into one dword, low half = a: one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  const floatx2_t f = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.f) & 0xFFFFu); }

template <typename T> __device__ __forceinline__ float load_f32(const T* p, size_t i);
template <> __device__ __forceinline__ float load_f32<float>(const float* p, size_t i) { return p[i]; }
template <> __device__ __forceinline__ float load_f32<bf16_t>(const bf16_t* p, size_t i) { return bf16_to_f32(p[i]); }

template <typename T> __device__ __forceinline__ void store_from_f32(T* p, size_t i, float v);
template <> __device__ __forceinline__ void store_from_f32<float>(float* p, size_t i, float v) { p[i] = v; }
template <> __device__ __forceinline__ void store_from_f32<bf16_t>(bf16_t* p, size_t i, float v) { p[i] = f32_to_bf16(v); }

// Fragment-major layout of a bf16 activation matrix X[rows, K] (K % 16 == 0), as the MFMA GEMMs read it:
// rows are grouped in tiles of 64, K in steps of 16; the 32 rows x 16 k of one (tile, k-step, half)
// form one 1 KiB block holding, for lane l of a wavefront, the 8 values X[32*half + l%32][16*step + 8*(l/32) .. +7]
// at element offset 8*l.  One such block is exactly the A operand of v_mfma_f32_32x32x16_bf16.
__host__ __device__ __forceinline__ size_t xf_offset(int row, int k, int K) {
  const int tile = row >> 6, half = (row >> 5) & 1, r = row & 31;
  const int step = k >> 4, kg = (k >> 3) & 1, e = k & 7;
  return ((((size_t)tile * (K >> 4) + step) * 2 + half) * 64 + (r + 32 * kg)) * 8 + e;
}
__host__ __device__ __forceinline__ size_t xf_elems(int rows, int K) { return (size_t)((rows + 63) / 64) * 64 * K; }

// Activation store policy: BF16 path writes fragment-major bf16, FP32 path writes row-major fp32.
template <bool BF16> struct Act;
template <> struct Act<true> {
  typedef bf16_t type;
  static __device__ __forceinline__ void store(bf16_t* p, int row, int k, int K, float v) { p[xf_offset(row, k, K)] = f32_to_bf16(v); }
  // four consecutive k (k % 4 == 0) are contiguous in the fragment-major layout
  static __device__ __forceinline__ void store4(bf16_t* p, int row, int k, int K, float a, float b, float c, float d) {
    uint2 v;
    v.x = pack_bf16x2(a, b);
    v.y = pack_bf16x2(c, d);
    *(uint2*)(p + xf_offset(row, k, K)) = v;
  }
};
template <> struct Act<false> {
  typedef float type;
  static __device__ __forceinline__ void store(float* p, int row, int k, int K, float v) { p[(size_t)row * K + k] = v; }
  static __device__ __forceinline__ void store4(float* p, int row, int k, int K, float a, float b, float c, float d) {
    *(float4*)(p + (size_t)row * K + k) = make_float4(a, b, c, d);
  }
};

// four consecutive values of a weight-typed vector (gain) or of a row-major activation
__device__ __forceinline__ float4 load4_f32(const float* p, size_t i) { return *(const float4*)(p + i); }
__device__ __forceinline__ float4 load4_f32(const bf16_t* p, size_t i) {
  const uint2 v = *(const uint2*)(p + i);
  return make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xFFFF0000u), __uint_as_float(v.y << 16),
                     __uint_as_float(v.y & 0xFFFF0000u));
}
// four consecutive values stored in the plain (row-major) storage type
__device__ __forceinline__ void store4_plain(float* p, size_t i, float a, float b, float c, float d) {
  *(float4*)(p + i) = make_float4(a, b, c, d);
}
__device__ __forceinline__ void store4_plain(bf16_t* p, size_t i, float a, float b, float c, float d) {
  uint2 v;
  v.x = pack_bf16x2(a, b);
  v.y = pack_bf16x2(c, d);
  *(uint2*)(p + i) = v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Butterfly all-reduce over the 64 lanes without the LDS crossbar that __shfl_xor goes through (ds_bpermute,
// ~100 clocks a step): step s hands every lane its own value and its partner's, in some order (a, b).  Steps 0, 1:
// DPP quad permutes (lane ^ 1, lane ^ 2); 2, 3: DPP mirrors within 8 and within 16 lanes (once a group of 4 or 8
// lanes agrees, the mirrored lane is as good a partner as lane ^ 4 or lane ^ 8); 4, 5: v_permlane16_swap and
// v_permlane32_swap.  For commutative, idempotent-or-associative combiners every lane ends with the wavefront's result.
template <int STEP>
__device__ __forceinline__ void xlane_partners(uint32_t x, uint32_t& a, uint32_t& b) {
  a = x;
  if constexpr (STEP == 0) b = (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, 0xB1, 0xF, 0xF, false);
  else if constexpr (STEP == 1) b = (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, 0x4E, 0xF, 0xF, false);
  else if constexpr (STEP == 2) b = (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, 0x141, 0xF, 0xF, false);
  else if constexpr (STEP == 3) b = (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, 0x140, 0xF, 0xF, false);
  else if constexpr (STEP == 4) { const auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false); a = r[0]; b = r[1]; }
  else { const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false); a = r[0]; b = r[1]; }
}
template <int STEP> __device__ __forceinline__ float xlane_max_step(float v) {
  uint32_t a, b;
  xlane_partners<STEP>(__float_as_uint(v), a, b);
  return fmaxf(__uint_as_float(a), __uint_as_float(b));
}
template <int STEP> __device__ __forceinline__ float xlane_sum_step(float v) {
  uint32_t a, b;
  xlane_partners<STEP>(__float_as_uint(v), a, b);
  return __uint_as_float(a) + __uint_as_float(b);
}
__device__ __forceinline__ float wave_max(float v) {
  v = xlane_max_step<0>(v); v = xlane_max_step<1>(v); v = xlane_max_step<2>(v);
  v = xlane_max_step<3>(v); v = xlane_max_step<4>(v); v = xlane_max_step<5>(v);
  return v;
}
// same result on every lane; the summation order differs from wave_sum's (used where the last ulp is free)
__device__ __forceinline__ float wave_sum_butterfly(float v) {
  v = xlane_sum_step<0>(v); v = xlane_sum_step<1>(v); v = xlane_sum_step<2>(v);
  v = xlane_sum_step<3>(v); v = xlane_sum_step<4>(v); v = xlane_sum_step<5>(v);
  return v;
}
// (value, index) of the wavefront's best entry: larger value first, ties -> smaller index
template <int STEP> __device__ __forceinline__ void xlane_best_step(float& v, int& i) {
  uint32_t va, vb, ia, ib;
  xlane_partners<STEP>(__float_as_uint(v), va, vb);
  xlane_partners<STEP>((uint32_t)i, ia, ib);
  const float fa = __uint_as_float(va), fb = __uint_as_float(vb);
  const bool first = fa > fb || (fa == fb && (int)ia < (int)ib);
  v = first ? fa : fb;
  i = first ? (int)ia : (int)ib;
}
__device__ __forceinline__ void wave_best_pair(float& v, int& i) {
  xlane_best_step<0>(v, i); xlane_best_step<1>(v, i); xlane_best_step<2>(v, i);
  xlane_best_step<3>(v, i); xlane_best_step<4>(v, i); xlane_best_step<5>(v, i);
}

// Block-wide sum for blockDim.x a multiple of 64, <= 1024.  `red` is a __shared__ float[17].
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  if (threadIdx.x == 0) {
    float s = 0.f;
    for (int i = 0; i < nw; ++i) s += red[i];
    red[16] = s;
  }
  __syncthreads();
  return red[16];
}
__device__ __forceinline__ float block_max(float v, float* red) {
  v = wave_max(v);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  if (threadIdx.x == 0) {
    float s = red[0];
    for (int i = 1; i < nw; ++i) s = fmaxf(s, red[i]);
    red[16] = s;
  }
  __syncthreads();
  return red[16];
}

// Runs a set-up call once per device (the device current at the call), thread-safe: kernel attributes such as the
// dynamic-LDS limit belong to the code object loaded on ONE device.
#include <mutex>
struct DeviceOnce {
  std::mutex mu;
  bool done[64] = {};
  template <typename F> hipError_t run(F&& f) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (done[dev]) return hipSuccess;
    e = f();
    if (e == hipSuccess) done[dev] = true;
    return e;
  }
};

// Launch with an optional start/stop event pair attached to the dispatch itself: the events then carry the
// kernel's own begin and end timestamps (what a kernel trace reports), not the time between two stream markers.
template <typename Kernel, typename Params>
inline void launch_with_events(Kernel kernel, dim3 grid, dim3 block, unsigned lds_bytes, hipStream_t st, hipEvent_t ev_start,
                               hipEvent_t ev_stop, const Params& p) {
  if (ev_start && ev_stop) hipExtLaunchKernelGGL(kernel, grid, block, lds_bytes, st, ev_start, ev_stop, 0, p);
  else hipLaunchKernelGGL(kernel, grid, block, lds_bytes, st, p);
}
