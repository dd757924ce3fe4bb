// Helpers shared by the BatchNorm kernels: vector loads/stores of four elements, fixed-order
// block reductions, activation derivative.
#pragma once
#include "common.h"

namespace hfta {

template <typename T, int VEC> struct Vec;
template <> struct Vec<float, 4> { typedef float4 type; };
template <> struct Vec<float, 1> { typedef float type; };
template <> struct Vec<bf16_raw, 4> { typedef uint2 type; };
template <> struct Vec<bf16_raw, 1> { typedef bf16_raw type; };

template <typename T, int VEC>
__device__ __forceinline__ void load_vec(const T* p, float (&v)[VEC]) {
  typename Vec<T, VEC>::type raw = *reinterpret_cast<const typename Vec<T, VEC>::type*>(p);
  const T* e = reinterpret_cast<const T*>(&raw);
#pragma unroll
  for (int i = 0; i < VEC; ++i) v[i] = Elem<T>::to_f32(e[i]);
}
template <typename T, int VEC>
__device__ __forceinline__ void store_vec(T* p, const float (&v)[VEC]) {
  typename Vec<T, VEC>::type raw;
  T* e = reinterpret_cast<T*>(&raw);
#pragma unroll
  for (int i = 0; i < VEC; ++i) e[i] = Elem<T>::from_f32(v[i]);
  *reinterpret_cast<typename Vec<T, VEC>::type*>(p) = raw;
}

// block-wide sum of two values; result valid in every thread
template <int NW>
__device__ __forceinline__ void block_sum2(float& a, float& b, float (*sh)[2]) {
  a = wave_sum(a);
  b = wave_sum(b);
  const int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) { sh[w][0] = a; sh[w][1] = b; }
  __syncthreads();
  float ra = 0.f, rb = 0.f;
#pragma unroll
  for (int i = 0; i < NW; i += 4) {          // fixed order, pairwise within groups of four waves
    ra += (sh[i][0] + sh[i + 1][0]) + (sh[i + 2][0] + sh[i + 3][0]);
    rb += (sh[i][1] + sh[i + 1][1]) + (sh[i + 2][1] + sh[i + 3][1]);
  }
  a = ra; b = rb;
}

__device__ __forceinline__ float act_grad(float pre, int act, float slope) {
  if (act == HFTA_ACT_RELU) return pre > 0.f ? 1.f : 0.f;
  if (act == HFTA_ACT_LEAKY) return pre > 0.f ? 1.f : slope;
  return 1.f;
}


// Channels whose data is large get one 1024-thread workgroup each (instead of 256 threads):
// 512 channels x 1024 threads fill the chip where 512 x 256 would leave it three quarters empty,
// and fewer channels are in flight at once.
static inline bool bn_wide_block(int64_t channel_bytes) { return channel_bytes >= 32 * 1024; }

// widest vector access every row of a strided [b][n][c][l] tensor allows: 4 elements or 1
static inline bool bn_vec4_ok(const void* p, const int64_t* s, int L, int dtype) {
  const size_t bytes = 4 * dtype_size(dtype);
  return L % 4 == 0 && reinterpret_cast<uintptr_t>(p) % bytes == 0 && s[0] % 4 == 0 && s[1] % 4 == 0 && s[2] % 4 == 0;
}

}  // namespace hfta
