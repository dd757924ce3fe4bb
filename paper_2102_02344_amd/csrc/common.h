// Shared device/host helpers for the fused-array kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "hfta.h"

namespace hfta {

typedef uint16_t bf16_raw;  // bf16 bit pattern; storage only

__device__ __forceinline__ float bf16_to_f32(bf16_raw h) {
  return __uint_as_float(((uint32_t)h) << 16);
}
// round to nearest even (the matrix-core generation's own conversion instruction)
__device__ __forceinline__ bf16_raw f32_to_bf16(float f) {
  const __bf16 b = (__bf16)f;
  return *reinterpret_cast<const bf16_raw*>(&b);
}
// two floats -> two bf16 in one 32-bit word (lo in the low half): one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {lo, hi};
  const bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
  return *reinterpret_cast<const uint32_t*>(&b);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
  static __device__ __forceinline__ float to_f32(float v) { return v; }
  static __device__ __forceinline__ float from_f32(float v) { return v; }
};
template <> struct Elem<bf16_raw> {
  static __device__ __forceinline__ float load(const bf16_raw* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(bf16_raw* p, float v) { *p = f32_to_bf16(v); }
  static __device__ __forceinline__ float to_f32(bf16_raw v) { return bf16_to_f32(v); }
  static __device__ __forceinline__ bf16_raw from_f32(float v) { return f32_to_bf16(v); }
};

// Walks the (sample n, chunk ch) pairs of one channel in steps of the workgroup size without a
// division per step (a 64-bit quotient per element chunk cost more vector-ALU time than the loads
// it addressed): the step is split once into whole rows and a remainder.
struct RowWalk {
  int n, ch, chunks, dn, dc;
  __device__ __forceinline__ RowWalk(int chunks_, int nt) : chunks(chunks_) {
    n = (int)threadIdx.x / chunks_;
    ch = (int)threadIdx.x - n * chunks_;
    dn = nt / chunks_;
    dc = nt - dn * chunks_;
  }
  __device__ __forceinline__ void step() {
    n += dn;
    ch += dc;
    if (ch >= chunks) { ch -= chunks; ++n; }
  }
};

__device__ __forceinline__ float apply_act(float x, int act, float slope) {
  switch (act) {
    case HFTA_ACT_RELU: return x > 0.f ? x : 0.f;
    case HFTA_ACT_LEAKY: return x > 0.f ? x : slope * x;
    case HFTA_ACT_TANH: return tanhf(x);
    case HFTA_ACT_GELU: return 0.5f * x * (1.f + erff(x * 0.70710678118654752f));
    default: return x;
  }
}

// wave64 reductions through the cross-lane shuffle network
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

static inline hipStream_t as_stream(void* s) { return (hipStream_t)s; }

static inline int launch_status() {
  return hipGetLastError() == hipSuccess ? HFTA_OK : HFTA_ELAUNCH;
}

static inline bool valid_dtype(int d) { return d == HFTA_F32 || d == HFTA_BF16; }
static inline bool valid_act(int a) { return a >= HFTA_ACT_NONE && a <= HFTA_ACT_GELU; }
static inline size_t dtype_size(int d) { return d == HFTA_BF16 ? 2 : 4; }

}  // namespace hfta
