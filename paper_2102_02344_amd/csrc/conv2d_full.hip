// Grouped Conv2d whose window covers the whole (unpadded) input image: one output pixel per sample,
// so the operator is the fused Linear of the fusion rules table (a batched matrix product per model)
// over the flattened window k = (c, y, x), which is contiguous in both the input and the weights:
//     Y[n][b, o]   = sum_k W[b][o][k] X[n][b][k]            (forward; the DCGAN discriminator's last layer)
//     dX[n][b][k]  = sum_o dY[n][b, o] W[b][o][k]           (also the forward of the generator's first
//                                                            transposed convolution, 1x1 -> 4x4)
//     dW[b][o][k]  = sum_n dY[n][b, o] X[n][b][k]
// Layers with at most 8 output channels (the discriminator's single logit) are bandwidth-bound
// vector work and get streaming kernels; everything else goes to the batched GEMM with the tensors'
// own strides (sample-major rows, model offset inside the row), no copies.
#include "gemm.h"

namespace hfta {

namespace {

constexpr int FULL_MAX_SMALL_CO = 8;

template <typename T> struct Vec16;                       // 16 bytes of storage as floats
template <> struct Vec16<bf16_raw> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void load(const bf16_raw* p, float (&f)[8]) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) { f[2 * i] = __uint_as_float(w[i] << 16); f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u); }
  }
  static __device__ __forceinline__ void store(bf16_raw* p, const float (&f)[8]) {
    *reinterpret_cast<uint4*>(p) = make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]),
                                              pack_bf16x2(f[6], f[7]));
  }
};
template <> struct Vec16<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void load(const float* p, float (&f)[4]) {
    const float4 v = *reinterpret_cast<const float4*>(p);
    f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
  }
  static __device__ __forceinline__ void store(float* p, const float (&f)[4]) {
    *reinterpret_cast<float4*>(p) = make_float4(f[0], f[1], f[2], f[3]);
  }
};

// One workgroup per (sample, model): Co dot products of length K against the same input row.
template <typename T>
__global__ __launch_bounds__(256) void full_fwd_small_kernel(const T* __restrict__ X, const T* __restrict__ Wt, const T* __restrict__ bias,
                                                             T* __restrict__ Y, int B, int Co, int K, int act, float slope) {
  constexpr int EPV = Vec16<T>::N;
  __shared__ float red[4][FULL_MAX_SMALL_CO];
  const int n = blockIdx.x, b = blockIdx.y, t = threadIdx.x;
  const T* x = X + ((int64_t)n * B + b) * K;
  const T* w = Wt + (int64_t)b * Co * K;
  float acc[FULL_MAX_SMALL_CO];
#pragma unroll
  for (int o = 0; o < FULL_MAX_SMALL_CO; ++o) acc[o] = 0.f;
  for (int k = t * EPV; k < K; k += 256 * EPV) {
    float xv[EPV];
    Vec16<T>::load(x + k, xv);
#pragma unroll
    for (int o = 0; o < FULL_MAX_SMALL_CO; ++o) {
      if (o < Co) {
        float wv[EPV];
        Vec16<T>::load(w + (int64_t)o * K + k, wv);
#pragma unroll
        for (int e = 0; e < EPV; ++e) acc[o] += xv[e] * wv[e];
      }
    }
  }
#pragma unroll
  for (int o = 0; o < FULL_MAX_SMALL_CO; ++o) {
    const float s = wave_sum(acc[o]);
    if ((t & 63) == 0) red[t >> 6][o] = s;
  }
  __syncthreads();
  if (t < Co) {
    float s = red[0][t] + red[1][t] + red[2][t] + red[3][t];
    if (bias) s += Elem<T>::load(bias + b * Co + t);
    Elem<T>::store(Y + ((int64_t)n * B + b) * Co + t, apply_act(s, act, slope));
  }
}

// dX[n][b][k .. k + EPV) = sum_o dY[n][b][o] W[b][o][k ..]
template <typename T>
__global__ __launch_bounds__(256) void full_dx_small_kernel(const T* __restrict__ dY, const T* __restrict__ Wt, T* __restrict__ dX, int B,
                                                            int Co, int K) {
  constexpr int EPV = Vec16<T>::N;
  const int n = blockIdx.y, b = blockIdx.z;
  const int k = (blockIdx.x * 256 + threadIdx.x) * EPV;
  if (k >= K) return;
  const T* dy = dY + ((int64_t)n * B + b) * Co;
  const T* w = Wt + (int64_t)b * Co * K + k;
  float out[EPV];
#pragma unroll
  for (int e = 0; e < EPV; ++e) out[e] = 0.f;
  for (int o = 0; o < Co; ++o) {
    const float g = Elem<T>::load(dy + o);
    float wv[EPV];
    Vec16<T>::load(w + (int64_t)o * K, wv);
#pragma unroll
    for (int e = 0; e < EPV; ++e) out[e] += g * wv[e];
  }
  Vec16<T>::store(dX + ((int64_t)n * B + b) * K + k, out);
}

// dW[b][o][k], k in pairs: a thread walks the samples with its pair, consecutive threads on consecutive pairs
template <typename T>
__global__ __launch_bounds__(256) void full_dw_small_kernel(const T* __restrict__ dY, const T* __restrict__ X, float* __restrict__ dW, int B,
                                                            int Nb, int Co, int K) {
  const int o = blockIdx.y, b = blockIdx.z;
  const int k = (blockIdx.x * 256 + threadIdx.x) * 2;
  if (k >= K) return;
  float s0 = 0.f, s1 = 0.f;
#pragma unroll 8
  for (int n = 0; n < Nb; ++n) {
    const float g = Elem<T>::load(dY + ((int64_t)n * B + b) * Co + o);
    const T* x = X + ((int64_t)n * B + b) * K + k;
    s0 += g * Elem<T>::load(x);
    s1 += g * Elem<T>::load(x + 1);
  }
  *reinterpret_cast<float2*>(dW + ((int64_t)b * Co + o) * K + k) = make_float2(s0, s1);
}

bool small_ok(int Nb, int B, int Co, int64_t K, int dtype, const void* p0, const void* p1, const void* p2) {
  const int epv = 16 / (int)dtype_size(dtype);
  return Co <= FULL_MAX_SMALL_CO && K % epv == 0 && Nb <= 65535 && B <= 65535 && reinterpret_cast<uintptr_t>(p0) % 16 == 0 &&
         reinterpret_cast<uintptr_t>(p1) % 16 == 0 && reinterpret_cast<uintptr_t>(p2) % 16 == 0;
}

GemmDesc full_desc(int B, int dtype) {
  GemmDesc d{};
  d.S = 1; d.G0 = B; d.G1 = 1;
  d.act = HFTA_ACT_NONE; d.dtype = dtype; d.splits = 1;
  return d;
}

}  // namespace

bool conv_full_applies(int H, int W, int kh, int kw, int pad, int Ci, int Nb) {
  return H == kh && W == kw && pad == 0 && (int64_t)Ci * kh * kw <= 0x7fffffff && (int64_t)Nb <= 0x7fffffff;
}

int conv_full_fwd(int B, int Nb, int Ci, int Co, int kh, int kw, int dtype, const void* X, const void* Wt, const void* bias, void* Y,
                  int act, float slope, hipStream_t st) {
  const int64_t K = (int64_t)Ci * kh * kw;
  if (small_ok(Nb, B, Co, K, dtype, X, Wt, X)) {
    const dim3 grid((unsigned)Nb, (unsigned)B);
    if (dtype == HFTA_BF16)
      hipLaunchKernelGGL(full_fwd_small_kernel<bf16_raw>, grid, dim3(256), 0, st, (const bf16_raw*)X, (const bf16_raw*)Wt,
                         (const bf16_raw*)bias, (bf16_raw*)Y, B, Co, (int)K, act, slope);
    else
      hipLaunchKernelGGL(full_fwd_small_kernel<float>, grid, dim3(256), 0, st, (const float*)X, (const float*)Wt, (const float*)bias,
                         (float*)Y, B, Co, (int)K, act, slope);
    return launch_status();
  }
  GemmDesc d = full_desc(B, dtype);
  d.A = X; d.Bm = Wt; d.C = Y;
  d.M = Nb; d.N = Co; d.K = (int)K;
  d.a_kc = true; d.a_ld = (int64_t)B * K; d.a_g0 = K;
  d.b_kc = true; d.b_ld = K; d.b_g0 = (int64_t)Co * K;
  d.c_ld = (int64_t)B * Co; d.c_g0 = Co;
  d.bias = bias; d.bias_mode = 2; d.bias_g0 = Co;
  d.act = act; d.slope = slope;
  return gemm_launch(d, st);
}

int conv_full_dx(int B, int Nb, int Ci, int Co, int kh, int kw, int dtype, const void* Wt, const void* dY, void* dX, hipStream_t st) {
  const int64_t K = (int64_t)Ci * kh * kw;
  if (small_ok(Nb, B, Co, K, dtype, Wt, dX, Wt)) {
    const int epv = 16 / (int)dtype_size(dtype);
    const dim3 grid((unsigned)((K / epv + 255) / 256), (unsigned)Nb, (unsigned)B);
    if (dtype == HFTA_BF16)
      hipLaunchKernelGGL(full_dx_small_kernel<bf16_raw>, grid, dim3(256), 0, st, (const bf16_raw*)dY, (const bf16_raw*)Wt, (bf16_raw*)dX, B,
                         Co, (int)K);
    else
      hipLaunchKernelGGL(full_dx_small_kernel<float>, grid, dim3(256), 0, st, (const float*)dY, (const float*)Wt, (float*)dX, B, Co, (int)K);
    return launch_status();
  }
  GemmDesc d = full_desc(B, dtype);
  d.A = dY; d.Bm = Wt; d.C = dX;
  d.M = Nb; d.N = (int)K; d.K = Co;
  d.a_kc = true; d.a_ld = (int64_t)B * Co; d.a_g0 = Co;
  d.b_kc = false; d.b_ld = K; d.b_g0 = (int64_t)Co * K;       // B[kk = o][n = k] = W[o][k]
  d.c_ld = (int64_t)B * K; d.c_g0 = K;
  return gemm_launch(d, st);
}

int conv_full_dw(int B, int Nb, int Ci, int Co, int kh, int kw, int dtype, const void* X, const void* dY, float* dW, hipStream_t st) {
  const int64_t K = (int64_t)Ci * kh * kw;
  if (Co <= FULL_MAX_SMALL_CO && K % 2 == 0 && Co <= 65535 && B <= 65535 && reinterpret_cast<uintptr_t>(dW) % 8 == 0) {
    const dim3 grid((unsigned)((K / 2 + 255) / 256), (unsigned)Co, (unsigned)B);
    if (dtype == HFTA_BF16)
      hipLaunchKernelGGL(full_dw_small_kernel<bf16_raw>, grid, dim3(256), 0, st, (const bf16_raw*)dY, (const bf16_raw*)X, dW, B, Nb, Co, (int)K);
    else
      hipLaunchKernelGGL(full_dw_small_kernel<float>, grid, dim3(256), 0, st, (const float*)dY, (const float*)X, dW, B, Nb, Co, (int)K);
    return launch_status();
  }
  GemmDesc d = full_desc(B, dtype);
  d.A = dY; d.Bm = X; d.C = dW;
  d.M = Co; d.N = (int)K; d.K = Nb;
  d.a_kc = false; d.a_ld = (int64_t)B * Co; d.a_g0 = Co;      // A[m = o][kk = n] = dY[n][b][o]
  d.b_kc = false; d.b_ld = (int64_t)B * K; d.b_g0 = K;        // B[kk = n][k]    = X[n][b][k]
  d.c_ld = K; d.c_g0 = (int64_t)Co * K;
  d.out_f32 = true;
  return gemm_launch(d, st);
}

}  // namespace hfta
