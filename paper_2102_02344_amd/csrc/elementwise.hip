// Support operators that close a training step: activations, dropout from an
// explicit mask, per-model LayerNorm, per-model losses.  All are HBM-bound
// streaming kernels; per-model reductions never mix models.
#include "common.h"

using namespace hfta;

namespace {

__device__ __forceinline__ float act_deriv_from_input(float x, int act, float slope) {
  switch (act) {
    case HFTA_ACT_RELU: return x > 0.f ? 1.f : 0.f;
    case HFTA_ACT_LEAKY: return x > 0.f ? 1.f : slope;
    case HFTA_ACT_TANH: { const float t = tanhf(x); return 1.f - t * t; }
    case HFTA_ACT_GELU: {
      const float cdf = 0.5f * (1.f + erff(x * 0.70710678118654752f));
      const float pdf = 0.39894228040143268f * expf(-0.5f * x * x);
      return cdf + x * pdf;
    }
    default: return 1.f;
  }
}
__device__ __forceinline__ float act_deriv_from_output(float y, int act, float slope) {
  switch (act) {
    case HFTA_ACT_RELU: return y > 0.f ? 1.f : 0.f;
    case HFTA_ACT_LEAKY: return y > 0.f ? 1.f : slope;
    case HFTA_ACT_TANH: return 1.f - y * y;
    default: return 1.f;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void act_fwd_kernel(const T* __restrict__ x, T* __restrict__ y, int64_t n, int act, float slope) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
    Elem<T>::store(y + i, apply_act(Elem<T>::load(x + i), act, slope));
}

template <typename T>
__global__ __launch_bounds__(256) void act_bwd_kernel(const T* __restrict__ z, const T* __restrict__ dy, T* __restrict__ dx,
                                                     int64_t n, int act, float slope, int from_output) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const float zz = Elem<T>::load(z + i);
    const float d = from_output ? act_deriv_from_output(zz, act, slope) : act_deriv_from_input(zz, act, slope);
    Elem<T>::store(dx + i, Elem<T>::load(dy + i) * d);
  }
}

// ---- 16-byte vector forms of the streaming operators ------------------------
// Used when every pointer is 16-byte aligned (tails run through the element kernels above).  The
// activation is a template parameter: one scalar branch per element would otherwise cost as much
// as the memory traffic.  For bf16 storage GELU and its derivative use erf from the
// Abramowitz-Stegun 7.1.26 rational form (|error| < 1.5e-7) and share one exponential.
template <typename T> struct V16;
template <> struct V16<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[4]) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
  }
  static __device__ __forceinline__ uint4 pack(const float (&f)[4]) {
    return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
  }
};
template <> struct V16<bf16_raw> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[8]) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) { f[2 * i] = __uint_as_float(w[i] << 16); f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u); }
  }
  static __device__ __forceinline__ uint4 pack(const float (&f)[8]) {
    return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]), pack_bf16x2(f[6], f[7]));
  }
};

// erf(|x|/sqrt 2) and exp(-x^2/2) together
__device__ __forceinline__ void erf_exp_fast(float x, float& erf_abs, float& ex) {
  const float z = fabsf(x) * 0.70710678118654752f;
  const float tt = __builtin_amdgcn_rcpf(fmaf(0.3275911f, z, 1.f));
  float poly = fmaf(tt, 1.061405429f, -1.453152027f);
  poly = fmaf(tt, poly, 1.421413741f);
  poly = fmaf(tt, poly, -0.284496736f);
  poly = fmaf(tt, poly, 0.254829592f);
  poly *= tt;
  ex = __builtin_amdgcn_exp2f(-z * z * 1.4426950408889634f);
  erf_abs = fmaf(-poly, ex, 1.f);
}

template <int ACT, bool FAST>
__device__ __forceinline__ float act_t(float x, float slope) {
  if (ACT == HFTA_ACT_RELU) return fmaxf(x, 0.f);
  if (ACT == HFTA_ACT_LEAKY) return x > 0.f ? x : slope * x;
  if (ACT == HFTA_ACT_TANH) return tanhf(x);
  if (ACT == HFTA_ACT_GELU) {
    if (FAST) {
      float ea, ex;
      erf_exp_fast(x, ea, ex);
      return 0.5f * x * (1.f + copysignf(ea, x));
    }
    return 0.5f * x * (1.f + erff(x * 0.70710678118654752f));
  }
  return x;
}
template <int ACT, bool FAST>
__device__ __forceinline__ float act_deriv_t(float x, float slope) {
  if (ACT == HFTA_ACT_GELU && FAST) {
    float ea, ex;
    erf_exp_fast(x, ea, ex);
    return fmaf(x * 0.39894228040143268f, ex, 0.5f * (1.f + copysignf(ea, x)));
  }
  return act_deriv_from_input(x, ACT, slope);
}

template <typename T, int ACT>
__global__ __launch_bounds__(256) void act_fwd_vec_kernel(const uint4* __restrict__ x, uint4* __restrict__ y, int64_t nvec, float slope) {
  constexpr int N = V16<T>::N;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * 256) {
    float f[N];
    V16<T>::unpack(x[i], f);
#pragma unroll
    for (int e = 0; e < N; ++e) f[e] = act_t<ACT, sizeof(T) == 2>(f[e], slope);
    y[i] = V16<T>::pack(f);
  }
}

template <typename T, int ACT, bool FROM_OUT>
__global__ __launch_bounds__(256) void act_bwd_vec_kernel(const uint4* __restrict__ z, const uint4* __restrict__ dy,
                                                         uint4* __restrict__ dx, int64_t nvec, float slope) {
  constexpr int N = V16<T>::N;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * 256) {
    float zz[N], d[N];
    V16<T>::unpack(z[i], zz);
    V16<T>::unpack(dy[i], d);
#pragma unroll
    for (int e = 0; e < N; ++e)
      d[e] *= FROM_OUT ? act_deriv_from_output(zz[e], ACT, slope) : act_deriv_t<ACT, sizeof(T) == 2>(zz[e], slope);
    dx[i] = V16<T>::pack(d);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void add_vec_kernel(const uint4* __restrict__ a, const uint4* __restrict__ b,
                                                     uint4* __restrict__ y, int64_t nvec) {
  constexpr int N = V16<T>::N;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * 256) {
    float fa[N], fb[N];
    V16<T>::unpack(a[i], fa);
    V16<T>::unpack(b[i], fb);
#pragma unroll
    for (int e = 0; e < N; ++e) fa[e] += fb[e];
    y[i] = V16<T>::pack(fa);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void add_kernel(const T* __restrict__ a, const T* __restrict__ b, T* __restrict__ y, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
    Elem<T>::store(y + i, Elem<T>::load(a + i) + Elem<T>::load(b + i));
}

template <typename T>
__global__ __launch_bounds__(256) void bias_act_nchw_kernel(T* __restrict__ y, const T* __restrict__ bias, int64_t K, int64_t HW,
                                                           int64_t total, int act, float slope) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t k = (i / HW) % K;
    const float b = bias ? Elem<T>::load(bias + k) : 0.f;
    Elem<T>::store(y + i, apply_act(Elem<T>::load(y + i) + b, act, slope));
  }
}

template <typename T>
__global__ __launch_bounds__(256) void dropout_kernel(const T* __restrict__ x, const uint8_t* __restrict__ mask, T* __restrict__ y,
                                                     int64_t n, float scale) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
    Elem<T>::store(y + i, mask[i] ? Elem<T>::load(x + i) * scale : 0.f);
}

// ---- LayerNorm: one wavefront per row of E elements -----------------------
template <typename T>
__global__ __launch_bounds__(256) void layernorm_fwd_kernel(const T* __restrict__ X, const float* __restrict__ w,
                                                           const float* __restrict__ bsh, float eps, float* __restrict__ save_mean,
                                                           float* __restrict__ save_invstd, T* __restrict__ Y, int R, int E,
                                                           int64_t rows) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int b = (int)(row / R);
  const T* x = X + row * E;
  float s = 0.f;
  for (int e = lane; e < E; e += 64) s += Elem<T>::load(x + e);
  const float mean = wave_sum(s) / (float)E;
  float q = 0.f;
  for (int e = lane; e < E; e += 64) { const float d = Elem<T>::load(x + e) - mean; q = fmaf(d, d, q); }
  const float invstd = 1.0f / sqrtf(wave_sum(q) / (float)E + eps);
  if (lane == 0) { save_mean[row] = mean; save_invstd[row] = invstd; }
  const float* wb = w + (int64_t)b * E;
  const float* bb = bsh + (int64_t)b * E;
  T* y = Y + row * E;
  for (int e = lane; e < E; e += 64)
    Elem<T>::store(y + e, fmaf((Elem<T>::load(x + e) - mean) * invstd, wb[e], bb[e]));
}

// dx per row; per-block partial dw/db over its rows go to the workspace [nblk][2][E] per model
template <typename T>
__global__ __launch_bounds__(256) void layernorm_bwd_kernel(const T* __restrict__ X, const T* __restrict__ dY, const float* __restrict__ w,
                                                           const float* __restrict__ save_mean, const float* __restrict__ save_invstd,
                                                           T* __restrict__ dX, float* __restrict__ part, int R, int E, int rows_per_block) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int b = blockIdx.y;
  const int r_begin = blockIdx.x * rows_per_block;
  const int r_end = min(R, r_begin + rows_per_block);
  const float* wb = w + (int64_t)b * E;
  for (int r = r_begin + wv; r < r_end; r += 4) {
    const int64_t row = (int64_t)b * R + r;
    const T* x = X + row * E;
    const T* dy = dY + row * E;
    const float mean = save_mean[row], invstd = save_invstd[row];
    float s1 = 0.f, s2 = 0.f;
    for (int e = lane; e < E; e += 64) {
      const float g = Elem<T>::load(dy + e) * wb[e];
      const float xh = (Elem<T>::load(x + e) - mean) * invstd;
      s1 += g; s2 = fmaf(g, xh, s2);
    }
    s1 = wave_sum(s1) / (float)E;
    s2 = wave_sum(s2) / (float)E;
    T* dx = dX + row * E;
    for (int e = lane; e < E; e += 64) {
      const float g = Elem<T>::load(dy + e) * wb[e];
      const float xh = (Elem<T>::load(x + e) - mean) * invstd;
      Elem<T>::store(dx + e, invstd * (g - s1 - xh * s2));
    }
  }
  // column partials: thread t owns columns t, t+256, ... and walks this block's rows in order
  float* pw = part + (((int64_t)b * gridDim.x + blockIdx.x) * 2) * E;
  for (int e = threadIdx.x; e < E; e += 256) {
    float aw = 0.f, ab = 0.f;
    for (int r = r_begin; r < r_end; ++r) {
      const int64_t row = (int64_t)b * R + r;
      const float d = Elem<T>::load(dY + row * E + e);
      const float xh = (Elem<T>::load(X + row * E + e) - save_mean[row]) * save_invstd[row];
      aw = fmaf(d, xh, aw); ab += d;
    }
    pw[e] = aw; pw[E + e] = ab;
  }
}

// np = 2: [dw | db] partial rows per block; np = 3: a third row, the column sums of the stored dX
__global__ __launch_bounds__(256) void layernorm_bwd_reduce_kernel(const float* __restrict__ part, float* __restrict__ dw,
                                                                  float* __restrict__ db, float* __restrict__ dxs, int E,
                                                                  int nblk, int np) {
  const int b = blockIdx.y;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= E) return;
  float aw = 0.f, ab = 0.f, ax = 0.f;
  for (int k = 0; k < nblk; ++k) {
    const float* pw = part + (((int64_t)b * nblk + k) * np) * E;
    aw += pw[e]; ab += pw[E + e];
    if (np == 3) ax += pw[2 * E + e];
  }
  dw[(int64_t)b * E + e] = aw;
  db[(int64_t)b * E + e] = ab;
  if (np == 3) dxs[(int64_t)b * E + e] = ax;
}

// ---- LayerNorm, register-resident rows ----------------------------------------
// One wavefront per row, a lane holds CH x 16 bytes of it (E <= CH * 64 * 16 / sizeof(T)), so the
// row is read from memory once: statistics, normalisation (and in the backward the per-column
// partial sums for dw, db) all work on registers.  Rows of a block are dealt round-robin to its
// four wavefronts; column partials are combined wave 0..3 in order, so results are reproducible.
template <typename T, int CH>
__global__ __launch_bounds__(256) void layernorm_fwd_vec_kernel(const uint4* __restrict__ X, const float* __restrict__ w,
                                                               const float* __restrict__ bsh, float eps,
                                                               float* __restrict__ save_mean, float* __restrict__ save_invstd,
                                                               uint4* __restrict__ Y, int R, int E, int64_t rows) {
  constexpr int N = V16<T>::N;
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int b = (int)(row / R);
  const int vpr = E / N;                                  // 16-byte vectors per row
  float f[CH][N];
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < CH; ++c) {
    const int v = lane + 64 * c;
    if (v < vpr) {
      V16<T>::unpack(X[row * vpr + v], f[c]);
#pragma unroll
      for (int e = 0; e < N; ++e) s += f[c][e];
    }
  }
  const float mean = wave_sum(s) / (float)E;
  float q = 0.f;
#pragma unroll
  for (int c = 0; c < CH; ++c)
    if (lane + 64 * c < vpr) {
#pragma unroll
      for (int e = 0; e < N; ++e) { const float d = f[c][e] - mean; q = fmaf(d, d, q); }
    }
  const float invstd = 1.0f / sqrtf(wave_sum(q) / (float)E + eps);
  if (lane == 0) { save_mean[row] = mean; save_invstd[row] = invstd; }
#pragma unroll
  for (int c = 0; c < CH; ++c) {
    const int v = lane + 64 * c;
    if (v < vpr) {
      const float* wp = w + (int64_t)b * E + v * N;
      const float* bp = bsh + (int64_t)b * E + v * N;
#pragma unroll
      for (int e = 0; e < N; ++e) f[c][e] = fmaf((f[c][e] - mean) * invstd, wp[e], bp[e]);
      Y[row * vpr + v] = V16<T>::pack(f[c]);
    }
  }
}

// SUMS: the incoming gradient is dY + dY2 (rounded to the storage type, as if a separate element-wise
// sum had stored it) when dY2 is given, and a third partial row carries the column sums of the
// stored dX (the bias gradient of the Linear that produced X's residual branch).
template <typename T, int CH, bool SUMS = false>
__global__ __launch_bounds__(256) void layernorm_bwd_vec_kernel(const uint4* __restrict__ X, const uint4* __restrict__ dY,
                                                               const float* __restrict__ w, const float* __restrict__ save_mean,
                                                               const float* __restrict__ save_invstd, uint4* __restrict__ dX,
                                                               float* __restrict__ part, int R, int E, int rows_per_block,
                                                               const uint4* __restrict__ dY2 = nullptr) {
  constexpr int N = V16<T>::N;
  constexpr int NP = SUMS ? 3 : 2;
  __shared__ float red[3][NP][CH * 64 * N];               // waves 1..3: [dw | db (| dx sums)] partials
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int b = blockIdx.y;
  const int r_begin = blockIdx.x * rows_per_block;
  const int r_end = min(R, r_begin + rows_per_block);
  const int vpr = E / N;
  float wl[CH][N], aw[CH][N], ab[CH][N], ax[SUMS ? CH : 1][N];
#pragma unroll
  for (int c = 0; c < CH; ++c)
#pragma unroll
    for (int e = 0; e < N; ++e) {
      const int col = (lane + 64 * c) * N + e;
      wl[c][e] = col < E ? w[(int64_t)b * E + col] : 0.f;
      aw[c][e] = 0.f; ab[c][e] = 0.f;
      if (SUMS) ax[c][e] = 0.f;
    }
  for (int r = r_begin + wv; r < r_end; r += 4) {
    const int64_t row = (int64_t)b * R + r;
    const float mean = save_mean[row], invstd = save_invstd[row];
    float xh[CH][N], g[CH][N];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int v = lane + 64 * c;
      if (v < vpr) {
        float x[N], d[N];
        V16<T>::unpack(X[row * vpr + v], x);
        V16<T>::unpack(dY[row * vpr + v], d);
        if (SUMS && dY2) {
          float d2[N];
          V16<T>::unpack(dY2[row * vpr + v], d2);
#pragma unroll
          for (int e = 0; e < N; ++e) d[e] += d2[e];
          V16<T>::unpack(V16<T>::pack(d), d);
        }
#pragma unroll
        for (int e = 0; e < N; ++e) {
          xh[c][e] = (x[e] - mean) * invstd;
          g[c][e] = d[e] * wl[c][e];
          s1 += g[c][e]; s2 = fmaf(g[c][e], xh[c][e], s2);
          aw[c][e] = fmaf(d[e], xh[c][e], aw[c][e]); ab[c][e] += d[e];
        }
      }
    }
    s1 = wave_sum(s1) / (float)E;
    s2 = wave_sum(s2) / (float)E;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int v = lane + 64 * c;
      if (v < vpr) {
        float o[N];
#pragma unroll
        for (int e = 0; e < N; ++e) o[e] = invstd * (g[c][e] - s1 - xh[c][e] * s2);
        const uint4 st = V16<T>::pack(o);
        dX[row * vpr + v] = st;
        if (SUMS) {
          V16<T>::unpack(st, o);
#pragma unroll
          for (int e = 0; e < N; ++e) ax[c][e] += o[e];
        }
      }
    }
  }
  if (wv > 0) {
#pragma unroll
    for (int c = 0; c < CH; ++c)
#pragma unroll
      for (int e = 0; e < N; ++e) {
        red[wv - 1][0][(lane + 64 * c) * N + e] = aw[c][e];
        red[wv - 1][1][(lane + 64 * c) * N + e] = ab[c][e];
        if (SUMS) red[wv - 1][NP - 1][(lane + 64 * c) * N + e] = ax[c][e];
      }
  }
  __syncthreads();
  if (wv == 0) {
    float* pw = part + (((int64_t)b * gridDim.x + blockIdx.x) * NP) * E;
#pragma unroll
    for (int c = 0; c < CH; ++c)
#pragma unroll
      for (int e = 0; e < N; ++e) {
        const int col = (lane + 64 * c) * N + e;
        if (col < E) {
          pw[col] = ((aw[c][e] + red[0][0][col]) + red[1][0][col]) + red[2][0][col];
          pw[E + col] = ((ab[c][e] + red[0][1][col]) + red[1][1][col]) + red[2][1][col];
          if (SUMS) pw[2 * E + col] = ((ax[c][e] + red[0][NP - 1][col]) + red[1][NP - 1][col]) + red[2][NP - 1][col];
        }
      }
  }
}

// ---- losses: one workgroup per model, fixed reduction order ----------------
__device__ __forceinline__ float block_sum_1024(float v, float* sh) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  float s = 0.f;
  const int nw = blockDim.x >> 6;
  for (int i = 0; i < nw; ++i) s += sh[i];
  return s;
}

template <typename T>
__global__ __launch_bounds__(1024) void softmax_xent_kernel(const T* __restrict__ logits, const int32_t* __restrict__ labels,
                                                           float* __restrict__ loss, T* __restrict__ dlogits, int R, int K) {
  __shared__ float sh[16];
  const int b = blockIdx.x;
  float acc = 0.f;
  const float invR = 1.f / (float)R;
  for (int r = threadIdx.x; r < R; r += blockDim.x) {
    const T* z = logits + ((int64_t)b * R + r) * K;
    T* dz = dlogits + ((int64_t)b * R + r) * K;
    const int lab = labels[(int64_t)b * R + r];
    float mx = -INFINITY;
    for (int k = 0; k < K; ++k) mx = fmaxf(mx, Elem<T>::load(z + k));
    float se = 0.f;
    for (int k = 0; k < K; ++k) se += expf(Elem<T>::load(z + k) - mx);
    const float lse = mx + logf(se);
    acc += lse - Elem<T>::load(z + lab);
    for (int k = 0; k < K; ++k) {
      const float pk = expf(Elem<T>::load(z + k) - lse);
      Elem<T>::store(dz + k, (pk - (k == lab ? 1.f : 0.f)) * invR);
    }
  }
  const float s = block_sum_1024(acc, sh);
  if (threadIdx.x == 0) loss[b] = s * invR;
}

template <typename T, int KIND>  // KIND 0: BCE on sigmoid(logits); 1: MSE
__global__ __launch_bounds__(1024) void pointwise_loss_kernel(const T* __restrict__ pred, const T* __restrict__ target,
                                                             float* __restrict__ loss, T* __restrict__ dpred, int64_t R,
                                                             int64_t sb, int64_t sr) {
  __shared__ float sh[16];
  const int b = blockIdx.x;
  float acc = 0.f;
  const float invR = 1.f / (float)R;
  for (int64_t i = threadIdx.x; i < R; i += blockDim.x) {
    const int64_t at = (int64_t)b * sb + i * sr;
    const float z = Elem<T>::load(pred + at);
    const float t = Elem<T>::load(target + at);
    float g;
    if (KIND == 0) {
      acc += fmaxf(z, 0.f) - z * t + log1pf(expf(-fabsf(z)));
      g = 1.f / (1.f + expf(-z)) - t;
    } else {
      const float d = z - t;
      acc = fmaf(d, d, acc);
      g = 2.f * d;
    }
    Elem<T>::store(dpred + at, g * invR);
  }
  const float s = block_sum_1024(acc, sh);
  if (threadIdx.x == 0) loss[b] = s * invR;
}

// Activation backward of a fused Linear's output fused with that Linear's bias gradient:
// dX = dY * act'(Z) over [B][M][F] and dbias[b][f] = sum_m dX[b][m][f] (of the values as stored), one
// pass.  A workgroup owns 16 pieces of 16 bytes along the features x 64 row lanes of one model; row
// lanes meet in LDS in a fixed order.
// SUM_ONLY: dx is already there (written by the full-width element-wise kernel); only its column sums
// are formed - the form for few models, where (features / 128) x B workgroups cannot carry the
// element-wise traffic.
template <typename T, int ACT, bool SUM_ONLY = false>
__global__ __launch_bounds__(1024) void act_bwd_colsum_kernel(const uint4* __restrict__ z, const uint4* __restrict__ dy,
                                                             uint4* __restrict__ dx, float* __restrict__ out, int M,
                                                             int F, float slope) {
  constexpr int N = V16<T>::N;
  __shared__ float part[64][16 * N + 1];
  const int b = blockIdx.y;
  const int cg = threadIdx.x & 15, rl = threadIdx.x >> 4;
  const int vpr = F / N;
  const int v = blockIdx.x * 16 + cg;
  float acc[N];
#pragma unroll
  for (int e = 0; e < N; ++e) acc[e] = 0.f;
  if (v < vpr) {
    const int64_t base = (int64_t)b * M * vpr + v;
#pragma unroll 4
    for (int r = rl; r < M; r += 64) {
      const int64_t at = base + (int64_t)r * vpr;
      float zz[N], d[N];
      if (SUM_ONLY) {
        V16<T>::unpack(dx[at], d);
      } else {
        V16<T>::unpack(z[at], zz);
        V16<T>::unpack(dy[at], d);
#pragma unroll
        for (int e = 0; e < N; ++e) d[e] *= act_deriv_t<ACT, sizeof(T) == 2>(zz[e], slope);
        const uint4 o = V16<T>::pack(d);
        dx[at] = o;
        V16<T>::unpack(o, d);               // the column sum is of the stored values
      }
#pragma unroll
      for (int e = 0; e < N; ++e) acc[e] += d[e];
    }
  }
#pragma unroll
  for (int e = 0; e < N; ++e) part[rl][cg * N + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < 16 * N) {
    const int col = blockIdx.x * 16 * N + threadIdx.x;
    if (col < F) {
      float s = 0.f;
      for (int r = 0; r < 64; ++r) s += part[r][threadIdx.x];
      out[(int64_t)b * F + col] = s;
    }
  }
}

// Long contiguous rows (a regression target per token and feature): one workgroup per model cannot
// pull a row through one compute unit fast enough, so both the loss and the gradient are full-width
// launches over all B*R elements in 16-byte pieces: chunk sums of the loss (64 per model, fixed
// order), their sum, then the element-wise gradient.  The gradient must not alias pred or target
// here (the chunk sums pass through its buffer before the inputs are read a second time).
template <int KIND>
__device__ __forceinline__ void pointwise_term(float z, float t, float& loss, float& g) {
  if (KIND == 0) {
    loss = fmaxf(z, 0.f) - z * t + log1pf(expf(-fabsf(z)));
    g = 1.f / (1.f + expf(-z)) - t;
  } else {
    const float d = z - t;
    loss = d * d;
    g = 2.f * d;
  }
}

template <typename T, int KIND>
__global__ __launch_bounds__(256) void pointwise_grad_vec_kernel(const uint4* __restrict__ pred, const uint4* __restrict__ target,
                                                                uint4* __restrict__ dpred, int64_t nvec, float invR) {
  constexpr int N = V16<T>::N;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * 256) {
    float z[N], t[N];
    V16<T>::unpack(pred[i], z);
    V16<T>::unpack(target[i], t);
#pragma unroll
    for (int e = 0; e < N; ++e) {
      float l, g;
      pointwise_term<KIND>(z[e], t[e], l, g);
      z[e] = g * invR;
    }
    dpred[i] = V16<T>::pack(z);
  }
}

// Loss of model b, first stage: workgroup (s, b) sums chunk s of the row and leaves the partial sum in
// the first floats of that model's dpred row, which the gradient launch overwrites afterwards (no
// scratch memory is needed, and the order of the additions is fixed).
constexpr int POINTWISE_CHUNKS = 64;
template <typename T, int KIND>
__global__ __launch_bounds__(1024) void pointwise_loss_part_kernel(const uint4* __restrict__ pred, const uint4* __restrict__ target,
                                                                  uint4* __restrict__ dpred, int64_t vec_per_row) {
  __shared__ float sh[16];
  constexpr int N = V16<T>::N;
  const int b = blockIdx.y;
  const int64_t per = (vec_per_row + POINTWISE_CHUNKS - 1) / POINTWISE_CHUNKS;
  const int64_t lo = (int64_t)blockIdx.x * per;
  const int64_t hi = lo + per < vec_per_row ? lo + per : vec_per_row;
  const uint4* pr = pred + (int64_t)b * vec_per_row;
  const uint4* tg = target + (int64_t)b * vec_per_row;
  float acc = 0.f;
#pragma unroll 4
  for (int64_t i = lo + threadIdx.x; i < hi; i += 1024) {
    float z[N], t[N];
    V16<T>::unpack(pr[i], z);
    V16<T>::unpack(tg[i], t);
#pragma unroll
    for (int e = 0; e < N; ++e) {
      float l, g;
      pointwise_term<KIND>(z[e], t[e], l, g);
      acc += l;
    }
  }
  const float s = block_sum_1024(acc, sh);
  if (threadIdx.x == 0) reinterpret_cast<float*>(dpred + (int64_t)b * vec_per_row)[blockIdx.x] = s;
}

// second stage: one wavefront per model adds the chunk sums in order
__global__ __launch_bounds__(64) void pointwise_loss_final_kernel(const uint4* __restrict__ dpred, float* __restrict__ loss,
                                                                 int64_t vec_per_row, float invR) {
  if (threadIdx.x != 0) return;
  const float* part = reinterpret_cast<const float*>(dpred + (int64_t)blockIdx.x * vec_per_row);
  float s = 0.f;
  for (int i = 0; i < POINTWISE_CHUNKS; ++i) s += part[i];
  loss[blockIdx.x] = s * invR;
}

// rows at least this long take the two-launch form when they are contiguous and 16-byte aligned
constexpr int64_t POINTWISE_WIDE_MIN_R = 1 << 16;

unsigned stream_blocks(int64_t n) {
  int64_t b = (n + 255) / 256;
  const int64_t cap = 256 * 32;
  return (unsigned)(b > cap ? cap : (b < 1 ? 1 : b));
}


static inline bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

template <typename T>
static void launch_act_fwd_vec(const void* X, void* Y, int64_t nvec, int act, float slope, hipStream_t st) {
  const dim3 g(stream_blocks(nvec)), b(256);
  const uint4* x = (const uint4*)X; uint4* y = (uint4*)Y;
  switch (act) {
    case HFTA_ACT_RELU: hipLaunchKernelGGL((act_fwd_vec_kernel<T, HFTA_ACT_RELU>), g, b, 0, st, x, y, nvec, slope); break;
    case HFTA_ACT_LEAKY: hipLaunchKernelGGL((act_fwd_vec_kernel<T, HFTA_ACT_LEAKY>), g, b, 0, st, x, y, nvec, slope); break;
    case HFTA_ACT_TANH: hipLaunchKernelGGL((act_fwd_vec_kernel<T, HFTA_ACT_TANH>), g, b, 0, st, x, y, nvec, slope); break;
    case HFTA_ACT_GELU: hipLaunchKernelGGL((act_fwd_vec_kernel<T, HFTA_ACT_GELU>), g, b, 0, st, x, y, nvec, slope); break;
    default: hipLaunchKernelGGL((act_fwd_vec_kernel<T, HFTA_ACT_NONE>), g, b, 0, st, x, y, nvec, slope); break;
  }
}
template <typename T, bool FROM_OUT>
static void launch_act_bwd_vec(const void* Z, const void* dY, void* dX, int64_t nvec, int act, float slope, hipStream_t st) {
  const dim3 g(stream_blocks(nvec)), b(256);
  const uint4* z = (const uint4*)Z; const uint4* dy = (const uint4*)dY; uint4* dx = (uint4*)dX;
  switch (act) {
    case HFTA_ACT_RELU: hipLaunchKernelGGL((act_bwd_vec_kernel<T, HFTA_ACT_RELU, FROM_OUT>), g, b, 0, st, z, dy, dx, nvec, slope); break;
    case HFTA_ACT_LEAKY: hipLaunchKernelGGL((act_bwd_vec_kernel<T, HFTA_ACT_LEAKY, FROM_OUT>), g, b, 0, st, z, dy, dx, nvec, slope); break;
    case HFTA_ACT_TANH: hipLaunchKernelGGL((act_bwd_vec_kernel<T, HFTA_ACT_TANH, FROM_OUT>), g, b, 0, st, z, dy, dx, nvec, slope); break;
    case HFTA_ACT_GELU: hipLaunchKernelGGL((act_bwd_vec_kernel<T, HFTA_ACT_GELU, FROM_OUT>), g, b, 0, st, z, dy, dx, nvec, slope); break;
    default: hipLaunchKernelGGL((act_bwd_vec_kernel<T, HFTA_ACT_NONE, FROM_OUT>), g, b, 0, st, z, dy, dx, nvec, slope); break;
  }
}

// Wide form of the pointwise losses; false when the layout does not allow it.
template <int KIND>
static bool launch_pointwise_wide(int B, int64_t R, int dtype, const void* pred, const void* target, float* loss,
                                  void* dpred, int64_t sb, int64_t sr, hipStream_t st) {
  const int per = dtype == HFTA_BF16 ? 8 : 4;
  if (sr != 1 || sb != R || R < POINTWISE_WIDE_MIN_R || R % per != 0 || !al16(pred) || !al16(target) || !al16(dpred) ||
      dpred == pred || dpred == target || B > 65535)
    return false;
  const int64_t vpr = R / per, nvec = vpr * B;
  const float invR = 1.f / (float)R;
  const uint4* p4 = (const uint4*)pred; const uint4* t4 = (const uint4*)target; uint4* d4 = (uint4*)dpred;
  // loss first (its partial sums pass through dpred), then the gradient over the whole of dpred
  const dim3 pg(POINTWISE_CHUNKS, (unsigned)B);
  if (dtype == HFTA_BF16)
    hipLaunchKernelGGL((pointwise_loss_part_kernel<bf16_raw, KIND>), pg, dim3(1024), 0, st, p4, t4, d4, vpr);
  else
    hipLaunchKernelGGL((pointwise_loss_part_kernel<float, KIND>), pg, dim3(1024), 0, st, p4, t4, d4, vpr);
  hipLaunchKernelGGL(pointwise_loss_final_kernel, dim3((unsigned)B), dim3(64), 0, st, (const uint4*)d4, loss, vpr, invR);
  if (dtype == HFTA_BF16)
    hipLaunchKernelGGL((pointwise_grad_vec_kernel<bf16_raw, KIND>), dim3(stream_blocks(nvec)), dim3(256), 0, st, p4, t4, d4, nvec, invR);
  else
    hipLaunchKernelGGL((pointwise_grad_vec_kernel<float, KIND>), dim3(stream_blocks(nvec)), dim3(256), 0, st, p4, t4, d4, nvec, invR);
  return true;
}

}  // namespace

extern "C" {

const char* hfta_status_string(int status) {
  switch (status) {
    case HFTA_OK: return "ok";
    case HFTA_EINVAL: return "invalid argument";
    case HFTA_EUNSUPPORTED: return "unsupported dtype / stride / size combination";
    case HFTA_EWORKSPACE: return "workspace missing or too small";
    case HFTA_ELAUNCH: return "HIP launch error";
    default: return "unknown status";
  }
}

int hfta_version(void) { return 100; }

int hfta_act_fwd(int64_t count, int dtype, const void* X, void* Y, int act, float slope, void* stream) {
  if (count <= 0 || !valid_dtype(dtype) || !X || !Y || !valid_act(act)) return HFTA_EINVAL;
  hipStream_t st = as_stream(stream);
  const int64_t epv = 16 / (int64_t)dtype_size(dtype);
  const int64_t nvec = (al16(X) && al16(Y)) ? count / epv : 0, done = nvec * epv;
  if (nvec > 0) {
    if (dtype == HFTA_BF16) launch_act_fwd_vec<bf16_raw>(X, Y, nvec, act, slope, st);
    else launch_act_fwd_vec<float>(X, Y, nvec, act, slope, st);
  }
  if (done < count) {
    const int64_t n = count - done;
    if (dtype == HFTA_BF16)
      hipLaunchKernelGGL(act_fwd_kernel<bf16_raw>, dim3(stream_blocks(n)), dim3(256), 0, st,
                         (const bf16_raw*)X + done, (bf16_raw*)Y + done, n, act, slope);
    else
      hipLaunchKernelGGL(act_fwd_kernel<float>, dim3(stream_blocks(n)), dim3(256), 0, st,
                         (const float*)X + done, (float*)Y + done, n, act, slope);
  }
  return launch_status();
}

int hfta_act_bwd(int64_t count, int dtype, const void* Z, const void* dY, void* dX, int act, float slope,
                 int from_output, void* stream) {
  if (count <= 0 || !valid_dtype(dtype) || !Z || !dY || !dX || !valid_act(act)) return HFTA_EINVAL;
  if (from_output && (act == HFTA_ACT_GELU || (act == HFTA_ACT_LEAKY && !(slope > 0.f)))) return HFTA_EUNSUPPORTED;
  hipStream_t st = as_stream(stream);
  const int64_t epv = 16 / (int64_t)dtype_size(dtype);
  const int64_t nvec = (al16(Z) && al16(dY) && al16(dX)) ? count / epv : 0, done = nvec * epv;
  if (nvec > 0) {
    if (dtype == HFTA_BF16) {
      if (from_output) launch_act_bwd_vec<bf16_raw, true>(Z, dY, dX, nvec, act, slope, st);
      else launch_act_bwd_vec<bf16_raw, false>(Z, dY, dX, nvec, act, slope, st);
    } else {
      if (from_output) launch_act_bwd_vec<float, true>(Z, dY, dX, nvec, act, slope, st);
      else launch_act_bwd_vec<float, false>(Z, dY, dX, nvec, act, slope, st);
    }
  }
  if (done < count) {
    const int64_t n = count - done;
    if (dtype == HFTA_BF16)
      hipLaunchKernelGGL(act_bwd_kernel<bf16_raw>, dim3(stream_blocks(n)), dim3(256), 0, st, (const bf16_raw*)Z + done,
                         (const bf16_raw*)dY + done, (bf16_raw*)dX + done, n, act, slope, from_output);
    else
      hipLaunchKernelGGL(act_bwd_kernel<float>, dim3(stream_blocks(n)), dim3(256), 0, st, (const float*)Z + done,
                         (const float*)dY + done, (float*)dX + done, n, act, slope, from_output);
  }
  return launch_status();
}

int hfta_act_bwd_colsum(int B, int M, int F, int dtype, const void* Z, const void* dY, void* dX, float* dbias, int act,
                        float slope, void* stream) {
  if (B <= 0 || M <= 0 || F <= 0 || !valid_dtype(dtype) || !Z || !dY || !dX || !dbias || !valid_act(act)) return HFTA_EINVAL;
  const int epv = 16 / (int)dtype_size(dtype);
  if (F % epv != 0 || !al16(Z) || !al16(dY) || !al16(dX) || B > 65535) return HFTA_EUNSUPPORTED;
  hipStream_t st = as_stream(stream);
  const dim3 g((unsigned)((F / epv + 15) / 16), (unsigned)B), blk(1024);
  const uint4* z = (const uint4*)Z; const uint4* dy = (const uint4*)dY; uint4* dx = (uint4*)dX;
  if ((int64_t)g.x * g.y < 128) {      // too few workgroups for the element-wise traffic: two launches
    const int64_t nvec = (int64_t)B * M * (F / epv);
    if (dtype == HFTA_BF16) {
      launch_act_bwd_vec<bf16_raw, false>(Z, dY, dX, nvec, act, slope, st);
      hipLaunchKernelGGL((act_bwd_colsum_kernel<bf16_raw, HFTA_ACT_NONE, true>), g, blk, 0, st, z, dy, dx, dbias, M, F, slope);
    } else {
      launch_act_bwd_vec<float, false>(Z, dY, dX, nvec, act, slope, st);
      hipLaunchKernelGGL((act_bwd_colsum_kernel<float, HFTA_ACT_NONE, true>), g, blk, 0, st, z, dy, dx, dbias, M, F, slope);
    }
    return launch_status();
  }
#define HFTA_ABC(T, A) hipLaunchKernelGGL((act_bwd_colsum_kernel<T, A>), g, blk, 0, st, z, dy, dx, dbias, M, F, slope)
#define HFTA_ABC_T(T) \
  switch (act) { \
    case HFTA_ACT_RELU: HFTA_ABC(T, HFTA_ACT_RELU); break; \
    case HFTA_ACT_LEAKY: HFTA_ABC(T, HFTA_ACT_LEAKY); break; \
    case HFTA_ACT_TANH: HFTA_ABC(T, HFTA_ACT_TANH); break; \
    case HFTA_ACT_GELU: HFTA_ABC(T, HFTA_ACT_GELU); break; \
    default: HFTA_ABC(T, HFTA_ACT_NONE); break; \
  }
  if (dtype == HFTA_BF16) { HFTA_ABC_T(bf16_raw) } else { HFTA_ABC_T(float) }
#undef HFTA_ABC_T
#undef HFTA_ABC
  return launch_status();
}

int hfta_add(int64_t count, int dtype, const void* A, const void* Bv, void* Y, void* stream) {
  if (count <= 0 || !valid_dtype(dtype) || !A || !Bv || !Y) return HFTA_EINVAL;
  hipStream_t st = as_stream(stream);
  const int64_t epv = 16 / (int64_t)dtype_size(dtype);
  const int64_t nvec = (al16(A) && al16(Bv) && al16(Y)) ? count / epv : 0, done = nvec * epv;
  if (nvec > 0) {
    if (dtype == HFTA_BF16)
      hipLaunchKernelGGL(add_vec_kernel<bf16_raw>, dim3(stream_blocks(nvec)), dim3(256), 0, st, (const uint4*)A,
                         (const uint4*)Bv, (uint4*)Y, nvec);
    else
      hipLaunchKernelGGL(add_vec_kernel<float>, dim3(stream_blocks(nvec)), dim3(256), 0, st, (const uint4*)A,
                         (const uint4*)Bv, (uint4*)Y, nvec);
  }
  if (done < count) {
    const int64_t n = count - done;
    if (dtype == HFTA_BF16)
      hipLaunchKernelGGL(add_kernel<bf16_raw>, dim3(stream_blocks(n)), dim3(256), 0, st, (const bf16_raw*)A + done,
                         (const bf16_raw*)Bv + done, (bf16_raw*)Y + done, n);
    else
      hipLaunchKernelGGL(add_kernel<float>, dim3(stream_blocks(n)), dim3(256), 0, st, (const float*)A + done,
                         (const float*)Bv + done, (float*)Y + done, n);
  }
  return launch_status();
}

int hfta_bias_act_nchw(int64_t Nb, int64_t K, int64_t HW, int dtype, void* Y, const void* bias, int act, float slope,
                       void* stream) {
  if (Nb <= 0 || K <= 0 || HW <= 0 || !valid_dtype(dtype) || !Y || !valid_act(act)) return HFTA_EINVAL;
  const int64_t total = Nb * K * HW;
  if (dtype == HFTA_BF16)
    hipLaunchKernelGGL(bias_act_nchw_kernel<bf16_raw>, dim3(stream_blocks(total)), dim3(256), 0, as_stream(stream),
                       (bf16_raw*)Y, (const bf16_raw*)bias, K, HW, total, act, slope);
  else
    hipLaunchKernelGGL(bias_act_nchw_kernel<float>, dim3(stream_blocks(total)), dim3(256), 0, as_stream(stream),
                       (float*)Y, (const float*)bias, K, HW, total, act, slope);
  return launch_status();
}

int hfta_dropout(int64_t count, int dtype, const void* X, const uint8_t* mask, float p, void* Y, void* stream) {
  if (count <= 0 || !valid_dtype(dtype) || !X || !mask || !Y || !(p >= 0.f) || !(p < 1.f)) return HFTA_EINVAL;
  const float scale = 1.f / (1.f - p);
  if (dtype == HFTA_BF16)
    hipLaunchKernelGGL(dropout_kernel<bf16_raw>, dim3(stream_blocks(count)), dim3(256), 0, as_stream(stream),
                       (const bf16_raw*)X, mask, (bf16_raw*)Y, count, scale);
  else
    hipLaunchKernelGGL(dropout_kernel<float>, dim3(stream_blocks(count)), dim3(256), 0, as_stream(stream),
                       (const float*)X, mask, (float*)Y, count, scale);
  return launch_status();
}

int hfta_layernorm_fwd(int B, int R, int E, int dtype, const void* X, const float* w, const float* b, float eps,
                       float* save_mean, float* save_invstd, void* Y, void* stream) {
  if (B <= 0 || R <= 0 || E <= 0 || !valid_dtype(dtype) || !X || !w || !b || !save_mean || !save_invstd || !Y || !(eps >= 0.f))
    return HFTA_EINVAL;
  const int64_t rows = (int64_t)B * R;
  if ((rows + 3) / 4 > 0x7fffffffLL) return HFTA_EINVAL;
  dim3 grid((unsigned)((rows + 3) / 4));
  const int epv = 16 / (int)dtype_size(dtype);
  if (al16(X) && al16(Y) && E % epv == 0 && E / epv <= 128) {      // rows fit one or two 16-byte pieces per lane
    hipStream_t st = as_stream(stream);
    const bool one = E / epv <= 64;
    if (dtype == HFTA_BF16) {
      if (one) hipLaunchKernelGGL((layernorm_fwd_vec_kernel<bf16_raw, 1>), grid, dim3(256), 0, st, (const uint4*)X, w, b, eps, save_mean, save_invstd, (uint4*)Y, R, E, rows);
      else hipLaunchKernelGGL((layernorm_fwd_vec_kernel<bf16_raw, 2>), grid, dim3(256), 0, st, (const uint4*)X, w, b, eps, save_mean, save_invstd, (uint4*)Y, R, E, rows);
    } else {
      if (one) hipLaunchKernelGGL((layernorm_fwd_vec_kernel<float, 1>), grid, dim3(256), 0, st, (const uint4*)X, w, b, eps, save_mean, save_invstd, (uint4*)Y, R, E, rows);
      else hipLaunchKernelGGL((layernorm_fwd_vec_kernel<float, 2>), grid, dim3(256), 0, st, (const uint4*)X, w, b, eps, save_mean, save_invstd, (uint4*)Y, R, E, rows);
    }
    return launch_status();
  }
  if (dtype == HFTA_BF16)
    hipLaunchKernelGGL(layernorm_fwd_kernel<bf16_raw>, grid, dim3(256), 0, as_stream(stream), (const bf16_raw*)X, w, b, eps,
                       save_mean, save_invstd, (bf16_raw*)Y, R, E, rows);
  else
    hipLaunchKernelGGL(layernorm_fwd_kernel<float>, grid, dim3(256), 0, as_stream(stream), (const float*)X, w, b, eps,
                       save_mean, save_invstd, (float*)Y, R, E, rows);
  return launch_status();
}

static int ln_blocks(int R) {
  int nb = (R + 63) / 64;
  return nb > 256 ? 256 : nb;
}

size_t hfta_layernorm_bwd_workspace_bytes(int B, int R, int E) {
  if (B <= 0 || R <= 0 || E <= 0) return 0;
  return (size_t)B * ln_blocks(R) * 2 * (size_t)E * sizeof(float);
}

int hfta_layernorm_bwd(int B, int R, int E, int dtype, const void* X, const void* dY, const float* w,
                       const float* save_mean, const float* save_invstd, void* dX, float* dw, float* db,
                       void* workspace, size_t ws_bytes, void* stream) {
  if (B <= 0 || R <= 0 || E <= 0 || !valid_dtype(dtype) || !X || !dY || !w || !save_mean || !save_invstd || !dX || !dw || !db)
    return HFTA_EINVAL;
  if (B > 65535) return HFTA_EUNSUPPORTED;
  if (!workspace || ws_bytes < hfta_layernorm_bwd_workspace_bytes(B, R, E)) return HFTA_EWORKSPACE;
  const int nblk = ln_blocks(R);
  const int rpb = (R + nblk - 1) / nblk;
  hipStream_t st = as_stream(stream);
  dim3 grid((unsigned)nblk, (unsigned)B);
  const int epv = 16 / (int)dtype_size(dtype);
  if (al16(X) && al16(dY) && al16(dX) && E % epv == 0 && E / epv <= 128) {
    const bool one = E / epv <= 64;
    float* part = (float*)workspace;
    if (dtype == HFTA_BF16) {
      if (one) hipLaunchKernelGGL((layernorm_bwd_vec_kernel<bf16_raw, 1>), grid, dim3(256), 0, st, (const uint4*)X, (const uint4*)dY, w, save_mean, save_invstd, (uint4*)dX, part, R, E, rpb);
      else hipLaunchKernelGGL((layernorm_bwd_vec_kernel<bf16_raw, 2>), grid, dim3(256), 0, st, (const uint4*)X, (const uint4*)dY, w, save_mean, save_invstd, (uint4*)dX, part, R, E, rpb);
    } else {
      if (one) hipLaunchKernelGGL((layernorm_bwd_vec_kernel<float, 1>), grid, dim3(256), 0, st, (const uint4*)X, (const uint4*)dY, w, save_mean, save_invstd, (uint4*)dX, part, R, E, rpb);
      else hipLaunchKernelGGL((layernorm_bwd_vec_kernel<float, 2>), grid, dim3(256), 0, st, (const uint4*)X, (const uint4*)dY, w, save_mean, save_invstd, (uint4*)dX, part, R, E, rpb);
    }
  } else if (dtype == HFTA_BF16)
    hipLaunchKernelGGL(layernorm_bwd_kernel<bf16_raw>, grid, dim3(256), 0, st, (const bf16_raw*)X, (const bf16_raw*)dY, w,
                       save_mean, save_invstd, (bf16_raw*)dX, (float*)workspace, R, E, rpb);
  else
    hipLaunchKernelGGL(layernorm_bwd_kernel<float>, grid, dim3(256), 0, st, (const float*)X, (const float*)dY, w, save_mean,
                       save_invstd, (float*)dX, (float*)workspace, R, E, rpb);
  if (launch_status() != HFTA_OK) return HFTA_ELAUNCH;
  hipLaunchKernelGGL(layernorm_bwd_reduce_kernel, dim3((unsigned)((E + 255) / 256), (unsigned)B), dim3(256), 0, st,
                     (const float*)workspace, dw, db, (float*)nullptr, E, nblk, 2);
  return launch_status();
}

size_t hfta_layernorm_bwd_sums_workspace_bytes(int B, int R, int E) {
  if (B <= 0 || R <= 0 || E <= 0) return 0;
  return (size_t)B * ln_blocks(R) * 3 * (size_t)E * sizeof(float);
}

int hfta_layernorm_bwd_sums(int B, int R, int E, int dtype, const void* X, const void* dY, const void* dY2, const float* w,
                            const float* save_mean, const float* save_invstd, void* dX, float* dw, float* db,
                            float* dx_colsum, void* workspace, size_t ws_bytes, void* stream) {
  if (B <= 0 || R <= 0 || E <= 0 || !valid_dtype(dtype) || !X || !dY || !w || !save_mean || !save_invstd || !dX || !dw ||
      !db || !dx_colsum)
    return HFTA_EINVAL;
  if (B > 65535) return HFTA_EUNSUPPORTED;
  if (!workspace || ws_bytes < hfta_layernorm_bwd_sums_workspace_bytes(B, R, E)) return HFTA_EWORKSPACE;
  const int epv = 16 / (int)dtype_size(dtype);
  if (!(al16(X) && al16(dY) && al16(dX) && (!dY2 || al16(dY2)) && E % epv == 0 && E / epv <= 128)) return HFTA_EUNSUPPORTED;
  const int nblk = ln_blocks(R);
  const int rpb = (R + nblk - 1) / nblk;
  hipStream_t st = as_stream(stream);
  dim3 grid((unsigned)nblk, (unsigned)B);
  const bool one = E / epv <= 64;
  float* part = (float*)workspace;
#define HFTA_LNS(T, CHN) hipLaunchKernelGGL((layernorm_bwd_vec_kernel<T, CHN, true>), grid, dim3(256), 0, st, (const uint4*)X, \
    (const uint4*)dY, w, save_mean, save_invstd, (uint4*)dX, part, R, E, rpb, (const uint4*)dY2)
  if (dtype == HFTA_BF16) { if (one) HFTA_LNS(bf16_raw, 1); else HFTA_LNS(bf16_raw, 2); }
  else { if (one) HFTA_LNS(float, 1); else HFTA_LNS(float, 2); }
#undef HFTA_LNS
  if (launch_status() != HFTA_OK) return HFTA_ELAUNCH;
  hipLaunchKernelGGL(layernorm_bwd_reduce_kernel, dim3((unsigned)((E + 255) / 256), (unsigned)B), dim3(256), 0, st,
                     (const float*)workspace, dw, db, dx_colsum, E, nblk, 3);
  return launch_status();
}

int hfta_softmax_xent(int B, int R, int K, int dtype, const void* logits, const int32_t* labels, float* loss,
                      void* dlogits, void* stream) {
  if (B <= 0 || R <= 0 || K <= 0 || !valid_dtype(dtype) || !logits || !labels || !loss || !dlogits) return HFTA_EINVAL;
  const int threads = R >= 1024 ? 1024 : ((R + 63) / 64) * 64;
  if (dtype == HFTA_BF16)
    hipLaunchKernelGGL(softmax_xent_kernel<bf16_raw>, dim3((unsigned)B), dim3(threads), 0, as_stream(stream),
                       (const bf16_raw*)logits, labels, loss, (bf16_raw*)dlogits, R, K);
  else
    hipLaunchKernelGGL(softmax_xent_kernel<float>, dim3((unsigned)B), dim3(threads), 0, as_stream(stream),
                       (const float*)logits, labels, loss, (float*)dlogits, R, K);
  return launch_status();
}

int hfta_bce_logits_strided(int B, int64_t R, int dtype, const void* logits, const void* targets, float* loss,
                            void* dlogits, int64_t stride_b, int64_t stride_r, void* stream) {
  if (B <= 0 || R <= 0 || !valid_dtype(dtype) || !logits || !targets || !loss || !dlogits) return HFTA_EINVAL;
  if (stride_b <= 0 || stride_r <= 0) return HFTA_EINVAL;
  if (launch_pointwise_wide<0>(B, R, dtype, logits, targets, loss, dlogits, stride_b, stride_r, as_stream(stream)))
    return launch_status();
  if (dtype == HFTA_BF16)
    hipLaunchKernelGGL((pointwise_loss_kernel<bf16_raw, 0>), dim3((unsigned)B), dim3(1024), 0, as_stream(stream),
                       (const bf16_raw*)logits, (const bf16_raw*)targets, loss, (bf16_raw*)dlogits, R, stride_b, stride_r);
  else
    hipLaunchKernelGGL((pointwise_loss_kernel<float, 0>), dim3((unsigned)B), dim3(1024), 0, as_stream(stream),
                       (const float*)logits, (const float*)targets, loss, (float*)dlogits, R, stride_b, stride_r);
  return launch_status();
}

int hfta_bce_logits(int B, int64_t R, int dtype, const void* logits, const void* targets, float* loss, void* dlogits,
                    void* stream) {
  return hfta_bce_logits_strided(B, R, dtype, logits, targets, loss, dlogits, R, 1, stream);
}

int hfta_mse(int B, int64_t R, int dtype, const void* pred, const void* target, float* loss, void* dpred, void* stream) {
  if (B <= 0 || R <= 0 || !valid_dtype(dtype) || !pred || !target || !loss || !dpred) return HFTA_EINVAL;
  if (launch_pointwise_wide<1>(B, R, dtype, pred, target, loss, dpred, R, 1, as_stream(stream))) return launch_status();
  if (dtype == HFTA_BF16)
    hipLaunchKernelGGL((pointwise_loss_kernel<bf16_raw, 1>), dim3((unsigned)B), dim3(1024), 0, as_stream(stream),
                       (const bf16_raw*)pred, (const bf16_raw*)target, loss, (bf16_raw*)dpred, R, R, (int64_t)1);
  else
    hipLaunchKernelGGL((pointwise_loss_kernel<float, 1>), dim3((unsigned)B), dim3(1024), 0, as_stream(stream),
                       (const float*)pred, (const float*)target, loss, (float*)dpred, R, R, (int64_t)1);
  return launch_status();
}

}  // extern "C"
