// Fused BatchNorm (training mode) over the channels of all B models.
//
// Conv-family layout (stride_l == 1): one workgroup per channel (b, c).  It
// streams the channel's Nb rows of L contiguous elements twice -- once for the
// statistics, once to normalise -- and the second pass of a channel follows its
// first immediately, so the re-read is served by L2 / Infinity Cache rather
// than HBM for all but the largest channels.  Statistics use sums shifted by
// the channel's first element, which keeps fp32 accurate when |mean| >> std.
// Reductions: per-lane partials -> wave64 shuffle reduction -> 4-entry LDS.
//
// Linear layout (L == 1, stride_c == 1, the table's [N, B, C] case): one thread
// per channel, coalesced across channels, two passes over the Nb samples.
#include <stdlib.h>
#include "bn_common.h"

using namespace hfta;

namespace {

constexpr int BN_UNROLL = 4;   // pieces a thread loads before it uses the first (conv layout)

struct BnFwdArgs {
  const void* X; void* Y;
  const float* gamma; const float* beta;
  float* running_mean; float* running_var; float* save_mean; float* save_invstd;
  int64_t xsb, xsn, xsc, ysb, ysn, ysc;
  int Nb, C, L, act;
  float eps, momentum, slope;
};

template <typename T, int VEC, int NT>
__global__ __launch_bounds__(NT) void bn_fwd_conv_kernel(BnFwdArgs p) {
  __shared__ float sh[NT / 64][2];
  const int c = blockIdx.x, b = blockIdx.y;
  const T* x = reinterpret_cast<const T*>(p.X) + b * p.xsb + c * p.xsc;
  T* y = reinterpret_cast<T*>(p.Y) + b * p.ysb + c * p.ysc;
  const int chunks = p.L / VEC;
  const float shift = Elem<T>::load(x);
  float s1 = 0.f, s2 = 0.f;
  for (RowWalk w(chunks, NT); w.n < p.Nb;) {
    // BN_UNROLL pieces per trip, their loads issued together (a piece past the end re-reads the
    // channel's first piece and is not used): the bytes in flight per thread set the bandwidth
    float v[BN_UNROLL][VEC];
    bool ok[BN_UNROLL];
#pragma unroll
    for (int u = 0; u < BN_UNROLL; ++u) {
      ok[u] = w.n < p.Nb;
      load_vec<T, VEC>(ok[u] ? x + w.n * p.xsn + w.ch * VEC : x, v[u]);
      w.step();
    }
#pragma unroll
    for (int u = 0; u < BN_UNROLL; ++u)
      if (ok[u]) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) { const float d = v[u][e] - shift; s1 += d; s2 = fmaf(d, d, s2); }
      }
  }
  block_sum2<NT / 64>(s1, s2, sh);
  const float m = (float)p.Nb * (float)p.L;
  const float dm = s1 / m;
  const float mean = shift + dm;
  float var = s2 / m - dm * dm;
  var = var < 0.f ? 0.f : var;
  const float invstd = 1.0f / sqrtf(var + p.eps);
  const int k = b * p.C + c;
  const float g = p.gamma[k], bt = p.beta[k];
  if (threadIdx.x == 0) {
    p.save_mean[k] = mean;
    p.save_invstd[k] = invstd;
    if (p.running_mean) {
      const float unb = m > 1.f ? var * (m / (m - 1.f)) : var;
      p.running_mean[k] = (1.f - p.momentum) * p.running_mean[k] + p.momentum * mean;
      p.running_var[k] = (1.f - p.momentum) * p.running_var[k] + p.momentum * unb;
    }
  }
  if (!p.Y) return;                      // statistics only: a consumer normalises on load
  for (RowWalk w(chunks, NT); w.n < p.Nb;) {
    float v[BN_UNROLL][VEC];
    int n[BN_UNROLL], ch[BN_UNROLL];
#pragma unroll
    for (int u = 0; u < BN_UNROLL; ++u) {
      n[u] = w.n; ch[u] = w.ch;
      load_vec<T, VEC>(n[u] < p.Nb ? x + n[u] * p.xsn + ch[u] * VEC : x, v[u]);
      w.step();
    }
#pragma unroll
    for (int u = 0; u < BN_UNROLL; ++u)
      if (n[u] < p.Nb) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[u][e] = apply_act(fmaf(g, (v[u][e] - mean) * invstd, bt), p.act, p.slope);
        store_vec<T, VEC>(y + n[u] * p.ysn + ch[u] * VEC, v[u]);
      }
  }
}



// Normalisation with given statistics (the forward kernel's second pass alone): what a consumer that
// normalises on load computes, written out.
template <typename T, int VEC, int NT>
__global__ __launch_bounds__(NT) void bn_apply_conv_kernel(BnFwdArgs p) {
  const int c = blockIdx.x, b = blockIdx.y, k = b * p.C + c;
  const T* x = reinterpret_cast<const T*>(p.X) + b * p.xsb + c * p.xsc;
  T* y = reinterpret_cast<T*>(p.Y) + b * p.ysb + c * p.ysc;
  const int chunks = p.L / VEC;
  const float mean = p.save_mean[k], invstd = p.save_invstd[k], g = p.gamma[k], bt = p.beta[k];
  for (RowWalk w(chunks, NT); w.n < p.Nb;) {
    float v[BN_UNROLL][VEC];
    int n[BN_UNROLL], ch[BN_UNROLL];
#pragma unroll
    for (int u = 0; u < BN_UNROLL; ++u) {
      n[u] = w.n; ch[u] = w.ch;
      load_vec<T, VEC>(n[u] < p.Nb ? x + n[u] * p.xsn + ch[u] * VEC : x, v[u]);
      w.step();
    }
#pragma unroll
    for (int u = 0; u < BN_UNROLL; ++u)
      if (n[u] < p.Nb) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[u][e] = apply_act(fmaf(g, (v[u][e] - mean) * invstd, bt), p.act, p.slope);
        store_vec<T, VEC>(y + n[u] * p.ysn + ch[u] * VEC, v[u]);
      }
  }
}

// Training statistics from partial sums that the producing convolution left behind (sums of (x - shift) and
// (x - shift)^2 per slice, shift = the channel's conv bias or 0), so that the tensor is read once, for the
// normalisation (bn_apply_conv_kernel), or not at all (a consumer normalises on load).  The partials lie
// [part][channel], so a workgroup takes 16 neighbouring channels -- 16 lanes read 128 contiguous bytes of one
// part, 64 such rows are in flight per step -- instead of one channel whose parts are a channel count apart.
// Per-lane sums in a fixed order, then a fixed-order tree over the 64 part lanes.
constexpr int BNS_C = 16, BNS_P = 64;
__global__ __launch_bounds__(BNS_C * BNS_P) void bn_stats_part_kernel(BnFwdArgs p, const float* __restrict__ part, int parts,
                                                                      const bf16_raw* __restrict__ shift_v) {
  __shared__ float2 red[BNS_P][BNS_C];
  const int cl = threadIdx.x & (BNS_C - 1), pl = threadIdx.x / BNS_C;
  const int c = blockIdx.x * BNS_C + cl, b = blockIdx.y;
  const bool live = c < p.C;
  const float2* pp = reinterpret_cast<const float2*>(part) + (int64_t)b * parts * p.C + (live ? c : 0);
  float s1 = 0.f, s2 = 0.f;
#pragma unroll 4
  for (int i = pl; i < parts; i += BNS_P) {
    const float2 v = pp[(int64_t)i * p.C];
    s1 += v.x; s2 += v.y;
  }
  red[pl][cl] = make_float2(s1, s2);
  __syncthreads();
  for (int h = BNS_P / 2; h > 0; h >>= 1) {
    if (pl < h) {
      const float2 a = red[pl][cl], o = red[pl + h][cl];
      red[pl][cl] = make_float2(a.x + o.x, a.y + o.y);
    }
    __syncthreads();
  }
  if (pl != 0 || !live) return;
  const int k = b * p.C + c;
  const float shift = shift_v ? bf16_to_f32(shift_v[k]) : 0.f;
  const float m = (float)p.Nb * (float)p.L;
  const float dm = red[0][cl].x / m;
  const float mean = shift + dm;
  float var = red[0][cl].y / m - dm * dm;
  var = var < 0.f ? 0.f : var;
  p.save_mean[k] = mean;
  p.save_invstd[k] = 1.0f / sqrtf(var + p.eps);
  if (p.running_mean) {
    const float unb = m > 1.f ? var * (m / (m - 1.f)) : var;
    p.running_mean[k] = (1.f - p.momentum) * p.running_mean[k] + p.momentum * mean;
    p.running_var[k] = (1.f - p.momentum) * p.running_var[k] + p.momentum * unb;
  }
}

// Linear layout [.., Nb, C] (channel stride 1, the fully connected head): a workgroup owns 64
// channels x 16 sample lanes, so the loads of a column are spread over lanes instead of walking one
// after the other through the memory latency; per-lane partial sums meet in LDS in a fixed order.
constexpr int BNL_C = 64, BNL_N = 16;

__device__ __forceinline__ float bnl_reduce(float v, float (*red)[BNL_C], int tx, int ty) {
  __syncthreads();                       // the previous reduction's readers are done
  red[ty][tx] = v;
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < BNL_N; ++j) s += red[j][tx];
  return s;
}

template <typename T>
__global__ __launch_bounds__(BNL_C * BNL_N) void bn_fwd_linear_kernel(BnFwdArgs p) {
  __shared__ float red[BNL_N][BNL_C];
  const int tx = threadIdx.x % BNL_C, ty = threadIdx.x / BNL_C;
  const int c = blockIdx.x * BNL_C + tx, b = blockIdx.y;
  const bool live = c < p.C;
  const int cc = live ? c : p.C - 1;
  const T* x = reinterpret_cast<const T*>(p.X) + b * p.xsb + cc;
  T* y = reinterpret_cast<T*>(p.Y) + b * p.ysb + cc;
  float s = 0.f;
  for (int n = ty; n < p.Nb; n += BNL_N) s += Elem<T>::load(x + n * p.xsn);
  const float m = (float)p.Nb;
  const float mean = bnl_reduce(s, red, tx, ty) / m;
  float q = 0.f;
  for (int n = ty; n < p.Nb; n += BNL_N) { const float d = Elem<T>::load(x + n * p.xsn) - mean; q = fmaf(d, d, q); }
  const float var = bnl_reduce(q, red, tx, ty) / m;
  const float invstd = 1.0f / sqrtf(var + p.eps);
  const int k = b * p.C + cc;
  const float g = p.gamma[k], bt = p.beta[k];
  if (live && ty == 0) {
    p.save_mean[k] = mean;
    p.save_invstd[k] = invstd;
    if (p.running_mean) {
      const float unb = m > 1.f ? var * (m / (m - 1.f)) : var;
      p.running_mean[k] = (1.f - p.momentum) * p.running_mean[k] + p.momentum * mean;
      p.running_var[k] = (1.f - p.momentum) * p.running_var[k] + p.momentum * unb;
    }
  }
  if (!live) return;
  for (int n = ty; n < p.Nb; n += BNL_N) {
    const float v = Elem<T>::load(x + n * p.xsn);
    Elem<T>::store(y + n * p.ysn, apply_act(fmaf(g, (v - mean) * invstd, bt), p.act, p.slope));
  }
}

struct BnBwdArgs {
  const void* X; const void* dY; void* dX;
  const float* gamma; const float* beta; const float* save_mean; const float* save_invstd;
  float* dgamma; float* dbeta; float* dx_sum;
  int64_t xsb, xsn, xsc, dysb, dysn, dysc, dxsb, dxsn, dxsc;
  int Nb, C, L, act;
  float slope;
};

template <typename T, int VEC, int NT>
__global__ __launch_bounds__(NT) void bn_bwd_conv_kernel(BnBwdArgs p) {
  __shared__ float sh[NT / 64][2];
  const int c = blockIdx.x, b = blockIdx.y, k = b * p.C + c;
  const T* x = reinterpret_cast<const T*>(p.X) + b * p.xsb + c * p.xsc;
  const T* dy = reinterpret_cast<const T*>(p.dY) + b * p.dysb + c * p.dysc;
  T* dx = reinterpret_cast<T*>(p.dX) + b * p.dxsb + c * p.dxsc;
  const float mean = p.save_mean[k], invstd = p.save_invstd[k], g = p.gamma[k], bt = p.beta[k];
  const int chunks = p.L / VEC;
  float s1 = 0.f, s2 = 0.f;
  for (RowWalk w(chunks, NT); w.n < p.Nb;) {
    float v[BN_UNROLL][VEC], d[BN_UNROLL][VEC];
    bool ok[BN_UNROLL];
#pragma unroll
    for (int u = 0; u < BN_UNROLL; ++u) {
      ok[u] = w.n < p.Nb;
      load_vec<T, VEC>(ok[u] ? x + w.n * p.xsn + w.ch * VEC : x, v[u]);
      load_vec<T, VEC>(ok[u] ? dy + w.n * p.dysn + w.ch * VEC : dy, d[u]);
      w.step();
    }
#pragma unroll
    for (int u = 0; u < BN_UNROLL; ++u)
      if (ok[u]) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const float xh = (v[u][e] - mean) * invstd;
          const float gr = d[u][e] * act_grad(fmaf(g, xh, bt), p.act, p.slope);
          s1 += gr;
          s2 = fmaf(gr, xh, s2);
        }
      }
  }
  block_sum2<NT / 64>(s1, s2, sh);
  if (threadIdx.x == 0) { p.dbeta[k] = s1; p.dgamma[k] = s2; }
  const float m = (float)p.Nb * (float)p.L;
  const float mb = s1 / m, mg = s2 / m, sc = g * invstd;
  float s3 = 0.f;
  for (RowWalk w(chunks, NT); w.n < p.Nb;) {
    float v[BN_UNROLL][VEC], d[BN_UNROLL][VEC];
    int n[BN_UNROLL], ch[BN_UNROLL];
#pragma unroll
    for (int u = 0; u < BN_UNROLL; ++u) {
      n[u] = w.n; ch[u] = w.ch;
      const bool ok = n[u] < p.Nb;
      load_vec<T, VEC>(ok ? x + n[u] * p.xsn + ch[u] * VEC : x, v[u]);
      load_vec<T, VEC>(ok ? dy + n[u] * p.dysn + ch[u] * VEC : dy, d[u]);
      w.step();
    }
#pragma unroll
    for (int u = 0; u < BN_UNROLL; ++u)
      if (n[u] < p.Nb) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const float xh = (v[u][e] - mean) * invstd;
          const float gr = d[u][e] * act_grad(fmaf(g, xh, bt), p.act, p.slope);
          v[u][e] = sc * (gr - mb - xh * mg);
          s3 += Elem<T>::to_f32(Elem<T>::from_f32(v[u][e]));     // the value as it is stored
        }
        store_vec<T, VEC>(dx + n[u] * p.dxsn + ch[u] * VEC, v[u]);
      }
  }
  if (p.dx_sum) {
    float dummy = 0.f;
    block_sum2<NT / 64>(s3, dummy, sh);
    if (threadIdx.x == 0) p.dx_sum[k] = s3;
  }
}

// The reduction half of the backward pass alone: dbeta, dgamma, and per channel the eight constants
// a consumer needs to form dX = sc * (g - mb - xhat * mg) by itself while it streams x and dY:
// coef[k] = {mean, invstd, gamma, beta, mb, mg, sc, 0}.  Nothing of size [Nb, C, L] is written.
template <typename T, int VEC, int NT>
__global__ __launch_bounds__(NT) void bn_bwd_conv_coef_kernel(BnBwdArgs p, float* __restrict__ coef) {
  __shared__ float sh[NT / 64][2];
  const int c = blockIdx.x, b = blockIdx.y, k = b * p.C + c;
  const T* x = reinterpret_cast<const T*>(p.X) + b * p.xsb + c * p.xsc;
  const T* dy = reinterpret_cast<const T*>(p.dY) + b * p.dysb + c * p.dysc;
  const float mean = p.save_mean[k], invstd = p.save_invstd[k], g = p.gamma[k], bt = p.beta[k];
  const int chunks = p.L / VEC;
  float s1 = 0.f, s2 = 0.f;
  for (RowWalk w(chunks, NT); w.n < p.Nb;) {
    float v[BN_UNROLL][VEC], d[BN_UNROLL][VEC];
    bool ok[BN_UNROLL];
#pragma unroll
    for (int u = 0; u < BN_UNROLL; ++u) {
      ok[u] = w.n < p.Nb;
      load_vec<T, VEC>(ok[u] ? x + w.n * p.xsn + w.ch * VEC : x, v[u]);
      load_vec<T, VEC>(ok[u] ? dy + w.n * p.dysn + w.ch * VEC : dy, d[u]);
      w.step();
    }
#pragma unroll
    for (int u = 0; u < BN_UNROLL; ++u)
      if (ok[u]) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const float xh = (v[u][e] - mean) * invstd;
          const float gr = d[u][e] * act_grad(fmaf(g, xh, bt), p.act, p.slope);
          s1 += gr;
          s2 = fmaf(gr, xh, s2);
        }
      }
  }
  block_sum2<NT / 64>(s1, s2, sh);
  if (threadIdx.x == 0) {
    p.dbeta[k] = s1;
    p.dgamma[k] = s2;
    const float m = (float)p.Nb * (float)p.L;
    float4* o = reinterpret_cast<float4*>(coef + (int64_t)k * 8);
    o[0] = make_float4(mean, invstd, g, bt);
    o[1] = make_float4(s1 / m, s2 / m, g * invstd, 0.f);
  }
}

// The same constants from the two sums handed over by the kernel that produced dY (sums[k] = {sum g, sum g xhat}).
__global__ __launch_bounds__(256) void bn_bwd_coef_sums_kernel(const float* __restrict__ sums, const float* __restrict__ gamma,
                                                               const float* __restrict__ beta, const float* __restrict__ mean,
                                                               const float* __restrict__ invstd, float* __restrict__ dgamma,
                                                               float* __restrict__ dbeta, float* __restrict__ coef, int n, float m) {
  const int k = blockIdx.x * 256 + threadIdx.x;
  if (k >= n) return;
  const float2 s = *reinterpret_cast<const float2*>(sums + (int64_t)k * 2);
  dbeta[k] = s.x;
  dgamma[k] = s.y;
  float4* o = reinterpret_cast<float4*>(coef + (int64_t)k * 8);
  o[0] = make_float4(mean[k], invstd[k], gamma[k], beta[k]);
  o[1] = make_float4(s.x / m, s.y / m, gamma[k] * invstd[k], 0.f);
}

template <typename T>
__global__ __launch_bounds__(BNL_C * BNL_N) void bn_bwd_linear_kernel(BnBwdArgs p) {
  __shared__ float red[BNL_N][BNL_C];
  const int tx = threadIdx.x % BNL_C, ty = threadIdx.x / BNL_C;
  const int c = blockIdx.x * BNL_C + tx, b = blockIdx.y;
  const bool live = c < p.C;
  const int cc = live ? c : p.C - 1;
  const int k = b * p.C + cc;
  const T* x = reinterpret_cast<const T*>(p.X) + b * p.xsb + cc;
  const T* dy = reinterpret_cast<const T*>(p.dY) + b * p.dysb + cc;
  T* dx = reinterpret_cast<T*>(p.dX) + b * p.dxsb + cc;
  const float mean = p.save_mean[k], invstd = p.save_invstd[k], g = p.gamma[k], bt = p.beta[k];
  float s1 = 0.f, s2 = 0.f;
  for (int n = ty; n < p.Nb; n += BNL_N) {
    const float xh = (Elem<T>::load(x + n * p.xsn) - mean) * invstd;
    const float gr = Elem<T>::load(dy + n * p.dysn) * act_grad(fmaf(g, xh, bt), p.act, p.slope);
    s1 += gr;
    s2 = fmaf(gr, xh, s2);
  }
  s1 = bnl_reduce(s1, red, tx, ty);
  s2 = bnl_reduce(s2, red, tx, ty);
  if (live && ty == 0) {
    p.dbeta[k] = s1;
    p.dgamma[k] = s2;
  }
  const float m = (float)p.Nb, mb = s1 / m, mg = s2 / m, sc = g * invstd;
  float s3 = 0.f;
  for (int n = ty; n < p.Nb; n += BNL_N) {
    const float xh = (Elem<T>::load(x + n * p.xsn) - mean) * invstd;
    const float gr = Elem<T>::load(dy + n * p.dysn) * act_grad(fmaf(g, xh, bt), p.act, p.slope);
    const T o = Elem<T>::from_f32(sc * (gr - mb - xh * mg));
    if (live) dx[n * p.dxsn] = o;
    s3 += Elem<T>::to_f32(o);
  }
  if (p.dx_sum) {                        // uniform over the grid
    s3 = bnl_reduce(s3, red, tx, ty);
    if (live && ty == 0) p.dx_sum[k] = s3;
  }
}

bool vec_ok(const void* p, const int64_t* s, int L, int dtype) {
  const int es = (int)dtype_size(dtype);
  const size_t bytes = 4 * es;
  return L % 4 == 0 && reinterpret_cast<uintptr_t>(p) % bytes == 0 && s[0] % 4 == 0 && s[1] % 4 == 0 && s[2] % 4 == 0;
}

// Evaluation mode: y = act(gamma (x - running_mean) / sqrt(running_var + eps) + beta), one read and one
// write; the channel's scale and shift are formed once per workgroup.
struct BnEvalArgs {
  const void* X; void* Y;
  const float* gamma; const float* beta; const float* running_mean; const float* running_var;
  int64_t xsb, xsn, xsc, ysb, ysn, ysc;
  int Nb, C, L, act;
  float eps, slope;
};

template <typename T, int VEC, int NT>
__global__ __launch_bounds__(NT) void bn_eval_conv_kernel(BnEvalArgs p) {
  const int c = blockIdx.x, b = blockIdx.y, k = b * p.C + c;
  const T* x = reinterpret_cast<const T*>(p.X) + b * p.xsb + c * p.xsc;
  T* y = reinterpret_cast<T*>(p.Y) + b * p.ysb + c * p.ysc;
  const float mean = p.running_mean[k];
  const float scale = p.gamma[k] * (1.0f / sqrtf(p.running_var[k] + p.eps)), bt = p.beta[k];
  const int chunks = p.L / VEC;
  for (RowWalk w(chunks, NT); w.n < p.Nb; w.step()) {
    float v[VEC];
    load_vec<T, VEC>(x + w.n * p.xsn + w.ch * VEC, v);
#pragma unroll
    for (int e = 0; e < VEC; ++e) v[e] = apply_act(fmaf(scale, v[e] - mean, bt), p.act, p.slope);
    store_vec<T, VEC>(y + w.n * p.ysn + w.ch * VEC, v);
  }
}

template <typename T>
__global__ __launch_bounds__(BNL_C * BNL_N) void bn_eval_linear_kernel(BnEvalArgs p) {
  const int tx = threadIdx.x % BNL_C, ty = threadIdx.x / BNL_C;
  const int c = blockIdx.x * BNL_C + tx, b = blockIdx.y;
  if (c >= p.C) return;
  const int k = b * p.C + c;
  const T* x = reinterpret_cast<const T*>(p.X) + b * p.xsb + c;
  T* y = reinterpret_cast<T*>(p.Y) + b * p.ysb + c;
  const float mean = p.running_mean[k];
  const float scale = p.gamma[k] * (1.0f / sqrtf(p.running_var[k] + p.eps)), bt = p.beta[k];
  for (int n = ty; n < p.Nb; n += BNL_N)
    Elem<T>::store(y + n * p.ysn, apply_act(fmaf(scale, Elem<T>::load(x + n * p.xsn) - mean, bt), p.act, p.slope));
}

int layout_kind(const int64_t* s, int L) {
  if (s[3] == 1) return 1;                 // conv family
  if (L == 1 && s[2] == 1) return 2;       // linear family
  return 0;
}

}  // namespace


namespace hfta {
// see bn_stats_part_kernel; conv layout only, bf16 (the producer is the streaming convolution)
int bn_fwd_from_partials(int B, int Nb, int C, int L, int dtype, const void* X, const int64_t xs[4], const float* gamma,
                         const float* beta, float eps, float momentum, float* running_mean, float* running_var,
                         float* save_mean, float* save_invstd, void* Y, const int64_t ys[4], int act, float slope,
                         const float* part, int parts, const void* shift, hipStream_t st) {
  // Y == nullptr: statistics only (mean, invstd, running statistics); nothing of size [Nb, C, L] is touched
  if (dtype != HFTA_BF16 || B > 65535 || layout_kind(xs, L) != 1 || (Y && layout_kind(ys, L) != 1)) return HFTA_EUNSUPPORTED;
  BnFwdArgs a{X, Y, gamma, beta, running_mean, running_var, save_mean, save_invstd,
              xs[0], xs[1], xs[2], Y ? ys[0] : 0, Y ? ys[1] : 0, Y ? ys[2] : 0, Nb, C, L, act, eps, momentum, slope};
  const bf16_raw* sv = (const bf16_raw*)shift;
  hipLaunchKernelGGL(bn_stats_part_kernel, dim3((unsigned)((C + BNS_C - 1) / BNS_C), (unsigned)B), dim3(BNS_C * BNS_P), 0, st, a, part,
                     parts, sv);
  const int rc = launch_status();
  if (!Y || rc != HFTA_OK) return rc;
  const dim3 grid((unsigned)C, (unsigned)B);
  const bool v4 = vec_ok(X, xs, L, dtype) && vec_ok(Y, ys, L, dtype);
  const bool big = bn_wide_block((int64_t)Nb * L * dtype_size(dtype));
  if (v4) { if (big) hipLaunchKernelGGL((bn_apply_conv_kernel<bf16_raw, 4, 1024>), grid, dim3(1024), 0, st, a);
            else hipLaunchKernelGGL((bn_apply_conv_kernel<bf16_raw, 4, 256>), grid, dim3(256), 0, st, a); }
  else { if (big) hipLaunchKernelGGL((bn_apply_conv_kernel<bf16_raw, 1, 1024>), grid, dim3(1024), 0, st, a);
         else hipLaunchKernelGGL((bn_apply_conv_kernel<bf16_raw, 1, 256>), grid, dim3(256), 0, st, a); }
  return launch_status();
}

// Training statistics of a conv-layout tensor alone (mean, invstd, running statistics): the first pass of
// the forward kernel, for a consumer that normalises on load.
int bn_stats_conv(int B, int Nb, int C, int L, int dtype, const void* X, const int64_t xs[4], const float* gamma,
                  const float* beta, float eps, float momentum, float* running_mean, float* running_var,
                  float* save_mean, float* save_invstd, hipStream_t st) {
  if (B > 65535 || layout_kind(xs, L) != 1) return HFTA_EUNSUPPORTED;
  BnFwdArgs a{X, nullptr, gamma, beta, running_mean, running_var, save_mean, save_invstd,
              xs[0], xs[1], xs[2], 0, 0, 0, Nb, C, L, HFTA_ACT_NONE, eps, momentum, 0.f};
  const dim3 grid((unsigned)C, (unsigned)B);
  const bool v4 = vec_ok(X, xs, L, dtype);
  const bool big = bn_wide_block((int64_t)Nb * L * dtype_size(dtype));
#define HFTA_BN_STATS(T, V) \
  do { if (big) hipLaunchKernelGGL((bn_fwd_conv_kernel<T, V, 1024>), grid, dim3(1024), 0, st, a); \
       else hipLaunchKernelGGL((bn_fwd_conv_kernel<T, V, 256>), grid, dim3(256), 0, st, a); } while (0)
  if (dtype == HFTA_BF16) { if (v4) HFTA_BN_STATS(bf16_raw, 4); else HFTA_BN_STATS(bf16_raw, 1); }
  else { if (v4) HFTA_BN_STATS(float, 4); else HFTA_BN_STATS(float, 1); }
#undef HFTA_BN_STATS
  return launch_status();
}

// Reduction half of the training backward pass over the [Nb, B*C, L] layout: dgamma, dbeta and the
// per-channel constants (eight floats, see the kernel) for a consumer that applies them itself.
int bn_bwd_coef(int B, int Nb, int C, int L, int dtype, const void* X, const int64_t xs[4], const void* dY,
                const int64_t dys[4], const float* gamma, const float* beta, const float* save_mean,
                const float* save_invstd, float* dgamma, float* dbeta, float* coef, int act, float slope, hipStream_t st) {
  if (B > 65535 || layout_kind(xs, L) != 1 || layout_kind(dys, L) != 1) return HFTA_EUNSUPPORTED;
  BnBwdArgs a{X, dY, nullptr, gamma, beta, save_mean, save_invstd, dgamma, dbeta, nullptr,
              xs[0], xs[1], xs[2], dys[0], dys[1], dys[2], 0, 0, 0, Nb, C, L, act, slope};
  const dim3 grid((unsigned)C, (unsigned)B);
  const bool v4 = vec_ok(X, xs, L, dtype) && vec_ok(dY, dys, L, dtype);
  const bool big = bn_wide_block((int64_t)Nb * L * dtype_size(dtype));
#define HFTA_BN_COEF(T, V) \
  do { if (big) hipLaunchKernelGGL((bn_bwd_conv_coef_kernel<T, V, 1024>), grid, dim3(1024), 0, st, a, coef); \
       else hipLaunchKernelGGL((bn_bwd_conv_coef_kernel<T, V, 256>), grid, dim3(256), 0, st, a, coef); } while (0)
  if (dtype == HFTA_BF16) { if (v4) HFTA_BN_COEF(bf16_raw, 4); else HFTA_BN_COEF(bf16_raw, 1); }
  else { if (v4) HFTA_BN_COEF(float, 4); else HFTA_BN_COEF(float, 1); }
#undef HFTA_BN_COEF
  return launch_status();
}
int bn_bwd_coef_from_sums(int B, int Nb, int C, int L, const float* sums, const float* gamma, const float* beta,
                          const float* save_mean, const float* save_invstd, float* dgamma, float* dbeta, float* coef,
                          hipStream_t st) {
  const int n = B * C;
  hipLaunchKernelGGL(bn_bwd_coef_sums_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, sums, gamma, beta, save_mean,
                     save_invstd, dgamma, dbeta, coef, n, (float)Nb * (float)L);
  return launch_status();
}
}  // namespace hfta

extern "C" {

int hfta_bn_fwd(int B, int Nb, int C, int L, int dtype, const void* X, const int64_t xs[4], const float* gamma,
                const float* beta, float eps, float momentum, float* running_mean, float* running_var,
                float* save_mean, float* save_invstd, void* Y, const int64_t ys[4], int act, float act_slope,
                void* stream) {
  if (B <= 0 || Nb <= 0 || C <= 0 || L <= 0 || !valid_dtype(dtype) || !X || !xs || !gamma || !beta || !save_mean ||
      !save_invstd || !Y || !ys || !(eps >= 0.f))
    return HFTA_EINVAL;
  if ((running_mean == nullptr) != (running_var == nullptr)) return HFTA_EINVAL;
  if (act != HFTA_ACT_NONE && act != HFTA_ACT_RELU && act != HFTA_ACT_LEAKY) return HFTA_EUNSUPPORTED;
  if (B > 65535) return HFTA_EUNSUPPORTED;
  const bool lin = (L == 1 && xs[2] == 1 && ys[2] == 1);
  const int kx = lin ? 2 : layout_kind(xs, L), ky = lin ? 2 : layout_kind(ys, L);
  if (kx == 0 || kx != ky) return HFTA_EUNSUPPORTED;
  BnFwdArgs a{X, Y, gamma, beta, running_mean, running_var, save_mean, save_invstd,
              xs[0], xs[1], xs[2], ys[0], ys[1], ys[2], Nb, C, L, act, eps, momentum, act_slope};
  hipStream_t st = as_stream(stream);
  if (kx == 2) {
    dim3 grid((unsigned)((C + BNL_C - 1) / BNL_C), (unsigned)B);
    if (dtype == HFTA_BF16) hipLaunchKernelGGL(bn_fwd_linear_kernel<bf16_raw>, grid, dim3(BNL_C * BNL_N), 0, st, a);
    else hipLaunchKernelGGL(bn_fwd_linear_kernel<float>, grid, dim3(BNL_C * BNL_N), 0, st, a);
    return launch_status();
  }
  dim3 grid((unsigned)C, (unsigned)B);
  const bool v4 = vec_ok(X, xs, L, dtype) && vec_ok(Y, ys, L, dtype);
  const bool big = bn_wide_block((int64_t)Nb * L * dtype_size(dtype));
#define HFTA_BN_FWD(T, V) \
  do { if (big) hipLaunchKernelGGL((bn_fwd_conv_kernel<T, V, 1024>), grid, dim3(1024), 0, st, a); \
       else hipLaunchKernelGGL((bn_fwd_conv_kernel<T, V, 256>), grid, dim3(256), 0, st, a); } while (0)
  if (dtype == HFTA_BF16) { if (v4) HFTA_BN_FWD(bf16_raw, 4); else HFTA_BN_FWD(bf16_raw, 1); }
  else { if (v4) HFTA_BN_FWD(float, 4); else HFTA_BN_FWD(float, 1); }
#undef HFTA_BN_FWD
  return launch_status();
}

int hfta_bn_apply_fwd(int B, int Nb, int C, int L, int dtype, const void* X, const int64_t xs[4], const float* gamma,
                      const float* beta, const float* mean, const float* invstd, void* Y, const int64_t ys[4], int act,
                      float act_slope, void* stream) {
  if (B <= 0 || Nb <= 0 || C <= 0 || L <= 0 || !valid_dtype(dtype) || !X || !xs || !gamma || !beta || !mean || !invstd ||
      !Y || !ys)
    return HFTA_EINVAL;
  if (act != HFTA_ACT_NONE && act != HFTA_ACT_RELU && act != HFTA_ACT_LEAKY) return HFTA_EUNSUPPORTED;
  if (B > 65535 || layout_kind(xs, L) != 1 || layout_kind(ys, L) != 1) return HFTA_EUNSUPPORTED;
  BnFwdArgs a{X, Y, gamma, beta, nullptr, nullptr, const_cast<float*>(mean), const_cast<float*>(invstd),
              xs[0], xs[1], xs[2], ys[0], ys[1], ys[2], Nb, C, L, act, 0.f, 0.f, act_slope};
  hipStream_t st = as_stream(stream);
  const dim3 grid((unsigned)C, (unsigned)B);
  const bool v4 = vec_ok(X, xs, L, dtype) && vec_ok(Y, ys, L, dtype);
  const bool big = bn_wide_block((int64_t)Nb * L * dtype_size(dtype));
#define HFTA_BN_APPLY(T, V) \
  do { if (big) hipLaunchKernelGGL((bn_apply_conv_kernel<T, V, 1024>), grid, dim3(1024), 0, st, a); \
       else hipLaunchKernelGGL((bn_apply_conv_kernel<T, V, 256>), grid, dim3(256), 0, st, a); } while (0)
  if (dtype == HFTA_BF16) { if (v4) HFTA_BN_APPLY(bf16_raw, 4); else HFTA_BN_APPLY(bf16_raw, 1); }
  else { if (v4) HFTA_BN_APPLY(float, 4); else HFTA_BN_APPLY(float, 1); }
#undef HFTA_BN_APPLY
  return launch_status();
}

int hfta_bn_eval_fwd(int B, int Nb, int C, int L, int dtype, const void* X, const int64_t xs[4], const float* gamma,
                     const float* beta, const float* running_mean, const float* running_var, float eps, void* Y,
                     const int64_t ys[4], int act, float act_slope, void* stream) {
  if (B <= 0 || Nb <= 0 || C <= 0 || L <= 0 || !valid_dtype(dtype) || !X || !xs || !gamma || !beta || !running_mean ||
      !running_var || !Y || !ys || !(eps >= 0.f))
    return HFTA_EINVAL;
  if (act != HFTA_ACT_NONE && act != HFTA_ACT_RELU && act != HFTA_ACT_LEAKY) return HFTA_EUNSUPPORTED;
  if (B > 65535) return HFTA_EUNSUPPORTED;
  const bool lin = (L == 1 && xs[2] == 1 && ys[2] == 1);
  const int kx = lin ? 2 : layout_kind(xs, L), ky = lin ? 2 : layout_kind(ys, L);
  if (kx == 0 || kx != ky) return HFTA_EUNSUPPORTED;
  BnEvalArgs a{X, Y, gamma, beta, running_mean, running_var, xs[0], xs[1], xs[2], ys[0], ys[1], ys[2],
               Nb, C, L, act, eps, act_slope};
  hipStream_t st = as_stream(stream);
  if (kx == 2) {
    dim3 grid((unsigned)((C + BNL_C - 1) / BNL_C), (unsigned)B);
    if (dtype == HFTA_BF16) hipLaunchKernelGGL(bn_eval_linear_kernel<bf16_raw>, grid, dim3(BNL_C * BNL_N), 0, st, a);
    else hipLaunchKernelGGL(bn_eval_linear_kernel<float>, grid, dim3(BNL_C * BNL_N), 0, st, a);
    return launch_status();
  }
  dim3 grid((unsigned)C, (unsigned)B);
  const bool v4 = vec_ok(X, xs, L, dtype) && vec_ok(Y, ys, L, dtype);
  const bool big = bn_wide_block((int64_t)Nb * L * dtype_size(dtype));
#define HFTA_BN_EVAL(T, V) \
  do { if (big) hipLaunchKernelGGL((bn_eval_conv_kernel<T, V, 1024>), grid, dim3(1024), 0, st, a); \
       else hipLaunchKernelGGL((bn_eval_conv_kernel<T, V, 256>), grid, dim3(256), 0, st, a); } while (0)
  if (dtype == HFTA_BF16) { if (v4) HFTA_BN_EVAL(bf16_raw, 4); else HFTA_BN_EVAL(bf16_raw, 1); }
  else { if (v4) HFTA_BN_EVAL(float, 4); else HFTA_BN_EVAL(float, 1); }
#undef HFTA_BN_EVAL
  return launch_status();
}

int hfta_bn_bwd(int B, int Nb, int C, int L, int dtype, const void* X, const int64_t xs[4], const void* dY,
                const int64_t dys[4], const float* gamma, const float* beta, const float* save_mean,
                const float* save_invstd, void* dX, const int64_t dxs[4], float* dgamma, float* dbeta, float* dx_sum,
                int act, float act_slope, void* stream) {
  if (B <= 0 || Nb <= 0 || C <= 0 || L <= 0 || !valid_dtype(dtype) || !X || !xs || !dY || !dys || !gamma || !beta ||
      !save_mean || !save_invstd || !dX || !dxs || !dgamma || !dbeta)
    return HFTA_EINVAL;
  if (act != HFTA_ACT_NONE && act != HFTA_ACT_RELU && act != HFTA_ACT_LEAKY) return HFTA_EUNSUPPORTED;
  if (B > 65535) return HFTA_EUNSUPPORTED;
  const bool lin = (L == 1 && xs[2] == 1 && dys[2] == 1 && dxs[2] == 1);
  const int kx = lin ? 2 : layout_kind(xs, L);
  if (kx == 0 || (!lin && (layout_kind(dys, L) != kx || layout_kind(dxs, L) != kx))) return HFTA_EUNSUPPORTED;
  BnBwdArgs a{X, dY, dX, gamma, beta, save_mean, save_invstd, dgamma, dbeta, dx_sum,
              xs[0], xs[1], xs[2], dys[0], dys[1], dys[2], dxs[0], dxs[1], dxs[2], Nb, C, L, act, act_slope};
  hipStream_t st = as_stream(stream);
  if (kx == 2) {
    dim3 grid((unsigned)((C + BNL_C - 1) / BNL_C), (unsigned)B);
    if (dtype == HFTA_BF16) hipLaunchKernelGGL(bn_bwd_linear_kernel<bf16_raw>, grid, dim3(BNL_C * BNL_N), 0, st, a);
    else hipLaunchKernelGGL(bn_bwd_linear_kernel<float>, grid, dim3(BNL_C * BNL_N), 0, st, a);
    return launch_status();
  }
  dim3 grid((unsigned)C, (unsigned)B);
  const bool v4 = vec_ok(X, xs, L, dtype) && vec_ok(dY, dys, L, dtype) && vec_ok(dX, dxs, L, dtype);
  const bool big = bn_wide_block((int64_t)Nb * L * dtype_size(dtype));
#define HFTA_BN_BWD(T, V) \
  do { if (big) hipLaunchKernelGGL((bn_bwd_conv_kernel<T, V, 1024>), grid, dim3(1024), 0, st, a); \
       else hipLaunchKernelGGL((bn_bwd_conv_kernel<T, V, 256>), grid, dim3(256), 0, st, a); } while (0)
  if (dtype == HFTA_BF16) { if (v4) HFTA_BN_BWD(bf16_raw, 4); else HFTA_BN_BWD(bf16_raw, 1); }
  else { if (v4) HFTA_BN_BWD(float, 4); else HFTA_BN_BWD(float, 1); }
#undef HFTA_BN_BWD
  return launch_status();
}

}  // extern "C"
