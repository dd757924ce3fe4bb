// BatchNorm + activation + max over the point axis as ONE operator, forward and backward.
//
// PointNet's global feature is max_l act(BN(z))[., l].  Fused, the activated tensor is never
// written and never read back: the forward streams z twice (statistics, then normalise-and-max)
// and writes only [B][Nb][C] values and indices; the backward needs z once, because the
// gradient arriving from the pool is non-zero at exactly one point per (sample, channel), so the
// two BatchNorm sums collapse to Nb gathered elements per channel.
//
// The forward is bit-identical to hfta_bn_fwd followed by hfta_maxpool_points (the maximum is
// taken over the activated values rounded to the storage type, lowest index on ties); the
// backward equals hfta_maxpool_points_bwd followed by hfta_bn_bwd up to fp32 summation order.
//
// One workgroup per channel (b, c); each wavefront owns whole rows (samples) in the second pass
// so that the argmax reduction stays inside a wave.
#include "bn_common.h"

using namespace hfta;

namespace {

struct BnPoolFwdArgs {
  const void* X; void* V; int32_t* idx;
  const float* gamma; const float* beta;
  float* running_mean; float* running_var; float* save_mean; float* save_invstd;
  int64_t xsb, xsn, xsc, vsb, vsn, vsc;
  int Nb, C, L, act;
  float eps, momentum, slope;
};

template <typename T, int VEC, int NT>
__global__ __launch_bounds__(NT) void bn_fwd_maxpool_kernel(BnPoolFwdArgs p) {
  constexpr int NW = NT / 64;
  __shared__ float sh[NW][2];
  const int c = blockIdx.x, b = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const T* x = reinterpret_cast<const T*>(p.X) + b * p.xsb + c * p.xsc;
  const int chunks = p.L / VEC;
  const float shift = Elem<T>::load(x);
  float s1 = 0.f, s2 = 0.f;
  // same element -> thread assignment and reduction order as the stand-alone BatchNorm forward,
  // so the statistics (and with them every activated value) come out bit-identical
  for (RowWalk w(chunks, NT); w.n < p.Nb; w.step()) {
    const int n = w.n, ch = w.ch;
    float v[VEC];
    load_vec<T, VEC>(x + n * p.xsn + ch * VEC, v);
#pragma unroll
    for (int e = 0; e < VEC; ++e) { const float d = v[e] - shift; s1 += d; s2 = fmaf(d, d, s2); }
  }
  block_sum2<NW>(s1, s2, sh);
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
  for (int n = wave; n < p.Nb; n += NW) {
    const T* row = x + n * p.xsn;
    float best = -INFINITY;
    int bi = 0x7fffffff;
    for (int ch = lane; ch < chunks; ch += 64) {
      float v[VEC];
      load_vec<T, VEC>(row + ch * VEC, v);
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        // the activated value exactly as hfta_bn_fwd would have stored it
        const float y = Elem<T>::to_f32(Elem<T>::from_f32(apply_act(fmaf(g, (v[e] - mean) * invstd, bt), p.act, p.slope)));
        if (y > best || bi == 0x7fffffff) { best = y; bi = ch * VEC + e; }
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float ov = __shfl_xor(best, o, 64);
      const int oi = __shfl_xor(bi, o, 64);
      if (oi != 0x7fffffff && (bi == 0x7fffffff || ov > best || (ov == best && oi < bi))) { best = ov; bi = oi; }
    }
    if (lane == 0) {
      const int64_t o = b * p.vsb + n * p.vsn + c * p.vsc;
      reinterpret_cast<T*>(p.V)[o] = Elem<T>::from_f32(best);
      p.idx[o] = bi;
    }
  }
}

struct BnPoolBwdArgs {
  const void* X; const void* dV; const int32_t* idx; void* dX;
  const float* gamma; const float* beta; const float* save_mean; const float* save_invstd;
  float* dgamma; float* dbeta; float* dx_sum;
  int64_t xsb, xsn, xsc, vsb, vsn, vsc, dxsb, dxsn, dxsc;
  int Nb, C, L, act;
  float slope;
};

template <typename T, int VEC, int NT>
__global__ __launch_bounds__(NT) void bn_bwd_maxpool_kernel(BnPoolBwdArgs p) {
  constexpr int NW = NT / 64;
  __shared__ float sh[NW][2];
  const int c = blockIdx.x, b = blockIdx.y, k = b * p.C + c;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const T* x = reinterpret_cast<const T*>(p.X) + b * p.xsb + c * p.xsc;
  const T* dv = reinterpret_cast<const T*>(p.dV) + b * p.vsb + c * p.vsc;
  const int32_t* ix = p.idx + b * p.vsb + c * p.vsc;
  T* dx = reinterpret_cast<T*>(p.dX) + b * p.dxsb + c * p.dxsc;
  const float mean = p.save_mean[k], invstd = p.save_invstd[k], g = p.gamma[k], bt = p.beta[k];
  // the incoming gradient is dV at the argmax point of each sample and zero elsewhere
  float s1 = 0.f, s2 = 0.f;
  for (int n = threadIdx.x; n < p.Nb; n += NT) {
    const int hit = min(max(ix[n * p.vsn], 0), p.L - 1);     // never address outside the row
    const float xh = (Elem<T>::load(x + n * p.xsn + hit) - mean) * invstd;
    const float gr = Elem<T>::load(dv + n * p.vsn) * act_grad(fmaf(g, xh, bt), p.act, p.slope);
    s1 += gr;
    s2 = fmaf(gr, xh, s2);
  }
  block_sum2<NW>(s1, s2, sh);
  if (threadIdx.x == 0) { p.dbeta[k] = s1; p.dgamma[k] = s2; }
  const float m = (float)p.Nb * (float)p.L;
  const float mb = s1 / m, mg = s2 / m, sc = g * invstd;
  const int chunks = p.L / VEC;
  float s3 = 0.f;
  for (int n = wave; n < p.Nb; n += NW) {
    const T* row = x + n * p.xsn;
    T* drow = dx + n * p.dxsn;
    const int hit = min(max(ix[n * p.vsn], 0), p.L - 1);
    const float gv = Elem<T>::load(dv + n * p.vsn);
    for (int ch = lane; ch < chunks; ch += 64) {
      float v[VEC];
      load_vec<T, VEC>(row + ch * VEC, v);
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const float xh = (v[e] - mean) * invstd;
        float gr = 0.f;
        if (ch * VEC + e == hit) gr = gv * act_grad(fmaf(g, xh, bt), p.act, p.slope);
        v[e] = sc * (gr - mb - xh * mg);
        s3 += Elem<T>::to_f32(Elem<T>::from_f32(v[e]));
      }
      store_vec<T, VEC>(drow + ch * VEC, v);
    }
  }
  if (p.dx_sum) {
    float dummy = 0.f;
    block_sum2<NW>(s3, dummy, sh);
    if (threadIdx.x == 0) p.dx_sum[k] = s3;
  }
}

bool act_ok(int act) { return act == HFTA_ACT_NONE || act == HFTA_ACT_RELU || act == HFTA_ACT_LEAKY; }

}  // namespace

extern "C" {

int hfta_bn_fwd_maxpool(int B, int Nb, int C, int L, int dtype, const void* X, const int64_t xs[4], const float* gamma,
                        const float* beta, float eps, float momentum, float* running_mean, float* running_var,
                        float* save_mean, float* save_invstd, void* V, int32_t* idx, const int64_t vs[3], int act,
                        float act_slope, void* stream) {
  if (B <= 0 || Nb <= 0 || C <= 0 || L <= 0 || !valid_dtype(dtype) || !X || !xs || !gamma || !beta || !save_mean ||
      !save_invstd || !V || !idx || !vs || !(eps >= 0.f))
    return HFTA_EINVAL;
  if ((running_mean == nullptr) != (running_var == nullptr)) return HFTA_EINVAL;
  if (!act_ok(act) || xs[3] != 1 || B > 65535) return HFTA_EUNSUPPORTED;
  BnPoolFwdArgs a{X, V, idx, gamma, beta, running_mean, running_var, save_mean, save_invstd,
                  xs[0], xs[1], xs[2], vs[0], vs[1], vs[2], Nb, C, L, act, eps, momentum, act_slope};
  dim3 grid((unsigned)C, (unsigned)B);
  hipStream_t st = as_stream(stream);
  const bool v4 = bn_vec4_ok(X, xs, L, dtype);
  const bool big = bn_wide_block((int64_t)Nb * L * dtype_size(dtype));
#define HFTA_LAUNCH(T, V_) \
  do { if (big) hipLaunchKernelGGL((bn_fwd_maxpool_kernel<T, V_, 1024>), grid, dim3(1024), 0, st, a); \
       else hipLaunchKernelGGL((bn_fwd_maxpool_kernel<T, V_, 256>), grid, dim3(256), 0, st, a); } while (0)
  if (dtype == HFTA_BF16) { if (v4) HFTA_LAUNCH(bf16_raw, 4); else HFTA_LAUNCH(bf16_raw, 1); }
  else { if (v4) HFTA_LAUNCH(float, 4); else HFTA_LAUNCH(float, 1); }
#undef HFTA_LAUNCH
  return launch_status();
}

int hfta_bn_bwd_maxpool(int B, int Nb, int C, int L, int dtype, const void* X, const int64_t xs[4], const void* dV,
                        const int32_t* idx, const int64_t vs[3], const float* gamma, const float* beta,
                        const float* save_mean, const float* save_invstd, void* dX, const int64_t dxs[4],
                        float* dgamma, float* dbeta, float* dx_sum, int act, float act_slope, void* stream) {
  if (B <= 0 || Nb <= 0 || C <= 0 || L <= 0 || !valid_dtype(dtype) || !X || !xs || !dV || !idx || !vs || !gamma || !beta ||
      !save_mean || !save_invstd || !dX || !dxs || !dgamma || !dbeta)
    return HFTA_EINVAL;
  if (!act_ok(act) || xs[3] != 1 || dxs[3] != 1 || B > 65535) return HFTA_EUNSUPPORTED;
  BnPoolBwdArgs a{X, dV, idx, dX, gamma, beta, save_mean, save_invstd, dgamma, dbeta, dx_sum,
                  xs[0], xs[1], xs[2], vs[0], vs[1], vs[2], dxs[0], dxs[1], dxs[2], Nb, C, L, act, act_slope};
  dim3 grid((unsigned)C, (unsigned)B);
  hipStream_t st = as_stream(stream);
  const bool v4 = bn_vec4_ok(X, xs, L, dtype) && bn_vec4_ok(dX, dxs, L, dtype);
  const bool big = bn_wide_block((int64_t)Nb * L * dtype_size(dtype));
#define HFTA_LAUNCH(T, V_) \
  do { if (big) hipLaunchKernelGGL((bn_bwd_maxpool_kernel<T, V_, 1024>), grid, dim3(1024), 0, st, a); \
       else hipLaunchKernelGGL((bn_bwd_maxpool_kernel<T, V_, 256>), grid, dim3(256), 0, st, a); } while (0)
  if (dtype == HFTA_BF16) { if (v4) HFTA_LAUNCH(bf16_raw, 4); else HFTA_LAUNCH(bf16_raw, 1); }
  else { if (v4) HFTA_LAUNCH(float, 4); else HFTA_LAUNCH(float, 1); }
#undef HFTA_LAUNCH
  return launch_status();
}

}  // extern "C"
