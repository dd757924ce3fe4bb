// Fused Adadelta over the parameter-major arena of all B models, and the per-model step
// learning-rate schedule (section "Our Proposal: HFTA", paragraph on optimizers and learning-rate
// schedulers: the hyper-parameters become vectors with one entry per model).
//
// Same single coalesced pass as the fused Adam: thread -> flat arena index -> (segment, model),
// four consecutive parameters per thread with 16-byte accesses when every segment allows it.
// HBM-bound: reads theta, g, v, u and writes theta, v, u (+ the bf16 copy the GEMMs read).
#include "common.h"

using namespace hfta;

namespace {

struct AdadeltaArgs {
  float* theta; const void* grad; float* sq; float* acc; bf16_raw* lowp;
  const float* lr; const float* rho; const float* eps; const float* wd;
  int64_t total;                                  // B * P
  int B, nseg;
  int64_t off[HFTA_ADAM_MAX_SEGMENTS + 1];        // per-model element offsets
};

struct AdadeltaHp { float lr, rho, eps, wd; };

__device__ __forceinline__ void adadelta_one(float& th, float g, float& v, float& u, const AdadeltaHp& h) {
  g = fmaf(h.wd, th, g);
  v = h.rho * v + (1.f - h.rho) * (g * g);
  const float d = sqrtf(u + h.eps) / sqrtf(v + h.eps) * g;
  u = h.rho * u + (1.f - h.rho) * (d * d);
  th = th - h.lr * d;
}

template <typename G, bool VEC4>
__global__ __launch_bounds__(256) void adadelta_multi_kernel(AdadeltaArgs p) {
  constexpr int W = VEC4 ? 4 : 1;
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * W;
  if (i >= p.total) return;
  int lo = 0, hi = p.nseg;                        // largest j with B*off[j] <= i
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if ((int64_t)p.B * p.off[mid] <= i) lo = mid; else hi = mid;
  }
  const int64_t n = p.off[lo + 1] - p.off[lo];
  const int b = (int)((i - (int64_t)p.B * p.off[lo]) / n);
  const AdadeltaHp h{p.lr[b], p.rho[b], p.eps[b], p.wd[b]};
  const G* gr = reinterpret_cast<const G*>(p.grad);
  if (VEC4) {
    float4 th = *reinterpret_cast<float4*>(p.theta + i);
    float4 v = *reinterpret_cast<float4*>(p.sq + i);
    float4 u = *reinterpret_cast<float4*>(p.acc + i);
    float g[4];
    if (sizeof(G) == 4) {
      *reinterpret_cast<float4*>(g) = *reinterpret_cast<const float4*>(gr + i);
    } else {
      const uint2 raw = *reinterpret_cast<const uint2*>(gr + i);
      g[0] = __uint_as_float(raw.x << 16); g[1] = __uint_as_float(raw.x & 0xffff0000u);
      g[2] = __uint_as_float(raw.y << 16); g[3] = __uint_as_float(raw.y & 0xffff0000u);
    }
    adadelta_one(th.x, g[0], v.x, u.x, h);
    adadelta_one(th.y, g[1], v.y, u.y, h);
    adadelta_one(th.z, g[2], v.z, u.z, h);
    adadelta_one(th.w, g[3], v.w, u.w, h);
    *reinterpret_cast<float4*>(p.theta + i) = th;
    *reinterpret_cast<float4*>(p.sq + i) = v;
    *reinterpret_cast<float4*>(p.acc + i) = u;
    if (p.lowp) *reinterpret_cast<uint2*>(p.lowp + i) = make_uint2(pack_bf16x2(th.x, th.y), pack_bf16x2(th.z, th.w));
  } else {
    float th = p.theta[i], v = p.sq[i], u = p.acc[i];
    adadelta_one(th, Elem<G>::load(gr + i), v, u, h);
    p.theta[i] = th; p.sq[i] = v; p.acc[i] = u;
    if (p.lowp) p.lowp[i] = f32_to_bf16(th);
  }
}

__global__ __launch_bounds__(64) void steplr_kernel(const float* base, const float* gamma, const int32_t* step_size,
                                                    int epoch, float* lr, int B) {
  const int b = blockIdx.x * 64 + threadIdx.x;
  if (b >= B) return;
  const int k = epoch / max(step_size[b], 1);
  lr[b] = (float)((double)base[b] * pow((double)gamma[b], (double)k));
}

}  // namespace

extern "C" int hfta_adadelta_step_multi(int B, int nseg, const int64_t* seg_offsets, int grad_dtype, float* theta,
                                        const void* grad, float* square_avg, float* acc_delta, void* theta_lowp,
                                        const float* lr, const float* rho, const float* eps, const float* weight_decay,
                                        void* stream) {
  if (B <= 0 || nseg <= 0 || !seg_offsets || !valid_dtype(grad_dtype) || !theta || !grad || !square_avg || !acc_delta ||
      !lr || !rho || !eps || !weight_decay)
    return HFTA_EINVAL;
  if (nseg > HFTA_ADAM_MAX_SEGMENTS || B > HFTA_ADAM_MAX_MODELS) return HFTA_EUNSUPPORTED;
  if (seg_offsets[0] != 0) return HFTA_EINVAL;
  AdadeltaArgs a;
  bool all4 = true;
  for (int j = 0; j <= nseg; ++j) {
    if (j > 0 && seg_offsets[j] <= seg_offsets[j - 1]) return HFTA_EINVAL;
    a.off[j] = seg_offsets[j];
    if (seg_offsets[j] % 4 != 0) all4 = false;
  }
  for (int j = nseg + 1; j <= HFTA_ADAM_MAX_SEGMENTS; ++j) a.off[j] = seg_offsets[nseg];
  auto al = [](const void* q, size_t k) { return reinterpret_cast<uintptr_t>(q) % k == 0; };
  const bool v4 = all4 && al(theta, 16) && al(square_avg, 16) && al(acc_delta, 16) &&
                  al(grad, grad_dtype == HFTA_BF16 ? 8 : 16) && (!theta_lowp || al(theta_lowp, 8));
  a.theta = theta; a.grad = grad; a.sq = square_avg; a.acc = acc_delta; a.lowp = (bf16_raw*)theta_lowp;
  a.lr = lr; a.rho = rho; a.eps = eps; a.wd = weight_decay;
  a.total = (int64_t)B * seg_offsets[nseg];
  a.B = B; a.nseg = nseg;
  const int64_t per_block = v4 ? 1024 : 256;
  const int64_t blocks = (a.total + per_block - 1) / per_block;
  if (blocks > 0x7fffffffLL) return HFTA_EINVAL;
  hipStream_t st = as_stream(stream);
  dim3 grid((unsigned)blocks);
  if (grad_dtype == HFTA_BF16) {
    if (v4) hipLaunchKernelGGL((adadelta_multi_kernel<bf16_raw, true>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((adadelta_multi_kernel<bf16_raw, false>), grid, dim3(256), 0, st, a);
  } else {
    if (v4) hipLaunchKernelGGL((adadelta_multi_kernel<float, true>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((adadelta_multi_kernel<float, false>), grid, dim3(256), 0, st, a);
  }
  return launch_status();
}

extern "C" int hfta_steplr(int B, const float* base_lr, const float* gamma, const int32_t* step_size, int epoch,
                           float* lr, void* stream) {
  if (B <= 0 || !base_lr || !gamma || !step_size || !lr || epoch < 0) return HFTA_EINVAL;
  hipLaunchKernelGGL(steplr_kernel, dim3((unsigned)((B + 63) / 64)), dim3(64), 0, as_stream(stream), base_lr, gamma,
                     step_size, epoch, lr, B);
  return launch_status();
}
