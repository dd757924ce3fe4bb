// Fused Adam: one coalesced pass over the parameter arena [B][P] of all models.
//
// grid.y is the model index, so a workgroup only ever touches one model: its
// five hyper-parameters are read once from the device arrays and the two bias
// corrections 1 - beta^t are formed once per workgroup in double precision
// (1 - 0.999^t loses most of its bits in fp32 for small t), then broadcast
// through LDS.  Each thread updates four consecutive parameters with 16-byte
// accesses.  HBM-bound: reads theta, g, m, v and writes theta, m, v (+ the bf16
// copy the GEMMs read).
#include "common.h"

using namespace hfta;

namespace {

struct AdamArgs {
  float* theta; const void* grad; float* m; float* v; bf16_raw* lowp;
  const float* lr; const float* beta1; const float* beta2; const float* eps; const float* wd;
  int64_t P;
  int t, decoupled;
};

struct AdamHp { float lr, b1, b2, eps, wd, inv_bc1, inv_bc2; };

__device__ __forceinline__ void adam_one(float& th, float g, float& m, float& v, const AdamHp& h, int decoupled) {
  if (decoupled) th = th * (1.f - h.lr * h.wd);
  else g = fmaf(h.wd, th, g);
  m = h.b1 * m + (1.f - h.b1) * g;
  v = h.b2 * v + (1.f - h.b2) * (g * g);
  const float mhat = m * h.inv_bc1;
  const float vhat = v * h.inv_bc2;
  th = th - h.lr * mhat / (sqrtf(vhat) + h.eps);
}

template <typename G, bool VEC4>
__global__ __launch_bounds__(256) void adam_kernel(AdamArgs p) {
  __shared__ AdamHp sh;
  const int b = blockIdx.y;
  if (threadIdx.x == 0) {
    AdamHp h;
    h.lr = p.lr[b]; h.b1 = p.beta1[b]; h.b2 = p.beta2[b]; h.eps = p.eps[b]; h.wd = p.wd[b];
    h.inv_bc1 = (float)(1.0 / (1.0 - pow((double)h.b1, (double)p.t)));
    h.inv_bc2 = (float)(1.0 / (1.0 - pow((double)h.b2, (double)p.t)));
    sh = h;
  }
  __syncthreads();
  const AdamHp h = sh;
  const int64_t base = (int64_t)b * p.P;
  const G* gr = reinterpret_cast<const G*>(p.grad) + base;
  if (VEC4) {
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= p.P) return;
    float4 th = *reinterpret_cast<float4*>(p.theta + base + i);
    float4 m = *reinterpret_cast<float4*>(p.m + base + i);
    float4 v = *reinterpret_cast<float4*>(p.v + base + i);
    float g[4];
    if (sizeof(G) == 4) {
      *reinterpret_cast<float4*>(g) = *reinterpret_cast<const float4*>(gr + i);
    } else {
      const uint2 raw = *reinterpret_cast<const uint2*>(gr + i);
      g[0] = __uint_as_float(raw.x << 16); g[1] = __uint_as_float(raw.x & 0xffff0000u);
      g[2] = __uint_as_float(raw.y << 16); g[3] = __uint_as_float(raw.y & 0xffff0000u);
    }
    adam_one(th.x, g[0], m.x, v.x, h, p.decoupled);
    adam_one(th.y, g[1], m.y, v.y, h, p.decoupled);
    adam_one(th.z, g[2], m.z, v.z, h, p.decoupled);
    adam_one(th.w, g[3], m.w, v.w, h, p.decoupled);
    *reinterpret_cast<float4*>(p.theta + base + i) = th;
    *reinterpret_cast<float4*>(p.m + base + i) = m;
    *reinterpret_cast<float4*>(p.v + base + i) = v;
    if (p.lowp) {
      uint2 o;
      o.x = pack_bf16x2(th.x, th.y);
      o.y = pack_bf16x2(th.z, th.w);
      *reinterpret_cast<uint2*>(p.lowp + base + i) = o;
    }
  } else {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= p.P) return;
    float th = p.theta[base + i], m = p.m[base + i], v = p.v[base + i];
    const float g = Elem<G>::load(gr + i);
    adam_one(th, g, m, v, h, p.decoupled);
    p.theta[base + i] = th; p.m[base + i] = m; p.v[base + i] = v;
    if (p.lowp) p.lowp[base + i] = f32_to_bf16(th);
  }
}

struct AdamMultiArgs {
  float* theta; const void* grad; float* m; float* v; bf16_raw* lowp;
  const float* lr; const float* beta1; const float* beta2; const float* eps; const float* wd;
  int64_t total;                                  // B * P
  int B, nseg, t, decoupled;
  int64_t off[HFTA_ADAM_MAX_SEGMENTS + 1];        // per-model element offsets
};

// Parameter-major arena: thread -> flat index -> (segment, model).  The bias
// corrections of all B models are formed once per workgroup in double.
template <typename G, bool VEC4>
__global__ __launch_bounds__(256) void adam_multi_kernel(AdamMultiArgs p) {
  extern __shared__ float bc[];                   // [B][2]
  for (int b = threadIdx.x; b < p.B; b += 256) {
    bc[2 * b] = (float)(1.0 / (1.0 - pow((double)p.beta1[b], (double)p.t)));
    bc[2 * b + 1] = (float)(1.0 / (1.0 - pow((double)p.beta2[b], (double)p.t)));
  }
  __syncthreads();
  constexpr int W = VEC4 ? 4 : 1;
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * W;
  if (i >= p.total) return;
  // binary search: largest j with B*off[j] <= i
  int lo = 0, hi = p.nseg;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if ((int64_t)p.B * p.off[mid] <= i) lo = mid; else hi = mid;
  }
  const int64_t n = p.off[lo + 1] - p.off[lo];
  const int b = (int)((i - (int64_t)p.B * p.off[lo]) / n);
  AdamHp h;
  h.lr = p.lr[b]; h.b1 = p.beta1[b]; h.b2 = p.beta2[b]; h.eps = p.eps[b]; h.wd = p.wd[b];
  h.inv_bc1 = bc[2 * b]; h.inv_bc2 = bc[2 * b + 1];
  const G* gr = reinterpret_cast<const G*>(p.grad);
  if (VEC4) {
    float4 th = *reinterpret_cast<float4*>(p.theta + i);
    float4 m = *reinterpret_cast<float4*>(p.m + i);
    float4 v = *reinterpret_cast<float4*>(p.v + i);
    float g[4];
    if (sizeof(G) == 4) {
      *reinterpret_cast<float4*>(g) = *reinterpret_cast<const float4*>(gr + i);
    } else {
      const uint2 raw = *reinterpret_cast<const uint2*>(gr + i);
      g[0] = __uint_as_float(raw.x << 16); g[1] = __uint_as_float(raw.x & 0xffff0000u);
      g[2] = __uint_as_float(raw.y << 16); g[3] = __uint_as_float(raw.y & 0xffff0000u);
    }
    adam_one(th.x, g[0], m.x, v.x, h, p.decoupled);
    adam_one(th.y, g[1], m.y, v.y, h, p.decoupled);
    adam_one(th.z, g[2], m.z, v.z, h, p.decoupled);
    adam_one(th.w, g[3], m.w, v.w, h, p.decoupled);
    *reinterpret_cast<float4*>(p.theta + i) = th;
    *reinterpret_cast<float4*>(p.m + i) = m;
    *reinterpret_cast<float4*>(p.v + i) = v;
    if (p.lowp) {
      uint2 o;
      o.x = pack_bf16x2(th.x, th.y);
      o.y = pack_bf16x2(th.z, th.w);
      *reinterpret_cast<uint2*>(p.lowp + i) = o;
    }
  } else {
    float th = p.theta[i], m = p.m[i], v = p.v[i];
    const float g = Elem<G>::load(gr + i);
    adam_one(th, g, m, v, h, p.decoupled);
    p.theta[i] = th; p.m[i] = m; p.v[i] = v;
    if (p.lowp) p.lowp[i] = f32_to_bf16(th);
  }
}

}  // namespace

extern "C" int hfta_adam_step_multi(int B, int nseg, const int64_t* seg_offsets, int grad_dtype, float* theta,
                                    const void* grad, float* m, float* v, void* theta_lowp, const float* lr,
                                    const float* beta1, const float* beta2, const float* eps,
                                    const float* weight_decay, int step_t, int decoupled_wd, void* stream) {
  if (B <= 0 || nseg <= 0 || !seg_offsets || !valid_dtype(grad_dtype) || !theta || !grad || !m || !v || !lr || !beta1 ||
      !beta2 || !eps || !weight_decay || step_t < 1)
    return HFTA_EINVAL;
  if (nseg > HFTA_ADAM_MAX_SEGMENTS || B > HFTA_ADAM_MAX_MODELS) return HFTA_EUNSUPPORTED;
  if (seg_offsets[0] != 0) return HFTA_EINVAL;
  AdamMultiArgs a;
  bool all4 = true;
  for (int j = 0; j <= nseg; ++j) {
    if (j > 0 && seg_offsets[j] <= seg_offsets[j - 1]) return HFTA_EINVAL;
    a.off[j] = seg_offsets[j];
    if (seg_offsets[j] % 4 != 0) all4 = false;
  }
  for (int j = nseg + 1; j <= HFTA_ADAM_MAX_SEGMENTS; ++j) a.off[j] = seg_offsets[nseg];
  auto al = [](const void* q, size_t k) { return reinterpret_cast<uintptr_t>(q) % k == 0; };
  const bool v4 = all4 && al(theta, 16) && al(m, 16) && al(v, 16) && al(grad, grad_dtype == HFTA_BF16 ? 8 : 16) &&
                  (!theta_lowp || al(theta_lowp, 8));
  a.theta = theta; a.grad = grad; a.m = m; a.v = v; a.lowp = (bf16_raw*)theta_lowp;
  a.lr = lr; a.beta1 = beta1; a.beta2 = beta2; a.eps = eps; a.wd = weight_decay;
  a.total = (int64_t)B * seg_offsets[nseg];
  a.B = B; a.nseg = nseg; a.t = step_t; a.decoupled = decoupled_wd ? 1 : 0;
  const int64_t per_block = v4 ? 1024 : 256;
  const int64_t blocks = (a.total + per_block - 1) / per_block;
  if (blocks > 0x7fffffffLL) return HFTA_EINVAL;
  const size_t shm = (size_t)B * 2 * sizeof(float);
  hipStream_t st = as_stream(stream);
  dim3 grid((unsigned)blocks);
  if (grad_dtype == HFTA_BF16) {
    if (v4) hipLaunchKernelGGL((adam_multi_kernel<bf16_raw, true>), grid, dim3(256), shm, st, a);
    else hipLaunchKernelGGL((adam_multi_kernel<bf16_raw, false>), grid, dim3(256), shm, st, a);
  } else {
    if (v4) hipLaunchKernelGGL((adam_multi_kernel<float, true>), grid, dim3(256), shm, st, a);
    else hipLaunchKernelGGL((adam_multi_kernel<float, false>), grid, dim3(256), shm, st, a);
  }
  return launch_status();
}

extern "C" int hfta_adam_step(int B, int64_t P, int grad_dtype, float* theta, const void* grad, float* m, float* v,
                              void* theta_lowp, const float* lr, const float* beta1, const float* beta2,
                              const float* eps, const float* weight_decay, int step_t, int decoupled_wd,
                              void* stream) {
  if (B <= 0 || P <= 0 || !valid_dtype(grad_dtype) || !theta || !grad || !m || !v || !lr || !beta1 || !beta2 || !eps ||
      !weight_decay || step_t < 1)
    return HFTA_EINVAL;
  if (B > 65535) return HFTA_EUNSUPPORTED;
  auto al = [](const void* q, size_t a) { return reinterpret_cast<uintptr_t>(q) % a == 0; };
  const bool v4 = P % 4 == 0 && al(theta, 16) && al(m, 16) && al(v, 16) && al(grad, grad_dtype == HFTA_BF16 ? 8 : 16) &&
                  (!theta_lowp || al(theta_lowp, 8));
  const int64_t per_block = v4 ? 1024 : 256;
  const int64_t blocks = (P + per_block - 1) / per_block;
  if (blocks > 0x7fffffffLL) return HFTA_EINVAL;
  AdamArgs a{theta, grad, m, v, (bf16_raw*)theta_lowp, lr, beta1, beta2, eps, weight_decay, P, step_t, decoupled_wd ? 1 : 0};
  dim3 grid((unsigned)blocks, (unsigned)B);
  hipStream_t st = as_stream(stream);
  if (grad_dtype == HFTA_BF16) {
    if (v4) hipLaunchKernelGGL((adam_kernel<bf16_raw, true>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((adam_kernel<bf16_raw, false>), grid, dim3(256), 0, st, a);
  } else {
    if (v4) hipLaunchKernelGGL((adam_kernel<float, true>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((adam_kernel<float, false>), grid, dim3(256), 0, st, a);
  }
  return launch_status();
}
