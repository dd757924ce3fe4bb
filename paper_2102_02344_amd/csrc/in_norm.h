// A tensor given as the previous block's stored pre-activation: its consumers form
//     x = act(gamma * ((z - mean) * invstd) + beta),   rounded to bf16,
// on the way into LDS with exactly the arithmetic of the BatchNorm forward kernels, so that they see the
// bits that block would have stored (fusion rules table, rows "BatchNorm1d" and the element-wise rows).
#pragma once
#include "common.h"

namespace hfta {

struct InNorm {                       // [B][C] fp32 each, as hfta_bn_fwd left them; gamma == nullptr: the tensor is taken as it is
  const float* gamma; const float* beta; const float* mean; const float* invstd;
  int act; float slope;
};

static inline bool in_norm_valid(const InNorm& n) {
  return n.gamma && n.beta && n.mean && n.invstd &&
         (n.act == HFTA_ACT_NONE || n.act == HFTA_ACT_RELU || n.act == HFTA_ACT_LEAKY);
}

// the four constants of channel k of model b: (mean, invstd, gamma, beta)
__device__ __forceinline__ float4 in_norm_consts(const InNorm& n, int64_t k) {
  return make_float4(n.mean[k], n.invstd[k], n.gamma[k], n.beta[k]);
}

__device__ __forceinline__ float in_norm_one(float z, const float4 cn, int act, float slope) {
  const float y = fmaf(cn.z, (z - cn.x) * cn.y, cn.w);
  float lo = act == HFTA_ACT_LEAKY ? slope * y : 0.f;      // what the activation returns where y <= 0
  if (act == HFTA_ACT_NONE) lo = y;
  return y > 0.f ? y : lo;
}

// four consecutive points of one channel (8 bytes of bf16); ok == false: the points lie past the sample's end and stay zero
__device__ __forceinline__ uint2 in_norm_apply4(uint2 q, const float4 cn, bool ok, int act, float slope) {
  float v[4] = {__uint_as_float(q.x << 16), __uint_as_float(q.x & 0xffff0000u), __uint_as_float(q.y << 16),
                __uint_as_float(q.y & 0xffff0000u)};
#pragma unroll
  for (int e = 0; e < 4; ++e) v[e] = ok ? in_norm_one(v[e], cn, act, slope) : 0.f;
  return make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
}

}  // namespace hfta
