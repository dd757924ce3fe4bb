// Max-pool over the point axis with argmax, and its scatter backward.
//
// One wavefront per row (b, n, c) of L contiguous points; four rows per
// workgroup.  A lane scans its strided share keeping (value, index) with a
// strict '>' so the lowest index wins inside the lane; the cross-lane butterfly
// prefers the larger value and, on equal values, the lower index, which makes
// the result the lowest point index attaining the maximum.  HBM-bound: every
// input byte is read exactly once.
#include "common.h"

using namespace hfta;

namespace {

struct PoolArgs {
  const void* X; void* V; int32_t* idx;
  int64_t xsb, xsn, xsc, vsb, vsn, vsc;
  int B, Nb, C, L;
  int64_t rows;
};

template <typename T, int VEC>
__global__ __launch_bounds__(256) void maxpool_fwd_kernel(PoolArgs p) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= p.rows) return;
  const int c = (int)(row % p.C);
  const int64_t bn = row / p.C;
  const int n = (int)(bn % p.Nb), b = (int)(bn / p.Nb);
  const T* x = reinterpret_cast<const T*>(p.X) + b * p.xsb + n * p.xsn + c * p.xsc;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  T bbits = T(0);
  if (VEC == 4) {
    // five pieces per lane in flight (a 2500-point row is two rounds); a piece past the row's end
    // re-reads the lane's first piece and is skipped
    constexpr int U = 5;
    const int chunks = p.L / 4;
    for (int ch0 = lane; ch0 < chunks; ch0 += 64 * U) {
      T e[U][4];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int ch = ch0 + 64 * u < chunks ? ch0 + 64 * u : ch0;
        if (sizeof(T) == 2) *reinterpret_cast<uint2*>(e[u]) = *reinterpret_cast<const uint2*>(x + ch * 4);
        else *reinterpret_cast<uint4*>(e[u]) = *reinterpret_cast<const uint4*>(x + ch * 4);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int ch = ch0 + 64 * u;
        if (ch < chunks) {
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const float v = Elem<T>::to_f32(e[u][k]);
            if (v > best || bi == 0x7fffffff) { best = v; bi = ch * 4 + k; bbits = e[u][k]; }
          }
        }
      }
    }
  } else {
    for (int l = lane; l < p.L; l += 64) {
      const T e = x[l];
      const float v = Elem<T>::to_f32(e);
      if (v > best || bi == 0x7fffffff) { best = v; bi = l; bbits = e; }
    }
  }
  uint32_t bits = (uint32_t)bbits;
  if (sizeof(T) == 4) bits = __float_as_uint(best);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(best, o, 64);
    const int oi = __shfl_xor(bi, o, 64);
    const uint32_t ob = __shfl_xor(bits, o, 64);
    if (oi != 0x7fffffff && (bi == 0x7fffffff || ov > best || (ov == best && oi < bi))) { best = ov; bi = oi; bits = ob; }
  }
  if (lane == 0) {
    const int64_t o = b * p.vsb + n * p.vsn + c * p.vsc;
    if (sizeof(T) == 2) reinterpret_cast<bf16_raw*>(p.V)[o] = (bf16_raw)bits;
    else reinterpret_cast<uint32_t*>(p.V)[o] = bits;
    p.idx[o] = bi;
  }
}

struct PoolBwdArgs {
  const void* dV; const int32_t* idx; void* dX;
  int64_t vsb, vsn, vsc, xsb, xsn, xsc;
  int B, Nb, C, L;
  int64_t rows;
};

template <typename T, int VEC>
__global__ __launch_bounds__(256) void maxpool_bwd_kernel(PoolBwdArgs p) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= p.rows) return;
  const int c = (int)(row % p.C);
  const int64_t bn = row / p.C;
  const int n = (int)(bn % p.Nb), b = (int)(bn / p.Nb);
  const int64_t o = b * p.vsb + n * p.vsn + c * p.vsc;
  const T g = reinterpret_cast<const T*>(p.dV)[o];
  const int hit = p.idx[o];
  T* dx = reinterpret_cast<T*>(p.dX) + b * p.xsb + n * p.xsn + c * p.xsc;
  if (VEC == 4) {
    const int chunks = p.L / 4;
    for (int ch = lane; ch < chunks; ch += 64) {
      T e[4] = {T(0), T(0), T(0), T(0)};
      if ((hit >> 2) == ch) e[hit & 3] = g;
      if (sizeof(T) == 2) *reinterpret_cast<uint2*>(dx + ch * 4) = *reinterpret_cast<uint2*>(e);
      else *reinterpret_cast<uint4*>(dx + ch * 4) = *reinterpret_cast<uint4*>(e);
    }
  } else {
    for (int l = lane; l < p.L; l += 64) dx[l] = (l == hit) ? g : T(0);
  }
}

bool vec4_ok(const void* ptr, int64_t sb, int64_t sn, int64_t sc, int L, int dtype) {
  const size_t bytes = 4 * dtype_size(dtype);
  return L % 4 == 0 && reinterpret_cast<uintptr_t>(ptr) % bytes == 0 && sb % 4 == 0 && sn % 4 == 0 && sc % 4 == 0;
}

}  // namespace

extern "C" {

int hfta_maxpool_points(int B, int Nb, int C, int L, int dtype, const void* X, const int64_t xs[4], void* V,
                        int32_t* idx, const int64_t vs[3], void* stream) {
  if (B <= 0 || Nb <= 0 || C <= 0 || L <= 0 || !valid_dtype(dtype) || !X || !xs || !V || !idx || !vs) return HFTA_EINVAL;
  if (xs[3] != 1) return HFTA_EUNSUPPORTED;
  const int64_t rows = (int64_t)B * Nb * C;
  if ((rows + 3) / 4 > 0x7fffffffLL) return HFTA_EINVAL;
  PoolArgs a{X, V, idx, xs[0], xs[1], xs[2], vs[0], vs[1], vs[2], B, Nb, C, L, rows};
  dim3 grid((unsigned)((rows + 3) / 4));
  hipStream_t st = as_stream(stream);
  const bool v4 = vec4_ok(X, xs[0], xs[1], xs[2], L, dtype);
  if (dtype == HFTA_BF16) {
    if (v4) hipLaunchKernelGGL((maxpool_fwd_kernel<bf16_raw, 4>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((maxpool_fwd_kernel<bf16_raw, 1>), grid, dim3(256), 0, st, a);
  } else {
    if (v4) hipLaunchKernelGGL((maxpool_fwd_kernel<float, 4>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((maxpool_fwd_kernel<float, 1>), grid, dim3(256), 0, st, a);
  }
  return launch_status();
}

int hfta_maxpool_points_bwd(int B, int Nb, int C, int L, int dtype, const void* dV, const int32_t* idx,
                            const int64_t vs[3], void* dX, const int64_t dxs[4], void* stream) {
  if (B <= 0 || Nb <= 0 || C <= 0 || L <= 0 || !valid_dtype(dtype) || !dV || !idx || !vs || !dX || !dxs) return HFTA_EINVAL;
  if (dxs[3] != 1) return HFTA_EUNSUPPORTED;
  const int64_t rows = (int64_t)B * Nb * C;
  if ((rows + 3) / 4 > 0x7fffffffLL) return HFTA_EINVAL;
  PoolBwdArgs a{dV, idx, dX, vs[0], vs[1], vs[2], dxs[0], dxs[1], dxs[2], B, Nb, C, L, rows};
  dim3 grid((unsigned)((rows + 3) / 4));
  hipStream_t st = as_stream(stream);
  const bool v4 = vec4_ok(dX, dxs[0], dxs[1], dxs[2], L, dtype);
  if (dtype == HFTA_BF16) {
    if (v4) hipLaunchKernelGGL((maxpool_bwd_kernel<bf16_raw, 4>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((maxpool_bwd_kernel<bf16_raw, 1>), grid, dim3(256), 0, st, a);
  } else {
    if (v4) hipLaunchKernelGGL((maxpool_bwd_kernel<float, 4>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((maxpool_bwd_kernel<float, 1>), grid, dim3(256), 0, st, a);
  }
  return launch_status();
}

}  // extern "C"
