// Support operators of a per-point (segmentation) head on a concatenation of feature maps with a
// tiled, point-independent part (fusion rules table: the concatenation and tiling are element-wise
// in the model index, so they are expressed through strides; "Conv1d" row for the head itself).
//
//   * a k=1 convolution over [per-point features | tiled vector] = convolution over the per-point
//     features + a per-(model, sample, channel) value broadcast along the points
//     (hfta_add_sample_bias), whose adjoint is the sum over the points (hfta_sum_points);
//   * feature maps live as channel slices of one [Nb][B*Ctot][L] buffer: nothing is copied to
//     concatenate; the gradient of a slice is added onto the gradient that arrives from the next
//     layer (hfta_add_strided), the max-pool's backward onto the last slice in place
//     (hfta_maxpool_points_bwd_add);
//   * softmax cross-entropy over the class axis of a [Nb][B*K][L] score tensor, one term per point
//     (hfta_softmax_xent_points).
// All are HBM-bound row kernels: one workgroup per row (b, n, c) of L contiguous points, 8- or
// 16-byte accesses when every row allows it.
#include "bn_common.h"

using namespace hfta;

namespace {

struct RowArgs {
  const void* A; const void* Bt; void* Y;
  int64_t asb, asn, asc, bsb, bsn, bsc, ysb, ysn, ysc;
  int64_t ssb, ssn, ssc;          // strides of the [B][Nb][C] per-sample tensor
  int Nb, C, L;
};

// MODE 0: Y = A + S[b,n,c];  MODE 1: Y = A + Bt
template <typename T, int VEC, int MODE>
__global__ __launch_bounds__(256) void row_add_kernel(RowArgs p) {
  const int c = blockIdx.x, n = blockIdx.y, b = blockIdx.z;
  const T* a = reinterpret_cast<const T*>(p.A) + b * p.asb + n * p.asn + c * p.asc;
  T* y = reinterpret_cast<T*>(p.Y) + b * p.ysb + n * p.ysn + c * p.ysc;
  const T* bt = reinterpret_cast<const T*>(p.Bt);
  float s = 0.f;
  if (MODE == 0) s = Elem<T>::load(bt + b * p.ssb + n * p.ssn + c * p.ssc);
  else bt += b * p.bsb + n * p.bsn + c * p.bsc;
  for (int l = threadIdx.x * VEC; l < p.L; l += 256 * VEC) {
    float v[VEC], w[VEC];
    load_vec<T, VEC>(a + l, v);
    if (MODE == 1) load_vec<T, VEC>(bt + l, w);
#pragma unroll
    for (int e = 0; e < VEC; ++e) v[e] += MODE == 0 ? s : w[e];
    store_vec<T, VEC>(y + l, v);
  }
}

// S[b,n,c] = sum_l X[b,n,c,l]: a thread adds its strided share, then a fixed-order block reduction
template <typename T, int VEC>
__global__ __launch_bounds__(256) void sum_points_kernel(RowArgs p) {
  __shared__ float sh[4];
  const int c = blockIdx.x, n = blockIdx.y, b = blockIdx.z;
  const T* a = reinterpret_cast<const T*>(p.A) + b * p.asb + n * p.asn + c * p.asc;
  float acc = 0.f;
  for (int l = threadIdx.x * VEC; l < p.L; l += 256 * VEC) {
    float v[VEC];
    load_vec<T, VEC>(a + l, v);
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc += v[e];
  }
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0)
    Elem<T>::store(reinterpret_cast<T*>(p.Y) + b * p.ssb + n * p.ssn + c * p.ssc, (sh[0] + sh[1]) + (sh[2] + sh[3]));
}

struct PoolAddArgs {
  const void* dV; const int32_t* idx; void* dX;
  int64_t vsb, vsn, vsc, xsb, xsn, xsc;
  int Nb, C, L;
  int64_t rows;
};

template <typename T>
__global__ __launch_bounds__(256) void maxpool_bwd_add_kernel(PoolAddArgs p) {
  const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (row >= p.rows) return;
  const int c = (int)(row % p.C);
  const int64_t bn = row / p.C;
  const int n = (int)(bn % p.Nb), b = (int)(bn / p.Nb);
  const int64_t vo = b * p.vsb + n * p.vsn + c * p.vsc;
  const int at = min(max(p.idx[vo], 0), p.L - 1);
  T* x = reinterpret_cast<T*>(p.dX) + b * p.xsb + n * p.xsn + c * p.xsc + at;
  Elem<T>::store(x, Elem<T>::load(x) + Elem<T>::load(reinterpret_cast<const T*>(p.dV) + vo));
}

struct XentArgs {
  const void* logits; void* dlogits; const int32_t* labels; float* partial;
  int64_t lsb, lsn, lsc, dsb, dsn, dsc;
  int Nb, K, L, blocks;
};

// one thread per point; the K scores of a point are L elements apart, consecutive lanes read consecutive points
template <typename T>
__global__ __launch_bounds__(256) void xent_points_kernel(XentArgs p) {
  __shared__ float sh[4];
  const int n = blockIdx.y, b = blockIdx.z;
  const int l = blockIdx.x * 256 + threadIdx.x;
  float term = 0.f;
  if (l < p.L) {
    const T* z = reinterpret_cast<const T*>(p.logits) + b * p.lsb + n * p.lsn + l;
    T* dz = reinterpret_cast<T*>(p.dlogits) + b * p.dsb + n * p.dsn + l;
    const int lab = p.labels[((int64_t)b * p.Nb + n) * p.L + l];
    float mx = -INFINITY;
    for (int k = 0; k < p.K; ++k) mx = fmaxf(mx, Elem<T>::load(z + k * p.lsc));
    float se = 0.f;
    for (int k = 0; k < p.K; ++k) se += expf(Elem<T>::load(z + k * p.lsc) - mx);
    const float lse = mx + logf(se);
    const float inv = 1.f / ((float)p.Nb * (float)p.L);
    float zl = 0.f;
    for (int k = 0; k < p.K; ++k) {
      const float zk = Elem<T>::load(z + k * p.lsc);
      if (k == lab) zl = zk;
      Elem<T>::store(dz + k * p.dsc, (expf(zk - lse) - (k == lab ? 1.f : 0.f)) * inv);
    }
    term = lse - zl;
  }
  term = wave_sum(term);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = term;
  __syncthreads();
  if (threadIdx.x == 0)
    p.partial[((int64_t)b * p.Nb + n) * p.blocks + blockIdx.x] = (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

__global__ __launch_bounds__(256) void xent_points_reduce_kernel(const float* partial, float* loss, int parts, float inv) {
  __shared__ float sh[4];
  const float* src = partial + (int64_t)blockIdx.x * parts;
  float acc = 0.f;
  for (int i = threadIdx.x; i < parts; i += 256) acc += src[i];
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) loss[blockIdx.x] = ((sh[0] + sh[1]) + (sh[2] + sh[3])) * inv;
}

bool grid_ok(int B, int Nb, int C) { return C <= 2147483647 && Nb <= 65535 && B <= 65535; }

template <int MODE>
int launch_row_add(int B, int Nb, int C, int L, int dtype, const RowArgs& a, bool v4, hipStream_t st) {
  dim3 grid((unsigned)C, (unsigned)Nb, (unsigned)B);
#define HFTA_LAUNCH(T, V_) hipLaunchKernelGGL((row_add_kernel<T, V_, MODE>), grid, dim3(256), 0, st, a)
  if (dtype == HFTA_BF16) { if (v4) HFTA_LAUNCH(bf16_raw, 4); else HFTA_LAUNCH(bf16_raw, 1); }
  else { if (v4) HFTA_LAUNCH(float, 4); else HFTA_LAUNCH(float, 1); }
#undef HFTA_LAUNCH
  return launch_status();
}

}  // namespace

extern "C" {

int hfta_add_sample_bias(int B, int Nb, int C, int L, int dtype, const void* Z, const int64_t zs[4], const void* S,
                         const int64_t ss[3], void* Y, const int64_t ys[4], void* stream) {
  if (B <= 0 || Nb <= 0 || C <= 0 || L <= 0 || !valid_dtype(dtype) || !Z || !zs || !S || !ss || !Y || !ys) return HFTA_EINVAL;
  if (zs[3] != 1 || ys[3] != 1 || !grid_ok(B, Nb, C)) return HFTA_EUNSUPPORTED;
  RowArgs a{};
  a.A = Z; a.Bt = S; a.Y = Y;
  a.asb = zs[0]; a.asn = zs[1]; a.asc = zs[2]; a.ysb = ys[0]; a.ysn = ys[1]; a.ysc = ys[2];
  a.ssb = ss[0]; a.ssn = ss[1]; a.ssc = ss[2];
  a.Nb = Nb; a.C = C; a.L = L;
  return launch_row_add<0>(B, Nb, C, L, dtype, a, bn_vec4_ok(Z, zs, L, dtype) && bn_vec4_ok(Y, ys, L, dtype), as_stream(stream));
}

int hfta_add_strided(int B, int Nb, int C, int L, int dtype, const void* A, const int64_t as[4], const void* Bt,
                     const int64_t bs[4], void* Y, const int64_t ys[4], void* stream) {
  if (B <= 0 || Nb <= 0 || C <= 0 || L <= 0 || !valid_dtype(dtype) || !A || !as || !Bt || !bs || !Y || !ys) return HFTA_EINVAL;
  if (as[3] != 1 || bs[3] != 1 || ys[3] != 1 || !grid_ok(B, Nb, C)) return HFTA_EUNSUPPORTED;
  RowArgs a{};
  a.A = A; a.Bt = Bt; a.Y = Y;
  a.asb = as[0]; a.asn = as[1]; a.asc = as[2]; a.bsb = bs[0]; a.bsn = bs[1]; a.bsc = bs[2];
  a.ysb = ys[0]; a.ysn = ys[1]; a.ysc = ys[2];
  a.Nb = Nb; a.C = C; a.L = L;
  const bool v4 = bn_vec4_ok(A, as, L, dtype) && bn_vec4_ok(Bt, bs, L, dtype) && bn_vec4_ok(Y, ys, L, dtype);
  return launch_row_add<1>(B, Nb, C, L, dtype, a, v4, as_stream(stream));
}

int hfta_sum_points(int B, int Nb, int C, int L, int dtype, const void* X, const int64_t xs[4], void* S,
                    const int64_t ss[3], void* stream) {
  if (B <= 0 || Nb <= 0 || C <= 0 || L <= 0 || !valid_dtype(dtype) || !X || !xs || !S || !ss) return HFTA_EINVAL;
  if (xs[3] != 1 || !grid_ok(B, Nb, C)) return HFTA_EUNSUPPORTED;
  RowArgs a{};
  a.A = X; a.Y = S;
  a.asb = xs[0]; a.asn = xs[1]; a.asc = xs[2]; a.ssb = ss[0]; a.ssn = ss[1]; a.ssc = ss[2];
  a.Nb = Nb; a.C = C; a.L = L;
  dim3 grid((unsigned)C, (unsigned)Nb, (unsigned)B);
  hipStream_t st = as_stream(stream);
  const bool v4 = bn_vec4_ok(X, xs, L, dtype);
#define HFTA_LAUNCH(T, V_) hipLaunchKernelGGL((sum_points_kernel<T, V_>), grid, dim3(256), 0, st, a)
  if (dtype == HFTA_BF16) { if (v4) HFTA_LAUNCH(bf16_raw, 4); else HFTA_LAUNCH(bf16_raw, 1); }
  else { if (v4) HFTA_LAUNCH(float, 4); else HFTA_LAUNCH(float, 1); }
#undef HFTA_LAUNCH
  return launch_status();
}

int hfta_maxpool_points_bwd_add(int B, int Nb, int C, int L, int dtype, const void* dV, const int32_t* idx,
                                const int64_t vs[3], void* dX, const int64_t dxs[4], void* stream) {
  if (B <= 0 || Nb <= 0 || C <= 0 || L <= 0 || !valid_dtype(dtype) || !dV || !idx || !vs || !dX || !dxs) return HFTA_EINVAL;
  if (dxs[3] != 1) return HFTA_EUNSUPPORTED;
  PoolAddArgs a{dV, idx, dX, vs[0], vs[1], vs[2], dxs[0], dxs[1], dxs[2], Nb, C, L, (int64_t)B * Nb * C};
  const unsigned blocks = (unsigned)((a.rows + 255) / 256);
  if (dtype == HFTA_BF16) hipLaunchKernelGGL(maxpool_bwd_add_kernel<bf16_raw>, dim3(blocks), dim3(256), 0, as_stream(stream), a);
  else hipLaunchKernelGGL(maxpool_bwd_add_kernel<float>, dim3(blocks), dim3(256), 0, as_stream(stream), a);
  return launch_status();
}

size_t hfta_softmax_xent_points_workspace_bytes(int B, int Nb, int L) {
  if (B <= 0 || Nb <= 0 || L <= 0) return 0;
  return (size_t)B * Nb * ((L + 255) / 256) * sizeof(float);
}

int hfta_softmax_xent_points(int B, int Nb, int K, int L, int dtype, const void* logits, const int64_t ls[4],
                             const int32_t* labels, float* loss, void* dlogits, const int64_t ds[4], void* workspace,
                             size_t ws_bytes, void* stream) {
  if (B <= 0 || Nb <= 0 || K <= 0 || L <= 0 || !valid_dtype(dtype) || !logits || !ls || !labels || !loss || !dlogits || !ds)
    return HFTA_EINVAL;
  if (ls[3] != 1 || ds[3] != 1 || !grid_ok(B, Nb, 1)) return HFTA_EUNSUPPORTED;
  if (!workspace || ws_bytes < hfta_softmax_xent_points_workspace_bytes(B, Nb, L)) return HFTA_EWORKSPACE;
  const int blocks = (L + 255) / 256;
  XentArgs a{logits, dlogits, labels, (float*)workspace, ls[0], ls[1], ls[2], ds[0], ds[1], ds[2], Nb, K, L, blocks};
  dim3 grid((unsigned)blocks, (unsigned)Nb, (unsigned)B);
  hipStream_t st = as_stream(stream);
  if (dtype == HFTA_BF16) hipLaunchKernelGGL(xent_points_kernel<bf16_raw>, grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL(xent_points_kernel<float>, grid, dim3(256), 0, st, a);
  if (launch_status() != HFTA_OK) return HFTA_ELAUNCH;
  hipLaunchKernelGGL(xent_points_reduce_kernel, dim3((unsigned)B), dim3(256), 0, st, (const float*)workspace, loss,
                     Nb * blocks, 1.f / ((float)Nb * (float)L));
  return launch_status();
}

}  // extern "C"
