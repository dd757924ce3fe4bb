// Fused Linear and fused k=1 Conv1d: argument checking and mapping of the
// forward / data-gradient / weight-gradient forms onto the batched GEMM core,
// plus the bias-gradient reductions.
#include "gemm.h"
#include <mutex>

namespace hfta {
int conv1x1_stream_fwd(int B, int Nb, int Ci, int Co, int L, const void* X, const int64_t xs[4], const void* W,
                       const void* bias, void* Y, const int64_t ys[4], int act, float slope, hipStream_t st,
                       float* stat_part = nullptr, const float* in_gamma = nullptr, const float* in_beta = nullptr,
                       const float* in_mean = nullptr, const float* in_invstd = nullptr, int in_act = 0, float in_slope = 0.f);
// BatchNorm forward whose statistics come from per-slice partial sums (bn.hip)
int bn_fwd_from_partials(int B, int Nb, int C, int L, int dtype, const void* X, const int64_t xs[4], const float* gamma,
                         const float* beta, float eps, float momentum, float* running_mean, float* running_var,
                         float* save_mean, float* save_invstd, void* Y, const int64_t ys[4], int act, float slope,
                         const float* part, int parts, const void* shift, hipStream_t st);
bool conv1x1_bn_bwd_streams(int B, int Ci, int Co, int L, int dtype);
size_t conv1x1_bn_bwd_stream_bytes(int B, int Nb, int Ci, int Co, int L);
int conv1x1_bn_bwd_stream(int B, int Nb, int Ci, int Co, int L, const void* X, const int64_t xs[4], const void* W,
                          const void* Z, const int64_t zs[4], const void* dY, const int64_t dys[4], const float* gamma,
                          const float* beta, const float* save_mean, const float* save_invstd, void* dX,
                          const int64_t dxs[4], float* dW, float* dbias, float* dgamma, float* dbeta, int act, float slope,
                          void* workspace, hipStream_t st, const float* in_gamma = nullptr, const float* in_beta = nullptr,
                          const float* in_mean = nullptr, const float* in_invstd = nullptr, int in_act = 0, float in_slope = 0.f,
                          const float* sums = nullptr, float* in_sums = nullptr);
bool conv1x1_bn_bwd_stream_sums(int Ci);
int bn_stats_conv(int B, int Nb, int C, int L, int dtype, const void* X, const int64_t xs[4], const float* gamma,
                  const float* beta, float eps, float momentum, float* running_mean, float* running_var,
                  float* save_mean, float* save_invstd, hipStream_t st);
}

using namespace hfta;

namespace {

// dbias of the fused Linear: column sums of dY[b] ([M][Fy]); 64 columns x 4 row slices per block.
// Forward of a k=1 convolution with at most 4 input channels (the point coordinates): no matrix
// instruction pays for K = 3.  A thread owns four consecutive points, keeps their Ci inputs in
// registers and walks the output channels; consecutive lanes write consecutive 8-byte pieces of an
// output row.  HBM-bound: Co rows written once.
struct TinyKArgs {
  const bf16_raw* X; const bf16_raw* W; const bf16_raw* bias; bf16_raw* Y;
  int64_t xsb, xsn, xsc, ysb, ysn, ysc;
  int Ci, Co, L, act;
  float slope;
};
__global__ __launch_bounds__(256) void conv1x1_tinyk_kernel(TinyKArgs p) {
  __shared__ float wl[256][4];                           // Co <= 256 (host): weights of the model, then its bias
  __shared__ float bl[256];
  const int n = blockIdx.y, b = blockIdx.z;
  for (int o = threadIdx.x; o < p.Co; o += 256) {
#pragma unroll
    for (int c = 0; c < 4; ++c) wl[o][c] = c < p.Ci ? bf16_to_f32(p.W[((int64_t)b * p.Co + o) * p.Ci + c]) : 0.f;
    bl[o] = p.bias ? bf16_to_f32(p.bias[(int64_t)b * p.Co + o]) : 0.f;
  }
  __syncthreads();
  const int l = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (l >= p.L) return;
  const bf16_raw* x = p.X + b * p.xsb + n * p.xsn + l;
  float xv[4][4];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    uint2 raw = make_uint2(0u, 0u);
    if (c < p.Ci) raw = *reinterpret_cast<const uint2*>(x + c * p.xsc);
    xv[c][0] = __uint_as_float(raw.x << 16); xv[c][1] = __uint_as_float(raw.x & 0xffff0000u);
    xv[c][2] = __uint_as_float(raw.y << 16); xv[c][3] = __uint_as_float(raw.y & 0xffff0000u);
  }
  bf16_raw* y = p.Y + b * p.ysb + n * p.ysn + l;
#pragma unroll 4
  for (int o = 0; o < p.Co; ++o) {
    float acc[4];
    const float4 wo = *reinterpret_cast<const float4*>(wl[o]);
    const float wc[4] = {wo.x, wo.y, wo.z, wo.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[e] = 0.f;
#pragma unroll
    for (int c = 0; c < 4; ++c)                          // channels past Ci: weight and input are zero
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[e] = fmaf(wc[c], xv[c][e], acc[e]);
    const float bo = bl[o];
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[e] = apply_act(acc[e] + bo, p.act, p.slope);
    *reinterpret_cast<uint2*>(y + o * p.ysc) = make_uint2(pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3]));
  }
}

// Wt[b][c][o] = W[b][o][c] (a few tens of KB per model)
__global__ __launch_bounds__(256) void transpose_w_kernel(const bf16_raw* __restrict__ W, bf16_raw* __restrict__ Wt,
                                                          int Co, int Ci, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const int o = (int)(i % Co);
  const int64_t bc = i / Co;
  const int c = (int)(bc % Ci);
  const int64_t b = bc / Ci;
  Wt[i] = W[(b * Co + o) * Ci + c];
}

template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(const T* __restrict__ dY, float* __restrict__ out,
                                                    int M, int Fy) {
  __shared__ float part[4][64];
  const int b = blockIdx.y;
  const int col = blockIdx.x * 64 + (threadIdx.x & 63);
  const int slice = threadIdx.x >> 6;
  float s = 0.f;
  if (col < Fy) {
    const T* p = dY + (int64_t)b * M * Fy + col;
    for (int r = slice; r < M; r += 4) s += Elem<T>::load(p + (int64_t)r * Fy);
  }
  part[slice][threadIdx.x & 63] = s;
  __syncthreads();
  if (slice == 0 && col < Fy)
    out[(int64_t)b * Fy + col] = (part[0][threadIdx.x] + part[1][threadIdx.x]) + (part[2][threadIdx.x] + part[3][threadIdx.x]);
}

// The same with 16-byte loads: 1024 threads = 16 column groups (one 16-byte piece of a row each,
// so a row's pieces are contiguous) x 64 row lanes; row lanes are summed through LDS in a fixed
// order.  Needs Fy a multiple of the piece and 16-byte aligned rows.
template <typename T>
__global__ __launch_bounds__(1024) void colsum_vec_kernel(const uint4* __restrict__ dY, float* __restrict__ out,
                                                         int M, int Fy) {
  constexpr int N = 16 / sizeof(T);
  __shared__ float part[64][16 * N + 1];
  const int b = blockIdx.y;
  const int cg = threadIdx.x & 15, rl = threadIdx.x >> 4;
  const int vpr = Fy / N;
  const int v = blockIdx.x * 16 + cg;
  float acc[N];
#pragma unroll
  for (int e = 0; e < N; ++e) acc[e] = 0.f;
  if (v < vpr) {
    const uint4* p = dY + (int64_t)b * M * vpr + v;
#pragma unroll 4
    for (int r = rl; r < M; r += 64) {
      const uint4 q = p[(int64_t)r * vpr];
      if (sizeof(T) == 2) {
        const uint32_t wds[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          acc[(2 * i) % N] += __uint_as_float(wds[i] << 16);
          acc[(2 * i + 1) % N] += __uint_as_float(wds[i] & 0xffff0000u);
        }
      } else {
        acc[0] += __uint_as_float(q.x); acc[1 % N] += __uint_as_float(q.y);
        acc[2 % N] += __uint_as_float(q.z); acc[3 % N] += __uint_as_float(q.w);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < N; ++e) part[rl][cg * N + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < 16 * N) {
    const int col = blockIdx.x * 16 * N + threadIdx.x;
    if (col < Fy) {
      float s = 0.f;
      for (int r = 0; r < 64; ++r) s += part[r][threadIdx.x];
      out[(int64_t)b * Fy + col] = s;
    }
  }
}

// dbias of the fused conv: sum over (n, l) of dY[b, n, o, :]; one workgroup per (o, b).
template <typename T>
__global__ __launch_bounds__(256) void rowsum_kernel(const T* __restrict__ dY, float* __restrict__ out,
                                                    int Nb, int Co, int L, int64_t sb, int64_t sn, int64_t sc) {
  __shared__ float part[4];
  const int o = blockIdx.x, b = blockIdx.y;
  const T* base = dY + b * sb + o * sc;
  float s = 0.f;
  const int64_t total = (int64_t)Nb * L;
  for (int64_t i = threadIdx.x; i < total; i += 256) {
    const int n = (int)(i / L), l = (int)(i - (int64_t)n * L);
    s += Elem<T>::load(base + n * sn + l);
  }
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) out[(int64_t)b * Co + o] = (part[0] + part[1]) + (part[2] + part[3]);
}

bool fits_i32(int64_t v) { return v > 0 && v <= 0x7fffffffLL; }

// Epilogue of the split forward of a Linear with few rows: Y = act(sum_s partial[s] + bias), the
// splits added in a fixed order; one thread per output element, consecutive threads on consecutive columns.
template <typename T>
__global__ __launch_bounds__(256) void splitk_bias_act_kernel(const float* __restrict__ partial, T* __restrict__ Y,
                                                              const T* __restrict__ bias, int64_t count, int MN, int N,
                                                              int splits, int act, float slope) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  float s = 0.f;
#pragma unroll 4
  for (int k = 0; k < splits; ++k) s += partial[(int64_t)k * count + i];
  if (bias) {
    const int64_t b = i / MN;
    s += Elem<T>::load(bias + b * N + (i - b * MN) % N);
  }
  Elem<T>::store(Y + i, apply_act(s, act, slope));
}

// Few rows, long reduction: one 128-row tile per model and column block leaves most of the chip
// idle and walks K in sequence; the reduction is cut into pieces of at least two k-tiles until
// about 256 workgroups exist.
int linear_fwd_splits(int B, int M, int Fx, int Fy, int dtype) {
  if (M > 64) return 1;
  const int bk = dtype == HFTA_BF16 ? GemmT<bf16_raw>::BK : GemmT<float>::BK;
  const int64_t tiles = (int64_t)((Fy + GEMM_BN - 1) / GEMM_BN) * B;
  const int tt = (Fx + bk - 1) / bk;
  int64_t want = (256 + tiles - 1) / tiles;
  if (want > tt / 2) want = tt / 2;
  if (want > 64) want = 64;
  return want < 2 ? 1 : (int)want;
}

GemmDesc base_desc(int dtype) {
  GemmDesc d{};
  d.S = 1; d.G0 = 1; d.G1 = 1;
  d.act = HFTA_ACT_NONE; d.slope = 0.f;
  d.dtype = dtype; d.out_f32 = false; d.splits = 1; d.partial = nullptr;
  d.bias = nullptr; d.bias_mode = 0; d.keep_partials = false;
  return d;
}

GemmDesc linear_dw_desc(int B, int M, int Fx, int Fy, int dtype, const void* X, const void* dY, float* dW) {
  GemmDesc d = base_desc(dtype);
  d.A = X; d.Bm = dY; d.C = dW;
  d.M = Fx; d.N = Fy; d.K = M; d.G0 = B;
  d.a_kc = false; d.a_ld = Fx; d.a_g0 = (int64_t)M * Fx;      // A[m=fx][k=row] = X[row][fx]
  d.b_kc = false; d.b_ld = Fy; d.b_g0 = (int64_t)M * Fy;
  d.c_ld = Fy; d.c_g0 = (int64_t)Fx * Fy;
  d.out_f32 = true;
  return d;
}

GemmDesc conv_dw_desc(int B, int Nb, int Ci, int Co, int L, int dtype, const void* X, const int64_t* xs,
                      const void* dY, const int64_t* dys, float* dW) {
  GemmDesc d = base_desc(dtype);
  d.A = dY; d.Bm = X; d.C = dW;
  d.M = Co; d.N = Ci; d.K = L; d.S = Nb; d.G0 = B;
  d.a_kc = true; d.a_ld = dys[2]; d.a_ss = dys[1]; d.a_g0 = dys[0];
  d.b_kc = true; d.b_ld = xs[2]; d.b_ss = xs[1]; d.b_g0 = xs[0];   // B[k=l][n=c] = X[c][l]
  d.c_ld = Ci; d.c_g0 = (int64_t)Co * Ci;
  d.out_f32 = true;
  return d;
}

// Built-in scratch of hfta_linear_fwd_static (split partials; every call on a GPU shares it).
__device__ __align__(256) unsigned char scratch[HFTA_LINEAR_FWD_STATIC_BYTES];

// Device address of `scratch` on the current device, looked up on the first call there.
float* static_scratch() {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr[kMaxDevices] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* q = nullptr;
    if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) {
      (void)hipGetLastError();
      return nullptr;
    }
    ptr[dev] = q;
  }
  return reinterpret_cast<float*>(ptr[dev]);
}

}  // namespace

extern "C" {

int hfta_linear_fwd(int B, int M, int Fx, int Fy, int dtype, const void* X, const void* W, const void* bias,
                    void* Y, int act, float act_slope, void* stream) {
  if (B <= 0 || M <= 0 || Fx <= 0 || Fy <= 0 || !X || !W || !Y || !valid_dtype(dtype) || !valid_act(act))
    return HFTA_EINVAL;
  if (!fits_i32((int64_t)M * Fx) || !fits_i32((int64_t)M * Fy) || !fits_i32((int64_t)Fx * Fy)) return HFTA_EINVAL;
  GemmDesc d = base_desc(dtype);
  d.A = X; d.Bm = W; d.C = Y;
  d.M = M; d.N = Fy; d.K = Fx; d.G0 = B;
  d.a_kc = true; d.a_ld = Fx; d.a_g0 = (int64_t)M * Fx;
  d.b_kc = false; d.b_ld = Fy; d.b_g0 = (int64_t)Fx * Fy;
  d.c_ld = Fy; d.c_g0 = (int64_t)M * Fy;
  d.bias = bias; d.bias_mode = 2; d.bias_g0 = Fy;
  d.act = act; d.slope = act_slope;
  return gemm_launch(d, as_stream(stream));
}

size_t hfta_linear_fwd_workspace_bytes(int B, int M, int Fx, int Fy, int dtype) {
  if (B <= 0 || M <= 0 || Fx <= 0 || Fy <= 0 || !valid_dtype(dtype)) return 0;
  const int splits = linear_fwd_splits(B, M, Fx, Fy, dtype);
  return splits > 1 ? (size_t)splits * B * M * Fy * sizeof(float) : 0;
}

// Split forward: fp32 partial products into `partial`, then the fixed-order sum with bias and act.
static int linear_fwd_split(int B, int M, int Fx, int Fy, int dtype, const void* X, const void* W, const void* bias,
                            void* Y, int act, float act_slope, int splits, float* partial, hipStream_t st) {
  GemmDesc d = base_desc(dtype);
  d.A = X; d.Bm = W; d.C = nullptr;
  d.M = M; d.N = Fy; d.K = Fx; d.G0 = B;
  d.a_kc = true; d.a_ld = Fx; d.a_g0 = (int64_t)M * Fx;
  d.b_kc = false; d.b_ld = Fy; d.b_g0 = (int64_t)Fx * Fy;
  d.c_ld = Fy; d.c_g0 = (int64_t)M * Fy;
  d.out_f32 = true; d.splits = splits; d.partial = partial; d.keep_partials = true;
  const int rc = gemm_launch(d, st);
  if (rc != HFTA_OK) return rc;
  const int64_t count = (int64_t)B * M * Fy;
  dim3 grid((unsigned)((count + 255) / 256));
  if (dtype == HFTA_BF16)
    hipLaunchKernelGGL(splitk_bias_act_kernel<bf16_raw>, grid, dim3(256), 0, st, d.partial, (bf16_raw*)Y,
                       (const bf16_raw*)bias, count, M * Fy, Fy, splits, act, act_slope);
  else
    hipLaunchKernelGGL(splitk_bias_act_kernel<float>, grid, dim3(256), 0, st, d.partial, (float*)Y,
                       (const float*)bias, count, M * Fy, Fy, splits, act, act_slope);
  return launch_status();
}

int hfta_linear_fwd_ws(int B, int M, int Fx, int Fy, int dtype, const void* X, const void* W, const void* bias,
                       void* Y, int act, float act_slope, void* workspace, size_t ws_bytes, void* stream) {
  if (B <= 0 || M <= 0 || Fx <= 0 || Fy <= 0 || !X || !W || !Y || !valid_dtype(dtype) || !valid_act(act))
    return HFTA_EINVAL;
  const int splits = linear_fwd_splits(B, M, Fx, Fy, dtype);
  if (splits <= 1) return hfta_linear_fwd(B, M, Fx, Fy, dtype, X, W, bias, Y, act, act_slope, stream);
  if (!fits_i32((int64_t)M * Fx) || !fits_i32((int64_t)M * Fy) || !fits_i32((int64_t)Fx * Fy)) return HFTA_EINVAL;
  const size_t need = (size_t)splits * B * M * Fy * sizeof(float);
  if (!workspace || ws_bytes < need) return HFTA_EWORKSPACE;
  return linear_fwd_split(B, M, Fx, Fy, dtype, X, W, bias, Y, act, act_slope, splits,
                          reinterpret_cast<float*>(workspace), as_stream(stream));
}

// hfta_linear_fwd_ws for callers that cannot allocate: the split partials live in `scratch`, a
// device array that is part of the library image.  In host code the array's name is only a
// handle; the memory is reached through the address hipGetSymbolAddress returns, looked up once
// per device (every GPU holds its own copy at its own address).
size_t hfta_linear_fwd_static_max_bytes(void) { return HFTA_LINEAR_FWD_STATIC_BYTES; }

int hfta_linear_fwd_static(int B, int M, int Fx, int Fy, int dtype, const void* X, const void* W, const void* bias,
                           void* Y, int act, float act_slope, void* stream) {
  if (B <= 0 || M <= 0 || Fx <= 0 || Fy <= 0 || !X || !W || !Y || !valid_dtype(dtype) || !valid_act(act))
    return HFTA_EINVAL;
  const int splits = linear_fwd_splits(B, M, Fx, Fy, dtype);
  if (splits <= 1) return hfta_linear_fwd(B, M, Fx, Fy, dtype, X, W, bias, Y, act, act_slope, stream);
  if (!fits_i32((int64_t)M * Fx) || !fits_i32((int64_t)M * Fy) || !fits_i32((int64_t)Fx * Fy)) return HFTA_EINVAL;
  const size_t need = (size_t)splits * B * M * Fy * sizeof(float);
  if (need > (size_t)HFTA_LINEAR_FWD_STATIC_BYTES) return HFTA_EWORKSPACE;   // beyond the built-in scratch
  float* partial = static_scratch();
  if (!partial) return HFTA_ELAUNCH;
  return linear_fwd_split(B, M, Fx, Fy, dtype, X, W, bias, Y, act, act_slope, splits, partial, as_stream(stream));
}

size_t hfta_linear_bwd_workspace_bytes(int B, int M, int Fx, int Fy, int dtype) {
  if (B <= 0 || M <= 0 || Fx <= 0 || Fy <= 0 || !valid_dtype(dtype)) return 0;
  GemmDesc d = linear_dw_desc(B, M, Fx, Fy, dtype, nullptr, nullptr, nullptr);
  return gemm_partial_bytes(d, gemm_pick_splits(d));
}

int hfta_linear_bwd(int B, int M, int Fx, int Fy, int dtype, const void* X, const void* W, const void* dY,
                    void* dX, float* dW, float* dbias, void* workspace, size_t ws_bytes, void* stream) {
  if (B <= 0 || M <= 0 || Fx <= 0 || Fy <= 0 || !dY || !valid_dtype(dtype)) return HFTA_EINVAL;
  if ((dX && !W) || (dW && !X)) return HFTA_EINVAL;
  if (!fits_i32((int64_t)M * Fx) || !fits_i32((int64_t)M * Fy) || !fits_i32((int64_t)Fx * Fy)) return HFTA_EINVAL;
  hipStream_t st = as_stream(stream);
  GemmDesc dw = linear_dw_desc(B, M, Fx, Fy, dtype, X, dY, dW);
  if (dW) {
    dw.splits = gemm_pick_splits(dw);
    const size_t need = gemm_partial_bytes(dw, dw.splits);
    if (need > 0 && (!workspace || ws_bytes < need)) return HFTA_EWORKSPACE;
    dw.partial = reinterpret_cast<float*>(workspace);
  }
  if (dX) {
    GemmDesc d = base_desc(dtype);
    d.A = dY; d.Bm = W; d.C = dX;
    d.M = M; d.N = Fx; d.K = Fy; d.G0 = B;
    d.a_kc = true; d.a_ld = Fy; d.a_g0 = (int64_t)M * Fy;
    d.b_kc = true; d.b_ld = Fy; d.b_g0 = (int64_t)Fx * Fy;    // B[k=fy][n=fx] = W[fx][fy]
    d.c_ld = Fx; d.c_g0 = (int64_t)M * Fx;
    int rc = gemm_launch(d, st);
    if (rc != HFTA_OK) return rc;
  }
  if (dW) {
    int rc = gemm_launch(dw, st);
    if (rc != HFTA_OK) return rc;
  }
  if (dbias) {
    dim3 grid((unsigned)((Fy + 63) / 64), (unsigned)B);
    const int epv = 16 / (int)dtype_size(dtype);
    if (Fy % epv == 0 && (reinterpret_cast<uintptr_t>(dY) & 15) == 0 && M >= 64) {
      dim3 vgrid((unsigned)((Fy / epv + 15) / 16), (unsigned)B);
      if (dtype == HFTA_BF16)
        hipLaunchKernelGGL(colsum_vec_kernel<bf16_raw>, vgrid, dim3(1024), 0, st, (const uint4*)dY, dbias, M, Fy);
      else
        hipLaunchKernelGGL(colsum_vec_kernel<float>, vgrid, dim3(1024), 0, st, (const uint4*)dY, dbias, M, Fy);
      return launch_status();
    }
    if (dtype == HFTA_BF16)
      hipLaunchKernelGGL(colsum_kernel<bf16_raw>, grid, dim3(256), 0, st, (const bf16_raw*)dY, dbias, M, Fy);
    else
      hipLaunchKernelGGL(colsum_kernel<float>, grid, dim3(256), 0, st, (const float*)dY, dbias, M, Fy);
    return launch_status();
  }
  return HFTA_OK;
}

static int check_conv1x1(int B, int Nb, int Ci, int Co, int L, int dtype) {
  if (B <= 0 || Nb <= 0 || Ci <= 0 || Co <= 0 || L <= 0 || !valid_dtype(dtype)) return HFTA_EINVAL;
  if (!fits_i32((int64_t)Ci * L) || !fits_i32((int64_t)Co * L) || !fits_i32((int64_t)Co * Ci)) return HFTA_EINVAL;
  if ((int64_t)B * Nb > 65535) return HFTA_EUNSUPPORTED;
  return HFTA_OK;
}

// stat_part / stat_done: see GemmDesc (only the GEMM path's persistent kernel can fill them)
static int conv1x1_fwd_impl(int B, int Nb, int Ci, int Co, int L, int dtype, const void* X, const int64_t xs[4],
                            const void* W, const void* bias, void* Y, const int64_t ys[4], int act, float act_slope,
                            void* stream, float* stat_part, bool* stat_done) {
  if (stat_done) *stat_done = false;
  int rc = check_conv1x1(B, Nb, Ci, Co, L, dtype);
  if (rc != HFTA_OK) return rc;
  if (!X || !W || !Y || !xs || !ys || !valid_act(act)) return HFTA_EINVAL;
  if (xs[3] != 1 || ys[3] != 1) return HFTA_EUNSUPPORTED;
  auto al8 = [](const void* q, const int64_t* st) {
    return reinterpret_cast<uintptr_t>(q) % 8 == 0 && st[0] % 4 == 0 && st[1] % 4 == 0 && st[2] % 4 == 0;
  };
  if (dtype == HFTA_BF16 && Ci <= 4 && Co <= 256 && L % 4 == 0 && al8(X, xs) && al8(Y, ys) && Nb <= 65535 && B <= 65535) {
    TinyKArgs a{(const bf16_raw*)X, (const bf16_raw*)W, (const bf16_raw*)bias, (bf16_raw*)Y, xs[0], xs[1], xs[2],
                ys[0], ys[1], ys[2], Ci, Co, L, act, act_slope};
    dim3 grid((unsigned)((L / 4 + 255) / 256), (unsigned)Nb, (unsigned)B);
    hipLaunchKernelGGL(conv1x1_tinyk_kernel, grid, dim3(256), 0, as_stream(stream), a);
    return launch_status();
  }
  if (dtype == HFTA_BF16) {   // wide layer, few input channels: streaming kernel
    rc = hfta::conv1x1_stream_fwd(B, Nb, Ci, Co, L, X, xs, W, bias, Y, ys, act, act_slope, as_stream(stream));
    if (rc != HFTA_EUNSUPPORTED) return rc;
  }
  GemmDesc d = base_desc(dtype);
  d.A = W; d.Bm = X; d.C = Y;
  d.M = Co; d.N = L; d.K = Ci; d.G0 = B; d.G1 = Nb;
  d.a_kc = true; d.a_ld = Ci; d.a_g0 = (int64_t)Co * Ci; d.a_g1 = 0;
  d.b_kc = false; d.b_ld = xs[2]; d.b_g0 = xs[0]; d.b_g1 = xs[1];
  d.c_ld = ys[2]; d.c_g0 = ys[0]; d.c_g1 = ys[1];
  d.bias = bias; d.bias_mode = 1; d.bias_g0 = Co; d.bias_g1 = 0;
  d.act = act; d.slope = act_slope;
  d.stat_part = stat_part; d.stat_done = stat_done;
  return gemm_launch(d, as_stream(stream));
}

int hfta_conv1x1_fwd(int B, int Nb, int Ci, int Co, int L, int dtype, const void* X, const int64_t xs[4],
                     const void* W, const void* bias, void* Y, const int64_t ys[4], int act, float act_slope,
                     void* stream) {
  return conv1x1_fwd_impl(B, Nb, Ci, Co, L, dtype, X, xs, W, bias, Y, ys, act, act_slope, stream, nullptr, nullptr);
}

// A k=1 convolution over [per-point maps | a vector tiled along the points] is the convolution over the
// per-point maps plus, per sample, the tiled vector's product with its block of the weights: that
// per-(sample, channel) term enters here as the accumulators' bias, so the sum is stored (rounded) once
// and no pass over Y adds it afterwards.
int hfta_conv1x1_fwd_sample_bias(int B, int Nb, int Ci, int Co, int L, int dtype, const void* X, const int64_t xs[4],
                                 const void* W, const void* S, const int64_t ss[3], void* Y, const int64_t ys[4], int act,
                                 float act_slope, void* stream) {
  int rc = check_conv1x1(B, Nb, Ci, Co, L, dtype);
  if (rc != HFTA_OK) return rc;
  if (!X || !W || !S || !Y || !xs || !ss || !ys || !valid_act(act)) return HFTA_EINVAL;
  if (xs[3] != 1 || ys[3] != 1 || ss[2] != 1) return HFTA_EUNSUPPORTED;
  GemmDesc d = base_desc(dtype);
  d.A = W; d.Bm = X; d.C = Y;
  d.M = Co; d.N = L; d.K = Ci; d.G0 = B; d.G1 = Nb;
  d.a_kc = true; d.a_ld = Ci; d.a_g0 = (int64_t)Co * Ci; d.a_g1 = 0;
  d.b_kc = false; d.b_ld = xs[2]; d.b_g0 = xs[0]; d.b_g1 = xs[1];
  d.c_ld = ys[2]; d.c_g0 = ys[0]; d.c_g1 = ys[1];
  d.bias = S; d.bias_mode = 1; d.bias_g0 = ss[0]; d.bias_g1 = ss[1];
  d.act = act; d.slope = act_slope;
  return gemm_launch(d, as_stream(stream));
}

// Conv1d k=1 + training-mode BatchNorm + activation.  When the streaming kernel takes the layer, its
// epilogue leaves per-slice sums of the stored values in the workspace and the BatchNorm reads Z
// once (normalisation only); otherwise the two operators run one after the other.
size_t hfta_conv1x1_bn_fwd_workspace_bytes(int B, int Nb, int Ci, int Co, int L, int dtype) {
  if (check_conv1x1(B, Nb, Ci, Co, L, dtype) != HFTA_OK || dtype != HFTA_BF16) return 0;
  return (size_t)B * Nb * ((L + 127) / 128) * Co * 2 * sizeof(float);
}

int hfta_conv1x1_bn_fwd(int B, int Nb, int Ci, int Co, int L, int dtype, const void* X, const int64_t xs[4],
                        const void* W, const void* bias, const float* gamma, const float* beta, float eps,
                        float momentum, float* running_mean, float* running_var, float* save_mean,
                        float* save_invstd, void* Z, const int64_t zs[4], void* Y, const int64_t ys[4], int act,
                        float act_slope, void* workspace, size_t ws_bytes, void* stream) {
  int rc = check_conv1x1(B, Nb, Ci, Co, L, dtype);
  if (rc != HFTA_OK) return rc;
  // Y == NULL: statistics only (the activated output is not formed; a consumer normalises Z on load)
  if (!X || !W || !Z || !xs || !zs || (Y && !ys) || !gamma || !beta || !save_mean || !save_invstd || !(eps >= 0.f))
    return HFTA_EINVAL;
  if ((running_mean == nullptr) != (running_var == nullptr)) return HFTA_EINVAL;
  if (act != HFTA_ACT_NONE && act != HFTA_ACT_RELU && act != HFTA_ACT_LEAKY) return HFTA_EUNSUPPORTED;
  if (xs[3] != 1 || zs[3] != 1 || (Y && ys[3] != 1)) return HFTA_EUNSUPPORTED;
  hipStream_t st = as_stream(stream);
  const size_t need = hfta_conv1x1_bn_fwd_workspace_bytes(B, Nb, Ci, Co, L, dtype);
  float* part = nullptr;
  if (dtype == HFTA_BF16 && need && workspace && ws_bytes >= need && reinterpret_cast<uintptr_t>(workspace) % 8 == 0) {
    part = reinterpret_cast<float*>(workspace);
    rc = hfta::conv1x1_stream_fwd(B, Nb, Ci, Co, L, X, xs, W, bias, Z, zs, HFTA_ACT_NONE, 0.f, st, part);
    if (rc == HFTA_OK)
      rc = hfta::bn_fwd_from_partials(B, Nb, Co, L, dtype, Z, zs, gamma, beta, eps, momentum, running_mean, running_var,
                                      save_mean, save_invstd, Y, ys, act, act_slope, part, Nb * ((L + 127) / 128), bias, st);
    if (rc != HFTA_EUNSUPPORTED) return rc;
  }
  // wide layers: the batched GEMM; its persistent 256 x 256 kernel leaves the same partial sums per 256-point tile
  bool stats = false;
  rc = conv1x1_fwd_impl(B, Nb, Ci, Co, L, dtype, X, xs, W, bias, Z, zs, HFTA_ACT_NONE, 0.f, stream, part, &stats);
  if (rc != HFTA_OK) return rc;
  if (stats) {
    rc = hfta::bn_fwd_from_partials(B, Nb, Co, L, dtype, Z, zs, gamma, beta, eps, momentum, running_mean, running_var,
                                    save_mean, save_invstd, Y, ys, act, act_slope, part, Nb * ((L + 255) / 256), bias, st);
    if (rc != HFTA_EUNSUPPORTED) return rc;
  }
  if (!Y)
    return hfta::bn_stats_conv(B, Nb, Co, L, dtype, Z, zs, gamma, beta, eps, momentum, running_mean, running_var, save_mean,
                               save_invstd, st);
  return hfta_bn_fwd(B, Nb, Co, L, dtype, Z, zs, gamma, beta, eps, momentum, running_mean, running_var, save_mean,
                     save_invstd, Y, ys, act, act_slope, stream);
}

// ---- the same pair of calls with the input given as the previous block's stored pre-activation ----
int hfta_conv1x1_bn_prenorm_supported(int B, int Nb, int Ci, int Co, int L, int dtype) {
  return check_conv1x1(B, Nb, Ci, Co, L, dtype) == HFTA_OK && dtype == HFTA_BF16 && Ci % 8 == 0 && Ci <= 128 && Co >= 64 &&
                 Co <= 128 && L % 4 == 0 && hfta::conv1x1_bn_bwd_streams(B, Ci, Co, L, dtype)
             ? 1 : 0;
}

static bool in_norm_ok(const float* g, const float* b, const float* m, const float* i, int act) {
  return g && b && m && i && (act == HFTA_ACT_NONE || act == HFTA_ACT_RELU || act == HFTA_ACT_LEAKY);
}

int hfta_conv1x1_bn_prenorm_fwd(int B, int Nb, int Ci, int Co, int L, int dtype, const void* Xpre, const int64_t xs[4],
                                const float* in_gamma, const float* in_beta, const float* in_mean, const float* in_invstd,
                                int in_act, float in_slope, const void* W, const void* bias, const float* gamma,
                                const float* beta, float eps, float momentum, float* running_mean, float* running_var,
                                float* save_mean, float* save_invstd, void* Z, const int64_t zs[4], void* Y,
                                const int64_t ys[4], int act, float act_slope, void* workspace, size_t ws_bytes,
                                void* stream) {
  int rc = check_conv1x1(B, Nb, Ci, Co, L, dtype);
  if (rc != HFTA_OK) return rc;
  if (!Xpre || !W || !Z || !xs || !zs || (Y && !ys) || !gamma || !beta || !save_mean || !save_invstd || !(eps >= 0.f))
    return HFTA_EINVAL;
  if (!in_gamma || !in_beta || !in_mean || !in_invstd) return HFTA_EINVAL;
  if ((running_mean == nullptr) != (running_var == nullptr)) return HFTA_EINVAL;
  if (!in_norm_ok(in_gamma, in_beta, in_mean, in_invstd, in_act)) return HFTA_EUNSUPPORTED;
  if (act != HFTA_ACT_NONE && act != HFTA_ACT_RELU && act != HFTA_ACT_LEAKY) return HFTA_EUNSUPPORTED;
  if (xs[3] != 1 || zs[3] != 1 || (Y && ys[3] != 1)) return HFTA_EUNSUPPORTED;
  if (!hfta_conv1x1_bn_prenorm_supported(B, Nb, Ci, Co, L, dtype)) return HFTA_EUNSUPPORTED;
  const size_t need = hfta_conv1x1_bn_fwd_workspace_bytes(B, Nb, Ci, Co, L, dtype);
  if (!workspace || ws_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 8 != 0) return HFTA_EWORKSPACE;
  hipStream_t st = as_stream(stream);
  float* part = reinterpret_cast<float*>(workspace);
  rc = hfta::conv1x1_stream_fwd(B, Nb, Ci, Co, L, Xpre, xs, W, bias, Z, zs, HFTA_ACT_NONE, 0.f, st, part, in_gamma, in_beta,
                                in_mean, in_invstd, in_act, in_slope);
  if (rc != HFTA_OK) return rc;
  return hfta::bn_fwd_from_partials(B, Nb, Co, L, dtype, Z, zs, gamma, beta, eps, momentum, running_mean, running_var,
                                    save_mean, save_invstd, Y, ys, act, act_slope, part, Nb * ((L + 127) / 128), bias, st);
}

// The data gradient of a narrow layer (Co <= 128, or Co <= 256 under at least 512 inputs) is a k=1 convolution of dY with the transposed
// weights: it takes the streaming forward kernel once W^T [B][Ci][Co] has been written to the workspace.
static bool dx_streams(int Ci, int Co, int L, int dtype) {
  return dtype == HFTA_BF16 && Co % 8 == 0 && L % 4 == 0 && ((Co <= 128 && Ci >= 64) || (Co <= 256 && Ci >= 512));
}
static size_t wt_offset(size_t partial_bytes) { return (partial_bytes + 255) & ~(size_t)255; }

size_t hfta_conv1x1_bwd_workspace_bytes(int B, int Nb, int Ci, int Co, int L, int dtype) {
  if (check_conv1x1(B, Nb, Ci, Co, L, dtype) != HFTA_OK) return 0;
  const int64_t unit[4] = {(int64_t)Ci * L, (int64_t)B * Ci * L, L, 1};
  GemmDesc d = conv_dw_desc(B, Nb, Ci, Co, L, dtype, nullptr, unit, nullptr, unit, nullptr);
  const size_t part = gemm_partial_bytes(d, gemm_pick_splits(d));
  return dx_streams(Ci, Co, L, dtype) ? wt_offset(part) + (size_t)B * Ci * Co * 2 : part;
}

int hfta_conv1x1_bwd(int B, int Nb, int Ci, int Co, int L, int dtype, const void* X, const int64_t xs[4],
                     const void* W, const void* dY, const int64_t dys[4], void* dX, const int64_t dxs[4],
                     float* dW, float* dbias, void* workspace, size_t ws_bytes, void* stream) {
  int rc = check_conv1x1(B, Nb, Ci, Co, L, dtype);
  if (rc != HFTA_OK) return rc;
  if (!dY || !dys) return HFTA_EINVAL;
  if ((dX && (!W || !dxs)) || (dW && (!X || !xs))) return HFTA_EINVAL;
  if (dys[3] != 1 || (dX && dxs[3] != 1) || (dW && xs[3] != 1)) return HFTA_EUNSUPPORTED;
  hipStream_t st = as_stream(stream);
  GemmDesc dw{};
  if (dW) {
    dw = conv_dw_desc(B, Nb, Ci, Co, L, dtype, X, xs, dY, dys, dW);
    dw.splits = gemm_pick_splits(dw);
    const size_t need = gemm_partial_bytes(dw, dw.splits);
    if (need > 0 && (!workspace || ws_bytes < need)) return HFTA_EWORKSPACE;
    dw.partial = reinterpret_cast<float*>(workspace);
  }
  bool dx_done = false;
  if (dX && dx_streams(Ci, Co, L, dtype) && workspace) {
    const size_t off = wt_offset(dW ? gemm_partial_bytes(dw, dw.splits) : 0);
    const size_t bytes = (size_t)B * Ci * Co * 2;
    if (ws_bytes >= off + bytes && reinterpret_cast<uintptr_t>(workspace) % 256 == 0) {
      bf16_raw* wt = reinterpret_cast<bf16_raw*>(reinterpret_cast<unsigned char*>(workspace) + off);
      const int64_t n = (int64_t)B * Ci * Co;
      hipLaunchKernelGGL(transpose_w_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                         (const bf16_raw*)W, wt, Co, Ci, n);
      rc = hfta::conv1x1_stream_fwd(B, Nb, Co, Ci, L, dY, dys, wt, nullptr, dX, dxs, HFTA_ACT_NONE, 0.f, st);
      if (rc == HFTA_OK) dx_done = true;
      else if (rc != HFTA_EUNSUPPORTED) return rc;
    }
  }
  if (dX && !dx_done) {
    GemmDesc d = base_desc(dtype);
    d.A = W; d.Bm = dY; d.C = dX;
    d.M = Ci; d.N = L; d.K = Co; d.G0 = B; d.G1 = Nb;
    d.a_kc = false; d.a_ld = Ci; d.a_g0 = (int64_t)Co * Ci; d.a_g1 = 0;   // A[m=c][k=o] = W[o][c]
    d.b_kc = false; d.b_ld = dys[2]; d.b_g0 = dys[0]; d.b_g1 = dys[1];
    d.c_ld = dxs[2]; d.c_g0 = dxs[0]; d.c_g1 = dxs[1];
    rc = gemm_launch(d, st);
    if (rc != HFTA_OK) return rc;
  }
  if (dW) {
    rc = gemm_launch(dw, st);
    if (rc != HFTA_OK) return rc;
  }
  if (dbias) {
    dim3 grid((unsigned)Co, (unsigned)B);
    if (dtype == HFTA_BF16)
      hipLaunchKernelGGL(rowsum_kernel<bf16_raw>, grid, dim3(256), 0, st, (const bf16_raw*)dY, dbias, Nb, Co, L,
                         dys[0], dys[1], dys[2]);
    else
      hipLaunchKernelGGL(rowsum_kernel<float>, grid, dim3(256), 0, st, (const float*)dY, dbias, Nb, Co, L,
                         dys[0], dys[1], dys[2]);
    return launch_status();
  }
  return HFTA_OK;
}


// BatchNorm backward + k=1 convolution backward in one call.  Shapes the one-pass kernel takes need
// its constants and partials only; every other case runs the two single operators with dz in the
// workspace: [dz, 256-byte aligned size][the convolution backward's own workspace].
static size_t cbb_fallback_dz_bytes(int B, int Nb, int Co, int L, int dtype) {
  return wt_offset((size_t)B * Nb * Co * L * dtype_size(dtype));
}

int hfta_conv1x1_bn_bwd_one_pass(int B, int Nb, int Ci, int Co, int L, int dtype) {
  return check_conv1x1(B, Nb, Ci, Co, L, dtype) == HFTA_OK && hfta::conv1x1_bn_bwd_streams(B, Ci, Co, L, dtype) ? 1 : 0;
}

size_t hfta_conv1x1_bn_bwd_workspace_bytes(int B, int Nb, int Ci, int Co, int L, int dtype) {
  if (check_conv1x1(B, Nb, Ci, Co, L, dtype) != HFTA_OK) return 0;
  if (hfta::conv1x1_bn_bwd_streams(B, Ci, Co, L, dtype)) return hfta::conv1x1_bn_bwd_stream_bytes(B, Nb, Ci, Co, L);
  return cbb_fallback_dz_bytes(B, Nb, Co, L, dtype) + hfta_conv1x1_bwd_workspace_bytes(B, Nb, Ci, Co, L, dtype);
}

int hfta_conv1x1_bn_bwd(int B, int Nb, int Ci, int Co, int L, int dtype, const void* X, const int64_t xs[4],
                        const void* W, const void* Z, const int64_t zs[4], const void* dY, const int64_t dys[4],
                        const float* gamma, const float* beta, const float* save_mean, const float* save_invstd,
                        void* dX, const int64_t dxs[4], float* dW, float* dbias, float* dgamma, float* dbeta,
                        const float* sums, int act, float act_slope, void* workspace, size_t ws_bytes, void* stream) {
  int rc = check_conv1x1(B, Nb, Ci, Co, L, dtype);
  if (rc != HFTA_OK) return rc;
  if (!X || !xs || !Z || !zs || !dY || !dys || !gamma || !beta || !save_mean || !save_invstd || !dW || !dgamma || !dbeta)
    return HFTA_EINVAL;
  if (dX && (!W || !dxs)) return HFTA_EINVAL;
  if (act != HFTA_ACT_NONE && act != HFTA_ACT_RELU && act != HFTA_ACT_LEAKY) return HFTA_EUNSUPPORTED;
  if (xs[3] != 1 || zs[3] != 1 || dys[3] != 1 || (dX && dxs[3] != 1)) return HFTA_EUNSUPPORTED;
  hipStream_t st = as_stream(stream);
  if (hfta::conv1x1_bn_bwd_streams(B, Ci, Co, L, dtype)) {
    if (!workspace || ws_bytes < hfta::conv1x1_bn_bwd_stream_bytes(B, Nb, Ci, Co, L)) return HFTA_EWORKSPACE;
    rc = hfta::conv1x1_bn_bwd_stream(B, Nb, Ci, Co, L, X, xs, W, Z, zs, dY, dys, gamma, beta, save_mean, save_invstd,
                                     dX, dxs, dW, dbias, dgamma, dbeta, act, act_slope, workspace, st, nullptr, nullptr, nullptr,
                                     nullptr, 0, 0.f, sums, nullptr);
    if (rc != HFTA_EUNSUPPORTED) return rc;
  }
  const size_t dzb = cbb_fallback_dz_bytes(B, Nb, Co, L, dtype);
  const size_t need = dzb + hfta_conv1x1_bwd_workspace_bytes(B, Nb, Ci, Co, L, dtype);
  if (!workspace || ws_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return HFTA_EWORKSPACE;
  const int64_t ds[4] = {(int64_t)Co * L, (int64_t)B * Co * L, L, 1};
  float* sink = nullptr;
  rc = hfta_bn_bwd(B, Nb, Co, L, dtype, Z, zs, dY, dys, gamma, beta, save_mean, save_invstd, workspace, ds, dgamma, dbeta,
                   dbias ? dbias : sink, act, act_slope, stream);
  if (rc != HFTA_OK) return rc;
  unsigned char* rest = reinterpret_cast<unsigned char*>(workspace) + dzb;
  return hfta_conv1x1_bwd(B, Nb, Ci, Co, L, dtype, X, xs, W, workspace, ds, dX, dxs, dW, nullptr, rest, ws_bytes - dzb, stream);
}


int hfta_conv1x1_bn_prenorm_bwd_gives_sums(int B, int Nb, int Ci, int Co, int L, int dtype) {
  return hfta_conv1x1_bn_prenorm_supported(B, Nb, Ci, Co, L, dtype) && hfta::conv1x1_bn_bwd_stream_sums(Ci) ? 1 : 0;
}

int hfta_conv1x1_bn_prenorm_bwd(int B, int Nb, int Ci, int Co, int L, int dtype, const void* Xpre, const int64_t xs[4],
                                const float* in_gamma, const float* in_beta, const float* in_mean, const float* in_invstd,
                                int in_act, float in_slope, const void* W, const void* Z, const int64_t zs[4],
                                const void* dY, const int64_t dys[4], const float* gamma, const float* beta,
                                const float* save_mean, const float* save_invstd, void* dX, const int64_t dxs[4],
                                float* dW, float* dbias, float* dgamma, float* dbeta, const float* sums, float* in_sums,
                                int act, float act_slope, void* workspace, size_t ws_bytes, void* stream) {
  int rc = check_conv1x1(B, Nb, Ci, Co, L, dtype);
  if (rc != HFTA_OK) return rc;
  if (in_sums && !dX) return HFTA_EINVAL;
  if (in_sums && !hfta_conv1x1_bn_prenorm_bwd_gives_sums(B, Nb, Ci, Co, L, dtype)) return HFTA_EUNSUPPORTED;
  if (!Xpre || !xs || !Z || !zs || !dY || !dys || !gamma || !beta || !save_mean || !save_invstd || !dW || !dgamma || !dbeta)
    return HFTA_EINVAL;
  if (!in_gamma || !in_beta || !in_mean || !in_invstd) return HFTA_EINVAL;
  if (dX && (!W || !dxs)) return HFTA_EINVAL;
  if (!in_norm_ok(in_gamma, in_beta, in_mean, in_invstd, in_act)) return HFTA_EUNSUPPORTED;
  if (act != HFTA_ACT_NONE && act != HFTA_ACT_RELU && act != HFTA_ACT_LEAKY) return HFTA_EUNSUPPORTED;
  if (xs[3] != 1 || zs[3] != 1 || dys[3] != 1 || (dX && dxs[3] != 1)) return HFTA_EUNSUPPORTED;
  if (!hfta_conv1x1_bn_prenorm_supported(B, Nb, Ci, Co, L, dtype)) return HFTA_EUNSUPPORTED;
  if (!workspace || ws_bytes < hfta::conv1x1_bn_bwd_stream_bytes(B, Nb, Ci, Co, L)) return HFTA_EWORKSPACE;
  return hfta::conv1x1_bn_bwd_stream(B, Nb, Ci, Co, L, Xpre, xs, W, Z, zs, dY, dys, gamma, beta, save_mean, save_invstd, dX,
                                     dxs, dW, dbias, dgamma, dbeta, act, act_slope, workspace, as_stream(stream), in_gamma,
                                     in_beta, in_mean, in_invstd, in_act, in_slope, sums, in_sums);
}

}  // extern "C"
