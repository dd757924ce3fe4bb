// Fused Conv2d with groups = B as an implicit GEMM on the matrix cores.
//
// The B models' convolutions are one launch: the model index is a batch
// dimension of the GEMM, never a channel-mixing dimension (fusion rules table,
// row "Conv2d": grouped convolution with G = B).  No im2col buffer exists: the
// operand tiles are gathered from the image / gradient tensors while they are
// staged into LDS, then the same 128x128 MFMA tile loop as the batched GEMM core
// runs on them.
//
//   forward        per (b, n):  Y[o][pix]  = sum_k W[o][k]   * col(X)[k][pix],   k = (c, ky, kx)
//   data gradient  per (b, n) and output-parity class: see conv_dx_kernel below
//   weight grad    per b:       dW[o][j]   = sum_{n,pix} dY[o][pix] * col(X)[pix][j], j = (c, ky, kx)
//
// The weight gradient's reduction over (n, pix) is split across workgroups with
// fp32 partials summed in a fixed order.
#include "gemm.h"

namespace hfta {
int conv_ig_forward(int B, int Nb, int Ci, int Co, int H, int W, int kh, int kw, int stride, int pad, const void* X,
                    const void* Wt, const void* bias, void* Y, int act, float slope, void* ws, size_t ws_bytes, hipStream_t st);
size_t conv_ig_fwd_split_bytes(int B, int Nb, int Ci, int Co, int H, int W);
size_t conv_ig_dx_split_bytes(int B, int Nb, int Ci, int Co, int H, int W);
size_t conv_ig_dx_pack_bytes(int B, int Ci, int Co);
bool conv_ig_dx_supported(int Nb, int Ci, int Co, int H, int W, int kh, int kw, int stride, int pad);
int conv_ig_dx(int B, int Nb, int Ci, int Co, int H, int W, int kh, int kw, int stride, int pad, const void* Wt,
               const void* dY, void* dX, void* pack, void* split_ws, hipStream_t st);
bool conv_full_applies(int H, int W, int kh, int kw, int pad, int Ci, int Nb);
int conv_full_fwd(int B, int Nb, int Ci, int Co, int kh, int kw, int dtype, const void* X, const void* Wt, const void* bias, void* Y,
                  int act, float slope, hipStream_t st);
int conv_full_dx(int B, int Nb, int Ci, int Co, int kh, int kw, int dtype, const void* Wt, const void* dY, void* dX, hipStream_t st);
int conv_full_dw(int B, int Nb, int Ci, int Co, int kh, int kw, int dtype, const void* X, const void* dY, float* dW, hipStream_t st);
bool conv_dx_fewc_supported(int Nb, int B, int Ci, int Co, int H, int W, int kh, int kw, int stride, int pad);
int conv_dx_fewc(int B, int Nb, int Ci, int Co, int H, int W, const void* Wt, const void* dY, void* dX, hipStream_t st);
bool conv_ig_dw_supported(int Nb, int Ci, int Co, int H, int W, int kh, int kw, int stride, int pad);
int conv_ig_dw_splits(int B, int Nb, int Ci, int Co, int H, int W);
int conv_ig_dw(int B, int Nb, int Ci, int Co, int H, int W, int kh, int kw, int stride, int pad, const void* X,
               const void* dY, float* dW, float* partial, hipStream_t st);
}

using namespace hfta;

namespace {

struct FastDiv {
  int d, shift;  // shift >= 0 when d is a power of two
  __host__ static FastDiv make(int d) {
    FastDiv f{d, -1};
    if (d > 0 && (d & (d - 1)) == 0) { f.shift = 0; while ((1 << f.shift) < d) ++f.shift; }
    return f;
  }
  __device__ __forceinline__ int div(int x) const { return shift >= 0 ? (x >> shift) : (x / d); }
  __device__ __forceinline__ void divmod(int x, int& q, int& r) const { q = div(x); r = x - q * d; }
};

enum { CONV_FWD = 0, CONV_DX = 1, CONV_DW = 2 };

struct ConvArgs {
  const void* X;    // fwd/dW: input image; dX: unused
  const void* Wt;   // fwd/dX: weights
  const void* dY;   // dX/dW: output gradient
  void* Out;        // fwd: Y; dX: dX; dW: dW (fp32) or unused when splits > 1
  const void* bias;
  float* partial;
  int B, Nb, Ci, Co, H, W, Ho, Wo, kh, kw, stride, pad;
  int M, N, K, S;   // GEMM view; S = outer reduction segments (dW: Nb)
  int tiles_n, tiles_per_seg, total_tiles, splits;
  int act, a_vec, c_vec;
  float slope;
  FastDiv d_kw, d_khkw, d_wo, d_w;
};

// ---- gather helpers ---------------------------------------------------------
// forward / weight-gradient im2col element: X[n][b*Ci + c][s*y + ky - p][s*x + kx - p] or 0
template <typename T>
__device__ __forceinline__ T x_at(const ConvArgs& p, const T* xb /* X + (n*B*Ci + b*Ci)*H*W */, int c, int iy, int ix) {
  if ((unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W) return xb[((int64_t)c * p.H + iy) * p.W + ix];
  return T(0);
}
// data-gradient element: dY[n][b*Co + o][(iy + p - ky)/s][(ix + p - kx)/s] when both divisions are exact
template <typename T>
__device__ __forceinline__ T dy_at(const ConvArgs& p, const T* dyb, int o, int ty, int tx) {
  if (ty < 0 || tx < 0) return T(0);
  int y = ty, x = tx;
  if (p.stride != 1) {
    y = ty / p.stride; x = tx / p.stride;
    if (y * p.stride != ty || x * p.stride != tx) return T(0);
  }
  if (y < p.Ho && x < p.Wo) return dyb[((int64_t)o * p.Ho + y) * p.Wo + x];
  return T(0);
}

// Stages one 128 x BK operand tile whose rows are GEMM rows/columns and whose 16-byte groups run
// along k, in the same LDS layout the MFMA loop of the GEMM core reads.
template <typename T, int MODE>
__global__ __launch_bounds__(GEMM_THREADS) void conv_gemm_kernel(ConvArgs p) {
  constexpr int BK = GemmT<T>::BK, KG = GemmT<T>::KG, NV = GemmT<T>::NV, KQ = GemmT<T>::KQ;
  __shared__ __attribute__((aligned(16))) unsigned char smem[2][2][GEMM_TILE_BYTES];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int tile_m = blockIdx.x / p.tiles_n, tile_n = blockIdx.x % p.tiles_n;
  const int m0 = tile_m * GEMM_BM, n0 = tile_n * GEMM_BN;
  const int split = blockIdx.z % p.splits, g = blockIdx.z / p.splits;
  // fwd / dX: g = b * Nb + n ; dW: g = b
  const int b = MODE == CONV_DW ? g : g / p.Nb;
  const int nimg = MODE == CONV_DW ? 0 : g % p.Nb;
  const int64_t HW = (int64_t)p.H * p.W, HoWo = (int64_t)p.Ho * p.Wo;
  const int khkw = p.kh * p.kw;

  const T* X = reinterpret_cast<const T*>(p.X);
  const T* Wt = reinterpret_cast<const T*>(p.Wt);
  const T* dY = reinterpret_cast<const T*>(p.dY);

  const int t_begin = (int)((int64_t)p.total_tiles * split / p.splits);
  const int t_end = (int)((int64_t)p.total_tiles * (split + 1) / p.splits);

  f32x16_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // thread -> elements.  A side (k-contiguous groups): group ga of rows ra and ra + 64.
  const int ga = t & 3, ra = t >> 2;
  // B side: k-quad kq, n-group ng (NV consecutive GEMM columns)
  const int kq = t % KQ, ng = t / KQ;
  // loop-invariant decomposition of this thread's B columns
  int cn_a[NV], cn_b[NV], cn_c[NV];   // fwd: (y, x, -) ; dX: (iy, ix, -) ; dW: (c, ky, kx)
#pragma unroll
  for (int e = 0; e < NV; ++e) {
    const int n = n0 + ng * NV + e;
    if (MODE == CONV_FWD) { p.d_wo.divmod(n, cn_a[e], cn_b[e]); cn_c[e] = 0; }
    else if (MODE == CONV_DX) { p.d_w.divmod(n, cn_a[e], cn_b[e]); cn_c[e] = 0; }
    else { int r; p.d_khkw.divmod(n, cn_a[e], r); p.d_kw.divmod(r, cn_b[e], cn_c[e]); }
  }

  uint4 qa[2];
  uint2 qb[4];
  auto issue = [&](int tt) {
    const int seg = tt / p.tiles_per_seg;
    const int k0 = (tt - seg * p.tiles_per_seg) * BK;
    // ---------------- A operand
    {
      const int k = k0 + ga * KG;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int m = m0 + ra + 64 * h;
        T tmp[KG];
        if (MODE == CONV_FWD) {
          // W[b*Co + m][k], k-contiguous
          const T* src = Wt + ((int64_t)b * p.Co + m) * p.K + k;
          if (p.a_vec && m < p.M && k + KG <= p.K && (p.K % KG) == 0) {
            qa[h] = *reinterpret_cast<const uint4*>(src);
            continue;
          }
#pragma unroll
          for (int e = 0; e < KG; ++e) tmp[e] = (m < p.M && k + e < p.K) ? src[e] : T(0);
        } else if (MODE == CONV_DX) {
          // Wt[c = m][k = (o, tap)] = W[b*Co + o][c][tap]: runs of kh*kw taps are contiguous
          if (p.a_vec && m < p.M && k + KG <= p.K && (khkw % KG) == 0) {
            const int o = p.d_khkw.div(k), tap = k - o * khkw;
            qa[h] = *reinterpret_cast<const uint4*>(Wt + (((int64_t)b * p.Co + o) * p.Ci + m) * khkw + tap);
            continue;
          }
#pragma unroll
          for (int e = 0; e < KG; ++e) {
            const int kk = k + e;
            if (m < p.M && kk < p.K) {
              const int o = p.d_khkw.div(kk), tap = kk - o * khkw;
              tmp[e] = Wt[(((int64_t)b * p.Co + o) * p.Ci + m) * khkw + tap];
            } else tmp[e] = T(0);
          }
        } else {
          // dY[seg][b*Co + m][pix = k], k-contiguous
          const T* src = dY + (((int64_t)seg * p.B + b) * p.Co + m) * HoWo + k;
          if (p.a_vec && m < p.M && k + KG <= p.K && (HoWo % KG) == 0) {
            qa[h] = *reinterpret_cast<const uint4*>(src);
            continue;
          }
#pragma unroll
          for (int e = 0; e < KG; ++e) tmp[e] = (m < p.M && k + e < p.K) ? src[e] : T(0);
        }
        qa[h] = *reinterpret_cast<const uint4*>(tmp);
      }
    }
    // ---------------- B operand: 4 k x NV n gathered elements
    {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int k = k0 + 4 * kq + j;
        T tmp[NV];
        if (MODE == CONV_FWD) {
          const T* xb = X + ((int64_t)nimg * p.B + b) * p.Ci * HW;
          int c, r, ky, kx;
          p.d_khkw.divmod(k, c, r);
          p.d_kw.divmod(r, ky, kx);
#pragma unroll
          for (int e = 0; e < NV; ++e) {
            const int n = n0 + ng * NV + e;
            tmp[e] = (k < p.K && n < p.N) ? x_at<T>(p, xb, c, cn_a[e] * p.stride + ky - p.pad, cn_b[e] * p.stride + kx - p.pad) : T(0);
          }
        } else if (MODE == CONV_DX) {
          const T* dyb = dY + ((int64_t)nimg * p.B + b) * p.Co * HoWo;
          int o, r, ky, kx;
          p.d_khkw.divmod(k, o, r);
          p.d_kw.divmod(r, ky, kx);
#pragma unroll
          for (int e = 0; e < NV; ++e) {
            const int n = n0 + ng * NV + e;
            tmp[e] = (k < p.K && n < p.N) ? dy_at<T>(p, dyb, o, cn_a[e] + p.pad - ky, cn_b[e] + p.pad - kx) : T(0);
          }
        } else {
          const T* xb = X + ((int64_t)seg * p.B + b) * p.Ci * HW;
          int y, x;
          p.d_wo.divmod(k, y, x);
#pragma unroll
          for (int e = 0; e < NV; ++e) {
            const int n = n0 + ng * NV + e;
            tmp[e] = (k < p.K && n < p.N) ? x_at<T>(p, xb, cn_a[e], y * p.stride + cn_b[e] - p.pad, x * p.stride + cn_c[e] - p.pad) : T(0);
          }
        }
        qb[j] = *reinterpret_cast<const uint2*>(tmp);
      }
    }
  };
  auto stash = [&](int buf) {
    store_kc(smem[buf][0], qa, t);
    if (sizeof(T) == 2) store_nc_bf16(smem[buf][1], qb, t);
    else store_nc_f32(smem[buf][1], qb, t);
  };

  if (t_begin < t_end) {
    issue(t_begin);
    stash(0);
    __syncthreads();
    int buf = 0;
    for (int tt = t_begin; tt < t_end; ++tt) {
      const bool more = tt + 1 < t_end;
      if (more) issue(tt + 1);
      mma_tile<T>(acc, smem[buf][0], smem[buf][1], wm, wn, lane);
      if (more) stash(buf ^ 1);
      __syncthreads();
      buf ^= 1;
    }
  }

  if (MODE == CONV_DW) {
    // fp32 output [b][M][N] (contiguous), through the partial buffer when split
    float* base = p.splits > 1 ? p.partial + ((int64_t)split * p.B + b) * (int64_t)p.M * p.N
                               : reinterpret_cast<float*>(p.Out) + (int64_t)b * p.M * p.N;
    store_tile<float, T, false>(acc, &smem[0][0][0], base, p.N, p.M, p.N, m0, n0, nullptr, 0, HFTA_ACT_NONE, 0.f, p.c_vec, t);
    return;
  }
  // fwd: Y[n][b*Co + m][pix]; dX: dX[n][b*Ci + m][ipx]
  T* out = reinterpret_cast<T*>(p.Out) + (((int64_t)nimg * p.B + b) * p.M) * (int64_t)p.N;
  const T* bias = (MODE == CONV_FWD && p.bias) ? reinterpret_cast<const T*>(p.bias) + (int64_t)b * p.Co : nullptr;
  store_tile<T, T>(acc, &smem[0][0][0], out, p.N, p.M, p.N, m0, n0, bias, 1, MODE == CONV_FWD ? p.act : HFTA_ACT_NONE,
                   p.slope, p.c_vec, t);
}

// ---- data gradient (and ConvTranspose2d forward), decomposed by output parity ---------------
// For stride s the input pixels fall into s*s classes (iy mod s, ix mod s).  Inside a class only the
// taps ky = ry + s*jy, kx = rx + s*jx contribute (ry = (py + pad) mod s), and they read dY at
// (qy - jy + cy, qx - jx + cx) for the class pixel (qy, qx): a stride-1 correlation with a
// ceil(kh/s) x ceil(kw/s) kernel.  One GEMM per class (grid.y), K = Co * KJ * KJ instead of
// Co * kh * kw, i.e. no multiplications by the structural zeros of the strided transpose
// (4x fewer MFMAs and gathers for 4x4 / stride 2).
struct ConvDxArgs {
  const void* Wt; const void* dY; void* dX;
  const void* Wp;    // weights regrouped per parity class, [b][class][Ci][K] (k-contiguous), or nullptr
  int B, Nb, Ci, Co, H, W, Ho, Wo, kh, kw, stride, pad;
  int KJ;            // taps per class and axis: ceil(k / stride)
  int Hqm, Wqm;      // class pixel grid (maximum over classes)
  int M, N, K;       // Ci, Hqm * Wqm, Co * KJ * KJ
  int tiles_n, k_tiles;
  FastDiv d_kj, d_kjkj, d_wqm, d_s;
};

// Regroups the weights for conv_dx_kernel: Wp[b][class][m][k = (o, jy, jx)] = W[b][o][m][ry + s jy][rx + s jx]
// (zero where the tap falls outside the kernel), so that the data-gradient kernel reads its A operand
// in 16-byte pieces instead of gathering single taps.
template <typename T>
__global__ __launch_bounds__(256) void conv_dx_pack_w_kernel(ConvDxArgs p, T* __restrict__ Wp, int64_t count) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  const int kk = (int)(i % p.K);
  int64_t r = i / p.K;
  const int m = (int)(r % p.Ci); r /= p.Ci;
  const int ncls = p.stride * p.stride;
  const int cls = (int)(r % ncls), b = (int)(r / ncls);
  int py, px, o, rr, jy, jx;
  p.d_s.divmod(cls, py, px);
  const int ry = (py + p.pad) % p.stride, rx = (px + p.pad) % p.stride;
  p.d_kjkj.divmod(kk, o, rr);
  p.d_kj.divmod(rr, jy, jx);
  const int ky = ry + p.stride * jy, kx = rx + p.stride * jx;
  const T* Wt = reinterpret_cast<const T*>(p.Wt);
  Wp[i] = (ky < p.kh && kx < p.kw) ? Wt[(((int64_t)b * p.Co + o) * p.Ci + m) * (p.kh * p.kw) + ky * p.kw + kx] : T(0);
}

template <typename T, bool PACKED>
__global__ __launch_bounds__(GEMM_THREADS) void conv_dx_kernel(ConvDxArgs p) {
  constexpr int BK = GemmT<T>::BK, KG = GemmT<T>::KG, NV = GemmT<T>::NV, KQ = GemmT<T>::KQ;
  __shared__ __attribute__((aligned(16))) unsigned char smem[2][2][GEMM_TILE_BYTES];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int tile_m = blockIdx.x / p.tiles_n, tile_n = blockIdx.x % p.tiles_n;
  const int m0 = tile_m * GEMM_BM, n0 = tile_n * GEMM_BN;
  const int cls = blockIdx.y;
  int py, px;
  p.d_s.divmod(cls, py, px);
  const int ry = (py + p.pad) % p.stride, rx = (px + p.pad) % p.stride;
  const int cy = (py + p.pad - ry) / p.stride, cx = (px + p.pad - rx) / p.stride;
  const int Hq = (p.H - py + p.stride - 1) / p.stride, Wq = (p.W - px + p.stride - 1) / p.stride;
  const int b = blockIdx.z / p.Nb, nimg = blockIdx.z % p.Nb;
  const int khkw = p.kh * p.kw, kjkj = p.KJ * p.KJ;
  const int64_t HoWo = (int64_t)p.Ho * p.Wo;
  const T* Wt = reinterpret_cast<const T*>(p.Wt) + (int64_t)b * p.Co * p.Ci * khkw;
  const T* Wpk = PACKED ? reinterpret_cast<const T*>(p.Wp) + ((int64_t)b * gridDim.y + cls) * p.Ci * (int64_t)p.K : nullptr;
  const T* dyb = reinterpret_cast<const T*>(p.dY) + ((int64_t)nimg * p.B + b) * p.Co * HoWo;

  f32x16_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int ga = t & 3, ra = t >> 2;
  const int kq = t % KQ, ng = t / KQ;
  int qy[NV], qx[NV];
#pragma unroll
  for (int e = 0; e < NV; ++e) p.d_wqm.divmod(n0 + ng * NV + e, qy[e], qx[e]);
  // this thread's pixels sit side by side in one row of the class grid (bf16: four of them, read as one 8-byte piece)
  const bool row4 = sizeof(T) == 2 && p.Wqm % NV == 0 && qy[0] < Hq && qx[0] + NV <= Wq;

  uint4 qa[2];
  uint2 qb[4];
  auto issue = [&](int tt) {
    const int k0 = tt * BK;
    if (PACKED) {
      const int k = k0 + ga * KG;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int m = m0 + ra + 64 * h;
        qa[h] = (m < p.M && k + KG <= p.K) ? *reinterpret_cast<const uint4*>(Wpk + (int64_t)m * p.K + k) : make_uint4(0, 0, 0, 0);
      }
    } else {
      const int k = k0 + ga * KG;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int m = m0 + ra + 64 * h;
        T tmp[KG];
#pragma unroll
        for (int e = 0; e < KG; ++e) {
          const int kk = k + e;
          int o, r, jy, jx;
          p.d_kjkj.divmod(kk, o, r);
          p.d_kj.divmod(r, jy, jx);
          const int ky = ry + p.stride * jy, kx = rx + p.stride * jx;
          tmp[e] = (m < p.M && kk < p.K && ky < p.kh && kx < p.kw)
                       ? Wt[((int64_t)o * p.Ci + m) * khkw + ky * p.kw + kx] : T(0);
        }
        qa[h] = *reinterpret_cast<const uint4*>(tmp);
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = k0 + 4 * kq + j;
      int o, r, jy, jx;
      p.d_kjkj.divmod(k, o, r);
      p.d_kj.divmod(r, jy, jx);
      const bool tap_ok = k < p.K && ry + p.stride * jy < p.kh && rx + p.stride * jx < p.kw;
      const int y0 = qy[0] - jy + cy, x0 = qx[0] - jx + cx;
      if (row4 && tap_ok && (unsigned)y0 < (unsigned)p.Ho && x0 >= 0 && x0 + NV <= p.Wo) {
        // four neighbouring dY values of one row; the address is only element-aligned
        __builtin_memcpy(&qb[j], dyb + ((int64_t)o * p.Ho + y0) * p.Wo + x0, sizeof(uint2));
        continue;
      }
      T tmp[NV];
#pragma unroll
      for (int e = 0; e < NV; ++e) {
        const int y = qy[e] - jy + cy, x = qx[e] - jx + cx;
        tmp[e] = (tap_ok && qy[e] < Hq && qx[e] < Wq && (unsigned)y < (unsigned)p.Ho && (unsigned)x < (unsigned)p.Wo)
                     ? dyb[((int64_t)o * p.Ho + y) * p.Wo + x] : T(0);
      }
      qb[j] = *reinterpret_cast<const uint2*>(tmp);
    }
  };
  auto stash = [&](int buf) {
    store_kc(smem[buf][0], qa, t);
    if (sizeof(T) == 2) store_nc_bf16(smem[buf][1], qb, t);
    else store_nc_f32(smem[buf][1], qb, t);
  };

  issue(0);
  stash(0);
  __syncthreads();
  int buf = 0;
  for (int tt = 0; tt < p.k_tiles; ++tt) {
    const bool more = tt + 1 < p.k_tiles;
    if (more) issue(tt + 1);
    mma_tile<T>(acc, smem[buf][0], smem[buf][1], wm, wn, lane);
    if (more) stash(buf ^ 1);
    __syncthreads();
    buf ^= 1;
  }

  // scatter the class tile into dX[n][b*Ci + c][py + s*qy][px + s*qx]
  constexpr int ES = sizeof(T);
  constexpr int RP = ES == 2 ? 128 : 64;
  constexpr int PITCH = ES == 2 ? EPI_PITCH2 : EPI_PITCH4;
  unsigned char* lds = &smem[0][0][0];
  T* out = reinterpret_cast<T*>(p.dX) + ((int64_t)nimg * p.B + b) * p.Ci * (int64_t)p.H * p.W;
#pragma unroll 1
  for (int pass = 0; pass < 128 / RP; ++pass) {
    stage_acc<T, T>(acc, lds, pass, p.M, m0, (const T*)nullptr, HFTA_ACT_NONE, 0.f, t);
    __syncthreads();
#pragma unroll 1
    for (int id = t; id < RP * 128; id += GEMM_THREADS) {
      const int r = id >> 7, cN = id & 127;
      const int m = m0 + pass * RP + r, n = n0 + cN;
      if (m >= p.M) continue;
      int y, x;
      p.d_wqm.divmod(n, y, x);
      if (y >= Hq || x >= Wq) continue;
      out[((int64_t)m * p.H + (py + p.stride * y)) * p.W + (px + p.stride * x)] =
          *reinterpret_cast<const T*>(lds + r * PITCH + cN * ES);
    }
    __syncthreads();
  }
}

__global__ void conv_splitk_reduce_kernel(const float* __restrict__ partial, float* __restrict__ out, int64_t count, int splits) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  float s = 0.f;
  for (int k = 0; k < splits; ++k) s += partial[(int64_t)k * count + i];
  out[i] = s;
}

// dbias[b*Co + o] = sum over (n, pix) of dY[n][b*Co + o][pix]
template <typename T>
__global__ __launch_bounds__(256) void conv_dbias_kernel(const T* __restrict__ dY, float* __restrict__ out, int Nb, int K, int64_t HoWo) {
  __shared__ float part[4];
  const int k = blockIdx.x;
  float s = 0.f;
  const int64_t total = (int64_t)Nb * HoWo;
  for (int64_t i = threadIdx.x; i < total; i += 256) {
    const int64_t n = i / HoWo, r = i - n * HoWo;
    s += Elem<T>::load(dY + (n * K + k) * HoWo + r);
  }
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) out[k] = (part[0] + part[1]) + (part[2] + part[3]);
}

// ---- lowering through a column buffer ------------------------------------------
// With a caller-supplied workspace the convolution becomes one large GEMM per model on the
// batched GEMM kernels: the sample index is folded into the GEMM's column dimension
// (N = Nb * Ho * Wo), so small images fill the tiles, and the operands are plain matrices.
//   col[b][k = (c, ky, kx)][n * Ho*Wo + pix]          (im2col_kernel)
//   forward   Y[b]    = W[b] (Co x K)  * col[b]        -> written straight into [Nb][B*Co][Ho*Wo]
//   weights   dW[b]   = dYp[b] (Co x N) * col[b]^T
//   data      dcol[b] = W[b]^T * dYp[b] (fp32),  dX = col2im(dcol)   (col2im_kernel: a gather, no atomics;
//             the per-tap partial sums stay fp32 so dX is rounded to the storage type once)
// dYp[b][co][n * Ho*Wo + pix] is the output gradient repacked model- and channel-major.
template <typename T, int V>
__global__ __launch_bounds__(256) void im2col_kernel(const T* __restrict__ X, T* __restrict__ col, int B, int Nb, int Ci,
                                                    int H, int W, int Ho, int Wo, int kh, int kw, int stride, int pad,
                                                    FastDiv d_khkw, FastDiv d_kw, FastDiv d_wov, FastDiv d_rows) {
  // one thread per V consecutive output pixels of a row; grid.y = k, grid.z = b
  const int K = Ci * kh * kw;
  const int b = blockIdx.z, k = blockIdx.y;
  int c, r, ky, kx;
  d_khkw.divmod(k, c, r);
  d_kw.divmod(r, ky, kx);
  const int wov = Wo / V;                                  // vectors per output row
  const int64_t N = (int64_t)Nb * Ho * Wo;
  T* dst = col + ((int64_t)b * K + k) * N;
  const int total = Nb * Ho * wov;
  for (int i = blockIdx.x * 256 + threadIdx.x; i < total; i += gridDim.x * 256) {
    int row, xv, n, y;
    d_wov.divmod(i, row, xv);
    d_rows.divmod(row, n, y);
    const int iy = y * stride + ky - pad;
    const T* src = X + (((int64_t)n * B + b) * Ci + c) * H * W + (int64_t)iy * W;
    T v[V];
#pragma unroll
    for (int e = 0; e < V; ++e) {
      const int ix = (xv * V + e) * stride + kx - pad;
      v[e] = ((unsigned)iy < (unsigned)H && (unsigned)ix < (unsigned)W) ? src[ix] : T(0);
    }
    T* o = dst + ((int64_t)n * Ho + y) * Wo + xv * V;
    if (V * sizeof(T) == 16) *reinterpret_cast<uint4*>(o) = *reinterpret_cast<const uint4*>(v);
    else if (V * sizeof(T) == 8) *reinterpret_cast<uint2*>(o) = *reinterpret_cast<const uint2*>(v);
    else {
#pragma unroll
      for (int e = 0; e < V; ++e) o[e] = v[e];
    }
  }
}

// dYp[b][co][n*HoWo + pix] = dY[n][b*Co + co][pix]
template <typename T>
__global__ __launch_bounds__(256) void pack_dy_kernel(const T* __restrict__ dY, T* __restrict__ dYp, int B, int Nb, int Co,
                                                     int HoWo, int vec) {
  const int bc = blockIdx.z * Co + blockIdx.y;             // b * Co + co
  const int64_t N = (int64_t)Nb * HoWo;
  constexpr int LV = 16 / (int)sizeof(T);
  if (vec) {                                               // aligned, and whole 16-byte pieces stay inside one sample
    const int64_t nv = N / LV;
    const int vps = HoWo / LV;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nv; i += (int64_t)gridDim.x * 256) {
      const int n = (int)(i / vps), pv = (int)(i - (int64_t)n * vps);
      reinterpret_cast<uint4*>(dYp + (int64_t)bc * N)[i] =
          reinterpret_cast<const uint4*>(dY + ((int64_t)n * B * Co + bc) * HoWo)[pv];
    }
    return;
  }
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < N; i += (int64_t)gridDim.x * 256) {
    const int n = (int)(i / HoWo), pix = (int)(i - (int64_t)n * HoWo);
    dYp[(int64_t)bc * N + i] = dY[((int64_t)n * B * Co + bc) * HoWo + pix];
  }
}

// dX[n][b*Ci + c][iy][ix] = sum over the taps that reach (iy, ix) of dcol[b][(c, ky, kx)][n, y, x]
template <typename T>
__global__ __launch_bounds__(256) void col2im_kernel(const float* __restrict__ dcol, T* __restrict__ dX, int B, int Nb, int Ci,
                                                    int H, int W, int Ho, int Wo, int kh, int kw, int stride, int pad) {
  const int b = blockIdx.z, c = blockIdx.y;
  const int bc = b * Ci + c;
  const int64_t N = (int64_t)Nb * Ho * Wo;
  const int K = Ci * kh * kw;
  const float* src = dcol + ((int64_t)b * K + (int64_t)c * kh * kw) * N;
  const int64_t total = (int64_t)Nb * H * W;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int n = (int)(i / (H * W));
    const int r = (int)(i - (int64_t)n * H * W);
    const int iy = r / W, ix = r - iy * W;
    float s = 0.f;
    for (int ky = 0; ky < kh; ++ky) {
      const int ty = iy + pad - ky;
      if (ty < 0 || ty % stride != 0) continue;
      const int y = ty / stride;
      if (y >= Ho) continue;
      for (int kx = 0; kx < kw; ++kx) {
        const int tx = ix + pad - kx;
        if (tx < 0 || tx % stride != 0) continue;
        const int x = tx / stride;
        if (x >= Wo) continue;
        s += src[(int64_t)(ky * kw + kx) * N + ((int64_t)n * Ho + y) * Wo + x];
      }
    }
    Elem<T>::store(dX + ((int64_t)n * B * Ci + bc) * H * W + r, s);
  }
}

// LDS-staged forms of the two lowering kernels: a block owns one channel of one model for NI
// samples, so the image (im2col) or the kh*kw column-buffer rows (col2im) are read from memory
// once, in whole contiguous runs, and the kh*kw-fold reuse happens in LDS.
template <typename T, int V>
__global__ __launch_bounds__(256) void im2col_lds_kernel(const T* __restrict__ X, T* __restrict__ col, int B, int Nb, int Ci,
                                                        int H, int W, int Ho, int Wo, int kh, int kw, int stride, int pad,
                                                        int NI, int vec_in, FastDiv d_howo, FastDiv d_wo) {
  extern __shared__ __attribute__((aligned(16))) unsigned char conv_dyn_smem[];
  T* img = reinterpret_cast<T*>(conv_dyn_smem);             // [NI][H*W]
  const int b = blockIdx.z, c = blockIdx.y, n0 = blockIdx.x * NI;
  const int ni = min(NI, Nb - n0);
  const int HW = H * W, HoWo = Ho * Wo, taps = kh * kw;
  const int64_t N = (int64_t)Nb * HoWo;
  constexpr int LV = 16 / (int)sizeof(T);
  if (vec_in) {                                             // 16-byte aligned images of whole 16-byte pieces
    const int vpi = HW / LV;
    for (int i = threadIdx.x; i < ni * vpi; i += 256) {
      const int n = i / vpi, r = i - n * vpi;
      reinterpret_cast<uint4*>(img)[i] =
          reinterpret_cast<const uint4*>(X + (((int64_t)(n0 + n) * B + b) * Ci + c) * HW)[r];
    }
  } else {
    for (int i = threadIdx.x; i < ni * HW; i += 256) {
      const int n = i / HW, r = i - n * HW;
      img[i] = X[(((int64_t)(n0 + n) * B + b) * Ci + c) * HW + r];
    }
  }
  __syncthreads();
  const int cnt = ni * HoWo;                                // a multiple of V (host)
  for (int tap = 0; tap < taps; ++tap) {
    const int ky = tap / kw, kx = tap - ky * kw;
    T* dst = col + ((int64_t)b * Ci * taps + (int64_t)c * taps + tap) * N + (int64_t)n0 * HoWo;
    for (int i = threadIdx.x * V; i < cnt; i += 256 * V) {
      T v[V];
#pragma unroll
      for (int e = 0; e < V; ++e) {
        int n, p, y, x;
        d_howo.divmod(i + e, n, p);
        d_wo.divmod(p, y, x);
        const int iy = y * stride + ky - pad, ix = x * stride + kx - pad;
        v[e] = ((unsigned)iy < (unsigned)H && (unsigned)ix < (unsigned)W) ? img[n * HW + iy * W + ix] : T(0);
      }
      if (V * sizeof(T) == 16) *reinterpret_cast<uint4*>(dst + i) = *reinterpret_cast<const uint4*>(v);
      else if (V * sizeof(T) == 8) *reinterpret_cast<uint2*>(dst + i) = *reinterpret_cast<const uint2*>(v);
      else {
#pragma unroll
        for (int e = 0; e < V; ++e) dst[i + e] = v[e];
      }
    }
  }
}

template <typename T, int V>
__global__ __launch_bounds__(256) void col2im_lds_kernel(const float* __restrict__ dcol, T* __restrict__ dX, int B, int Nb, int Ci,
                                                        int H, int W, int Ho, int Wo, int kh, int kw, int stride, int pad,
                                                        int NI, FastDiv d_hw, FastDiv d_w, FastDiv d_s) {
  extern __shared__ __attribute__((aligned(16))) unsigned char conv_dyn_smem[];
  float* rows = reinterpret_cast<float*>(conv_dyn_smem);    // [kh*kw][NI*Ho*Wo], fp32 partial sums
  const int b = blockIdx.z, c = blockIdx.y, n0 = blockIdx.x * NI;
  const int ni = min(NI, Nb - n0);
  const int HW = H * W, HoWo = Ho * Wo, taps = kh * kw;
  const int64_t N = (int64_t)Nb * HoWo;
  const int seg = NI * HoWo, cnt = ni * HoWo;
  constexpr int LV = 4;
  for (int tap = 0; tap < taps; ++tap) {
    const float* src = dcol + ((int64_t)b * Ci * taps + (int64_t)c * taps + tap) * N + (int64_t)n0 * HoWo;
    if (HoWo % LV == 0) {
      for (int i = threadIdx.x; i < cnt / LV; i += 256)
        reinterpret_cast<uint4*>(rows + tap * seg)[i] = reinterpret_cast<const uint4*>(src)[i];
    } else {
      for (int i = threadIdx.x; i < cnt; i += 256) rows[tap * seg + i] = src[i];
    }
  }
  __syncthreads();
  const int out = ni * HW;                                  // a multiple of V (host)
  T* dst = dX + (((int64_t)n0 * B + b) * Ci + c) * HW;      // sample n at + n * B*Ci*HW
  for (int i = threadIdx.x * V; i < out; i += 256 * V) {
    T v[V];
    int n0e = 0, r0 = 0;
#pragma unroll
    for (int e = 0; e < V; ++e) {
      int n, r, iy, ix;
      d_hw.divmod(i + e, n, r);
      d_w.divmod(r, iy, ix);
      if (e == 0) { n0e = n; r0 = r; }
      float sum = 0.f;
      int qy, ry, qx, rx;
      d_s.divmod(iy + pad, qy, ry);                         // taps ky = ry, ry + s, ...: y = qy, qy - 1, ...
      d_s.divmod(ix + pad, qx, rx);
      for (int ky = ry, y = qy; ky < kh; ky += stride, --y) {
        if ((unsigned)y >= (unsigned)Ho) continue;
        for (int kx = rx, x = qx; kx < kw; kx += stride, --x) {
          if ((unsigned)x >= (unsigned)Wo) continue;
          sum += rows[(ky * kw + kx) * seg + n * HoWo + y * Wo + x];
        }
      }
      v[e] = Elem<T>::from_f32(sum);
    }
    T* d = dst + (int64_t)n0e * B * Ci * HW + r0;           // V | H*W: the V elements share a sample
    if (V * sizeof(T) == 16) *reinterpret_cast<uint4*>(d) = *reinterpret_cast<const uint4*>(v);
    else if (V * sizeof(T) == 8) *reinterpret_cast<uint2*>(d) = *reinterpret_cast<const uint2*>(v);
    else {
#pragma unroll
      for (int e = 0; e < V; ++e) d[e] = v[e];
    }
  }
}

struct ConvGeom { int Ho, Wo; };

int check_conv(int B, int Nb, int Ci, int Co, int H, int W, int kh, int kw, int stride, int pad, int dtype, ConvGeom* g) {
  if (B <= 0 || Nb <= 0 || Ci <= 0 || Co <= 0 || H <= 0 || W <= 0 || kh <= 0 || kw <= 0 || stride <= 0 || pad < 0 ||
      !valid_dtype(dtype))
    return HFTA_EINVAL;
  if (H + 2 * pad < kh || W + 2 * pad < kw) return HFTA_EINVAL;
  g->Ho = (H + 2 * pad - kh) / stride + 1;
  g->Wo = (W + 2 * pad - kw) / stride + 1;
  const int64_t lim = 0x7fffffffLL;
  if ((int64_t)Ci * kh * kw > lim || (int64_t)Ci * H * W > lim || (int64_t)Co * g->Ho * g->Wo > lim ||
      (int64_t)Co * kh * kw > lim || (int64_t)Nb * g->Ho * g->Wo > lim)
    return HFTA_EINVAL;
  if ((int64_t)B * Nb > 65535) return HFTA_EUNSUPPORTED;
  return HFTA_OK;
}

ConvArgs base_args(int B, int Nb, int Ci, int Co, int H, int W, int kh, int kw, int stride, int pad, ConvGeom g) {
  ConvArgs a{};
  a.B = B; a.Nb = Nb; a.Ci = Ci; a.Co = Co; a.H = H; a.W = W; a.Ho = g.Ho; a.Wo = g.Wo;
  a.kh = kh; a.kw = kw; a.stride = stride; a.pad = pad;
  a.S = 1; a.splits = 1; a.act = HFTA_ACT_NONE; a.slope = 0.f;
  a.d_kw = FastDiv::make(kw); a.d_khkw = FastDiv::make(kh * kw); a.d_wo = FastDiv::make(g.Wo); a.d_w = FastDiv::make(W);
  return a;
}

void finish_tiles(ConvArgs& a, int dtype) {
  const int BK = dtype == HFTA_BF16 ? GemmT<bf16_raw>::BK : GemmT<float>::BK;
  a.tiles_n = (a.N + GEMM_BN - 1) / GEMM_BN;
  a.tiles_per_seg = (a.K + BK - 1) / BK;
  a.total_tiles = a.S * a.tiles_per_seg;
}

int dw_splits(const ConvArgs& a) {
  const int64_t tiles = (int64_t)((a.M + GEMM_BM - 1) / GEMM_BM) * a.tiles_n * a.B;
  if (tiles >= 512 || a.total_tiles < 16) return 1;
  int64_t want = (1024 + tiles - 1) / tiles, cap = a.total_tiles / 8;
  if (want > cap) want = cap;
  if (want > 256) want = 256;
  if ((int64_t)a.B * want > 65535) want = 65535 / a.B;
  return want < 1 ? 1 : (int)want;
}

int store_bytes(const void* p, int64_t n, int es) {
  for (int w = 16; w >= 8; w >>= 1)
    if (reinterpret_cast<uintptr_t>(p) % w == 0 && n % (w / es) == 0) return w;
  return 0;
}

template <int MODE>
int launch_conv(ConvArgs a, int dtype, unsigned gz, hipStream_t st) {
  if (MODE == CONV_DW) a.c_vec = store_bytes(a.splits > 1 ? (const void*)a.partial : a.Out, a.N, 4);
  else a.c_vec = store_bytes(a.Out, a.N, (int)dtype_size(dtype));
  dim3 grid((unsigned)(((a.M + GEMM_BM - 1) / GEMM_BM) * a.tiles_n), 1, gz);
  if (dtype == HFTA_BF16) hipLaunchKernelGGL((conv_gemm_kernel<bf16_raw, MODE>), grid, dim3(GEMM_THREADS), 0, st, a);
  else hipLaunchKernelGGL((conv_gemm_kernel<float, MODE>), grid, dim3(GEMM_THREADS), 0, st, a);
  return launch_status();
}


// ---- host side of the lowered path ---------------------------------------------
size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct Lowered {
  int64_t K, N, HoWo;
  size_t col_bytes, dcol_bytes, dyp_bytes, part_bytes;   // dcol: fp32 per-tap partial sums of the data gradient
};

GemmDesc lowered_dw_desc(int B, int Co, const Lowered& L, int dtype) {
  GemmDesc d{};
  d.S = 1; d.G0 = B; d.G1 = 1;
  d.M = Co; d.N = (int)L.K; d.K = (int)L.N;
  d.a_kc = true; d.a_ld = L.N; d.a_g0 = (int64_t)Co * L.N;
  d.b_kc = true; d.b_ld = L.N; d.b_g0 = L.K * L.N;
  d.c_ld = L.K; d.c_g0 = (int64_t)Co * L.K;
  d.act = HFTA_ACT_NONE; d.dtype = dtype; d.out_f32 = true; d.splits = 1;
  return d;
}

bool lowered_sizes(int B, int Nb, int Ci, int Co, ConvGeom g, int kh, int kw, int dtype, Lowered* L) {
  L->K = (int64_t)Ci * kh * kw;
  L->HoWo = (int64_t)g.Ho * g.Wo;
  L->N = (int64_t)Nb * L->HoWo;
  if (L->N > 0x7fffffffLL || L->K > 0x7fffffffLL || L->K * L->N > ((int64_t)1 << 40) || B > 65535 || L->K > 65535 ||
      Co > 65535 || Ci > 65535)
    return false;
  const size_t es = dtype_size(dtype);
  L->col_bytes = align256((size_t)B * L->K * L->N * es);
  L->dcol_bytes = align256((size_t)B * L->K * L->N * sizeof(float));
  L->dyp_bytes = align256((size_t)B * Co * L->N * es);
  GemmDesc d = lowered_dw_desc(B, Co, *L, dtype);
  L->part_bytes = align256(gemm_partial_bytes(d, gemm_pick_splits(d)));
  return true;
}

unsigned row_blocks(int64_t items) {
  int64_t b = (items + 255) / 256;
  return (unsigned)(b > 64 ? 64 : (b < 1 ? 1 : b));
}

constexpr size_t CONV_LDS_BUDGET = 48 * 1024;

// samples per block: enough output pixels to keep 256 threads busy, within the LDS budget
static int pick_ni(int Nb, int per_sample_out, size_t per_sample_lds) {
  int ni = (2048 + per_sample_out - 1) / per_sample_out;
  if (ni > Nb) ni = Nb;
  while (ni > 1 && (size_t)ni * per_sample_lds > CONV_LDS_BUDGET) --ni;
  return ni < 1 ? 1 : ni;
}

template <typename T>
int launch_im2col_t(const void* X, void* col, int B, int Nb, int Ci, int H, int W, ConvGeom g, int kh, int kw, int stride,
                    int pad, hipStream_t st) {
  const int K = Ci * kh * kw;
  const T* x = (const T*)X;
  T* cb = (T*)col;
  const size_t img_bytes = (size_t)H * W * sizeof(T);
  if (img_bytes <= CONV_LDS_BUDGET && Ci <= 65535) {
    const int HoWo = g.Ho * g.Wo;
    const int ni = pick_ni(Nb, HoWo, img_bytes);
    int V = 16 / (int)sizeof(T);
    while (V > 1 && HoWo % V != 0) V >>= 1;
    const dim3 gr((unsigned)((Nb + ni - 1) / ni), (unsigned)Ci, (unsigned)B);
    const size_t lds = (size_t)ni * img_bytes;
    const FastDiv dh = FastDiv::make(HoWo), dw = FastDiv::make(g.Wo);
    const int vec_in = (H * W) % (16 / (int)sizeof(T)) == 0 && reinterpret_cast<uintptr_t>(X) % 16 == 0;
#define HFTA_IM2COL_L(VV) hipLaunchKernelGGL((im2col_lds_kernel<T, VV>), gr, dim3(256), lds, st, x, cb, B, Nb, Ci, H, W, g.Ho, g.Wo, kh, kw, stride, pad, ni, vec_in, dh, dw)
    if (V == 8) HFTA_IM2COL_L(8); else if (V == 4) HFTA_IM2COL_L(4); else if (V == 2) HFTA_IM2COL_L(2); else HFTA_IM2COL_L(1);
#undef HFTA_IM2COL_L
    return launch_status();
  }
  int V = 16 / (int)sizeof(T);
  while (V > 1 && g.Wo % V != 0) V >>= 1;
  const dim3 gr(row_blocks((int64_t)Nb * g.Ho * (g.Wo / V)), (unsigned)K, (unsigned)B);
  const FastDiv a = FastDiv::make(kh * kw), b2 = FastDiv::make(kw), c = FastDiv::make(g.Wo / V), d = FastDiv::make(g.Ho);
#define HFTA_IM2COL(VV) hipLaunchKernelGGL((im2col_kernel<T, VV>), gr, dim3(256), 0, st, x, cb, B, Nb, Ci, H, W, g.Ho, g.Wo, kh, kw, stride, pad, a, b2, c, d)
  if (V == 8) HFTA_IM2COL(8); else if (V == 4) HFTA_IM2COL(4); else if (V == 2) HFTA_IM2COL(2); else HFTA_IM2COL(1);
#undef HFTA_IM2COL
  return launch_status();
}

template <typename T>
int launch_col2im_t(const void* dcol, void* dX, int B, int Nb, int Ci, int H, int W, ConvGeom g, int kh, int kw, int stride,
                    int pad, hipStream_t st) {
  const int HoWo = g.Ho * g.Wo, HW = H * W;
  const size_t per_sample = (size_t)kh * kw * HoWo * sizeof(float);
  if (per_sample <= CONV_LDS_BUDGET) {
    const int ni = pick_ni(Nb, HW, per_sample);
    int V = 16 / (int)sizeof(T);
    while (V > 1 && (HW % V != 0 || reinterpret_cast<uintptr_t>(dX) % (V * sizeof(T)) != 0)) V >>= 1;
    const dim3 gr((unsigned)((Nb + ni - 1) / ni), (unsigned)Ci, (unsigned)B);
    const size_t lds = (size_t)ni * per_sample;
    const FastDiv dhw = FastDiv::make(HW), dw = FastDiv::make(W), ds = FastDiv::make(stride);
#define HFTA_COL2IM_L(VV) hipLaunchKernelGGL((col2im_lds_kernel<T, VV>), gr, dim3(256), lds, st, (const float*)dcol, (T*)dX, B, Nb, Ci, H, W, g.Ho, g.Wo, kh, kw, stride, pad, ni, dhw, dw, ds)
    if (V == 8) HFTA_COL2IM_L(8); else if (V == 4) HFTA_COL2IM_L(4); else if (V == 2) HFTA_COL2IM_L(2); else HFTA_COL2IM_L(1);
#undef HFTA_COL2IM_L
    return launch_status();
  }
  const dim3 cgrid(row_blocks((int64_t)Nb * HW), (unsigned)Ci, (unsigned)B);
  hipLaunchKernelGGL(col2im_kernel<T>, cgrid, dim3(256), 0, st, (const float*)dcol, (T*)dX, B, Nb, Ci, H, W, g.Ho, g.Wo, kh, kw,
                     stride, pad);
  return launch_status();
}

int lowered_fwd(int B, int Nb, int Ci, int Co, int H, int W, int kh, int kw, int stride, int pad, int dtype, ConvGeom g,
                const Lowered& L, const void* X, const void* Wt, const void* bias, void* Y, int act, float slope,
                void* ws, hipStream_t st) {
  int rc = dtype == HFTA_BF16 ? launch_im2col_t<bf16_raw>(X, ws, B, Nb, Ci, H, W, g, kh, kw, stride, pad, st)
                              : launch_im2col_t<float>(X, ws, B, Nb, Ci, H, W, g, kh, kw, stride, pad, st);
  if (rc != HFTA_OK) return rc;
  GemmDesc d{};
  d.S = 1; d.G0 = B; d.G1 = 1;
  d.A = Wt; d.Bm = ws; d.C = Y;
  d.M = Co; d.N = (int)L.N; d.K = (int)L.K;
  d.a_kc = true; d.a_ld = L.K; d.a_g0 = (int64_t)Co * L.K;
  d.b_kc = false; d.b_ld = L.N; d.b_g0 = L.K * L.N;
  d.c_ld = L.HoWo; d.c_g0 = (int64_t)Co * L.HoWo;
  d.c_seg = (int)L.HoWo; d.c_seg_stride = (int64_t)B * Co * L.HoWo;
  d.bias = bias; d.bias_mode = 1; d.bias_g0 = Co;
  d.act = act; d.slope = slope; d.dtype = dtype; d.out_f32 = false; d.splits = 1;
  return gemm_launch(d, st);
}

}  // namespace

extern "C" {

size_t hfta_conv2d_grouped_fwd_workspace_bytes(int B, int Nb, int Ci, int Co, int H, int W, int kh, int kw, int stride,
                                               int pad, int dtype) {
  ConvGeom g;
  Lowered L;
  if (check_conv(B, Nb, Ci, Co, H, W, kh, kw, stride, pad, dtype, &g) != HFTA_OK) return 0;
  // the sample-folded implicit GEMM splits long reductions with few tiles over k (fp32 partial slices)
  const size_t ig = (dtype == HFTA_BF16 && kh == 4 && kw == 4 && stride == 2 && pad == 1) ? conv_ig_fwd_split_bytes(B, Nb, Ci, Co, H, W) : 0;
  if (!lowered_sizes(B, Nb, Ci, Co, g, kh, kw, dtype, &L)) return ig;
  return L.col_bytes > ig ? L.col_bytes : ig;
}

int hfta_conv2d_grouped_fwd(int B, int Nb, int Ci, int Co, int H, int W, int kh, int kw, int stride, int pad, int dtype,
                            const void* X, const void* Wt, const void* bias, void* Y, int act, float act_slope,
                            void* workspace, size_t ws_bytes, void* stream) {
  ConvGeom g;
  int rc = check_conv(B, Nb, Ci, Co, H, W, kh, kw, stride, pad, dtype, &g);
  if (rc != HFTA_OK) return rc;
  if (!X || !Wt || !Y || !valid_act(act)) return HFTA_EINVAL;
  // a window that covers the whole image: the operator is a batched Linear over the flattened window
  if (conv_full_applies(H, W, kh, kw, pad, Ci, Nb))
    return conv_full_fwd(B, Nb, Ci, Co, kh, kw, dtype, X, Wt, bias, Y, act, act_slope, as_stream(stream));
  // bf16, 4x4 / stride 2 / pad 1, power-of-two output grids: the sample-folded implicit GEMM (no workspace)
  if (dtype == HFTA_BF16) {
    rc = conv_ig_forward(B, Nb, Ci, Co, H, W, kh, kw, stride, pad, X, Wt, bias, Y, act, act_slope, workspace, ws_bytes,
                         as_stream(stream));
    if (rc != HFTA_EUNSUPPORTED) return rc;
  }
  Lowered L;
  // images of 16x16 outputs and more fill the implicit kernel's 128-column tiles by themselves, and
  // it moves no column buffer: measured faster there; below that the sample-folded GEMM wins
  const bool big_image = (int64_t)g.Ho * g.Wo >= 256;
  if (!big_image && workspace && reinterpret_cast<uintptr_t>(workspace) % 256 == 0 &&
      lowered_sizes(B, Nb, Ci, Co, g, kh, kw, dtype, &L) && ws_bytes >= L.col_bytes) {
    rc = lowered_fwd(B, Nb, Ci, Co, H, W, kh, kw, stride, pad, dtype, g, L, X, Wt, bias, Y, act, act_slope, workspace,
                     as_stream(stream));
    if (rc != HFTA_EUNSUPPORTED) return rc;
  }
  ConvArgs a = base_args(B, Nb, Ci, Co, H, W, kh, kw, stride, pad, g);
  a.X = X; a.Wt = Wt; a.Out = Y; a.bias = bias; a.act = act; a.slope = act_slope;
  a.a_vec = reinterpret_cast<uintptr_t>(Wt) % 16 == 0;
  a.M = Co; a.N = g.Ho * g.Wo; a.K = Ci * kh * kw;
  finish_tiles(a, dtype);
  return launch_conv<CONV_FWD>(a, dtype, (unsigned)(B * Nb), as_stream(stream));
}

// Regrouped weights of the implicit data gradient (optional: the kernel gathers single taps without them).
static size_t dx_pack_bytes(int B, int Ci, int Co, int kh, int kw, int stride, int dtype, ConvGeom g) {
  if (dtype == HFTA_BF16 && conv_ig_dx_supported(1, Ci, Co, 2 * g.Ho, 2 * g.Wo, kh, kw, stride, 1) && kh == 4 && stride == 2)
    return conv_ig_dx_pack_bytes(B, Ci, Co);
  const bool implicit_dx = (int64_t)g.Ho * g.Wo >= 256 && Ci >= 32;
  const int kmax = kh > kw ? kh : kw, KJ = (kmax + stride - 1) / stride;
  const int64_t K = (int64_t)Co * KJ * KJ;
  const int kg = 16 / (int)dtype_size(dtype);
  if (!implicit_dx || K % kg != 0 || K > 0x7fffffffLL) return 0;
  return (size_t)B * stride * stride * Ci * K * dtype_size(dtype);
}

static size_t implicit_bwd_bytes(int B, int Nb, int Ci, int Co, int H, int W, int kh, int kw, int stride, int pad,
                                 int dtype, ConvGeom g) {
  ConvArgs a = base_args(B, Nb, Ci, Co, H, W, kh, kw, stride, pad, g);
  a.M = Co; a.N = Ci * kh * kw; a.K = g.Ho * g.Wo; a.S = Nb;
  finish_tiles(a, dtype);
  const int sp = dw_splits(a);
  size_t need = sp > 1 ? (size_t)sp * B * (size_t)a.M * a.N * sizeof(float) : 0;
  if (dtype == HFTA_BF16 && conv_ig_dw_supported(Nb, Ci, Co, H, W, kh, kw, stride, pad)) {
    const int isp = conv_ig_dw_splits(B, Nb, Ci, Co, H, W);
    const size_t ig = isp > 1 ? (size_t)isp * B * (size_t)a.M * a.N * sizeof(float) : 0;
    if (ig > need) need = ig;
  }
  return need;
}

static bool ig_dx_applies(int Nb, int Ci, int Co, int H, int W, int kh, int kw, int stride, int pad, int dtype) {
  return dtype == HFTA_BF16 && conv_ig_dx_supported(Nb, Ci, Co, H, W, kh, kw, stride, pad);
}

/* What the implicit-GEMM path needs (the weight gradient's split partials and the data gradient's
 * regrouped weights; may be 0). */
size_t hfta_conv2d_grouped_bwd_min_workspace_bytes(int B, int Nb, int Ci, int Co, int H, int W, int kh, int kw,
                                                   int stride, int pad, int dtype) {
  ConvGeom g;
  if (check_conv(B, Nb, Ci, Co, H, W, kh, kw, stride, pad, dtype, &g) != HFTA_OK) return 0;
  const size_t imp = implicit_bwd_bytes(B, Nb, Ci, Co, H, W, kh, kw, stride, pad, dtype, g);
  const size_t pk = ig_dx_applies(Nb, Ci, Co, H, W, kh, kw, stride, pad, dtype) ? conv_ig_dx_pack_bytes(B, Ci, Co) : 0;
  // behind the weight gradient's partials: the data gradient's k-split slices, then its regrouped weights
  return pk ? align256(imp) + align256(conv_ig_dx_split_bytes(B, Nb, Ci, Co, H, W)) + pk : imp;
}

/* The size that enables the column-buffer path; anything from the implicit path's own need (the
 * split partials of the weight gradient, possibly 0) upwards is accepted and selects that path. */
size_t hfta_conv2d_grouped_bwd_workspace_bytes(int B, int Nb, int Ci, int Co, int H, int W, int kh, int kw, int stride,
                                               int pad, int dtype) {
  ConvGeom g;
  if (check_conv(B, Nb, Ci, Co, H, W, kh, kw, stride, pad, dtype, &g) != HFTA_OK) return 0;
  const size_t imp = implicit_bwd_bytes(B, Nb, Ci, Co, H, W, kh, kw, stride, pad, dtype, g);
  Lowered L;
  if (!lowered_sizes(B, Nb, Ci, Co, g, kh, kw, dtype, &L)) return imp;
  const size_t low = L.dcol_bytes + L.dyp_bytes + L.part_bytes;
  const size_t base = low > imp ? low : imp;
  const size_t pk = dx_pack_bytes(B, Ci, Co, kh, kw, stride, dtype, g);
  const size_t dxs = ig_dx_applies(Nb, Ci, Co, H, W, kh, kw, stride, pad, dtype) ? align256(conv_ig_dx_split_bytes(B, Nb, Ci, Co, H, W)) : 0;
  return pk ? align256(base) + dxs + pk : base;      // (k-split slices and) regrouped weights behind everything else
}

int hfta_conv2d_grouped_bwd(int B, int Nb, int Ci, int Co, int H, int W, int kh, int kw, int stride, int pad, int dtype,
                            const void* X, const void* Wt, const void* dY, void* dX, float* dW, float* dbias,
                            void* workspace, size_t ws_bytes, void* stream) {
  ConvGeom g;
  int rc = check_conv(B, Nb, Ci, Co, H, W, kh, kw, stride, pad, dtype, &g);
  if (rc != HFTA_OK) return rc;
  if (!dY || (dX && !Wt) || (dW && !X)) return HFTA_EINVAL;
  hipStream_t st = as_stream(stream);
  Lowered L;
  if (conv_full_applies(H, W, kh, kw, pad, Ci, Nb)) {      // whole-image window: batched Linear gradients
    if (dX) {
      rc = conv_full_dx(B, Nb, Ci, Co, kh, kw, dtype, Wt, dY, dX, st);
      if (rc != HFTA_OK) return rc;
      dX = nullptr;
    }
    if (dW) {
      rc = conv_full_dw(B, Nb, Ci, Co, kh, kw, dtype, X, dY, dW, st);
      if (rc != HFTA_OK) return rc;
      dW = nullptr;
    }
  }
  // at most 4 input channels: direct vector arithmetic (a matrix tile would be 95 % empty)
  if (dX && dtype == HFTA_BF16 && conv_dx_fewc_supported(Nb, B, Ci, Co, H, W, kh, kw, stride, pad)) {
    rc = conv_dx_fewc(B, Nb, Ci, Co, H, W, Wt, dY, dX, st);
    if (rc == HFTA_OK) dX = nullptr;
    else if (rc != HFTA_EUNSUPPORTED) return rc;
  }
  // Data gradient as an implicit GEMM over (sample, pixel) columns per parity class: its regrouped
  // weights take the last bytes of the workspace (every other user starts at its front, and both the
  // minimum and the full size leave that room).
  if (dX && workspace && ig_dx_applies(Nb, Ci, Co, H, W, kh, kw, stride, pad, dtype)) {
    const size_t pk = align256(conv_ig_dx_pack_bytes(B, Ci, Co));
    const size_t need = hfta_conv2d_grouped_bwd_min_workspace_bytes(B, Nb, Ci, Co, H, W, kh, kw, stride, pad, dtype);
    const size_t end = ws_bytes & ~(size_t)255;
    if (ws_bytes >= need && end >= pk && reinterpret_cast<uintptr_t>(workspace) % 256 == 0) {
      const size_t dxs = align256(conv_ig_dx_split_bytes(B, Nb, Ci, Co, H, W));
      unsigned char* wend = reinterpret_cast<unsigned char*>(workspace) + end;
      rc = conv_ig_dx(B, Nb, Ci, Co, H, W, kh, kw, stride, pad, Wt, dY, dX, wend - pk, dxs ? wend - pk - dxs : nullptr, st);
      if (rc == HFTA_OK) dX = nullptr;
      else if (rc != HFTA_EUNSUPPORTED) return rc;
    }
  }
  // Weight gradient as an implicit GEMM over 8-channel column groups; its k-split partials start the workspace.
  if (dW && dtype == HFTA_BF16 && conv_ig_dw_supported(Nb, Ci, Co, H, W, kh, kw, stride, pad)) {
    const int sp = conv_ig_dw_splits(B, Nb, Ci, Co, H, W);
    const size_t need = sp > 1 ? (size_t)sp * B * (size_t)Co * Ci * 16 * sizeof(float) : 0;
    if (need && (!workspace || ws_bytes < need)) return HFTA_EWORKSPACE;
    rc = conv_ig_dw(B, Nb, Ci, Co, H, W, kh, kw, stride, pad, X, dY, dW, need ? reinterpret_cast<float*>(workspace) : nullptr, st);
    if (rc == HFTA_OK) dW = nullptr;
    else if (rc != HFTA_EUNSUPPORTED) return rc;
  }
  // the data gradient of large images with enough channels stays on the implicit kernel (see the
  // forward); everything else goes through the column buffer when the workspace allows
  const bool implicit_dx = (int64_t)g.Ho * g.Wo >= 256 && Ci >= 32;
  if ((dW || (dX && !implicit_dx)) && workspace && reinterpret_cast<uintptr_t>(workspace) % 256 == 0 &&
      lowered_sizes(B, Nb, Ci, Co, g, kh, kw, dtype, &L) && ws_bytes >= L.dcol_bytes + L.dyp_bytes + L.part_bytes) {
    unsigned char* wsb = reinterpret_cast<unsigned char*>(workspace);
    void* colb = wsb;
    void* dyp = wsb + L.dcol_bytes;
    float* part = reinterpret_cast<float*>(wsb + L.dcol_bytes + L.dyp_bytes);
    const dim3 pgrid(row_blocks(L.N), (unsigned)Co, (unsigned)B);
    const int pvec = L.HoWo % (16 / (int64_t)dtype_size(dtype)) == 0 && reinterpret_cast<uintptr_t>(dY) % 16 == 0;
    if (dtype == HFTA_BF16)
      hipLaunchKernelGGL(pack_dy_kernel<bf16_raw>, pgrid, dim3(256), 0, st, (const bf16_raw*)dY, (bf16_raw*)dyp, B, Nb, Co,
                         (int)L.HoWo, pvec);
    else
      hipLaunchKernelGGL(pack_dy_kernel<float>, pgrid, dim3(256), 0, st, (const float*)dY, (float*)dyp, B, Nb, Co,
                         (int)L.HoWo, pvec);
    if (launch_status() != HFTA_OK) return HFTA_ELAUNCH;
    if (dW) {
      rc = dtype == HFTA_BF16 ? launch_im2col_t<bf16_raw>(X, colb, B, Nb, Ci, H, W, g, kh, kw, stride, pad, st)
                              : launch_im2col_t<float>(X, colb, B, Nb, Ci, H, W, g, kh, kw, stride, pad, st);
      if (rc != HFTA_OK) return rc;
      GemmDesc d = lowered_dw_desc(B, Co, L, dtype);
      d.A = dyp; d.Bm = colb; d.C = dW;
      d.splits = gemm_pick_splits(d);
      d.partial = part;
      rc = gemm_launch(d, st);
      if (rc != HFTA_OK) return rc;
    }
    if (dX && !implicit_dx) {
      GemmDesc d{};
      d.S = 1; d.G0 = B; d.G1 = 1;
      d.A = Wt; d.Bm = dyp; d.C = colb;
      d.M = (int)L.K; d.N = (int)L.N; d.K = Co;
      d.a_kc = false; d.a_ld = L.K; d.a_g0 = (int64_t)Co * L.K;      // A[m = k][kk = co] = W[co][k]
      d.b_kc = false; d.b_ld = L.N; d.b_g0 = (int64_t)Co * L.N;
      d.c_ld = L.N; d.c_g0 = L.K * L.N;
      d.act = HFTA_ACT_NONE; d.dtype = dtype; d.out_f32 = true; d.splits = 1;   // fp32 partial sums per tap
      rc = gemm_launch(d, st);
      if (rc != HFTA_OK) return rc;
      rc = dtype == HFTA_BF16 ? launch_col2im_t<bf16_raw>(colb, dX, B, Nb, Ci, H, W, g, kh, kw, stride, pad, st)
                              : launch_col2im_t<float>(colb, dX, B, Nb, Ci, H, W, g, kh, kw, stride, pad, st);
      if (rc != HFTA_OK) return rc;
    }
    dW = nullptr;                      // done; what is left (implicit dX, dbias) follows
    if (!implicit_dx) dX = nullptr;
  }
  ConvArgs w = base_args(B, Nb, Ci, Co, H, W, kh, kw, stride, pad, g);
  if (dW) {
    w.X = X; w.dY = dY; w.Out = dW;
    w.a_vec = reinterpret_cast<uintptr_t>(dY) % 16 == 0;
    w.M = Co; w.N = Ci * kh * kw; w.K = g.Ho * g.Wo; w.S = Nb;
    finish_tiles(w, dtype);
    w.splits = dw_splits(w);
    if (w.splits > 1) {
      const size_t need = (size_t)w.splits * B * (size_t)w.M * w.N * sizeof(float);
      if (!workspace || ws_bytes < need) return HFTA_EWORKSPACE;
      w.partial = reinterpret_cast<float*>(workspace);
    }
  }
  if (dX) {
    ConvDxArgs a{};
    a.Wt = Wt; a.dY = dY; a.dX = dX;
    a.B = B; a.Nb = Nb; a.Ci = Ci; a.Co = Co; a.H = H; a.W = W; a.Ho = g.Ho; a.Wo = g.Wo;
    a.kh = kh; a.kw = kw; a.stride = stride; a.pad = pad;
    const int kmax = kh > kw ? kh : kw;
    a.KJ = (kmax + stride - 1) / stride;
    a.Hqm = (H + stride - 1) / stride; a.Wqm = (W + stride - 1) / stride;
    a.M = Ci; a.N = a.Hqm * a.Wqm;
    if ((int64_t)Co * a.KJ * a.KJ > 0x7fffffffLL || stride * stride > 65535) return HFTA_EUNSUPPORTED;
    a.K = Co * a.KJ * a.KJ;
    const int BK = dtype == HFTA_BF16 ? GemmT<bf16_raw>::BK : GemmT<float>::BK;
    a.tiles_n = (a.N + GEMM_BN - 1) / GEMM_BN;
    a.k_tiles = (a.K + BK - 1) / BK;
    a.d_kj = FastDiv::make(a.KJ); a.d_kjkj = FastDiv::make(a.KJ * a.KJ);
    a.d_wqm = FastDiv::make(a.Wqm); a.d_s = FastDiv::make(stride);
    dim3 grid((unsigned)(((a.M + GEMM_BM - 1) / GEMM_BM) * a.tiles_n), (unsigned)(stride * stride), (unsigned)(B * Nb));
    // regrouped weights live at the end of a full-size workspace; a smaller workspace selects the gathering variant
    const size_t pk = dx_pack_bytes(B, Ci, Co, kh, kw, stride, dtype, g);
    const size_t full = hfta_conv2d_grouped_bwd_workspace_bytes(B, Nb, Ci, Co, H, W, kh, kw, stride, pad, dtype);
    if (pk && workspace && ws_bytes >= full && reinterpret_cast<uintptr_t>(workspace) % 256 == 0) {
      unsigned char* wp = reinterpret_cast<unsigned char*>(workspace) + (full - pk);
      a.Wp = wp;
      const int64_t count = (int64_t)(pk / dtype_size(dtype));
      dim3 pg((unsigned)((count + 255) / 256));
      if (dtype == HFTA_BF16) {
        hipLaunchKernelGGL(conv_dx_pack_w_kernel<bf16_raw>, pg, dim3(256), 0, st, a, reinterpret_cast<bf16_raw*>(wp), count);
        hipLaunchKernelGGL((conv_dx_kernel<bf16_raw, true>), grid, dim3(GEMM_THREADS), 0, st, a);
      } else {
        hipLaunchKernelGGL(conv_dx_pack_w_kernel<float>, pg, dim3(256), 0, st, a, reinterpret_cast<float*>(wp), count);
        hipLaunchKernelGGL((conv_dx_kernel<float, true>), grid, dim3(GEMM_THREADS), 0, st, a);
      }
    } else if (dtype == HFTA_BF16) {
      hipLaunchKernelGGL((conv_dx_kernel<bf16_raw, false>), grid, dim3(GEMM_THREADS), 0, st, a);
    } else {
      hipLaunchKernelGGL((conv_dx_kernel<float, false>), grid, dim3(GEMM_THREADS), 0, st, a);
    }
    if (launch_status() != HFTA_OK) return HFTA_ELAUNCH;
  }
  if (dW) {
    rc = launch_conv<CONV_DW>(w, dtype, (unsigned)(B * w.splits), st);
    if (rc != HFTA_OK) return rc;
    if (w.splits > 1) {
      const int64_t count = (int64_t)B * w.M * w.N;
      hipLaunchKernelGGL(conv_splitk_reduce_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st,
                         (const float*)w.partial, dW, count, w.splits);
      if (launch_status() != HFTA_OK) return HFTA_ELAUNCH;
    }
  }
  if (dbias) {
    const int64_t HoWo = (int64_t)g.Ho * g.Wo;
    if (dtype == HFTA_BF16)
      hipLaunchKernelGGL(conv_dbias_kernel<bf16_raw>, dim3((unsigned)(B * Co)), dim3(256), 0, st, (const bf16_raw*)dY, dbias,
                         Nb, B * Co, HoWo);
    else
      hipLaunchKernelGGL(conv_dbias_kernel<float>, dim3((unsigned)(B * Co)), dim3(256), 0, st, (const float*)dY, dbias, Nb,
                         B * Co, HoWo);
    return launch_status();
  }
  return HFTA_OK;
}

}  // extern "C"
