// Batched, strided GEMM core on the CDNA4 matrix cores.
//
// One kernel serves the three forms of the fused Linear and the fused k=1
// Conv1d (forward, data gradient, weight gradient): every model of the array is
// one slice of the batch, so B weight sets are one launch (the fusion rules
// table's "baddbmm" / grouped-convolution rows).
//
//   C[g][m][n] = epilogue( sum_{s<S} sum_{k<K} A[g][s][m][k] * B[g][s][k][n] )
//
// g = (g0, g1) is a two-level batch index; s is an outer reduction index (the
// sample axis of the k=1 convolution's weight gradient).  Each operand is
// addressed by element strides and must be contiguous along exactly one of its
// two matrix dims; C is contiguous along n.
//
// Tiling: 256 threads = 4 wavefronts compute a 128x128 tile of C; each wavefront
// owns a 64x64 quadrant as 2x2 MFMA 32x32 blocks with fp32 accumulators.
// Operand tiles are staged through LDS as [row][64 B of k + 16 B pad] so that a
// lane's MFMA fragment (16 B along k) is one conflict-free ds_read_b128;
// operands that are contiguous along m/n in memory are transposed in registers
// on their way into LDS.  Global loads of tile t+1 are issued before the MFMAs
// of tile t (register-staged double buffering, two LDS buffers, one barrier per
// k-tile).
#pragma once
#include "common.h"
#include <type_traits>

namespace hfta {

struct GemmDesc {
  const void* A;
  const void* Bm;
  void* C;
  int M, N, K, S;
  int G0, G1;
  int64_t a_ld, a_ss, a_g0, a_g1;  // a_ld: stride of A's non-contiguous matrix dim
  int64_t b_ld, b_ss, b_g0, b_g1;
  int64_t c_ld, c_g0, c_g1;
  bool a_kc, b_kc;                 // operand contiguous along k (else along m / n)
  const void* bias;                // storage dtype, or nullptr
  int bias_mode;                   // 1: per row m, 2: per column n
  int64_t bias_g0, bias_g1;
  int act;
  float slope;
  int dtype;                       // storage type of A and B (and of C unless out_f32)
  bool out_f32;
  int splits;                      // > 1: fp32 partials [split][G0*G1][M][N] go to `partial`
  float* partial;
  bool keep_partials;              // splits > 1: leave the partials unsummed (the caller's epilogue adds them); C unused
  // C's columns in segments of c_seg (0 = one contiguous row): column n lives at
  // (n / c_seg) * c_seg_stride + n % c_seg past the row start (an [N][C][HW] image tensor seen as [C][N*HW])
  int c_seg;
  int64_t c_seg_stride;
  // BatchNorm statistics of the output taken in the epilogue (bf16 k=1 convolution forward in the persistent
  // 256 x 256 kernel only): per (group, 256-column tile, row m) the sums of (c - bias[m]) and (c - bias[m])^2 over
  // the tile's columns, [G0*G1][tiles_n][M][2] floats, from the values as they are stored.  *stat_done is set
  // when the kernel that writes them was launched (otherwise nothing touched stat_part).
  float* stat_part;
  bool* stat_done;
};

struct GemmArgs {
  const void* A;
  const void* Bm;
  void* C;
  const void* bias;
  float* partial;
  int64_t a_ld, a_ss, a_g0, a_g1;
  int64_t b_ld, b_ss, b_g0, b_g1;
  int64_t c_ld, c_g0, c_g1;
  int64_t bias_g0, bias_g1;
  int M, N, K, S, G1;
  int tiles_m, tiles_n, tiles_per_seg, total_tiles, splits;
  int a_vec, b_vec, c_vec, p_vec;
  int bias_mode, act;
  float slope;
  uint32_t a_extent, b_extent;   // bytes from an operand slice's first to one past its last element
  uint32_t c_extent;             // same for one output slice, or 0 when it does not fit 31 bits
  int c_seg;
  int64_t c_seg_stride;
  float* stat_part;              // see GemmDesc
};

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

constexpr int GEMM_BM = 128, GEMM_BN = 128, GEMM_THREADS = 256;
constexpr int GEMM_PITCH = 80;                       // bytes per LDS row: 64 B of k + 16 B pad
constexpr int GEMM_TILE_BYTES = 128 * GEMM_PITCH;    // one operand tile

template <typename T> struct GemmT;
template <> struct GemmT<bf16_raw> { static constexpr int KG = 8, BK = 32, NV = 4, KQ = 8; };
template <> struct GemmT<float>    { static constexpr int KG = 4, BK = 16, NV = 2, KQ = 4; };

// ---- global -> registers ------------------------------------------------
// K-contiguous operand: thread t stages 16-byte group (t % 4) of rows t/4 and t/4 + 64.
template <typename T>
__device__ __forceinline__ void load_kc(uint4 (&q)[2], const T* base, int64_t ld, int row0, int rows,
                                        int k0, int K, int vec, int t) {
  constexpr int KG = GemmT<T>::KG;
  const int g = t & 3;
  const int k = k0 + g * KG;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int r = row0 + (t >> 2) + 64 * h;
    const T* src = base + (int64_t)r * ld + k;
    if (vec == 2 && r < rows && k + KG <= K) {
      q[h] = *reinterpret_cast<const uint4*>(src);
    } else if (vec == 1 && r < rows && k + KG <= K) {     // rows only 8-byte aligned
      const uint2 lo = *reinterpret_cast<const uint2*>(src);
      const uint2 hi = *reinterpret_cast<const uint2*>(src + KG / 2);
      q[h] = make_uint4(lo.x, lo.y, hi.x, hi.y);
    } else {
      T tmp[KG];
#pragma unroll
      for (int e = 0; e < KG; ++e) tmp[e] = (r < rows && k + e < K) ? src[e] : T(0);
      q[h] = *reinterpret_cast<const uint4*>(tmp);
    }
  }
}
__device__ __forceinline__ void store_kc(unsigned char* tile, const uint4 (&q)[2], int t) {
#pragma unroll
  for (int h = 0; h < 2; ++h)
    *reinterpret_cast<uint4*>(tile + ((t >> 2) + 64 * h) * GEMM_PITCH + (t & 3) * 16) = q[h];
}

// m/n-contiguous operand: thread t stages a 4(k) x NV(n) block: k-quad t % KQ, n-group t / KQ.
template <typename T>
__device__ __forceinline__ void load_nc(uint2 (&q)[4], const T* base, int64_t ld, int col0, int cols,
                                        int k0, int K, int vec, int t) {
  constexpr int NV = GemmT<T>::NV, KQ = GemmT<T>::KQ;
  const int kq = t % KQ, ng = t / KQ;
  const int c = col0 + ng * NV;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int k = k0 + 4 * kq + j;
    const T* src = base + (int64_t)k * ld + c;
    if (vec && k < K && c + NV <= cols) {
      q[j] = *reinterpret_cast<const uint2*>(src);
    } else {
      T tmp[NV];
#pragma unroll
      for (int e = 0; e < NV; ++e) tmp[e] = (k < K && c + e < cols) ? src[e] : T(0);
      q[j] = *reinterpret_cast<const uint2*>(tmp);
    }
  }
}
__device__ __forceinline__ void store_nc_bf16(unsigned char* tile, const uint2 (&q)[4], int t) {
  const int kq = t % 8, ng = t / 8;
  // q[j] = 4 bf16 along n for k = 4kq + j; emit 4 rows (n) of 4 bf16 along k
  const uint32_t a0 = q[0].x, a1 = q[1].x, a2 = q[2].x, a3 = q[3].x;
  const uint32_t b0 = q[0].y, b1 = q[1].y, b2 = q[2].y, b3 = q[3].y;
  uint2 o[4];
  o[0] = make_uint2((a0 & 0xffffu) | (a1 << 16), (a2 & 0xffffu) | (a3 << 16));
  o[1] = make_uint2((a0 >> 16) | (a1 & 0xffff0000u), (a2 >> 16) | (a3 & 0xffff0000u));
  o[2] = make_uint2((b0 & 0xffffu) | (b1 << 16), (b2 & 0xffffu) | (b3 << 16));
  o[3] = make_uint2((b0 >> 16) | (b1 & 0xffff0000u), (b2 >> 16) | (b3 & 0xffff0000u));
#pragma unroll
  for (int i = 0; i < 4; ++i)
    *reinterpret_cast<uint2*>(tile + (ng * 4 + i) * GEMM_PITCH + kq * 8) = o[i];
}
__device__ __forceinline__ void store_nc_f32(unsigned char* tile, const uint2 (&q)[4], int t) {
  const int kq = t % 4, ng = t / 4;
  *reinterpret_cast<uint4*>(tile + (ng * 2 + 0) * GEMM_PITCH + kq * 16) = make_uint4(q[0].x, q[1].x, q[2].x, q[3].x);
  *reinterpret_cast<uint4*>(tile + (ng * 2 + 1) * GEMM_PITCH + kq * 16) = make_uint4(q[0].y, q[1].y, q[2].y, q[3].y);
}

template <typename T, bool KC> struct Stager;
template <typename T> struct Stager<T, true> {
  uint4 q[2];
  __device__ __forceinline__ void load(const T* base, int64_t ld, int r0, int rows, int k0, int K, int vec, int t) {
    load_kc<T>(q, base, ld, r0, rows, k0, K, vec, t);
  }
  __device__ __forceinline__ void store(unsigned char* tile, int t) { store_kc(tile, q, t); }
};
template <> struct Stager<bf16_raw, false> {
  uint2 q[4];
  __device__ __forceinline__ void load(const bf16_raw* base, int64_t ld, int r0, int rows, int k0, int K, int vec, int t) {
    load_nc<bf16_raw>(q, base, ld, r0, rows, k0, K, vec, t);
  }
  __device__ __forceinline__ void store(unsigned char* tile, int t) { store_nc_bf16(tile, q, t); }
};
template <> struct Stager<float, false> {
  uint2 q[4];
  __device__ __forceinline__ void load(const float* base, int64_t ld, int r0, int rows, int k0, int K, int vec, int t) {
    load_nc<float>(q, base, ld, r0, rows, k0, K, vec, t);
  }
  __device__ __forceinline__ void store(unsigned char* tile, int t) { store_nc_f32(tile, q, t); }
};

// ---- MFMA on one k-tile ---------------------------------------------------
// The B fragment is passed as the MFMA's first operand, so the accumulators hold the
// TRANSPOSED block: lane l owns row m = l % 32 and columns n = 8*(v/4) + 4*(l/32) + v%4 of each
// 32x32 block, i.e. four consecutive n per group of four registers -- what a row-major store wants.
template <typename T>
__device__ __forceinline__ void mma_tile(f32x16_t (&acc)[2][2], const unsigned char* As,
                                         const unsigned char* Bs, int wm, int wn, int lane);
template <>
__device__ __forceinline__ void mma_tile<bf16_raw>(f32x16_t (&acc)[2][2], const unsigned char* As,
                                                   const unsigned char* Bs, int wm, int wn, int lane) {
  const int r = lane & 31, gsel = lane >> 5;
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    bf16x8_t a[2], b[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      a[i] = *reinterpret_cast<const bf16x8_t*>(As + (wm * 64 + i * 32 + r) * GEMM_PITCH + (2 * s + gsel) * 16);
      b[i] = *reinterpret_cast<const bf16x8_t*>(Bs + (wn * 64 + i * 32 + r) * GEMM_PITCH + (2 * s + gsel) * 16);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
  }
}
template <>
__device__ __forceinline__ void mma_tile<float>(f32x16_t (&acc)[2][2], const unsigned char* As,
                                                const unsigned char* Bs, int wm, int wn, int lane) {
  const int r = lane & 31, gsel = lane >> 5;
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    float4 a[2], b[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      a[i] = *reinterpret_cast<const float4*>(As + (wm * 64 + i * 32 + r) * GEMM_PITCH + (2 * s + gsel) * 16);
      b[i] = *reinterpret_cast<const float4*>(Bs + (wn * 64 + i * 32 + r) * GEMM_PITCH + (2 * s + gsel) * 16);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(b[j].x, a[i].x, acc[i][j], 0, 0, 0);
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(b[j].y, a[i].y, acc[i][j], 0, 0, 0);
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(b[j].z, a[i].z, acc[i][j], 0, 0, 0);
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(b[j].w, a[i].w, acc[i][j], 0, 0, 0);
      }
  }
}

// ---- epilogue: accumulators -> LDS -> wide row-major global stores ------------
// The 128x128 tile is staged through LDS (all 128 rows at once for 2-byte outputs, two passes of
// 64 rows for 4-byte outputs) so that every global store is a 16-byte (or 8-byte, when the row
// pitch only allows that) piece of a contiguous row segment.  Requires the k-loop's last barrier.
constexpr int EPI_PITCH2 = 128 * 2 + 8;    // bytes, 2-byte outputs: 8-byte aligned rows
constexpr int EPI_PITCH4 = 128 * 4 + 16;   // bytes, 4-byte outputs: 16-byte aligned rows

__device__ __forceinline__ float cheap_act(float x, int act, float slope) {
  if (act == HFTA_ACT_RELU) return x > 0.f ? x : 0.f;
  if (act == HFTA_ACT_LEAKY) return x > 0.f ? x : slope * x;
  return x;
}

// Activation kinds the staging code is specialised for: the three select-only ones are resolved
// at compile time (a run-time switch costs a scalar branch per element, and the epilogue's vector
// ALU work is what bounds the memory-bound shapes); ACT_ANY evaluates the run-time `act`.
enum { EPI_NONE = 0, EPI_RELU = 1, EPI_LEAKY = 2, EPI_ANY = 3 };

template <int KIND>
__device__ __forceinline__ float epi_act(float x, int act, float slope) {
  if (KIND == EPI_NONE) return x;
  if (KIND == EPI_RELU) return fmaxf(x, 0.f);
  if (KIND == EPI_LEAKY) return x > 0.f ? x : slope * x;
  return apply_act(x, act, slope);
}

// Phase 1 of the epilogue: accumulators (+ bias, activation) -> LDS staging tile in the output
// type.  `pass` selects the 64-row half for 4-byte outputs (two passes), ignored for 2-byte
// outputs (all 128 rows at once).  COLB: the bias is per column n (else per row m).  The caller
// owns the barriers around it.
template <typename OutT, typename BiasT, int KIND, bool COLB>
__device__ __forceinline__ void stage_pass(f32x16_t (&acc)[2][2], unsigned char* lds, int pass, int M, int N,
                                           int m0, int n0, const BiasT* bias, int act, float slope, int t) {
  constexpr int ES = sizeof(OutT);
  constexpr int RP = ES == 2 ? 128 : 64;
  constexpr int PITCH = ES == 2 ? EPI_PITCH2 : EPI_PITCH4;
  const int lane = t & 63, wave = t >> 6, wm = wave >> 1, wn = wave & 1;
  const int ml = lane & 31, nq = (lane >> 5) * 4;
  if (RP == 128 || wm == pass) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int rl = (RP == 128 ? wm * 64 : 0) + i * 32 + ml;
      const int m = m0 + wm * 64 + i * 32 + ml;
      float bm = 0.f;
      if (!COLB && bias && m < M) bm = Elem<BiasT>::load(bias + m);
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int nl = wn * 64 + j * 32 + 8 * q + nq;
          float x[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            x[e] = acc[i][j][4 * q + e] + bm;
            if (COLB && n0 + nl + e < N) x[e] += Elem<BiasT>::load(bias + n0 + nl + e);
            x[e] = epi_act<KIND>(x[e], act, slope);
          }
          unsigned char* dst = lds + rl * PITCH + nl * ES;
          if (ES == 2) {
            uint2 o;
            o.x = pack_bf16x2(x[0], x[1]);
            o.y = pack_bf16x2(x[2], x[3]);
            *reinterpret_cast<uint2*>(dst) = o;
          } else {
            *reinterpret_cast<float4*>(dst) = make_float4(x[0], x[1], x[2], x[3]);
          }
        }
    }
  }
}

// Row-bias / no-bias staging with one of the select-only activations (used directly by kernels
// that interleave their own work between staging and stores).
template <typename OutT, typename BiasT>
__device__ __forceinline__ void stage_acc(f32x16_t (&acc)[2][2], unsigned char* lds, int pass, int M, int m0,
                                          const BiasT* row_bias, int act, float slope, int t) {
  if (act == HFTA_ACT_RELU) stage_pass<OutT, BiasT, EPI_RELU, false>(acc, lds, pass, M, 0, m0, 0, row_bias, act, slope, t);
  else if (act == HFTA_ACT_LEAKY) stage_pass<OutT, BiasT, EPI_LEAKY, false>(acc, lds, pass, M, 0, m0, 0, row_bias, act, slope, t);
  else stage_pass<OutT, BiasT, EPI_NONE, false>(acc, lds, pass, M, 0, m0, 0, row_bias, act, slope, t);
}

// Phase 2: staged rows -> global memory.  VB = bytes per lane (16, 8: whole aligned pieces of a
// row, consecutive lanes on consecutive pieces so a wavefront's store covers whole row segments;
// 0: single elements).  INTERIOR: the tile lies wholly inside the matrix, no per-lane checks.
__device__ __forceinline__ int64_t col_offset(int n, int c_seg, int64_t c_seg_stride) {
  if (c_seg <= 0) return n;
  const int q = n / c_seg;
  return (int64_t)q * c_seg_stride + (n - q * c_seg);
}

template <typename OutT, int VB, bool INTERIOR>
__device__ __forceinline__ void store_rows(const unsigned char* lds, OutT* Cb, int64_t c_ld, int M, int N,
                                           int mbase, int n0, int t, int c_seg, int64_t c_seg_stride) {
  constexpr int ES = sizeof(OutT);
  constexpr int RP = ES == 2 ? 128 : 64;
  constexpr int PITCH = ES == 2 ? EPI_PITCH2 : EPI_PITCH4;
  if constexpr (VB > 0) {
    constexpr int EPV = VB / ES;                         // elements per piece
    constexpr int PPR = 128 / EPV;                       // pieces per row
    constexpr int RPI = GEMM_THREADS / PPR;              // rows per iteration
    const int r0 = t / PPR, c = t % PPR;
    const unsigned char* src = lds + r0 * PITCH + c * VB;
    const int n = n0 + c * EPV;
    OutT* dst = Cb + (int64_t)(mbase + r0) * c_ld + col_offset(n, c_seg, c_seg_stride);
#pragma unroll 4
    for (int it = 0; it < RP / RPI; ++it) {
      const int m = mbase + r0 + it * RPI;
      typedef typename std::conditional<VB == 16, uint4, uint2>::type V;
      const V v = *reinterpret_cast<const V*>(src + it * RPI * PITCH);
      OutT* d = dst + (int64_t)it * RPI * c_ld;
      if (INTERIOR || (m < M && n + EPV <= N)) {
        *reinterpret_cast<V*>(d) = v;
      } else if (m < M && n < N) {
        const OutT* e = reinterpret_cast<const OutT*>(&v);
#pragma unroll
        for (int k = 0; k < EPV; ++k)
          if (n + k < N) d[k] = e[k];
      }
    }
  } else {
#pragma unroll 2
    for (int it = 0; it < RP * 128 / GEMM_THREADS; ++it) {
      const int id = t + GEMM_THREADS * it;
      const int r = id / 128, c = id % 128;
      const int m = mbase + r, n = n0 + c;
      if (m < M && n < N)
        Cb[(int64_t)m * c_ld + col_offset(n, c_seg, c_seg_stride)] = *reinterpret_cast<const OutT*>(lds + r * PITCH + c * ES);
    }
  }
}

// The whole epilogue of a 128x128 tile.  ALLOW_FULL = false leaves out the per-column-bias and
// transcendental-activation code for kernels whose host side never asks for them.
template <typename OutT, typename BiasT, bool ALLOW_FULL = true>
__device__ __forceinline__ void store_tile(f32x16_t (&acc)[2][2], unsigned char* lds, OutT* Cb, int64_t c_ld,
                                           int M, int N, int m0, int n0, const BiasT* bias, int bias_mode,
                                           int act, float slope, int c_vec, int t, int c_seg = 0,
                                           int64_t c_seg_stride = 0) {
  constexpr int RP = sizeof(OutT) == 2 ? 128 : 64;       // rows per pass
  const bool colb = bias && bias_mode == 2;
  const bool full = ALLOW_FULL && (colb || act == HFTA_ACT_TANH || act == HFTA_ACT_GELU);
  const BiasT* rb = bias_mode == 1 ? bias : nullptr;
  const bool interior = m0 + 128 <= M && n0 + 128 <= N;
#pragma unroll
  for (int pass = 0; pass < 128 / RP; ++pass) {
    if (full) {
      if (colb) stage_pass<OutT, BiasT, EPI_ANY, true>(acc, lds, pass, M, N, m0, n0, bias, act, slope, t);
      else stage_pass<OutT, BiasT, EPI_ANY, false>(acc, lds, pass, M, N, m0, n0, rb, act, slope, t);
    } else {
      stage_acc<OutT, BiasT>(acc, lds, pass, M, m0, rb, act, slope, t);
    }
    __syncthreads();
    const int mbase = m0 + pass * RP;
    if (c_vec == 16) {
      if (interior) store_rows<OutT, 16, true>(lds, Cb, c_ld, M, N, mbase, n0, t, c_seg, c_seg_stride);
      else store_rows<OutT, 16, false>(lds, Cb, c_ld, M, N, mbase, n0, t, c_seg, c_seg_stride);
    } else if (c_vec == 8) {
      if (interior) store_rows<OutT, 8, true>(lds, Cb, c_ld, M, N, mbase, n0, t, c_seg, c_seg_stride);
      else store_rows<OutT, 8, false>(lds, Cb, c_ld, M, N, mbase, n0, t, c_seg, c_seg_stride);
    } else {
      store_rows<OutT, 0, false>(lds, Cb, c_ld, M, N, mbase, n0, t, c_seg, c_seg_stride);
    }
    if (pass + 1 < 128 / RP) __syncthreads();
  }
}

// ---- the kernel -----------------------------------------------------------
template <typename T, bool A_KC, bool B_KC, typename OutT>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_kernel(GemmArgs p) {
  constexpr int BK = GemmT<T>::BK;
  __shared__ __attribute__((aligned(16))) unsigned char smem[2][2][GEMM_TILE_BYTES];

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  // XCD-aware placement: the hardware deals workgroups round-robin over the 8 XCDs (each with its
  // own L2) in linear-id order.  Re-number so that every XCD walks one contiguous range of
  // (batch, tile) work: the tiles of one batch item -- which share its operands -- meet in one
  // L2, and inside a batch item the m-tiles that share a B tile run back to back.
  int bx = blockIdx.x, bz = blockIdx.z;
  {
    const int total = gridDim.x * gridDim.z, per = total >> 3;
    const int lin = blockIdx.x + gridDim.x * blockIdx.z;
    if (lin < (per << 3)) {
      const int l2 = (lin & 7) * per + (lin >> 3);
      bz = l2 / gridDim.x;
      bx = l2 - bz * gridDim.x;
    }
  }
  const int tile_m = bx % p.tiles_m, tile_n = bx / p.tiles_m;
  const int m0 = tile_m * GEMM_BM, n0 = tile_n * GEMM_BN;
  const int split = bz % p.splits, g = bz / p.splits;
  const int g0 = g / p.G1, g1 = g % p.G1;

  const T* Ab = reinterpret_cast<const T*>(p.A) + g0 * p.a_g0 + g1 * p.a_g1;
  const T* Bb = reinterpret_cast<const T*>(p.Bm) + g0 * p.b_g0 + g1 * p.b_g1;

  const int t_begin = (int)((int64_t)p.total_tiles * split / p.splits);
  const int t_end = (int)((int64_t)p.total_tiles * (split + 1) / p.splits);

  f32x16_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  Stager<T, A_KC> sa;
  Stager<T, B_KC> sb;
  auto issue = [&](int tt) {
    const int seg = tt / p.tiles_per_seg;
    const int k0 = (tt - seg * p.tiles_per_seg) * BK;
    sa.load(Ab + seg * p.a_ss, p.a_ld, m0, p.M, k0, p.K, p.a_vec, t);
    sb.load(Bb + seg * p.b_ss, p.b_ld, n0, p.N, k0, p.K, p.b_vec, t);
  };

  if (t_begin < t_end) {
    issue(t_begin);
    sa.store(smem[0][0], t);
    sb.store(smem[0][1], t);
    __syncthreads();
    int buf = 0;
    for (int tt = t_begin; tt < t_end; ++tt) {
      const bool more = tt + 1 < t_end;
      if (more) issue(tt + 1);
      mma_tile<T>(acc, smem[buf][0], smem[buf][1], wm, wn, lane);
      if (more) {
        sa.store(smem[buf ^ 1][0], t);
        sb.store(smem[buf ^ 1][1], t);
      }
      __syncthreads();
      buf ^= 1;
    }
  }

  if (p.splits > 1) {
    float* Pb = p.partial + ((int64_t)split * (gridDim.z / p.splits) + g) * (int64_t)p.M * p.N;
    store_tile<float, T, false>(acc, &smem[0][0][0], Pb, p.N, p.M, p.N, m0, n0, nullptr, 0, HFTA_ACT_NONE, 0.f, p.p_vec, t);
    return;
  }
  OutT* Cb = reinterpret_cast<OutT*>(p.C) + g0 * p.c_g0 + g1 * p.c_g1;
  const T* bias = p.bias ? reinterpret_cast<const T*>(p.bias) + g0 * p.bias_g0 + g1 * p.bias_g1 : nullptr;
  // bf16 operands with an fp32 result (weight gradients) never carry a column bias or a
  // transcendental activation (checked by the host)
  store_tile<OutT, T, sizeof(T) == sizeof(OutT)>(acc, &smem[0][0][0], Cb, p.c_ld, p.M, p.N, m0, n0, bias, p.bias_mode, p.act, p.slope, p.c_vec, t, p.c_seg, p.c_seg_stride);
}

int gemm_pick_splits(const GemmDesc& d);
size_t gemm_partial_bytes(const GemmDesc& d, int splits);
int gemm_launch(const GemmDesc& d, hipStream_t stream);

}  // namespace hfta
