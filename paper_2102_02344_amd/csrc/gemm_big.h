// Compute-bound variant of the batched GEMM core: 256x256 output tile per 512-thread workgroup.
//
// The 128x128 kernel in gemm.h reads 32 bytes of LDS per MFMA cycle and wave, which is the
// whole LDS bandwidth of a compute unit, and moves 64 flop per byte it pulls from L2.  For the
// MLP-sized GEMMs (M, N >= 256, K >= 512) this kernel doubles both ratios: eight wavefronts in a
// 2 (m) x 4 (n) grid each own a 128x64 block (4 x 2 MFMA 32x32x16 blocks, 128 fp32
// accumulators), k-tiles are 64 elements (128 bytes per row) staged in LDS as
// [row][128 B + 16 B pad], double-buffered.  Two k-tiles are in flight in registers behind the
// one being multiplied; their loads are branch-free raw buffer loads (out-of-range offset =
// zeros, no memory request; see gemm_pf.h), so the hardware overlaps them with the MFMAs.
// One workgroup per compute unit (147 KB LDS).  bf16 storage only.
//
// The epilogue is specialised at compile time (BIG_*): with one workgroup per compute unit
// nothing overlaps it, and a run-time switch per element or an exact erf costs as much as the
// k-loop of a K = 512 problem.
//
// Two kernels: gemm_big_kernel (one tile per workgroup; every epilogue kind) and, further down,
// gemm_bigp_kernel (persistent: as many workgroups as compute units walk the tiles, with the
// loads, the bias and the stores of neighbouring tiles overlapped; select-kind epilogues), which
// the launcher takes whenever a launch has more tiles than compute units.
#pragma once
#include "gemm_pf.h"

namespace hfta {

constexpr int BIG_BM = 256, BIG_BN = 256, BIG_THREADS = 512, BIG_G = 8;
constexpr int BIG_BK = 64;                               // bf16 elements per k-tile
constexpr int BIG_PITCH = 16 * BIG_G + 16;               // 144 bytes
constexpr int BIG_TILE = 256 * BIG_PITCH;                // 36864 bytes per operand tile
constexpr int BIG_SMEM = 4 * BIG_TILE;                   // two operands, two stages
constexpr int BIG_EPI_PITCH = 256 * 2 + 8;               // bf16 staging row (8-byte aligned)
constexpr int BIG_EPI_PITCH4 = 256 * 4 + 16;             // fp32 staging row
constexpr int BIG_PF = 2;                                // k-tiles in flight in registers

// Epilogue kinds.  SEL: y = max(x, 0) + neg_slope * min(x, 0) -- identity (1), ReLU (0) and
// LeakyReLU (slope) without a branch.  GELU here is x * Phi(x) with erf from the Abramowitz-Stegun
// 7.1.26 rational form (|error| < 1.5e-7, far below bf16 resolution), TANH the library's.
enum { BIG_SEL = 0, BIG_TANH = 1, BIG_GELU = 2, BIG_NONE = 3 };

__device__ __forceinline__ float gelu_as(float x) {
  const float z = fabsf(x) * 0.70710678118654752f;
  const float tt = __builtin_amdgcn_rcpf(fmaf(0.3275911f, z, 1.f));
  float poly = fmaf(tt, 1.061405429f, -1.453152027f);
  poly = fmaf(tt, poly, 1.421413741f);
  poly = fmaf(tt, poly, -0.284496736f);
  poly = fmaf(tt, poly, 0.254829592f);
  poly *= tt;
  const float e = __builtin_amdgcn_exp2f(-z * z * 1.4426950408889634f);
  const float erf_abs = fmaf(-poly, e, 1.f);
  const float erf_x = copysignf(erf_abs, x);
  return 0.5f * x * (1.f + erf_x);
}

template <int ACT>
__device__ __forceinline__ float big_act(float x, float neg_slope) {
  if (ACT == BIG_NONE) return x;
  if (ACT == BIG_SEL) return fmaf(neg_slope, fminf(x, 0.f), fmaxf(x, 0.f));
  if (ACT == BIG_TANH) return tanhf(x);
  return gelu_as(x);
}

// RP staged rows x 256 columns -> global memory: consecutive lanes on consecutive 16- or 8-byte
// pieces of a row, so a wavefront's store covers whole row segments.
template <typename OutT, int THREADS>
__device__ __forceinline__ void big_store_rows(const unsigned char* smem, OutT* Cb, int64_t c_ld, int M, int N,
                                               int mbase, int n0, int c_vec, int t, int c_seg, int64_t c_seg_stride) {
  constexpr int ES = sizeof(OutT);
  constexpr int RP = ES == 2 ? 128 : 64;
  constexpr int PITCH = ES == 2 ? BIG_EPI_PITCH : BIG_EPI_PITCH4;
  if (c_vec == 16) {
    constexpr int EPV = 16 / ES, PPR = 256 / EPV, RPI = THREADS / PPR;
    const int r0 = t / PPR, c = t % PPR, n = n0 + c * EPV;
#pragma unroll 4
    for (int it = 0; it < RP / RPI; ++it) {
      const int rr = r0 + it * RPI, m = mbase + rr;
      const uint4 v = *reinterpret_cast<const uint4*>(smem + rr * PITCH + c * 16);
      OutT* dst = Cb + (int64_t)m * c_ld + col_offset(n, c_seg, c_seg_stride);
      if (m < M && n + EPV <= N) {
        *reinterpret_cast<uint4*>(dst) = v;
      } else if (m < M && n < N) {
        const OutT* e = reinterpret_cast<const OutT*>(&v);
#pragma unroll
        for (int k = 0; k < EPV; ++k)
          if (n + k < N) dst[k] = e[k];
      }
    }
  } else {
    constexpr int EPV = 8 / ES, PPR = 256 / EPV, RPI = THREADS / PPR;
    const int r0 = t / PPR, c = t % PPR, n = n0 + c * EPV;
#pragma unroll 4
    for (int it = 0; it < RP / RPI; ++it) {
      const int rr = r0 + it * RPI, m = mbase + rr;
      const uint2 v = *reinterpret_cast<const uint2*>(smem + rr * PITCH + c * 8);
      OutT* dst = Cb + (int64_t)m * c_ld + col_offset(n, c_seg, c_seg_stride);
      if (m < M && n + EPV <= N && c_vec == 8) {
        *reinterpret_cast<uint2*>(dst) = v;
      } else if (m < M && n < N) {
        const OutT* e = reinterpret_cast<const OutT*>(&v);
#pragma unroll
        for (int k = 0; k < EPV; ++k)
          if (n + k < N) dst[k] = e[k];
      }
    }
  }
}

// k-contiguous operand: 256 rows x 8 chunks of 16 bytes per k-tile, 4 chunks per thread
template <bool V16> struct BigOpKc {
  typedef uint4 Regs[4];
  uint32_t off[4];
  int kg;
  __device__ __forceinline__ void init(int row0, int rows, int64_t ld, int t) {
    kg = (t & 7) * 8;
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      const int r = row0 + (t >> 3) + 64 * h;
      off[h] = r < rows ? (uint32_t)((int64_t)r * ld * 2) + (uint32_t)kg * 2u : PF_OOB;
    }
  }
  __device__ __forceinline__ void load(Regs& q, __amdgpu_buffer_rsrc_t rs, int k0, int K) const {
    const int k = k0 + kg;
    if (V16) {
      const bool ok = k + 8 <= K;
#pragma unroll
      for (int h = 0; h < 4; ++h) {
        const pf_u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)(ok ? off[h] + (uint32_t)k0 * 2u : PF_OOB), 0, 0);
        q[h] = make_uint4(v.x, v.y, v.z, v.w);
      }
    } else {
      const bool ok0 = k + 4 <= K, ok1 = k + 8 <= K;
#pragma unroll
      for (int h = 0; h < 4; ++h) {
        const uint32_t o = off[h] + (uint32_t)k0 * 2u;
        const pf_u32x2 lo = __builtin_amdgcn_raw_buffer_load_b64(rs, (int)(ok0 ? o : PF_OOB), 0, 0);
        const pf_u32x2 hi = __builtin_amdgcn_raw_buffer_load_b64(rs, (int)(ok1 ? o + 8u : PF_OOB), 0, 0);
        q[h] = make_uint4(lo.x, lo.y, hi.x, hi.y);
      }
    }
  }
  static __device__ __forceinline__ void store(unsigned char* tile, const Regs& q, int t) {
#pragma unroll
    for (int h = 0; h < 4; ++h)
      *reinterpret_cast<uint4*>(tile + ((t >> 3) + 64 * h) * BIG_PITCH + (t & 7) * 16) = q[h];
  }
};

// m/n-contiguous operand kept in its natural layout in LDS ([64 k][256 n], 576-byte rows: the same
// 36864 bytes as the k-major tile) and transposed by the LDS transpose read on the way into the
// matrix-instruction fragments: no register shuffles, global loads and LDS stores of 16 bytes (N16)
// or 8 bytes (rows only 8-byte aligned, e.g. 2500 points).  A thread owns chunk t%32 (8 columns) of
// rows t/32 + 16h.
constexpr int BIG_NPITCH = 256 * 2 + 64;
static_assert(64 * BIG_NPITCH == BIG_TILE, "natural-layout tile must fit the k-major tile's bytes");
template <bool N16> struct BigOpNt {
  typedef uint4 Regs[4];
  uint32_t off0, off1;    // byte offsets of the chunk's two 8-byte halves in row k = t/32, or out of range
  uint32_t ldb;
  __device__ __forceinline__ void init(int col0, int cols, int64_t ld, int t) {
    ldb = (uint32_t)(ld * 2);
    const int c = col0 + (t & 31) * 8, kr = t >> 5;
    off0 = c + 4 <= cols ? (uint32_t)kr * ldb + (uint32_t)c * 2u : PF_OOB;
    off1 = c + 8 <= cols ? (uint32_t)kr * ldb + (uint32_t)c * 2u + 8u : PF_OOB;
  }
  __device__ __forceinline__ void load(Regs& q, __amdgpu_buffer_rsrc_t rs, int k0, int K) const {
    const int kr = (int)(threadIdx.x >> 5);
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      const bool ok = k0 + kr + 16 * h < K;
      const uint32_t kb = (uint32_t)(k0 + 16 * h) * ldb;
      if (N16) {               // host side: columns a multiple of 8, so the halves are in or out together
        const pf_u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)(ok && off1 != PF_OOB ? off0 + kb : PF_OOB), 0, 0);
        q[h] = make_uint4(v.x, v.y, v.z, v.w);
      } else {
        const pf_u32x2 lo = __builtin_amdgcn_raw_buffer_load_b64(rs, (int)(ok && off0 != PF_OOB ? off0 + kb : PF_OOB), 0, 0);
        const pf_u32x2 hi = __builtin_amdgcn_raw_buffer_load_b64(rs, (int)(ok && off1 != PF_OOB ? off1 + kb : PF_OOB), 0, 0);
        q[h] = make_uint4(lo.x, lo.y, hi.x, hi.y);
      }
    }
  }
  static __device__ __forceinline__ void store(unsigned char* tile, const Regs& q, int t) {
#pragma unroll
    for (int h = 0; h < 4; ++h)
      *reinterpret_cast<uint4*>(tile + ((t >> 5) + 16 * h) * BIG_NPITCH + (t & 31) * 16) = q[h];
  }
};

template <bool KC, bool V16, bool N16> struct BigOp;
template <bool V16, bool N16> struct BigOp<true, V16, N16> : BigOpKc<V16> {};
template <bool V16, bool N16> struct BigOp<false, V16, N16> : BigOpNt<N16> {};

// Fragment of the 32x32x16 matrix instruction for the 32 rows (columns of the natural tile) from
// `base` and k-step s: lane l holds row base + l%32 and k = 16s + 8(l/32) + 0..7.
typedef short big_v4s __attribute__((ext_vector_type(4)));
template <bool KC>
__device__ __forceinline__ bf16x8_t big_frag(const unsigned char* tile, int base, int s, int lane) {
  if (KC) return *reinterpret_cast<const bf16x8_t*>(tile + (base + (lane & 31)) * BIG_PITCH + (lane >> 5) * 16 + s * 32);
  // Transpose read: in every group of 16 lanes, lane r supplies the address of four neighbouring
  // columns in one k-row, and lane i = 4a + c receives column c of the rows supplied by lanes
  // a, a+4, a+8, a+12.  With lane r pointing at k-row r/4 and column quad r%4, lane i of the group
  // ends up with column i of the group's 16 and four consecutive k.
  const int r16 = lane & 15;
  const unsigned char* a0 = tile + (16 * s + 8 * (lane >> 5) + (r16 >> 2)) * BIG_NPITCH +
                            (base + 16 * ((lane >> 4) & 1) + 4 * (r16 & 3)) * 2;
  typedef __attribute__((address_space(3))) big_v4s* lds_v4s;
  const big_v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(a0));
  const big_v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(a0 + 4 * BIG_NPITCH));
  union { big_v4s h[2]; bf16x8_t v; } u;
  u.h[0] = lo; u.h[1] = hi;
  return u.v;
}

// COLB: bias per column n (the fused Linear's), else per row m or none.
template <bool A_KC, bool B_KC, typename OutT, bool V16, bool COLB, int ACT, bool N16 = false>
__global__ __launch_bounds__(BIG_THREADS) void gemm_big_kernel(GemmArgs p) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[BIG_SMEM];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 2, wn = wave & 3;               // 2 x 4 waves, 128 x 64 each
  // XCD-aware renumbering (see gemm_kernel)
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
  const int m0 = tile_m * BIG_BM, n0 = tile_n * BIG_BN;
  // split-K: this workgroup reduces k-tiles [t_begin, t_end) and writes an fp32 partial tile
  const int split = bz % p.splits, g = bz / p.splits;
  const int g0 = g / p.G1, g1 = g % p.G1;
  const int t_begin = (int)((int64_t)p.total_tiles * split / p.splits);
  const bf16_raw* Ab = reinterpret_cast<const bf16_raw*>(p.A) + g0 * p.a_g0 + g1 * p.a_g1;
  const bf16_raw* Bb = reinterpret_cast<const bf16_raw*>(p.Bm) + g0 * p.b_g0 + g1 * p.b_g1;

  f32x16_t acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  BigOp<A_KC, V16, N16> oa;
  BigOp<B_KC, V16, N16> ob;
  oa.init(m0, p.M, p.a_ld, t);
  ob.init(n0, p.N, p.b_ld, t);
  typename BigOp<A_KC, V16, N16>::Regs ra[BIG_PF];
  typename BigOp<B_KC, V16, N16>::Regs rb[BIG_PF];
  const int t_end = (int)((int64_t)p.total_tiles * (split + 1) / p.splits);
  auto issue = [&](int set, int tt) {
    const bool live = tt < t_end;
    const int Ke = live ? p.K : 0;      // a dead tile has no valid k: every offset out of range
    const int tc = live ? tt : 0;
    const int seg = tc / p.tiles_per_seg;
    const int k0 = (tc - seg * p.tiles_per_seg) * BIG_BK;
    oa.load(ra[set], pf_rsrc(Ab + seg * p.a_ss, p.a_extent), k0, Ke);
    ob.load(rb[set], pf_rsrc(Bb + seg * p.b_ss, p.b_extent), k0, Ke);
  };
  auto tileA = [&](int buf) { return smem + buf * 2 * BIG_TILE; };
  auto tileB = [&](int buf) { return smem + buf * 2 * BIG_TILE + BIG_TILE; };

#pragma unroll
  for (int d = 0; d < BIG_PF; ++d) issue(d, t_begin + d);
  oa.store(tileA(0), ra[0], t);
  ob.store(tileB(0), rb[0], t);
  __syncthreads();
  int buf = 0;
  const int r = lane & 31, gsel = lane >> 5;
  bool done = false;
  for (int base = t_begin; !done; base += BIG_PF) {
#pragma unroll
    for (int d = 0; d < BIG_PF; ++d) {
      const int cur = base + d;
      issue(d, cur + BIG_PF);
      const unsigned char* As = tileA(buf);
      const unsigned char* Bs = tileB(buf);
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        bf16x8_t a[4], b[2];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = big_frag<A_KC>(As, wm * 128 + i * 32, s, lane);
#pragma unroll
        for (int j = 0; j < 2; ++j) b[j] = big_frag<B_KC>(Bs, wn * 64 + j * 32, s, lane);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
      }
      if (cur + 1 >= t_end) { done = true; break; }
      oa.store(tileA(buf ^ 1), ra[(d + 1) % BIG_PF], t);
      ob.store(tileB(buf ^ 1), rb[(d + 1) % BIG_PF], t);
      __syncthreads();
      buf ^= 1;
    }
  }
  __syncthreads();

  // epilogue: bias + activation in registers, staged through LDS in the output type in passes of
  // 128 rows (2-byte outputs) / 64 rows (4-byte outputs), then 16- or 8-byte row-major stores.
  // lane l holds row m = l % 32 and columns 8*(v/4) + 4*(l/32) + v%4 of each 32x32 block.
  constexpr int ES = sizeof(OutT);
  constexpr int RP = ES == 2 ? 128 : 64;
  constexpr int PITCH = ES == 2 ? BIG_EPI_PITCH : BIG_EPI_PITCH4;
  const bool to_partial = ES == 4 && p.splits > 1;
  OutT* Cb = to_partial
      ? reinterpret_cast<OutT*>(p.partial) + ((int64_t)split * (gridDim.z / p.splits) + g) * (int64_t)p.M * p.N
      : reinterpret_cast<OutT*>(p.C) + g0 * p.c_g0 + g1 * p.c_g1;
  const int64_t c_ld = to_partial ? p.N : p.c_ld;
  const int c_vec = to_partial ? p.p_vec : p.c_vec;
  const int c_seg = to_partial ? 0 : p.c_seg;
  const bf16_raw* bias = p.bias ? reinterpret_cast<const bf16_raw*>(p.bias) + g0 * p.bias_g0 + g1 * p.bias_g1 : nullptr;
  const int ml = lane & 31, nq = (lane >> 5) * 4;
  const float neg_slope = p.slope;

  float cb[2][4][4];                                     // this lane's 32 column biases
  if (COLB) {
    const __amdgpu_buffer_rsrc_t rbias = pf_rsrc(bias, (uint32_t)p.N * 2u);
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = n0 + wn * 64 + j * 32 + 8 * q + nq;
        const pf_u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rbias, (int)(n + 4 <= p.N ? (uint32_t)n * 2u : PF_OOB), 0, 0);
        cb[j][q][0] = __uint_as_float(v.x << 16);
        cb[j][q][1] = __uint_as_float(v.x & 0xffff0000u);
        cb[j][q][2] = __uint_as_float(v.y << 16);
        cb[j][q][3] = __uint_as_float(v.y & 0xffff0000u);
      }
  }

#pragma unroll
  for (int pass = 0; pass < 256 / RP; ++pass) {
    if (wm == pass * RP / 128) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = i * 32;                          // first row of this block inside the wave's 128
        if (row / RP != (pass * RP % 128) / RP) continue;
        const int rl = row % RP + ml;
        const int m = m0 + wm * 128 + row + ml;
        float bm = 0.f;
        if (!COLB && bias && m < p.M) bm = bf16_to_f32(bias[m]);
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int nl = wn * 64 + j * 32 + 8 * q + nq;
            float x[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
              x[e] = big_act<ACT>(acc[i][j][4 * q + e] + (COLB ? cb[j][q][e] : bm), neg_slope);
            unsigned char* dst = smem + rl * PITCH + nl * ES;
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
    __syncthreads();
    big_store_rows<OutT, BIG_THREADS>(smem, Cb, c_ld, p.M, p.N, m0 + pass * RP, n0, c_vec, t, c_seg, p.c_seg_stride);
    if (pass + 1 < 256 / RP) __syncthreads();
  }
}

// ---- persistent variant ------------------------------------------------------------------
// One workgroup per compute unit walks the output tiles lin = blockIdx.x, blockIdx.x + gridDim.x, ...
// of the same XCD-aware numbering.  With one workgroup per compute unit nothing overlaps a tile's
// launch, first loads, bias fetch and epilogue, which together cost as much as nine k-tiles; here
// the loader runs two k-tiles ahead across tile boundaries, so the next tile's first two k-tiles
// (and this tile's bias) are in flight while the last two k-tiles are multiplied and the epilogue
// runs.  Rows of k-tiles come in pairs (an odd count multiplies one all-zero k-tile), which keeps
// the register sets' roles fixed at a tile boundary.  Stores are raw buffer stores (a piece outside
// the matrix gets an out-of-range offset and is dropped), so the epilogue is straight-line code and
// the wait for the prefetched loads does not have to cover the stores behind them.  The epilogue
// is vector-ALU bound (two waves per SIMD, nothing to overlap it), so no activation (BIG_NONE) is a
// compile-time case of its own rather than a select with slope 1.
// Host side guarantees: operands loadable in whole pieces of the width the instantiation uses,
// output rows aligned to the store piece (16 or 8 bytes), N a multiple of it, output slice below
// 2 GiB.
// rows staged per epilogue pass: the whole tile for 2-byte outputs (133 KB of the 144 KB the k-loop's
// tiles leave free: every wave converts at the same time), a quarter of it for 4-byte outputs
constexpr int BIGP_RP(int es) { return es == 2 ? 256 : 64; }
static_assert(256 * BIG_EPI_PITCH <= BIG_SMEM && 64 * BIG_EPI_PITCH4 <= BIG_SMEM, "staging must fit the tile buffers");

template <typename OutT, int VB>
__device__ __forceinline__ void bigp_store_rows(const unsigned char* smem, __amdgpu_buffer_rsrc_t rc, uint32_t c_ldb,
                                                int M, int mbase, uint32_t col_byte, int t) {
  constexpr int ES = sizeof(OutT);
  constexpr int RP = BIGP_RP(ES);
  constexpr int PITCH = ES == 2 ? BIG_EPI_PITCH : BIG_EPI_PITCH4;
  constexpr int EPV = VB / ES, PPR = 256 / EPV, RPI = BIG_THREADS / PPR;
  const int r0 = t / PPR, c = t % PPR;
  constexpr int NIT = RP / RPI;                          // pieces per thread, read NB at a time
  constexpr int NB = ES == 2 ? 4 : 2;
  typedef typename std::conditional<VB == 16, uint4, uint2>::type V;
#pragma unroll
  for (int h = 0; h < NIT; h += NB) {
    V v[NB];
#pragma unroll
    for (int it = 0; it < NB; ++it)
      v[it] = *reinterpret_cast<const V*>(smem + (r0 + (h + it) * RPI) * PITCH + c * VB);
#pragma unroll
    for (int it = 0; it < NB; ++it) {
      const int m = mbase + r0 + (h + it) * RPI;
      const uint32_t off = (m < M && col_byte != PF_OOB) ? (uint32_t)m * c_ldb + col_byte : PF_OOB;
      if constexpr (VB == 16) {
        pf_u32x4 w; w.x = v[it].x; w.y = v[it].y; w.z = v[it].z; w.w = v[it].w;
        __builtin_amdgcn_raw_buffer_store_b128(w, rc, (int)off, 0, 0);
      } else {
        pf_u32x2 w; w.x = v[it].x; w.y = v[it].y;
        __builtin_amdgcn_raw_buffer_store_b64(w, rc, (int)off, 0, 0);
      }
    }
  }
}

struct BigCoord { int m0, n0, g0, g1, split, g, t_begin, t_end; };

// STATS (2-byte output, row bias or none, no activation): while a tile sits staged in LDS on its way out, two
// threads per row add its 256 stored values and their squares (two-element dot products), origin moved to the
// row's bias, and leave one pair per (group, column tile, row): the BatchNorm that follows a k=1 convolution
// takes its statistics from these and reads the output once.  Columns past N hold the bias itself (their B
// operand was read as zeros) and add nothing to the shifted sums.
typedef __bf16 big_bf16x2 __attribute__((ext_vector_type(2)));
template <bool A_KC, bool B_KC, typename OutT, bool COLB, int ACT, bool V16, bool N16, bool STATS = false>
__global__ __launch_bounds__(BIG_THREADS) void gemm_bigp_kernel(GemmArgs p, int vgx, int vtotal) {
  static_assert(!STATS || (sizeof(OutT) == 2 && !COLB && ACT == BIG_NONE && BIG_THREADS == 512), "statistics epilogue: bf16 out, row bias, no activation");
  __shared__ __attribute__((aligned(16))) unsigned char smem[BIG_SMEM];
  __shared__ uint2 sbias[64];                            // this tile's 256 column biases (an object of its own:
                                                         // its reads need not wait for the staging writes)
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  constexpr int ES = sizeof(OutT);
  constexpr int RP = BIGP_RP(ES);
  constexpr int PITCH = ES == 2 ? BIG_EPI_PITCH : BIG_EPI_PITCH4;
  constexpr int EPV = 16 / ES;
  const bool to_partial = ES == 4 && p.splits > 1;
  const int groups = vtotal / vgx / p.splits;            // G0 * G1

  // tile lin of the virtual (tiles, 1, groups * splits) grid, renumbered as in gemm_big_kernel
  auto coord = [&](int lin) {
    int bx, bz;
    const int per = vtotal >> 3;
    const int l2 = lin < (per << 3) ? (lin & 7) * per + (lin >> 3) : lin;
    bz = l2 / vgx;
    bx = l2 - bz * vgx;
    BigCoord c;
    c.m0 = (bx % p.tiles_m) * BIG_BM;
    c.n0 = (bx / p.tiles_m) * BIG_BN;
    c.split = bz % p.splits;
    c.g = bz / p.splits;
    c.g0 = c.g / p.G1;
    c.g1 = c.g % p.G1;
    c.t_begin = (int)((int64_t)p.total_tiles * c.split / p.splits);
    c.t_end = (int)((int64_t)p.total_tiles * (c.split + 1) / p.splits);
    return c;
  };

  // loader state: the tile whose k-tiles are being fetched
  BigOp<A_KC, V16, N16> oa;
  BigOp<B_KC, V16, N16> ob;
  typename BigOp<A_KC, V16, N16>::Regs ra[BIG_PF];
  typename BigOp<B_KC, V16, N16>::Regs rb[BIG_PF];
  const bf16_raw* Ab;
  const bf16_raw* Bb;
  int l_end;
  auto aim = [&](const BigCoord& c, bool live) {
    Ab = reinterpret_cast<const bf16_raw*>(p.A) + c.g0 * p.a_g0 + c.g1 * p.a_g1;
    Bb = reinterpret_cast<const bf16_raw*>(p.Bm) + c.g0 * p.b_g0 + c.g1 * p.b_g1;
    l_end = live ? c.t_end : 0;
    oa.init(c.m0, p.M, p.a_ld, t);
    ob.init(c.n0, p.N, p.b_ld, t);
  };
  auto issue = [&](int set, int tt) {
    const bool live = tt < l_end;
    const int Ke = live ? p.K : 0;      // a dead k-tile has no valid k: every offset out of range
    const int tc = live ? tt : 0;
    const int seg = tc / p.tiles_per_seg;
    const int k0 = (tc - seg * p.tiles_per_seg) * BIG_BK;
    oa.load(ra[set], pf_rsrc(Ab + seg * p.a_ss, p.a_extent), k0, Ke);
    ob.load(rb[set], pf_rsrc(Bb + seg * p.b_ss, p.b_extent), k0, Ke);
  };
  auto tileA = [&](int buf) { return smem + buf * 2 * BIG_TILE; };
  auto tileB = [&](int buf) { return smem + buf * 2 * BIG_TILE + BIG_TILE; };

  f32x16_t acc[4][2];
  auto multiply = [&](int buf) {
    const unsigned char* As = tileA(buf);
    const unsigned char* Bs = tileB(buf);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      bf16x8_t a[4], b[2];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = big_frag<A_KC>(As, wm * 128 + i * 32, s, lane);
#pragma unroll
      for (int j = 0; j < 2; ++j) b[j] = big_frag<B_KC>(Bs, wn * 64 + j * 32, s, lane);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
    }
  };

  const int ml = lane & 31, nq = (lane >> 5) * 4;
  const float neg_slope = p.slope;
  // The bias is the accumulators' initial value, so the epilogue (vector-ALU bound) does not add
  // it.  Column biases of the tile about to start sit in `sbias` (wave 0 fetches the 256 of them);
  // row biases in four registers per lane.  The resource's extent does the bounds check (N is a
  // multiple of 4 for a column bias, so an 8-byte piece is inside or outside as a whole; no bias =
  // empty extent = zeros).
  unsigned short bmp[4] = {0, 0, 0, 0};
  auto fetch_bias = [&](const BigCoord& c, pf_u32x2& bcol) {
    const bf16_raw* bias = p.bias ? reinterpret_cast<const bf16_raw*>(p.bias) + c.g0 * p.bias_g0 + c.g1 * p.bias_g1 : nullptr;
    if (COLB) {
      const __amdgpu_buffer_rsrc_t rbias = pf_rsrc(bias, (uint32_t)p.N * 2u);
      bcol = __builtin_amdgcn_raw_buffer_load_b64(rbias, (int)(t < 64 ? (uint32_t)(c.n0 + 4 * t) * 2u : PF_OOB), 0, 0);
    } else {
      const __amdgpu_buffer_rsrc_t rbias = pf_rsrc(bias, bias ? (uint32_t)p.M * 2u : 0u);
      const uint32_t mb = (uint32_t)(c.m0 + wm * 128 + ml) * 2u;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        bmp[i] = __builtin_amdgcn_raw_buffer_load_b16(rbias, (int)(mb + (uint32_t)(i * 32) * 2u), 0, 0);
    }
  };
  auto park_bias = [&](const pf_u32x2& bcol) {
    if (COLB && wave_s == 0) {
      uint2 bv; bv.x = bcol.x; bv.y = bcol.y;
      sbias[(int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u))] = bv;
    }
  };

  BigCoord cur = coord(blockIdx.x);
  aim(cur, true);
  issue(0, cur.t_begin);
  issue(1, cur.t_begin + 1);
  {
    pf_u32x2 bcol;
    bcol.x = 0u; bcol.y = 0u;
    fetch_bias(cur, bcol);
    park_bias(bcol);
  }
  oa.store(tileA(0), ra[0], t);
  ob.store(tileB(0), rb[0], t);
  __syncthreads();

  // A pair multiplies the k-tile in LDS buffer 0 (its partner is in flight in register set 1), then
  // the partner from buffer 1; the loads it issues are two k-tiles ahead, and in the last pair of a
  // tile they belong to the next tile (or are dead after the last one).
  for (int lin = blockIdx.x;;) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float cbv[4];
        if (COLB) {
          const uint2 cb = sbias[(wn * 64 + j * 32 + 8 * q + nq) >> 2];
          cbv[0] = __uint_as_float(cb.x << 16);
          cbv[1] = __uint_as_float(cb.x & 0xffff0000u);
          cbv[2] = __uint_as_float(cb.y << 16);
          cbv[3] = __uint_as_float(cb.y & 0xffff0000u);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int e = 0; e < 4; ++e)
            acc[i][j][4 * q + e] = COLB ? cbv[e] : __uint_as_float((uint32_t)bmp[i] << 16);
      }

    const int pairs = (cur.t_end - cur.t_begin + 1) >> 1;
    const int nlin = lin + (int)gridDim.x;
    const bool more = nlin < vtotal;
    BigCoord nxt = cur;
    pf_u32x2 bcol;
    bcol.x = 0u; bcol.y = 0u;
    int tt = cur.t_begin + 2;
    for (int pr = 1;; ++pr, tt += 2) {
      const bool last = pr >= pairs;
      if (last) {
        if (more) nxt = coord(nlin);
        aim(nxt, more);
        tt = nxt.t_begin;
        fetch_bias(nxt, bcol);               // the next tile's (a repeat of this one's after the last)
      }
      issue(0, tt);
      multiply(0);
      oa.store(tileA(1), ra[1], t);
      ob.store(tileB(1), rb[1], t);
      __syncthreads();
      issue(1, tt + 1);
      multiply(1);
      if (last) break;
      oa.store(tileA(0), ra[0], t);
      ob.store(tileB(0), rb[0], t);
      __syncthreads();
    }
    // (thread index rebuilt from the wave number in a scalar register and the lane count, so that
    // it is not carried in a vector register through the k-loop)
    const int lane_e = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    park_bias(bcol);
    __syncthreads();

    // epilogue (see gemm_big_kernel): lane l holds row l % 32 and columns 8*(v/4) + 4*(l/32) + v%4
    {
      OutT* Cb = to_partial
          ? reinterpret_cast<OutT*>(p.partial) + ((int64_t)cur.split * groups + cur.g) * (int64_t)p.M * p.N
          : reinterpret_cast<OutT*>(p.C) + cur.g0 * p.c_g0 + cur.g1 * p.c_g1;
      const uint32_t c_ldb = (uint32_t)((to_partial ? (int64_t)p.N : p.c_ld) * ES);
      const __amdgpu_buffer_rsrc_t rc = pf_rsrc(Cb, to_partial ? (uint32_t)((int64_t)p.M * p.N * 4) : p.c_extent);
      // this thread's store column; computed here from opaque copies so that neither it nor the
      // segment division's reciprocal is carried in registers through the k-loop
      int tq = wave_s * 64 + lane_e, cs = p.c_seg;
      asm volatile("" : "+v"(tq), "+s"(cs));
      const int vb = to_partial ? p.p_vec : p.c_vec;     // 16- or 8-byte store pieces
      const int epv = vb / ES;
      const int n = cur.n0 + (tq % (256 / epv)) * epv;
      const uint32_t col_byte = n + epv <= p.N
          ? (uint32_t)((to_partial ? (int64_t)n : col_offset(n, cs, p.c_seg_stride)) * ES) : PF_OOB;
#pragma unroll
      for (int pass = 0; pass < 256 / RP; ++pass) {
        if (RP >= 128 ? (wm * 128) / RP == pass : wm == pass * RP / 128) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            if (RP < 128 && (i * 32) / RP != (pass * RP % 128) / RP) continue;   // this 32-row block's pass
            const int rl = (wm * 128 + i * 32) % RP + ml;
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const int nl = wn * 64 + j * 32 + 8 * q + nq;
                float x[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) x[e] = big_act<ACT>(acc[i][j][4 * q + e], neg_slope);
                unsigned char* dst = smem + rl * PITCH + nl * ES;
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
        __syncthreads();
        if (vb == 16) bigp_store_rows<OutT, 16>(smem, rc, c_ldb, p.M, cur.m0 + pass * RP, col_byte, t);
        else bigp_store_rows<OutT, 8>(smem, rc, c_ldb, p.M, cur.m0 + pass * RP, col_byte, t);
        if constexpr (STATS) {             // RP == 256: the whole tile is staged in this one pass
          const int row = t >> 1, half = t & 1, m = cur.m0 + row;
          const unsigned char* src = smem + row * PITCH + half * 256;
          const big_bf16x2 ones = __builtin_bit_cast(big_bf16x2, 0x3f803f80u);
          float s1 = 0.f, s2 = 0.f;
#pragma unroll 8
          for (int q = 0; q < 32; ++q) {
            const uint2 v = *reinterpret_cast<const uint2*>(src + q * 8);
            const big_bf16x2 lo = __builtin_bit_cast(big_bf16x2, v.x), hi = __builtin_bit_cast(big_bf16x2, v.y);
            s1 = __builtin_amdgcn_fdot2_f32_bf16(lo, ones, s1, false);
            s2 = __builtin_amdgcn_fdot2_f32_bf16(lo, lo, s2, false);
            s1 = __builtin_amdgcn_fdot2_f32_bf16(hi, ones, s1, false);
            s2 = __builtin_amdgcn_fdot2_f32_bf16(hi, hi, s2, false);
          }
          const bf16_raw* rb_ = p.bias ? reinterpret_cast<const bf16_raw*>(p.bias) + cur.g0 * p.bias_g0 + cur.g1 * p.bias_g1 : nullptr;
          const float shift = (rb_ && m < p.M) ? bf16_to_f32(rb_[m]) : 0.f;
          s2 = fmaf(shift, fmaf(128.f, shift, -2.f * s1), s2);   // sum (c - b)^2 = sum c^2 - 2 b sum c + 128 b^2
          s1 = fmaf(-128.f, shift, s1);
          s1 += __shfl_xor(s1, 1, 64);
          s2 += __shfl_xor(s2, 1, 64);
          if (half == 0 && m < p.M)
            *reinterpret_cast<float2*>(p.stat_part + (((int64_t)cur.g * p.tiles_n + cur.n0 / BIG_BN) * p.M + m) * 2) = make_float2(s1, s2);
        }
        __syncthreads();
      }
    }
    if (!more) break;
    oa.store(tileA(0), ra[0], t);
    ob.store(tileB(0), rb[0], t);
    __syncthreads();
    cur = nxt;
    lin = nlin;
  }
}

}  // namespace hfta
