// Compute-bound variant of the batched GEMM core: 256x256 output tile per 512-thread workgroup.
//
// The 128x128 kernel in gemm.h reads 32 bytes of LDS per MFMA cycle and wave, which is the
// whole LDS bandwidth of a compute unit, and moves 64 flop per byte it pulls from L2.  For the
// MLP-sized GEMMs (M, N >= 256, K >= 128) this kernel doubles both ratios: eight wavefronts in a
// 2 (m) x 4 (n) grid each own a 128x64 block (4 x 2 MFMA 32x32x16 blocks, 128 fp32
// accumulators), k-tiles are 64 elements (128 bytes per row) staged in LDS as
// [row][128 B + 16 B pad], double-buffered, with the next k-tile's global loads parked in
// registers while the current one is multiplied.  One workgroup per compute unit (147 KB LDS).
// bf16 storage only; operands must satisfy the fast-path alignment rules of the 128x128 kernel.
#pragma once
#include "gemm.h"

namespace hfta {

constexpr int BIG_BM = 256, BIG_BN = 256, BIG_THREADS = 512, BIG_G = 8;
constexpr int BIG_BK = 64;                               // bf16 elements per k-tile
constexpr int BIG_PITCH = 16 * BIG_G + 16;               // 144 bytes
constexpr int BIG_TILE = 256 * BIG_PITCH;                // 36864 bytes per operand tile
constexpr int BIG_SMEM = 4 * BIG_TILE;                   // two operands, two stages
constexpr int BIG_EPI_PITCH = 256 * 2 + 8;               // bf16 staging row (8-byte aligned)
constexpr int BIG_EPI_PITCH4 = 256 * 4 + 16;             // fp32 staging row

// k-contiguous operand: 256 rows x 8 chunks of 16 bytes, 4 chunks per thread
struct BigStageKc {
  uint4 q[4];
  __device__ __forceinline__ void load(const bf16_raw* base, int64_t ld, int row0, int rows, int k0, int K, int vec, int t) {
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      const int id = t + BIG_THREADS * h;
      const int g = id & 7, r = row0 + (id >> 3);
      const int k = k0 + g * 8;
      const bf16_raw* src = base + (int64_t)r * ld + k;
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (vec == 2) {
        if (r < rows && k + 8 <= K) v = *reinterpret_cast<const uint4*>(src);
      } else {
        if (r < rows && k + 4 <= K) { const uint2 lo = *reinterpret_cast<const uint2*>(src); v.x = lo.x; v.y = lo.y; }
        if (r < rows && k + 8 <= K) { const uint2 hi = *reinterpret_cast<const uint2*>(src + 4); v.z = hi.x; v.w = hi.y; }
      }
      q[h] = v;
    }
  }
  __device__ __forceinline__ void store(unsigned char* tile, int t) const {
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      const int id = t + BIG_THREADS * h;
      *reinterpret_cast<uint4*>(tile + (id >> 3) * BIG_PITCH + (id & 7) * 16) = q[h];
    }
  }
};

// m/n-contiguous operand: [64 k][256 n] as 16 k-quads x 64 n-groups of 4(k) x 4(n) blocks, 2 per thread
struct BigStageNc {
  uint2 q[2][4];
  __device__ __forceinline__ void load(const bf16_raw* base, int64_t ld, int col0, int cols, int k0, int K, int vec, int t) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int id = t + BIG_THREADS * h;
      const int kq = (id >> 9) * 8 + (id & 7), ng = (id >> 3) & 63;
      const int c = col0 + ng * 4;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int k = k0 + 4 * kq + j;
        uint2 v = make_uint2(0u, 0u);
        if (k < K && c + 4 <= cols) v = *reinterpret_cast<const uint2*>(base + (int64_t)k * ld + c);
        q[h][j] = v;
      }
    }
  }
  __device__ __forceinline__ void store(unsigned char* tile, int t) const {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int id = t + BIG_THREADS * h;
      const int kq = (id >> 9) * 8 + (id & 7), ng = (id >> 3) & 63;
      const uint32_t a0 = q[h][0].x, a1 = q[h][1].x, a2 = q[h][2].x, a3 = q[h][3].x;
      const uint32_t b0 = q[h][0].y, b1 = q[h][1].y, b2 = q[h][2].y, b3 = q[h][3].y;
      uint2 o[4];
      o[0] = make_uint2((a0 & 0xffffu) | (a1 << 16), (a2 & 0xffffu) | (a3 << 16));
      o[1] = make_uint2((a0 >> 16) | (a1 & 0xffff0000u), (a2 >> 16) | (a3 & 0xffff0000u));
      o[2] = make_uint2((b0 & 0xffffu) | (b1 << 16), (b2 & 0xffffu) | (b3 << 16));
      o[3] = make_uint2((b0 >> 16) | (b1 & 0xffff0000u), (b2 >> 16) | (b3 & 0xffff0000u));
#pragma unroll
      for (int i = 0; i < 4; ++i)
        *reinterpret_cast<uint2*>(tile + (ng * 4 + i) * BIG_PITCH + kq * 8) = o[i];
    }
  }
};

template <bool KC> struct BigStage;
template <> struct BigStage<true> : BigStageKc {};
template <> struct BigStage<false> : BigStageNc {};

// SLOW = true: per-column bias and/or tanh / GELU.  The fp32 accumulators are staged and bias +
// activation run once per element in the rolled store loop (see store_tile_impl in gemm.h).
template <bool A_KC, bool B_KC, typename OutT, bool SLOW>
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
  const int g0 = bz / p.G1, g1 = bz % p.G1;
  const bf16_raw* Ab = reinterpret_cast<const bf16_raw*>(p.A) + g0 * p.a_g0 + g1 * p.a_g1;
  const bf16_raw* Bb = reinterpret_cast<const bf16_raw*>(p.Bm) + g0 * p.b_g0 + g1 * p.b_g1;

  f32x16_t acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  BigStage<A_KC> sa;
  BigStage<B_KC> sb;
  auto issue = [&](int tt) {
    const int seg = tt / p.tiles_per_seg;
    const int k0 = (tt - seg * p.tiles_per_seg) * BIG_BK;
    sa.load(Ab + seg * p.a_ss, p.a_ld, m0, p.M, k0, p.K, p.a_vec, t);
    sb.load(Bb + seg * p.b_ss, p.b_ld, n0, p.N, k0, p.K, p.b_vec, t);
  };
  auto tileA = [&](int buf) { return smem + buf * 2 * BIG_TILE; };
  auto tileB = [&](int buf) { return smem + buf * 2 * BIG_TILE + BIG_TILE; };

  issue(0);
  sa.store(tileA(0), t);
  sb.store(tileB(0), t);
  __syncthreads();
  int buf = 0;
  const int r = lane & 31, gsel = lane >> 5;
  for (int tt = 0; tt < p.total_tiles; ++tt) {
    const bool more = tt + 1 < p.total_tiles;
    if (more) issue(tt + 1);
    const unsigned char* As = tileA(buf) + (wm * 128 + r) * BIG_PITCH + gsel * 16;
    const unsigned char* Bs = tileB(buf) + (wn * 64 + r) * BIG_PITCH + gsel * 16;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      bf16x8_t a[4], b[2];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = *reinterpret_cast<const bf16x8_t*>(As + i * 32 * BIG_PITCH + s * 32);
#pragma unroll
      for (int j = 0; j < 2; ++j) b[j] = *reinterpret_cast<const bf16x8_t*>(Bs + j * 32 * BIG_PITCH + s * 32);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
    }
    if (more) {
      sa.store(tileA(buf ^ 1), t);
      sb.store(tileB(buf ^ 1), t);
    }
    __syncthreads();
    buf ^= 1;
  }

  // epilogue: stage through LDS in passes of 128 rows (2-byte staging) / 64 rows (4-byte staging),
  // then wide row stores.  lane l holds row m = l % 32 and columns 8*(v/4) + 4*(l/32) + v%4 of
  // each 32x32 block.
  constexpr int ES = SLOW ? 4 : (int)sizeof(OutT);       // staged element size
  constexpr int OS = sizeof(OutT);
  constexpr int RP = ES == 2 ? 128 : 64;
  constexpr int PITCH = ES == 2 ? BIG_EPI_PITCH : BIG_EPI_PITCH4;
  constexpr int EPC = 16 / ES, CPR = 256 / EPC;
  OutT* Cb = reinterpret_cast<OutT*>(p.C) + g0 * p.c_g0 + g1 * p.c_g1;
  const bf16_raw* bias = p.bias ? reinterpret_cast<const bf16_raw*>(p.bias) + g0 * p.bias_g0 + g1 * p.bias_g1 : nullptr;
  const int ml = lane & 31, nq = (lane >> 5) * 4;
#pragma unroll 1
  for (int pass = 0; pass < 256 / RP; ++pass) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = wm * 128 + i * 32;                 // first row of this block inside the tile
      if (row / RP != pass) continue;
      const int rl = row % RP + ml;
      const int m = m0 + row + ml;
      float bm = 0.f;
      if (bias && p.bias_mode == 1 && m < p.M) bm = bf16_to_f32(bias[m]);
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int nl = wn * 64 + j * 32 + 8 * q + nq;
          float x[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            x[e] = acc[i][j][4 * q + e] + bm;
            if (!SLOW) x[e] = cheap_act(x[e], p.act, p.slope);
          }
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
    __syncthreads();
#pragma unroll 1
    for (int id = t; id < RP * CPR; id += BIG_THREADS) {
      const int rr = id / CPR, c = id % CPR;
      const int m = m0 + pass * RP + rr, n = n0 + c * EPC;
      if (m >= p.M || n >= p.N) continue;
      const unsigned char* src = smem + rr * PITCH + c * 16;
      OutT* dst = Cb + (int64_t)m * p.c_ld + n;
      if (SLOW) {
        const float4 v = *reinterpret_cast<const float4*>(src);
        float x[4] = {v.x, v.y, v.z, v.w};
        OutT o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (bias && p.bias_mode == 2 && n + e < p.N) x[e] += bf16_to_f32(bias[n + e]);
          o[e] = Elem<OutT>::from_f32(apply_act(x[e], p.act, p.slope));
        }
        if (n + 4 <= p.N && p.c_vec >= 4 * OS) {
          if (OS == 2) *reinterpret_cast<uint2*>(dst) = *reinterpret_cast<const uint2*>(o);
          else *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(o);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (n + e < p.N) dst[e] = o[e];
        }
      } else {
        const uint2 lo = *reinterpret_cast<const uint2*>(src);
        const uint2 hi = *reinterpret_cast<const uint2*>(src + 8);
        if (p.c_vec == 16 && n + EPC <= p.N) {
          *reinterpret_cast<uint4*>(dst) = make_uint4(lo.x, lo.y, hi.x, hi.y);
        } else if (p.c_vec >= 8 && n + EPC <= p.N) {
          *reinterpret_cast<uint2*>(dst) = lo;
          *reinterpret_cast<uint2*>(dst + EPC / 2) = hi;
        } else {
          OutT e[EPC];
          *reinterpret_cast<uint2*>(e) = lo;
          *reinterpret_cast<uint2*>(reinterpret_cast<unsigned char*>(e) + 8) = hi;
#pragma unroll
          for (int k = 0; k < EPC; ++k)
            if (n + k < p.N) dst[k] = e[k];
        }
      }
    }
    __syncthreads();
  }
}

}  // namespace hfta
