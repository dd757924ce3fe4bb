// Deep-prefetch variant of the 128x128 bf16 GEMM kernel.
//
// Same tiling, LDS layout, MFMA schedule and epilogue as gemm_kernel; what differs is how operand
// tiles travel from memory to LDS.  PF k-tiles are in flight in registers at any time instead of
// one, which is what a workgroup needs to keep HBM busy when the k-loop does little arithmetic per
// byte (the fused k=1 convolutions of a point-cloud model: K = 64..1024 against millions of
// columns).  For the hardware to overlap them, the loads of a step must not sit under control
// flow: every load is a raw buffer load whose offset is either inside the operand slice or a
// fixed out-of-range value, for which the hardware returns zeros and makes no memory request.
// Rows / columns beyond the matrix, k beyond K and k-tiles beyond the end of the loop are all
// expressed that way, so the steady-state loop issues PF-1 tiles ahead with no branches.
//
// Eligibility (checked by the host): bf16 operands, every 8-byte (16-byte when V16) piece of an
// operand either wholly inside or wholly outside the matrix, each operand slice below 2 GiB.
#pragma once
#include "gemm.h"

namespace hfta {

typedef uint32_t pf_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t pf_u32x2 __attribute__((ext_vector_type(2)));
constexpr uint32_t PF_OOB = 0x80000000u;   // >= any slice extent: the load returns zeros

__device__ __forceinline__ __amdgpu_buffer_rsrc_t pf_rsrc(const void* p, uint32_t bytes) {
  // raw buffer (stride 0), 32-bit data format; the range check is offset >= bytes
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// Per-thread addressing of one operand; q-sets (the staged data) are kept apart so that several
// tiles can be in flight with one copy of the offsets.
template <bool KC, bool V16> struct PfOperand;

template <bool V16> struct PfOperand<true, V16> {   // k-contiguous: rows t/4 and t/4+64, 16-byte group t%4
  typedef uint4 Regs[2];
  uint32_t off[2];
  int kg;
  __device__ __forceinline__ void init(int row0, int rows, int64_t ld, int t) {
    kg = (t & 3) * 8;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int r = row0 + (t >> 2) + 64 * h;
      off[h] = r < rows ? (uint32_t)((int64_t)r * ld * 2) + (uint32_t)kg * 2u : PF_OOB;
    }
  }
  __device__ __forceinline__ void load(Regs& q, __amdgpu_buffer_rsrc_t rs, int k0, int K) const {
    const int k = k0 + kg;
    if (V16) {
      const bool ok = k + 8 <= K;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const pf_u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)(ok ? off[h] + (uint32_t)k0 * 2u : PF_OOB), 0, 0);
        q[h] = make_uint4(v.x, v.y, v.z, v.w);
      }
    } else {
      const bool ok0 = k + 4 <= K, ok1 = k + 8 <= K;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const uint32_t o = off[h] + (uint32_t)k0 * 2u;
        const pf_u32x2 lo = __builtin_amdgcn_raw_buffer_load_b64(rs, (int)(ok0 ? o : PF_OOB), 0, 0);
        const pf_u32x2 hi = __builtin_amdgcn_raw_buffer_load_b64(rs, (int)(ok1 ? o + 8u : PF_OOB), 0, 0);
        q[h] = make_uint4(lo.x, lo.y, hi.x, hi.y);
      }
    }
  }
  static __device__ __forceinline__ void store(unsigned char* tile, const Regs& q, int t) { store_kc(tile, q, t); }
};

// m/n-contiguous operand: kept in its natural layout in LDS ([32 k][128 n], 320-byte rows = the k-major
// tile's 10240 bytes) and transposed by the LDS transpose read on the way into the matrix-instruction
// fragments.  A thread owns chunk t%16 (8 columns) of k-rows t/16 and t/16 + 16; N16: the chunk is one
// 16-byte piece (row starts 16-byte aligned, columns a multiple of 8), else two 8-byte pieces.
constexpr int PF_NPITCH = 128 * 2 + 64;
static_assert(32 * PF_NPITCH == GEMM_TILE_BYTES, "natural-layout tile must fit the k-major tile's bytes");
template <bool N16> struct PfOperandNt {
  typedef uint4 Regs[2];
  uint32_t off0, off1;
  uint32_t ldb;
  __device__ __forceinline__ void init(int col0, int cols, int64_t ld, int t) {
    ldb = (uint32_t)(ld * 2);
    const int c = col0 + (t & 15) * 8, kr = t >> 4;
    off0 = c + 4 <= cols ? (uint32_t)kr * ldb + (uint32_t)c * 2u : PF_OOB;
    off1 = c + 8 <= cols ? (uint32_t)kr * ldb + (uint32_t)c * 2u + 8u : PF_OOB;
  }
  __device__ __forceinline__ void load(Regs& q, __amdgpu_buffer_rsrc_t rs, int k0, int K) const {
    const int kr = (int)(threadIdx.x >> 4);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const bool ok = k0 + kr + 16 * h < K;
      const uint32_t kb = (uint32_t)(k0 + 16 * h) * ldb;
      if (N16) {
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
    for (int h = 0; h < 2; ++h)
      *reinterpret_cast<uint4*>(tile + ((t >> 4) + 16 * h) * PF_NPITCH + (t & 15) * 16) = q[h];
  }
};
template <bool V16> struct PfOperand<false, V16> : PfOperandNt<V16> {};   // for this operand kind V16 means N16

// Fragment for the 32 rows (columns of a natural-layout tile) from `base`, k-step s of the 32-deep tile:
// lane l holds row base + l%32 and k = 16s + 8(l/32) + 0..7.  Transpose read: in every group of 16
// lanes, lane r supplies the address of four neighbouring columns in one k-row and lane i = 4a + c
// receives column c of the rows supplied by lanes a, a+4, a+8, a+12; with lane r on k-row r/4 and
// column quad r%4, lane i ends up with column i of the group's 16 and four consecutive k.
typedef short pf_v4s __attribute__((ext_vector_type(4)));
template <bool KC>
__device__ __forceinline__ bf16x8_t pf_frag(const unsigned char* tile, int base, int s, int lane) {
  if (KC) return *reinterpret_cast<const bf16x8_t*>(tile + (base + (lane & 31)) * GEMM_PITCH + (2 * s + (lane >> 5)) * 16);
  const int r16 = lane & 15;
  const unsigned char* a0 = tile + (16 * s + 8 * (lane >> 5) + (r16 >> 2)) * PF_NPITCH +
                            (base + 16 * ((lane >> 4) & 1) + 4 * (r16 & 3)) * 2;
  typedef __attribute__((address_space(3))) pf_v4s* lds_v4s;
  union { pf_v4s h[2]; bf16x8_t v; } u;
  u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(a0));
  u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(a0 + 4 * PF_NPITCH));
  return u.v;
}

template <bool A_KC, bool B_KC>
__device__ __forceinline__ void pf_mma_tile(f32x16_t (&acc)[2][2], const unsigned char* As, const unsigned char* Bs,
                                            int wm, int wn, int lane) {
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    bf16x8_t a[2], b[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      a[i] = pf_frag<A_KC>(As, wm * 64 + i * 32, s, lane);
      b[i] = pf_frag<B_KC>(Bs, wn * 64 + i * 32, s, lane);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
  }
}

template <bool A_KC, bool B_KC, typename OutT, bool V16, int PF, bool N16 = false>
// three workgroups per compute unit: the register budget this asks for (<= 168) makes the compiler keep
// the accumulators in ordinary registers (120-137 in all), 40 KB of LDS each; four spill
__global__ __launch_bounds__(GEMM_THREADS, 3) void gemm_pf_kernel(GemmArgs p) {
  typedef bf16_raw T;
  constexpr int BK = GemmT<T>::BK;
  __shared__ __attribute__((aligned(16))) unsigned char smem[2][2][GEMM_TILE_BYTES];

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  int bx = blockIdx.x, bz = blockIdx.z;
  {  // XCD-aware renumbering, as in gemm_kernel
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

  PfOperand<A_KC, A_KC ? V16 : N16> oa;
  PfOperand<B_KC, B_KC ? V16 : N16> ob;
  oa.init(m0, p.M, p.a_ld, t);
  ob.init(n0, p.N, p.b_ld, t);
  typename PfOperand<A_KC, A_KC ? V16 : N16>::Regs ra[PF];
  typename PfOperand<B_KC, B_KC ? V16 : N16>::Regs rb[PF];

  auto issue = [&](int set, int tt) {
    const bool live = tt < t_end;
    const int Ke = live ? p.K : 0;      // a dead tile has no valid k: every offset out of range
    const int tc = live ? tt : t_begin;
    const int seg = tc / p.tiles_per_seg;
    const int k0 = (tc - seg * p.tiles_per_seg) * BK;
    oa.load(ra[set], pf_rsrc(Ab + seg * p.a_ss, p.a_extent), k0, Ke);
    ob.load(rb[set], pf_rsrc(Bb + seg * p.b_ss, p.b_extent), k0, Ke);
  };

  if (t_begin < t_end) {
#pragma unroll
    for (int d = 0; d < PF; ++d) issue(d, t_begin + d);
    oa.store(smem[0][0], ra[0], t);
    ob.store(smem[0][1], rb[0], t);
    __syncthreads();
    int buf = 0;
    bool done = false;
    for (int base = t_begin; !done; base += PF) {
#pragma unroll
      for (int d = 0; d < PF; ++d) {
        const int cur = base + d;          // tile in LDS buffer `buf`; it came through register set d
        issue(d, cur + PF);                // set d is free again; beyond the end: zeros, no traffic
        pf_mma_tile<A_KC, B_KC>(acc, smem[buf][0], smem[buf][1], wm, wn, lane);
        if (cur + 1 >= t_end) { done = true; break; }
        oa.store(smem[buf ^ 1][0], ra[(d + 1) % PF], t);
        ob.store(smem[buf ^ 1][1], rb[(d + 1) % PF], t);
        __syncthreads();
        buf ^= 1;
      }
    }
    __syncthreads();
  }

  if (p.splits > 1) {
    float* Pb = p.partial + ((int64_t)split * (gridDim.z / p.splits) + g) * (int64_t)p.M * p.N;
    store_tile<float, T, false>(acc, &smem[0][0][0], Pb, p.N, p.M, p.N, m0, n0, nullptr, 0, HFTA_ACT_NONE, 0.f, p.p_vec, t);
    return;
  }
  OutT* Cb = reinterpret_cast<OutT*>(p.C) + g0 * p.c_g0 + g1 * p.c_g1;
  const T* bias = p.bias ? reinterpret_cast<const T*>(p.bias) + g0 * p.bias_g0 + g1 * p.bias_g1 : nullptr;
  // fp32 results of bf16 operands are weight gradients: the host never pairs them with a column bias
  // or a transcendental activation, and leaving that code out halves the kernel's registers
  store_tile<OutT, T, sizeof(OutT) == 2>(acc, &smem[0][0][0], Cb, p.c_ld, p.M, p.N, m0, n0, bias, p.bias_mode, p.act, p.slope, p.c_vec, t, p.c_seg, p.c_seg_stride);
}

int gemm_pf_launch(const GemmDesc& d, const GemmArgs& a, bool v16, bool n16, dim3 grid, hipStream_t st);

}  // namespace hfta
