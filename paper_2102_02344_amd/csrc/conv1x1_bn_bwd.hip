// Backward of the fused Conv1d(k=1) -> BatchNorm1d (training) -> activation block of the point-cloud
// models (fusion rules table, rows "Conv1d" and "BatchNorm1d"; the per-point layers 64 -> 64 -> 128
// of the classification network) as ONE streaming pass over the activations.
//
// With dY the gradient at the block's output, z the stored convolution output and x its input,
//     g  = dY * act'(gamma * xhat + beta),          xhat = (z - mean) * invstd
//     dz = gamma * invstd * (g - mean(g) - xhat * mean(g * xhat))                  (BatchNorm)
//     dX[ci][l] = sum_co W[co][ci] dz[co][l],   dW[co][ci] = sum_{n,l} dz[co][l] x[ci][l],
//     dbias[co] = sum_{n,l} dz[co][l]                                               (convolution)
// The two means need all of dY and z once (a reduction kernel of the BatchNorm file leaves them as
// per-channel constants); everything else is done here per 128-point slice: the slice of dY and z
// comes from HBM once, dz is formed in registers, rounded to the storage type (so that the result is
// the one of the two single operators run back to back with dz stored in between) and laid into LDS
// twice -- [point][co] as the k-contiguous operand of the dX product and [co][point] as the one of
// the dW product -- next to the x slice.  dz itself never goes to HBM: against BatchNorm backward,
// data gradient and weight gradient as three kernels this leaves out one store and two loads of a
// [Nb, B*Co, L] tensor and one load of dY and z.
//
// A workgroup (eight wavefronts) is persistent: it walks over `tiles / G` slices of one model, keeps
// that model's W^T tile and per-channel constants in LDS and its share of dW in accumulator
// registers.  The next DEPTH slices are in flight in registers, each set reissued as soon as its
// slice has been laid into LDS; a round of DEPTH slices has no exit in its middle (a slice past the
// end runs empty), so that the wait on the oldest set leaves the younger ones in flight.  Measured:
// one or two slices ahead are enough, three or four change nothing (the [Nb, C, L] layout makes every
// slice 64..128 separate 256-byte row segments, and that access pattern, not the number of bytes in
// flight, is what holds the kernel at about 4 TB/s), so DEPTH is set by the register budget.  At the
// end every workgroup writes fp32 partials of dW and dbias; a second kernel adds the partials of a
// model in a fixed order.  Loads are raw buffer loads: anything outside an operand is an
// out-of-range offset that returns zeros without a memory request.
#include "gemm_pf.h"
#include "bn_common.h"
#include "in_norm.h"

namespace hfta {

int bn_bwd_coef(int B, int Nb, int C, int L, int dtype, const void* X, const int64_t xs[4], const void* dY,
                const int64_t dys[4], const float* gamma, const float* beta, const float* save_mean,
                const float* save_invstd, float* dgamma, float* dbeta, float* coef, int act, float slope, hipStream_t st);
int bn_bwd_coef_from_sums(int B, int Nb, int C, int L, const float* sums, const float* gamma, const float* beta,
                          const float* save_mean, const float* save_invstd, float* dgamma, float* dbeta, float* coef,
                          hipStream_t st);

namespace {

struct CbbArgs {
  const bf16_raw* dY; const bf16_raw* Z; const bf16_raw* X; const bf16_raw* W;
  bf16_raw* dX;                  // nullptr: no data gradient (the network's first layer)
  const float* coef;             // [B][Co][8]: mean, invstd, gamma, beta, mean(g), mean(g xhat), gamma*invstd, 0
  float* part;                   // [G * KS][B*Co*Ci + B*Co + 2*B*Ci]: dW partials, dbias partials, partials of the input block's two sums
  int64_t dy_g0, dy_g1, dy_ld, z_g0, z_g1, z_ld, x_g0, x_g1, x_ld, dx_g0, dx_g1, dx_ld;
  int B, Ci, Co, L, Nb, G, slices, act, w_vec;           // w_vec: rows of W can be read eight bytes at a time
  float slope;
  uint32_t dy_extent, z_extent, x_extent, w_extent;
  // in_gamma != nullptr: X is the previous block's stored pre-activation; x = act_in(BatchNorm_in(X)), rounded to
  // bf16, is formed on the way into LDS with the arithmetic of the BatchNorm kernels.  [B][Ci] each.
  const float* in_gamma; const float* in_beta; const float* in_mean; const float* in_invstd;
  int in_act; float in_slope;
  // With in_gamma and dX: also leave, per input channel, the two reductions the INPUT block's BatchNorm backward
  // needs over its output gradient (= dX as stored) and its pre-activation (= X): sum g and sum g xhat with
  // g = dX * act_in'(.), xhat = (X - in_mean) * in_invstd.  The same thread loads a piece of X and stores that
  // piece of dX, so this costs no memory traffic; that block's own pass over both tensors goes away.
  int in_sums;
};

__device__ __forceinline__ float lo_f32(uint32_t v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ float hi_f32(uint32_t v) { return __uint_as_float(v & 0xffff0000u); }

constexpr int CBB_THREADS = 512;

// CO, CI: channel tiles (64 or 128) that hold Co and Ci.
template <int CO, int CI, bool HAS_DX>
struct CbbCfg {
  // Without a data gradient a 64 x 64 layer needs half the registers and LDS: two workgroups share a
  // compute unit (one lays its slice into LDS while the other runs its matrix instructions).
  static constexpr int WGS = (CO == 64 && CI == 64 && !HAS_DX) ? 2 : 1;
  static constexpr int SUBO = CO / 32;                 // 32-channel blocks of dY / z
  static constexpr int BPT = SUBO / 2;                 // 4 x 4 blocks of dY (and of z) per thread and slice
  static constexpr int XPT = CI / 16;                  // 8-byte pieces of x per thread and slice
  static constexpr int DEPTH = WGS == 2 ? 1 : ((CO == 64 && CI == 64) ? 2 : ((CO == 128 && CI == 128) ? 1 : 2));   // register budget
  static constexpr int PT = CO * 2 + 16;               // row pitch of the k = co tiles (W^T, dz^T), bytes
  static constexpr int PN = 128 * 2 + 16;              // row pitch of the k = point tiles (dz, x)
  static constexpr int PS = 128 * 2 + 8;               // row pitch of the dX tile on its way out
  static constexpr int WT_BYTES = CI * PT, DZT_BYTES = 128 * PT, DZN_BYTES = CO * PN, XN_BYTES = CI * PN;
  static constexpr int ST_BYTES = CI * PS, CF_BYTES = CO * 32;
  static constexpr bool OVERLAY = (CO == 128 && CI == 128);   // the dX tile goes out over dz^T (LDS would not hold both)
  static constexpr int XC_BYTES = CI * 16;             // the input block's BatchNorm constants (with a data gradient: own region; without: over W^T)
  static constexpr bool SUMS = HAS_DX && CI <= 64;     // can leave the input block's two sums (LDS and registers hold the extra state)
  static constexpr int ZR_BYTES = SUMS ? CI * 256 : 0; // the raw x pieces of the slice, each kept for the thread that loaded it
  static constexpr int SMEM0 = WT_BYTES + DZT_BYTES + DZN_BYTES + XN_BYTES + CF_BYTES + (OVERLAY ? 0 : ST_BYTES) + (HAS_DX ? XC_BYTES : 0);
  static constexpr int SMEM = SMEM0 + ZR_BYTES;
  static constexpr int DXT = CI / 64;                  // 32 x 32 tiles of dX per wavefront (CI/32 x 4 tiles, 8 wavefronts)
  static constexpr int WTILES = (CO / 32) * (CI / 32); // 32 x 32 tiles of dW
  static constexpr int KS = WTILES == 4 ? 2 : 1;       // four tiles: the slice's points are split over two wavefronts per tile
  static constexpr int NU = WTILES * KS / 8;           // (tile, point half) units per wavefront
  static constexpr int MMA_UNROLL = 2;                 // k-steps whose operand fragments are in registers at once (register budget)
  static_assert(DZT_BYTES + DZN_BYTES >= ST_BYTES, "staging tile must fit over the two dz tiles");
  static_assert(DZT_BYTES + DZN_BYTES >= 32 * CO * 4, "dbias scratch must fit over the two dz tiles");
  static_assert(SMEM * WGS <= 160 * 1024, "LDS");
};

// (The launch bound is the register budget: 2 * CBB_THREADS threads per compute unit where two workgroups share one.)
template <int CO, int CI, bool HAS_DX>
__global__ __launch_bounds__((CbbCfg<CO, CI, HAS_DX>::WGS * CBB_THREADS)) void cbb_kernel(CbbArgs p) {
  typedef CbbCfg<CO, CI, HAS_DX> K;
  constexpr int PT = K::PT, PN = K::PN, PS = K::PS, BPT = K::BPT, XPT = K::XPT, DEPTH = K::DEPTH;
  __shared__ __attribute__((aligned(16))) unsigned char smem[K::SMEM];
  unsigned char* Wts = smem;
  unsigned char* dzT = Wts + K::WT_BYTES;
  unsigned char* dzN = dzT + K::DZT_BYTES;
  unsigned char* xN = dzN + K::DZN_BYTES;
  unsigned char* cfb = xN + K::XN_BYTES;
  unsigned char* stg = K::OVERLAY ? dzT : cfb + K::CF_BYTES;
  const float4* cf = reinterpret_cast<const float4*>(cfb);
  float4* xc = reinterpret_cast<float4*>(HAS_DX ? cfb + K::CF_BYTES + (K::OVERLAY ? 0 : K::ST_BYTES) : Wts);
  static_assert(HAS_DX || K::WT_BYTES >= K::XC_BYTES, "constants fit over the unused W^T tile");
  unsigned char* zraw = smem + K::SMEM0;
  const bool sums_on = K::SUMS && p.in_sums;
  const float in_neg = p.in_act == HFTA_ACT_RELU ? 0.f : (p.in_act == HFTA_ACT_LEAKY ? p.in_slope : 1.f);

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int r = lane & 31, gsel = lane >> 5;
  const int kq = t % 8, ng = (t / 8) % 32, sh = t / 256;   // 4 x 4 blocks: channel group of four, point group of four, 32-channel block parity
  const int b = blockIdx.x / p.G, w = blockIdx.x - b * p.G;
  const int tiles = p.Nb * p.slices;
  // contiguous share of the model's slices: consecutive slices of one sample follow each other in time
  const int share = (tiles + p.G - 1) / p.G, ubeg = w * share, uend = min(tiles, ubeg + share);
  constexpr bool has_dx = HAS_DX;
  // derivative of the activation where its argument is not positive (1 where it is): one select per element
  const float act_neg = p.act == HFTA_ACT_RELU ? 0.f : (p.act == HFTA_ACT_LEAKY ? p.slope : 1.f);

  // ---- once per workgroup: per-channel constants and W^T ([ci][co], transposed in registers) ----
  // constants of channel k = 32 s + 4 kq + j live in slot (4 s + j) * 8 + kq of two float4 arrays: the eight
  // channel groups kq a wavefront reads at once are 128 contiguous bytes (no bank conflict)
  if (t < 2 * CO) {
    const int k = t >> 1, slot = ((k >> 5) * 4 + (k & 3)) * 8 + ((k >> 2) & 7);
    float4 c = make_float4(0.f, 0.f, 0.f, 0.f);
    if (k < p.Co) c = *reinterpret_cast<const float4*>(p.coef + ((int64_t)b * p.Co + k) * 8 + (t & 1) * 4);
    reinterpret_cast<float4*>(cfb)[(t & 1) * CO + slot] = c;
  }
  const bool xin = p.in_gamma != nullptr;
  if (xin)
    for (int k = t; k < CI; k += CBB_THREADS) {
      const int64_t g = (int64_t)b * p.Ci + k;
      xc[k] = k < p.Ci ? make_float4(p.in_mean[g], p.in_invstd[g], p.in_gamma[g], p.in_beta[g]) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  if (has_dx && !p.w_vec) {
    // rows of W not 8-byte aligned (Ci % 4 != 0, e.g. three input channels): element by element, once per workgroup
    for (int i = t; i < K::WT_BYTES / 4; i += CBB_THREADS) reinterpret_cast<uint32_t*>(Wts)[i] = 0u;
    __syncthreads();
    const bf16_raw* wb = p.W + (int64_t)b * p.Co * p.Ci;
    for (int i = t; i < p.Co * p.Ci; i += CBB_THREADS) {
      const int co = i / p.Ci, ci = i - co * p.Ci;
      *reinterpret_cast<bf16_raw*>(Wts + ci * PT + co * 2) = wb[i];
    }
  } else if (has_dx) {
    const __amdgpu_buffer_rsrc_t rw = pf_rsrc(p.W + (int64_t)b * p.Co * p.Ci, p.w_extent);
    const int c = ng * 4;                    // ci
    uint2 q[BPT][4];
#pragma unroll
    for (int i = 0; i < BPT; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int k = (sh + 2 * i) * 32 + 4 * kq + j;   // co
        const bool ok = k < p.Co && c + 4 <= p.Ci;
        const pf_u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rw, (int)(ok ? ((uint32_t)k * (uint32_t)p.Ci + (uint32_t)c) * 2u : PF_OOB), 0, 0);
        q[i][j] = make_uint2(v.x, v.y);
      }
    if (CI == 128 || ng < CI / 4) {
#pragma unroll
      for (int i = 0; i < BPT; ++i) {
        const uint32_t a0 = q[i][0].x, a1 = q[i][1].x, a2 = q[i][2].x, a3 = q[i][3].x;
        const uint32_t b0 = q[i][0].y, b1 = q[i][1].y, b2 = q[i][2].y, b3 = q[i][3].y;
        uint2 o[4];
        o[0] = make_uint2((a0 & 0xffffu) | (a1 << 16), (a2 & 0xffffu) | (a3 << 16));
        o[1] = make_uint2((a0 >> 16) | (a1 & 0xffff0000u), (a2 >> 16) | (a3 & 0xffff0000u));
        o[2] = make_uint2((b0 & 0xffffu) | (b1 << 16), (b2 & 0xffffu) | (b3 << 16));
        o[3] = make_uint2((b0 >> 16) | (b1 & 0xffff0000u), (b2 >> 16) | (b3 & 0xffff0000u));
#pragma unroll
        for (int e = 0; e < 4; ++e)
          *reinterpret_cast<uint2*>(Wts + (ng * 4 + e) * PT + (sh + 2 * i) * 64 + kq * 8) = o[e];
      }
    }
  }
  __syncthreads();

  // ---- slices in flight: dY and z as 4 x 4 blocks (channel rows 4 kq + j, points 4 ng ..), x by rows ----
  struct Regs { uint2 d[BPT][4], z[BPT][4], x[XPT]; };
  Regs q[DEPTH];
  const uint32_t dy_ldb = (uint32_t)(p.dy_ld * 2), z_ldb = (uint32_t)(p.z_ld * 2), x_ldb = (uint32_t)(p.x_ld * 2);
  auto issue = [&](Regs& g, int u) {
    const bool live = u < uend;
    const int n = live ? u / p.slices : 0;
    const int l0 = live ? (u - n * p.slices) * 128 : 0;
    const __amdgpu_buffer_rsrc_t rd = pf_rsrc(p.dY + b * p.dy_g0 + n * p.dy_g1, p.dy_extent);
    const __amdgpu_buffer_rsrc_t rz = pf_rsrc(p.Z + b * p.z_g0 + n * p.z_g1, p.z_extent);
    const __amdgpu_buffer_rsrc_t rx = pf_rsrc(p.X + b * p.x_g0 + n * p.x_g1, p.x_extent);
    const int c = l0 + ng * 4;
    const bool cok = live && c + 4 <= p.L;
#pragma unroll
    for (int i = 0; i < BPT; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int k = (sh + 2 * i) * 32 + 4 * kq + j;
        const bool ok = cok && k < p.Co;
        const pf_u32x2 vd = __builtin_amdgcn_raw_buffer_load_b64(rd, (int)(ok ? (uint32_t)k * dy_ldb + (uint32_t)c * 2u : PF_OOB), 0, 0);
        const pf_u32x2 vz = __builtin_amdgcn_raw_buffer_load_b64(rz, (int)(ok ? (uint32_t)k * z_ldb + (uint32_t)c * 2u : PF_OOB), 0, 0);
        g.d[i][j] = make_uint2(vd.x, vd.y);
        g.z[i][j] = make_uint2(vz.x, vz.y);
      }
#pragma unroll
    for (int i = 0; i < XPT; ++i) {
      const int id = t + CBB_THREADS * i, row = id >> 5, cx = l0 + (id & 31) * 4;
      const bool ok = live && row < p.Ci && cx + 4 <= p.L;
      const pf_u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rx, (int)(ok ? (uint32_t)row * x_ldb + (uint32_t)cx * 2u : PF_OOB), 0, 0);
      g.x[i] = make_uint2(v.x, v.y);
    }
  };

  constexpr int TCI = CI / 32, NU = K::NU, KS = K::KS, DXT = K::DXT;
  f32x16_t wacc[NU];
#pragma unroll
  for (int i = 0; i < NU; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) wacc[i][v] = 0.f;
  float bsum[BPT][4];
#pragma unroll
  for (int i = 0; i < BPT; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) bsum[i][j] = 0.f;
  constexpr int SPT = K::SUMS ? XPT : 1;     // this thread's rows (t / 32 + 16 i) are the same in every slice
  float isum1[SPT], isum2[SPT];
#pragma unroll
  for (int i = 0; i < SPT; ++i) isum1[i] = isum2[i] = 0.f;

#pragma unroll
  for (int d = 0; d < DEPTH; ++d) issue(q[d], ubeg + d);
  for (int u0 = ubeg; u0 < uend; u0 += DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      // No way out of the loop from inside a round: a slice past the last one runs as an empty slice (its
      // loads request nothing, every point is "past the sample's end"), so the only back edge is taken with
      // all DEPTH slices reissued in order and the waits on the oldest one leave the younger ones in flight.
      const int u = u0 + d;
      const bool live = u < uend;
      const int n = live ? u / p.slices : 0, l0 = live ? (u - n * p.slices) * 128 : p.slices * 128;
      const bool cok = l0 + ng * 4 + 4 <= p.L;
      // ---- dz of this slice, rounded, into both LDS tiles; x into its tile ----
#pragma unroll
      for (int i = 0; i < BPT; ++i) {
        if (i > 0) __builtin_amdgcn_sched_barrier(0);      // one block's temporaries at a time
        const int s = sh + 2 * i;
        float dz[4][4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int k = s * 32 + 4 * kq + j;
          const float4 c0 = cf[(s * 4 + j) * 8 + kq], c1 = cf[CO + (s * 4 + j) * 8 + kq];
          const uint2 qd = q[d].d[i][j], qz = q[d].z[i][j];
          const float dd[4] = {lo_f32(qd.x), hi_f32(qd.x), lo_f32(qd.y), hi_f32(qd.y)};
          const float zz[4] = {lo_f32(qz.x), hi_f32(qz.x), lo_f32(qz.y), hi_f32(qz.y)};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float xh = (zz[e] - c0.x) * c0.y;
            const float gr = dd[e] * (fmaf(c0.z, xh, c0.w) > 0.f ? 1.f : act_neg);
            const float v = c1.z * (gr - c1.x - xh * c1.y);
            dz[j][e] = cok ? v : 0.f;        // points past the sample's end add nothing to dW and dbias
          }
          uint2 o;
          o.x = pack_bf16x2(dz[j][0], dz[j][1]);
          o.y = pack_bf16x2(dz[j][2], dz[j][3]);
          *reinterpret_cast<uint2*>(dzN + k * PN + ng * 8) = o;
          bsum[i][j] += (lo_f32(o.x) + hi_f32(o.x)) + (lo_f32(o.y) + hi_f32(o.y));   // the values as the products see them
        }
        if (has_dx) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            uint2 o;
            o.x = pack_bf16x2(dz[0][e], dz[1][e]);
            o.y = pack_bf16x2(dz[2][e], dz[3][e]);
            *reinterpret_cast<uint2*>(dzT + (ng * 4 + e) * PT + s * 64 + kq * 8) = o;
          }
        }
      }
#pragma unroll
      for (int i = 0; i < XPT; ++i) {
        const int id = t + CBB_THREADS * i;
        uint2 xv = q[d].x[i];
        if (K::SUMS && sums_on) *reinterpret_cast<uint2*>(zraw + id * 8) = xv;
        if (xin) {
          xv = in_norm_apply4(xv, xc[id >> 5], l0 + (id & 31) * 4 + 4 <= p.L, p.in_act, p.in_slope);
        }
        *reinterpret_cast<uint2*>(xN + (id >> 5) * PN + (id & 31) * 8) = xv;
      }
      __syncthreads();
      issue(q[d], u + DEPTH);                // past the last slice: nothing is requested

      // ---- dW += dz x^T: (tile, point half) units of this wavefront ----
#pragma unroll
      for (int i = 0; i < NU; ++i) {
        const int id = wave + 8 * i, tile = KS == 2 ? (id & 3) : id, kh = KS == 2 ? (id >> 2) : 0;
        const int tco = tile / TCI, tci = tile % TCI;
#pragma unroll(K::MMA_UNROLL)
        for (int s = 0; s < 8 / KS; ++s) {
          const int ks = kh * (8 / KS) + s;
          const bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(dzN + (tco * 32 + r) * PN + (2 * ks + gsel) * 16);
          const bf16x8_t bb = *reinterpret_cast<const bf16x8_t*>(xN + (tci * 32 + r) * PN + (2 * ks + gsel) * 16);
          wacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bb, wacc[i], 0, 0, 0);
        }
      }
      if (has_dx) {
        // ---- dX tile [ci][point] = W^T dz: wavefront -> point quarter wave % 4, ci blocks wave / 4 (+ 2) ----
        const int tp = wave & 3;
        f32x16_t acc[DXT];
#pragma unroll
        for (int i = 0; i < DXT; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
#pragma unroll(K::MMA_UNROLL)
        for (int s = 0; s < CO / 16; ++s) {
          const bf16x8_t bb = *reinterpret_cast<const bf16x8_t*>(dzT + (tp * 32 + r) * PT + (2 * s + gsel) * 16);
#pragma unroll
          for (int i = 0; i < DXT; ++i) {
            const bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(Wts + (((wave >> 2) + 2 * i) * 32 + r) * PT + (2 * s + gsel) * 16);
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bb, a, acc[i], 0, 0, 0);
          }
        }
        if (K::OVERLAY) __syncthreads();     // every wavefront is done with dz^T before the tile on its way out lands there
        // accumulator (rows = points, one ci per lane) -> [ci][point] rows in LDS
#pragma unroll
        for (int i = 0; i < DXT; ++i)
#pragma unroll
          for (int qq = 0; qq < 4; ++qq) {
            uint2 o;
            o.x = pack_bf16x2(acc[i][4 * qq], acc[i][4 * qq + 1]);
            o.y = pack_bf16x2(acc[i][4 * qq + 2], acc[i][4 * qq + 3]);
            *reinterpret_cast<uint2*>(stg + (((wave >> 2) + 2 * i) * 32 + r) * PS + (tp * 32 + 8 * qq + 4 * gsel) * 2) = o;
          }
        __syncthreads();
        bf16_raw* dXb = p.dX + b * p.dx_g0 + n * p.dx_g1;
#pragma unroll
        for (int i = 0; i < XPT; ++i) {
          const int id = t + CBB_THREADS * i, row = id >> 5, c = l0 + (id & 31) * 4;
          const uint2 v = *reinterpret_cast<const uint2*>(stg + row * PS + (id & 31) * 8);
          const bool okp = row < p.Ci && c + 4 <= p.L;
          if (okp) *reinterpret_cast<uint2*>(dXb + (int64_t)row * p.dx_ld + c) = v;
          if (K::SUMS && sums_on) {
            const uint2 zr = *reinterpret_cast<const uint2*>(zraw + id * 8);
            const float4 ic = xc[row];       // mean, invstd, gamma, beta of the input block
            const float dd[4] = {lo_f32(v.x), hi_f32(v.x), lo_f32(v.y), hi_f32(v.y)};
            const float zz[4] = {lo_f32(zr.x), hi_f32(zr.x), lo_f32(zr.y), hi_f32(zr.y)};
            float a1 = 0.f, a2 = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float xh = (zz[e] - ic.x) * ic.y;
              const float gr = dd[e] * (fmaf(ic.z, xh, ic.w) > 0.f ? 1.f : in_neg);
              a1 += gr;
              a2 = fmaf(gr, xh, a2);
            }
            isum1[K::SUMS ? i : 0] += okp ? a1 : 0.f;
            isum2[K::SUMS ? i : 0] += okp ? a2 : 0.f;
          }
        }
        if (K::OVERLAY) __syncthreads();     // read out before the next slice's dz lands
      } else {
        __syncthreads();                     // operands read before the next slice lands
      }
    }
  }

  // ---- this workgroup's partials: [G * KS] slots of dW (+ dbias in the slots of point half 0) ----
  const int64_t nW = (int64_t)p.B * p.Co * p.Ci, nB = (int64_t)p.B * p.Co, stride = nW + nB + 2 * (int64_t)p.B * p.Ci;
  if (K::SUMS && sums_on) {
    // the 32 lanes that share a row add up; every slot of this workgroup gets its entry (zeros past the first)
#pragma unroll
    for (int i = 0; i < SPT; ++i) {
      float a1 = isum1[i], a2 = isum2[i];
#pragma unroll
      for (int m = 16; m >= 1; m >>= 1) {
        a1 += __shfl_xor(a1, m, 64);
        a2 += __shfl_xor(a2, m, 64);
      }
      const int row = (t >> 5) + 16 * i;
      if ((t & 31) == 0 && row < p.Ci)
#pragma unroll
        for (int kh = 0; kh < KS; ++kh)
          *reinterpret_cast<float2*>(p.part + (int64_t)(w * KS + kh) * stride + nW + nB + ((int64_t)b * p.Ci + row) * 2) =
              kh == 0 ? make_float2(a1, a2) : make_float2(0.f, 0.f);
    }
  }
#pragma unroll
  for (int i = 0; i < NU; ++i) {
    const int id = wave + 8 * i, tile = KS == 2 ? (id & 3) : id, kh = KS == 2 ? (id >> 2) : 0;
    const int tco = tile / TCI, tci = tile % TCI;
    float* pw = p.part + (int64_t)(w * KS + kh) * stride + (int64_t)b * p.Co * p.Ci;
    const int ci = tci * 32 + r;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int co = tco * 32 + 8 * (v >> 2) + 4 * gsel + (v & 3);
      if (co < p.Co && ci < p.Ci) pw[(int64_t)co * p.Ci + ci] = wacc[i][v];
    }
  }
  __syncthreads();                           // (overlay or not) nobody reads dz^T any more
  float* sc = reinterpret_cast<float*>(dzT);               // [32 point groups][CO]
#pragma unroll
  for (int i = 0; i < BPT; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) sc[ng * CO + (sh + 2 * i) * 32 + 4 * kq + j] = bsum[i][j];
  __syncthreads();
  if (t < KS * CO && (t % CO) < p.Co) {
    const int kh = t / CO, co = t % CO;
    float s = 0.f;
    if (kh == 0) {
#pragma unroll 8
      for (int i = 0; i < 32; ++i) s += sc[i * CO + co];
    }
    p.part[(int64_t)(w * KS + kh) * stride + nW + (int64_t)b * p.Co + co] = s;
  }
}

// out[i] = sum over the G workgroup partials in a fixed order (four interleaved chains combined as
// (0+1)+(2+3)); the first nW outputs are dW, the next nB dbias, the last nS (0 if not asked for) the
// input block's sums.
__global__ __launch_bounds__(256) void cbb_reduce_kernel(const float* __restrict__ part, float* __restrict__ dW,
                                                         float* __restrict__ dbias, float* __restrict__ sums, int64_t nW,
                                                         int64_t nB, int64_t nS, int64_t stride, int G) {
  __shared__ float sh[4][64];
  const int q = threadIdx.x >> 6, li = threadIdx.x & 63;
  const int64_t i = (int64_t)blockIdx.x * 64 + li, count = nW + nB + nS;
  float s = 0.f;
  if (i < count) {
#pragma unroll 8
    for (int k = q; k < G; k += 4) s += part[(int64_t)k * stride + i];
  }
  sh[q][li] = s;
  __syncthreads();
  if (q == 0 && i < count) {
    const float v = (sh[0][li] + sh[1][li]) + (sh[2][li] + sh[3][li]);
    if (i < nW) dW[i] = v;
    else if (i < nW + nB) { if (dbias) dbias[i - nW] = v; }
    else sums[i - nW - nB] = v;
  }
}

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

int cbb_groups(int B, int Nb, int L, int per_cu) {
  const int tiles = Nb * ((L + 127) / 128);
  int G = 256 * per_cu / B;                 // workgroups the chip holds at once, per model
  if (G < 1) G = 1;
  if (G > tiles) G = tiles;
  return G;
}

// CbbCfg::WGS of the kernel the shape takes (the workspace is sized for the larger count: no data gradient)
int cbb_per_cu(int Ci, int Co, bool has_dx) { return (Ci <= 64 && Co <= 64 && !has_dx) ? 2 : 1; }

int cbb_point_halves(int Ci, int Co) { return (Ci <= 64 && Co <= 64) ? 2 : 1; }   // CbbCfg::KS of the kernel the shape takes

}  // namespace

// The shapes the one-pass kernel takes (the caller has checked B, Nb, Ci, Co, L > 0).
// ... and can leave the input block's two sums on the way (a data gradient and on-load normalisation are asked for)
bool conv1x1_bn_bwd_stream_sums(int Ci) { return Ci <= 64; }

bool conv1x1_bn_bwd_streams(int B, int Ci, int Co, int L, int dtype) {
  return dtype == HFTA_BF16 && Ci <= 128 && Co <= 128 && L % 4 == 0 && B <= 65535;
}

size_t conv1x1_bn_bwd_stream_bytes(int B, int Nb, int Ci, int Co, int L) {
  const size_t slots = (size_t)cbb_groups(B, Nb, L, cbb_per_cu(Ci, Co, false)) * cbb_point_halves(Ci, Co);
  return align256((size_t)B * Co * 8 * sizeof(float)) + slots * ((size_t)B * Co * Ci + (size_t)B * Co + 2 * (size_t)B * Ci) * sizeof(float);
}

// HFTA_EUNSUPPORTED: alignment or strides are not the kernel's (nothing has been launched).
int conv1x1_bn_bwd_stream(int B, int Nb, int Ci, int Co, int L, const void* X, const int64_t xs[4], const void* W,
                          const void* Z, const int64_t zs[4], const void* dY, const int64_t dys[4], const float* gamma,
                          const float* beta, const float* save_mean, const float* save_invstd, void* dX,
                          const int64_t dxs[4], float* dW, float* dbias, float* dgamma, float* dbeta, int act, float slope,
                          void* workspace, hipStream_t st, const float* in_gamma, const float* in_beta,
                          const float* in_mean, const float* in_invstd, int in_act, float in_slope, const float* sums,
                          float* in_sums) {
  auto al = [](const void* q, size_t a) { return (reinterpret_cast<uintptr_t>(q) % a) == 0; };
  auto s4 = [](const int64_t* s) { return s[0] % 4 == 0 && s[1] % 4 == 0 && s[2] % 4 == 0 && s[2] > 0 && s[3] == 1; };
  if (!al(X, 8) || !al(Z, 8) || !al(dY, 8) || !s4(xs) || !s4(zs) || !s4(dys) || !al(workspace, 16)) return HFTA_EUNSUPPORTED;
  if (dX && (!s4(dxs) || !al(dX, 8))) return HFTA_EUNSUPPORTED;
  if (in_gamma && (!in_beta || !in_mean || !in_invstd ||
                   (in_act != HFTA_ACT_NONE && in_act != HFTA_ACT_RELU && in_act != HFTA_ACT_LEAKY)))
    return HFTA_EUNSUPPORTED;
  if (in_sums && (!in_gamma || !dX || !conv1x1_bn_bwd_stream_sums(Ci))) return HFTA_EUNSUPPORTED;
  auto ext = [&](const int64_t* s, int C) { return ((int64_t)(C - 1) * s[2] + L) * 2; };
  const int64_t w_ext = (int64_t)Co * Ci * 2;
  if (ext(xs, Ci) >= (int64_t)1 << 31 || ext(zs, Co) >= (int64_t)1 << 31 || ext(dys, Co) >= (int64_t)1 << 31 || w_ext >= (int64_t)1 << 31)
    return HFTA_EUNSUPPORTED;
  float* coef = reinterpret_cast<float*>(workspace);
  float* part = reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(workspace) + align256((size_t)B * Co * 8 * sizeof(float)));
  // the two sums of this block's BatchNorm backward: from the successor's backward, or a pass over dY and z
  int rc = sums ? bn_bwd_coef_from_sums(B, Nb, Co, L, sums, gamma, beta, save_mean, save_invstd, dgamma, dbeta, coef, st)
                : bn_bwd_coef(B, Nb, Co, L, HFTA_BF16, Z, zs, dY, dys, gamma, beta, save_mean, save_invstd, dgamma, dbeta, coef, act, slope, st);
  if (rc != HFTA_OK) return rc;
  CbbArgs a;
  a.dY = (const bf16_raw*)dY; a.Z = (const bf16_raw*)Z; a.X = (const bf16_raw*)X; a.W = (const bf16_raw*)W;
  a.dX = (bf16_raw*)dX; a.coef = coef; a.part = part;
  a.dy_g0 = dys[0]; a.dy_g1 = dys[1]; a.dy_ld = dys[2];
  a.z_g0 = zs[0]; a.z_g1 = zs[1]; a.z_ld = zs[2];
  a.x_g0 = xs[0]; a.x_g1 = xs[1]; a.x_ld = xs[2];
  a.dx_g0 = dX ? dxs[0] : 0; a.dx_g1 = dX ? dxs[1] : 0; a.dx_ld = dX ? dxs[2] : 0;
  a.B = B; a.Ci = Ci; a.Co = Co; a.L = L; a.Nb = Nb;
  a.G = cbb_groups(B, Nb, L, cbb_per_cu(Ci, Co, dX != nullptr));
  a.slices = (L + 127) / 128;
  a.act = act; a.slope = slope;
  a.in_gamma = in_gamma; a.in_beta = in_beta; a.in_mean = in_mean; a.in_invstd = in_invstd;
  a.in_act = in_act; a.in_slope = in_slope;
  a.in_sums = in_sums ? 1 : 0;
  a.w_vec = (W && al(W, 8) && Ci % 4 == 0) ? 1 : 0;
  a.dy_extent = (uint32_t)ext(dys, Co); a.z_extent = (uint32_t)ext(zs, Co); a.x_extent = (uint32_t)ext(xs, Ci);
  a.w_extent = (uint32_t)w_ext;
  const dim3 grid((unsigned)(B * a.G));
#define HFTA_CBB(CO_, CI_) \
  do { if (dX) hipLaunchKernelGGL((cbb_kernel<CO_, CI_, true>), grid, dim3(CBB_THREADS), 0, st, a); \
       else hipLaunchKernelGGL((cbb_kernel<CO_, CI_, false>), grid, dim3(CBB_THREADS), 0, st, a); } while (0)
  if (Co <= 64 && Ci <= 64) HFTA_CBB(64, 64);
  else if (Co <= 64) HFTA_CBB(64, 128);
  else if (Ci <= 64) HFTA_CBB(128, 64);
  else HFTA_CBB(128, 128);
#undef HFTA_CBB
  rc = launch_status();
  if (rc != HFTA_OK) return rc;
  const int64_t nW = (int64_t)B * Co * Ci, nB = (int64_t)B * Co, nSall = 2 * (int64_t)B * Ci, nS = in_sums ? nSall : 0;
  hipLaunchKernelGGL(cbb_reduce_kernel, dim3((unsigned)((nW + nB + nS + 63) / 64)), dim3(256), 0, st, part, dW, dbias, in_sums, nW, nB,
                     nS, nW + nB + nSall, a.G * cbb_point_halves(Ci, Co));
  return launch_status();
}

}  // namespace hfta
