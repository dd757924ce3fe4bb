// Streaming forward kernel of the fused k=1 Conv1d for layers with at most 128 (256) input channels
// (fusion rules table, Conv1d row; the point-cloud models' 64 -> 64 ... 128 -> 1024 layers).
//
// Per model b and sample n:  Y[co][l] = sum_ci W[b][co][ci] * X[ci][l] + bias[b][co], with Ci <= 128
// (<= 256 for layers at least 512 channels wide, e.g. the data gradient of a 2880 -> 256 layer):
// the whole reduction fits one LDS tile, so a generic k-loop kernel spends its time in launch,
// prologue and epilogue latencies, not in the matrix cores or in HBM.  Here one workgroup owns one
// 128-point slice of one sample, keeps that X tile (transposed, [point][ci]) in LDS, and walks
// over all 128-row tiles of W: X is read from HBM exactly once, the W tile of step i+1 is in
// flight in registers while step i runs its MFMAs, and the stores of step i drain while step i+1
// computes.  Loads are raw buffer loads: anything outside the operand (rows >= Co, ci >= Ci,
// points >= L, the W tile after the last) is an out-of-range offset that returns zeros without a
// memory request, so the loop has no branches around its loads.
#include "gemm_pf.h"
#include "in_norm.h"

namespace hfta {

// 128 < Ci <= 256 keeps a 256-deep X tile and W tile in LDS (one workgroup per compute unit): it
// beats the k-loop GEMM only when many W tiles share one X tile.
constexpr int STREAM_WIDE_MIN_CO = 512;

typedef __bf16 stat_bf16x2 __attribute__((ext_vector_type(2)));   // operand of the two-element dot product

struct StreamArgs {
  const bf16_raw* W;
  const bf16_raw* X;
  bf16_raw* Y;
  const bf16_raw* bias;
  int64_t x_g0, x_g1, x_ld;
  int64_t y_g0, y_g1, y_ld;
  int Ci, Co, L, Nb;
  int tiles_co;
  int act, c_vec;
  float slope;
  uint32_t w_extent, x_extent;
  // BatchNorm statistics of the output, taken from the values as they are stored (nullptr: off):
  // per (model, sample, 128-point slice) and channel the sums of (y - bias) and (y - bias)^2 over the
  // slice's points, [b * Nb + n][slice][Co][2]; the activation must be none.
  float* stat_part;
  // Input given as the previous block's stored pre-activation (XF kernels): x = act_in(gamma (X - mean) invstd + beta),
  // rounded to bf16, is formed on the way into LDS with the arithmetic of the BatchNorm kernels, so the
  // product sees the bits that block would have stored.  [B][Ci] each.
  const float* in_gamma; const float* in_beta; const float* in_mean; const float* in_invstd;
  int in_act; float in_slope;
};

// ONE: the layer has a single 128-row W tile (Co <= 128), so the X tile is dead once the matrix
// instructions have run and the output staging tile may lie over it: 37 KB of LDS instead of 52 KB
// at KT = 64, i.e. four workgroups per compute unit instead of three (register budget via launch
// bounds).
template <int KT, bool ONE = false, bool XF = false>
__global__ __launch_bounds__(GEMM_THREADS, ONE ? 4 : 1) void conv1x1_stream_kernel(StreamArgs p) {
  constexpr int PITCH = KT * 2 + 16;                   // bytes per LDS row: KT bf16 + pad
  constexpr int TILE = 128 * PITCH;
  constexpr int STAGE = 128 * EPI_PITCH2;
  constexpr int SREG = TILE > STAGE ? TILE : STAGE;    // W tile, then the output staging tile
  constexpr int SUB = KT / 32;
  constexpr int SMEM = ONE ? (2 * TILE > STAGE ? 2 * TILE : STAGE) : TILE + SREG;
  __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM + (XF ? KT * 16 : 0)];
  unsigned char* Xs = ONE ? smem + TILE : smem;        // ONE: [W tile | X tile], staging over both
  unsigned char* Ws = ONE ? smem : smem + TILE;

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  int bx = blockIdx.x, bz = blockIdx.z;
  {  // XCD-aware renumbering: each XCD walks a contiguous range of (sample, slice) work
    const int total = gridDim.x * gridDim.z, per = total >> 3;
    const int lin = blockIdx.x + gridDim.x * blockIdx.z;
    if (lin < (per << 3)) {
      const int l2 = (lin & 7) * per + (lin >> 3);
      bz = l2 / gridDim.x;
      bx = l2 - bz * gridDim.x;
    }
  }
  const int b = bz / p.Nb, n = bz % p.Nb;
  const int l0 = bx * 128;

  const __amdgpu_buffer_rsrc_t rw = pf_rsrc(p.W + (int64_t)b * p.Co * p.Ci, p.w_extent);
  const __amdgpu_buffer_rsrc_t rx = pf_rsrc(p.X + b * p.x_g0 + n * p.x_g1, p.x_extent);

  if (XF) {                              // the input block's BatchNorm constants, one float4 per input channel
    float4* ic = reinterpret_cast<float4*>(smem + SMEM);
    for (int k = t; k < KT; k += GEMM_THREADS) {
      const int64_t g = (int64_t)b * p.Ci + k;
      ic[k] = k < p.Ci ? make_float4(p.in_mean[g], p.in_invstd[g], p.in_gamma[g], p.in_beta[g]) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    __syncthreads();
  }
  // ---- X tile: 4(ci) x 4(points) blocks, transposed in registers on the way into LDS ----
  {
    // (Which lanes take which block does not matter to the memory system: whole 256-byte row segments per half
    // wavefront or 128 bytes of four rows per wavefront instead of this 64-byte-per-row mapping time the same.)
    const int kq = t % 8, ng = t / 8;
    const int c = l0 + ng * 4;
    const uint32_t ldb = (uint32_t)(p.x_ld * 2);
    uint2 q[SUB][4];
#pragma unroll
    for (int s = 0; s < SUB; ++s)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int k = s * 32 + 4 * kq + j;
        const bool ok = k < p.Ci && c + 4 <= p.L;
        const pf_u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rx, (int)(ok ? (uint32_t)k * ldb + (uint32_t)c * 2u : PF_OOB), 0, 0);
        q[s][j] = make_uint2(v.x, v.y);
      }
    if (XF) {
      const float4* ic = reinterpret_cast<const float4*>(smem + SMEM);
      const bool cok = c + 4 <= p.L;       // points past the sample's end stay zero (the statistics epilogue counts on it)
#pragma unroll
      for (int s = 0; s < SUB; ++s)
#pragma unroll
        for (int j = 0; j < 4; ++j) q[s][j] = in_norm_apply4(q[s][j], ic[s * 32 + 4 * kq + j], cok, p.in_act, p.in_slope);
    }
#pragma unroll
    for (int s = 0; s < SUB; ++s) {
      const uint32_t a0 = q[s][0].x, a1 = q[s][1].x, a2 = q[s][2].x, a3 = q[s][3].x;
      const uint32_t b0 = q[s][0].y, b1 = q[s][1].y, b2 = q[s][2].y, b3 = q[s][3].y;
      uint2 o[4];
      o[0] = make_uint2((a0 & 0xffffu) | (a1 << 16), (a2 & 0xffffu) | (a3 << 16));
      o[1] = make_uint2((a0 >> 16) | (a1 & 0xffff0000u), (a2 >> 16) | (a3 & 0xffff0000u));
      o[2] = make_uint2((b0 & 0xffffu) | (b1 << 16), (b2 & 0xffffu) | (b3 << 16));
      o[3] = make_uint2((b0 >> 16) | (b1 & 0xffff0000u), (b2 >> 16) | (b3 & 0xffff0000u));
#pragma unroll
      for (int i = 0; i < 4; ++i)
        *reinterpret_cast<uint2*>(Xs + (ng * 4 + i) * PITCH + s * 64 + kq * 8) = o[i];
    }
  }

  // ---- W tiles: rows t/4 and t/4+64, 16-byte group t%4 of every 32-wide k block ----
  const int wr = t >> 2, wg = (t & 3) * 8;
  uint4 wq[SUB][2];
  auto load_w = [&](int ct) {
#pragma unroll
    for (int s = 0; s < SUB; ++s)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int row = ct * 128 + wr + 64 * h, k = s * 32 + wg;
        const bool ok = row < p.Co && k + 8 <= p.Ci;
        const pf_u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rw, (int)(ok ? ((uint32_t)row * (uint32_t)p.Ci + (uint32_t)k) * 2u : PF_OOB), 0, 0);
        wq[s][h] = make_uint4(v.x, v.y, v.z, v.w);
      }
  };
  load_w(0);

  bf16_raw* Yb = p.Y + b * p.y_g0 + n * p.y_g1;
  const bf16_raw* bias = p.bias ? p.bias + (int64_t)b * p.Co : nullptr;
  const int r = lane & 31, gsel = lane >> 5;

  for (int ct = 0; ct < p.tiles_co; ++ct) {
#pragma unroll
    for (int s = 0; s < SUB; ++s)
#pragma unroll
      for (int h = 0; h < 2; ++h)
        *reinterpret_cast<uint4*>(Ws + (wr + 64 * h) * PITCH + (s * 32 + wg) * 2) = wq[s][h];
    __syncthreads();
    load_w(ct + 1);                      // past the last tile: rows >= Co, zeros, no traffic

    f32x16_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
#pragma unroll
    for (int s = 0; s < KT / 16; ++s) {
      bf16x8_t a[2], bb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        a[i] = *reinterpret_cast<const bf16x8_t*>(Ws + (wm * 64 + i * 32 + r) * PITCH + (2 * s + gsel) * 16);
        bb[i] = *reinterpret_cast<const bf16x8_t*>(Xs + (wn * 64 + i * 32 + r) * PITCH + (2 * s + gsel) * 16);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bb[j], a[i], acc[i][j], 0, 0, 0);
    }
    __syncthreads();                     // every wavefront is done with the W tile
    store_tile<bf16_raw, bf16_raw, false>(acc, Ws, Yb, p.y_ld, p.Co, p.L, ct * 128, l0, bias, 1, p.act, p.slope, p.c_vec, t);
    if (p.stat_part) {
      // the staged tile [128 channels][128 points] is still in LDS: two threads per channel add their
      // 64 points with two-element dot products (sum of z and of z^2 of the rounded values), then
      // move both sums to the channel's bias as origin, the form the partial sums are kept in.  A
      // point past the slice's end holds the bias itself (its X column was read as zeros), i.e. it
      // adds nothing to the shifted sums, so all 64 columns count.
      const int row = t >> 1, half = t & 1;
      const int m = ct * 128 + row;
      const float shift = (bias && m < p.Co) ? bf16_to_f32(bias[m]) : 0.f;
      const unsigned char* src = Ws + row * EPI_PITCH2 + half * 128;
      const stat_bf16x2 ones = __builtin_bit_cast(stat_bf16x2, 0x3f803f80u);
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const uint2 v = *reinterpret_cast<const uint2*>(src + q * 8);
        const stat_bf16x2 lo = __builtin_bit_cast(stat_bf16x2, v.x), hi = __builtin_bit_cast(stat_bf16x2, v.y);
        s1 = __builtin_amdgcn_fdot2_f32_bf16(lo, ones, s1, false);
        s2 = __builtin_amdgcn_fdot2_f32_bf16(lo, lo, s2, false);
        s1 = __builtin_amdgcn_fdot2_f32_bf16(hi, ones, s1, false);
        s2 = __builtin_amdgcn_fdot2_f32_bf16(hi, hi, s2, false);
      }
      s2 = fmaf(shift, fmaf(64.f, shift, -2.f * s1), s2);      // sum (z - c)^2 = sum z^2 - 2 c sum z + 64 c^2
      s1 = fmaf(-64.f, shift, s1);
      s1 += __shfl_xor(s1, 1, 64);
      s2 += __shfl_xor(s2, 1, 64);
      if (half == 0 && m < p.Co)
        *reinterpret_cast<float2*>(p.stat_part + (((int64_t)bz * gridDim.x + bx) * p.Co + m) * 2) = make_float2(s1, s2);
    }
    __syncthreads();                     // staging tile read out before the next W tile lands
  }
}

// Returns HFTA_OK when launched, HFTA_EUNSUPPORTED when the problem is not this kernel's.
// in_gamma != nullptr: X is the previous block's stored pre-activation, normalised and activated on load
// (Ci <= 128 only).
int conv1x1_stream_fwd(int B, int Nb, int Ci, int Co, int L, const void* X, const int64_t xs[4], const void* W,
                       const void* bias, void* Y, const int64_t ys[4], int act, float slope, hipStream_t st,
                       float* stat_part, const float* in_gamma, const float* in_beta, const float* in_mean,
                       const float* in_invstd, int in_act, float in_slope) {
  auto al = [](const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; };
  if (Ci > 256 || Ci % 8 != 0 || Co < 64 || L % 4 != 0) return HFTA_EUNSUPPORTED;
  if (Ci > 128 && Co < STREAM_WIDE_MIN_CO) return HFTA_EUNSUPPORTED;
  if (act == HFTA_ACT_TANH || act == HFTA_ACT_GELU || (stat_part && act != HFTA_ACT_NONE)) return HFTA_EUNSUPPORTED;
  if (in_gamma && (Ci > 128 || !in_beta || !in_mean || !in_invstd ||
                   (in_act != HFTA_ACT_NONE && in_act != HFTA_ACT_RELU && in_act != HFTA_ACT_LEAKY)))
    return HFTA_EUNSUPPORTED;
  if (!al(W, 16) || !al(X, 8) || xs[0] % 4 || xs[1] % 4 || xs[2] % 4 || xs[2] <= 0) return HFTA_EUNSUPPORTED;
  const int64_t x_ext = ((int64_t)(Ci - 1) * xs[2] + L) * 2, w_ext = (int64_t)Co * Ci * 2;
  if (x_ext >= (int64_t)1 << 31 || w_ext >= (int64_t)1 << 31) return HFTA_EUNSUPPORTED;
  StreamArgs a;
  a.W = (const bf16_raw*)W; a.X = (const bf16_raw*)X; a.Y = (bf16_raw*)Y; a.bias = (const bf16_raw*)bias;
  a.x_g0 = xs[0]; a.x_g1 = xs[1]; a.x_ld = xs[2];
  a.y_g0 = ys[0]; a.y_g1 = ys[1]; a.y_ld = ys[2];
  a.Ci = Ci; a.Co = Co; a.L = L; a.Nb = Nb;
  a.tiles_co = (Co + 127) / 128;
  a.act = act; a.slope = slope;
  a.c_vec = 0;
  for (int w = 16; w >= 8; w >>= 1) {
    const int q = w / 2;
    if (al(Y, w) && ys[0] % q == 0 && ys[1] % q == 0 && ys[2] % q == 0) { a.c_vec = w; break; }
  }
  a.w_extent = (uint32_t)w_ext; a.x_extent = (uint32_t)x_ext;
  a.stat_part = stat_part;
  a.in_gamma = in_gamma; a.in_beta = in_beta; a.in_mean = in_mean; a.in_invstd = in_invstd;
  a.in_act = in_act; a.in_slope = in_slope;
  dim3 grid((unsigned)((L + 127) / 128), 1, (unsigned)(B * Nb));
  if (in_gamma) {
    if (Ci <= 64 && Co <= 128) hipLaunchKernelGGL((conv1x1_stream_kernel<64, true, true>), grid, dim3(GEMM_THREADS), 0, st, a);
    else if (Ci <= 64) hipLaunchKernelGGL((conv1x1_stream_kernel<64, false, true>), grid, dim3(GEMM_THREADS), 0, st, a);
    else hipLaunchKernelGGL((conv1x1_stream_kernel<128, false, true>), grid, dim3(GEMM_THREADS), 0, st, a);
    return launch_status();
  }
  if (Ci <= 64 && Co <= 128) hipLaunchKernelGGL((conv1x1_stream_kernel<64, true>), grid, dim3(GEMM_THREADS), 0, st, a);
  else if (Ci <= 64) hipLaunchKernelGGL(conv1x1_stream_kernel<64>, grid, dim3(GEMM_THREADS), 0, st, a);
  else if (Ci <= 128) hipLaunchKernelGGL(conv1x1_stream_kernel<128>, grid, dim3(GEMM_THREADS), 0, st, a);
  else hipLaunchKernelGGL(conv1x1_stream_kernel<256>, grid, dim3(GEMM_THREADS), 0, st, a);
  return launch_status();
}

}  // namespace hfta
