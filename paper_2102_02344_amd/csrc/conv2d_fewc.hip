// Data gradient of a grouped 4x4 / stride 2 / pad 1 convolution with at most 4 input channels (the
// DCGAN generator's last transposed convolution 64 -> 3 and the discriminator's first layer 3 -> 64;
// fusion rules table, rows "Conv2d" / "ConvTranspose2d").  With 3 rows a matrix-instruction tile is
// 95 % empty and the column-tile gather of the implicit GEMM costs as much as for a full tile, so
// this is plain vector arithmetic:
//     dX[c][2qy+py][2qx+px] = sum_o sum_{(ky,r) in S(py)} sum_{(kx,s) in S(px)} W[o][c][ky][kx] dY[o][qy-1+r][qx-1+s]
//     S(0) = {(1,1), (3,0)},  S(1) = {(0,2), (2,1)}
// One thread owns one q pixel: the 2x2 output block of every channel (4 Ci accumulators) against the
// 3x3 neighbourhood of dY, 16 Ci multiply-adds per output channel o.  A workgroup covers 32 x 8 q
// pixels; dY goes through LDS eight channels at a time (10 x 34 halo tile); the weights are the same
// for every thread of a workgroup and are read with scalar loads (they occupy the scalar unit and
// scalar registers, not LDS bandwidth or vector instructions).
#include "common.h"

namespace hfta {

namespace {

constexpr int FC_TX = 32, FC_TY = 8, FC_OC = 8;            // q tile, channels of dY per LDS stage
constexpr int FC_PW = FC_TX + 2 + 2;                       // halo row pitch (elements)

struct FewcArgs {
  const bf16_raw* Wt; const bf16_raw* dY; bf16_raw* dX;
  int B, Nb, Co, H, W, Hq, Wq, tiles_x;
};

template <int CI>
__global__ __launch_bounds__(256) void conv_dx_fewc_kernel(FewcArgs p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_raw* tile = reinterpret_cast<bf16_raw*>(smem);                           // [2][FC_OC][FC_TY + 2][FC_PW]
  const int t = threadIdx.x, tx = t & (FC_TX - 1), ty = t >> 5;
  const int qx0 = (blockIdx.x % p.tiles_x) * FC_TX, qy0 = (blockIdx.x / p.tiles_x) * FC_TY;
  const int n = blockIdx.y, b = blockIdx.z;
  const int64_t P = (int64_t)p.Hq * p.Wq;
  const bf16_raw* dy = p.dY + ((int64_t)n * p.B + b) * p.Co * P;
  const uint32_t* __restrict__ w2 = reinterpret_cast<const uint32_t*>(p.Wt + (int64_t)b * p.Co * CI * 16);   // pairs (kx, kx + 1)

  constexpr int TILE_EL = FC_OC * (FC_TY + 2) * FC_PW;
  constexpr int PER_THREAD = (FC_OC * (FC_TY + 2) * (FC_TX + 2) + 255) / 256;
  bf16_raw stage[PER_THREAD];
  auto fetch = [&](int o0) {
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      const int e = t + 256 * i;
      const int col = e % (FC_TX + 2), r = e / (FC_TX + 2);
      const int row = r % (FC_TY + 2), oc = r / (FC_TY + 2);
      const int y = qy0 - 1 + row, x = qx0 - 1 + col, o = o0 + oc;
      const bool ok = oc < FC_OC && o < p.Co && y >= 0 && y < p.Hq && x >= 0 && x < p.Wq;
      const bf16_raw v = dy[ok ? (int64_t)o * P + (int64_t)y * p.Wq + x : 0];     // always a valid address: no load under a branch
      stage[i] = ok ? v : (bf16_raw)0;
    }
  };
  auto park = [&](int buf) {
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      const int e = t + 256 * i;
      const int col = e % (FC_TX + 2), r = e / (FC_TX + 2);
      const int row = r % (FC_TY + 2), oc = r / (FC_TY + 2);
      if (oc < FC_OC) tile[buf * TILE_EL + (oc * (FC_TY + 2) + row) * FC_PW + col] = stage[i];
    }
  };

  float acc[CI][2][2];
#pragma unroll
  for (int c = 0; c < CI; ++c) acc[c][0][0] = acc[c][0][1] = acc[c][1][0] = acc[c][1][1] = 0.f;

  fetch(0);
  park(0);
  __syncthreads();
  int buf = 0;
  for (int o0 = 0; o0 < p.Co; o0 += FC_OC) {
    const bool more = o0 + FC_OC < p.Co;
    if (more) fetch(o0 + FC_OC);
#pragma unroll 2
    for (int oc = 0; oc < FC_OC; ++oc) {
      if (o0 + oc >= p.Co) break;
      const bf16_raw* tp = tile + buf * TILE_EL + (oc * (FC_TY + 2) + ty) * FC_PW + tx;
      float d[3][3];
#pragma unroll
      for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s) d[r][s] = bf16_to_f32(tp[r * FC_PW + s]);
      const uint32_t* wq = w2 + (size_t)(o0 + oc) * CI * 8;      // uniform address: scalar loads
#pragma unroll
      for (int c = 0; c < CI; ++c) {
        float4 k[4];                                            // rows ky = 0..3
#pragma unroll
        for (int ky = 0; ky < 4; ++ky) {
          const uint32_t lo = wq[c * 8 + ky * 2], hi = wq[c * 8 + ky * 2 + 1];
          k[ky] = make_float4(__uint_as_float(lo << 16), __uint_as_float(lo & 0xffff0000u), __uint_as_float(hi << 16),
                              __uint_as_float(hi & 0xffff0000u));
        }
        const float4 k0 = k[0], k1 = k[1], k2 = k[2], k3 = k[3];
        // py = 0: (ky 1, r 1), (ky 3, r 0);  py = 1: (ky 0, r 2), (ky 2, r 1); the same pairs along x
#define HFTA_FC4(A, w0, x0, w1, x1, w2, x2, w3, x3) A = fmaf(w3, x3, fmaf(w2, x2, fmaf(w1, x1, fmaf(w0, x0, A))))
        HFTA_FC4(acc[c][0][0], k1.y, d[1][1], k1.w, d[1][0], k3.y, d[0][1], k3.w, d[0][0]);
        HFTA_FC4(acc[c][0][1], k1.x, d[1][2], k1.z, d[1][1], k3.x, d[0][2], k3.z, d[0][1]);
        HFTA_FC4(acc[c][1][0], k0.y, d[2][1], k0.w, d[2][0], k2.y, d[1][1], k2.w, d[1][0]);
        HFTA_FC4(acc[c][1][1], k0.x, d[2][2], k0.z, d[2][1], k2.x, d[1][2], k2.z, d[1][1]);
#undef HFTA_FC4
      }
    }
    if (more) park(buf ^ 1);
    __syncthreads();
    buf ^= 1;
  }
  const int qx = qx0 + tx, qy = qy0 + ty;
  if (qx < p.Wq && qy < p.Hq) {
    bf16_raw* out = p.dX + (((int64_t)n * p.B + b) * CI) * p.H * p.W + (int64_t)(2 * qy) * p.W + 2 * qx;
#pragma unroll
    for (int c = 0; c < CI; ++c) {
      *reinterpret_cast<uint32_t*>(out + (int64_t)c * p.H * p.W) = pack_bf16x2(acc[c][0][0], acc[c][0][1]);
      *reinterpret_cast<uint32_t*>(out + (int64_t)c * p.H * p.W + p.W) = pack_bf16x2(acc[c][1][0], acc[c][1][1]);
    }
  }
}

}  // namespace

bool conv_dx_fewc_supported(int Nb, int B, int Ci, int Co, int H, int W, int kh, int kw, int stride, int pad) {
  return kh == 4 && kw == 4 && stride == 2 && pad == 1 && Ci >= 1 && Ci <= 4 && H % 2 == 0 && W % 2 == 0 && Nb <= 65535 && B <= 65535;
}

int conv_dx_fewc(int B, int Nb, int Ci, int Co, int H, int W, const void* Wt, const void* dY, void* dX, hipStream_t st) {
  if (reinterpret_cast<uintptr_t>(dX) % 4 != 0 || reinterpret_cast<uintptr_t>(Wt) % 4 != 0) return HFTA_EUNSUPPORTED;
  FewcArgs a{(const bf16_raw*)Wt, (const bf16_raw*)dY, (bf16_raw*)dX, B, Nb, Co, H, W, H / 2, W / 2, (W / 2 + FC_TX - 1) / FC_TX};
  const size_t lds = 2 * FC_OC * (FC_TY + 2) * FC_PW * 2;
  const dim3 grid((unsigned)(a.tiles_x * ((a.Hq + FC_TY - 1) / FC_TY)), (unsigned)Nb, (unsigned)B);
#define HFTA_FEWC(C) \
  hipLaunchKernelGGL(conv_dx_fewc_kernel<C>, grid, dim3(256), lds, st, a)
  switch (Ci) {
    case 1: HFTA_FEWC(1); break;
    case 2: HFTA_FEWC(2); break;
    case 3: HFTA_FEWC(3); break;
    default: HFTA_FEWC(4); break;
  }
#undef HFTA_FEWC
  return launch_status();
}

}  // namespace hfta
