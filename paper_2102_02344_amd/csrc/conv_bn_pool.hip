// Fused backward of  k=1 Conv1d -> BatchNorm (+ ReLU / LeakyReLU) -> max over points,
// the tail of a point-cloud model's per-point MLP (fusion rules table rows "Conv1d" and
// "BatchNorm1d" plus the point max-pool), without ever forming the dense gradient of the
// convolution's [Nb, B*Co, L] output.
//
// The pooled gradient reaches the convolution output z only at the Nb argmax points of a channel,
// so BatchNorm's backward is, per channel c (m = Nb*L, xhat = (z - mean) * invstd, a = gamma*invstd):
//     dz[n,c,l] = s[n,c] * [l == idx[n,c]]  -  p0'[c]  -  p1[c] * z[n,c,l]
//     s = a * dv * act'(.),  p1 = a*invstd*dgamma/m,  p0' = a*(dbeta - invstd*mean*dgamma)/m
// with dbeta, dgamma sums over the Nb argmax elements only.  Substituting z = W x + bias:
//     dX[n][:,l] = sum_{c: idx[n,c] = l} s[n,c] W[c,:]  -  v  -  G x[n][:,l]
//         G = sum_c p1[c] W[c,:]^T W[c,:]   (Ci x Ci),   v = sum_c p0[c] W[c,:],  p0 = p0' + p1*bias
//     dW[c,:]    = sum_n s[n,c] x[n][:, idx[n,c]]  -  a[c] (dbeta[c] E[x] + invstd dgamma[c] Cov(z_c, x))
//         E[x] = SX / m,  Cov(z_c, x) = (W[c,:] XX + bias SX) / m - mean[c] E[x],  XX = sum_{n,l} x x^T,  SX = sum_{n,l} x
// so the work is one Ci x Ci Gram matrix of the layer input (a split-K GEMM), one Ci -> Ci
// convolution with a scatter of the argmax columns in its epilogue, and small per-model algebra:
// the 1.3 GB tensor of the headline workload is neither read nor written.
#include "gemm_pf.h"
#include "bn_common.h"
#include "in_norm.h"

using namespace hfta;

namespace {

struct CbpChan { float a, dbeta, dgamma, invstd, mean, bias; };

struct CbpArgs {
  const bf16_raw* X; const bf16_raw* W; const bf16_raw* bias; const bf16_raw* Z; const bf16_raw* dV;
  const int32_t* idx;
  const float* zhit;  // [B][Nb][Co] convolution output at the argmax (then Z is not read), or null
  const float* Tin;   // [B][Co][Ci] W XX from the forward operator, or null: computed here
  const float* gamma; const float* beta; const float* save_mean; const float* save_invstd;
  bf16_raw* dX; float* dW; float* dbias; float* dgamma; float* dbeta;
  int64_t xsb, xsn, xsc, zsb, zsn, zsc, vsb, vsn, vsc, dxsb, dxsn, dxsc;
  int B, Nb, Ci, Co, L, act;
  float slope;
  InNorm in;          // X given as the previous block's stored pre-activation (gamma == nullptr: X as it is)
  // workspace
  CbpChan* chan;      // [B][Co]
  float* p0;          // [B][Co]
  float* p1;          // [B][Co]
  float* s;           // [B][Nb][Co]
  float* XX;          // [B][Ci][Ci]
  float* SX;          // [B][Ci]
  bf16_raw* negG;     // [B][Ci][Ci]
  float* v;           // [B][Ci]
  bf16_raw* xg;       // [B][Nb][Co][Ci]: the input column at each argmax point
  float* SXpart;      // [B][Nb][tiles][Ci]
  uint32_t* skey;     // [B][Nb][Co]: argmax positions sorted by point, point << 10 | channel
  float* sval;        // [B][Nb][Co]: s in that order
  int* toff;          // [B][Nb][tiles + 1]: where each 128-point tile starts in the sorted order
  int c_vec;
  uint32_t x_extent, g_extent;
};

// ---- per channel: dbeta, dgamma from the Nb argmax elements; coefficients ----------------
__global__ __launch_bounds__(64) void cbp_coef_kernel(CbpArgs p) {
  const int c = blockIdx.x, b = blockIdx.y, k = b * p.Co + c;
  const int lane = threadIdx.x;
  const float mean = p.save_mean[k], invstd = p.save_invstd[k], g = p.gamma[k], bt = p.beta[k];
  float s1 = 0.f, s2 = 0.f;
  for (int n = lane; n < p.Nb; n += 64) {
    const int hit = min(max(p.idx[b * p.vsb + n * p.vsn + c * p.vsc], 0), p.L - 1);
    const float z = p.zhit ? p.zhit[((int64_t)b * p.Nb + n) * p.Co + c]
                           : bf16_to_f32(p.Z[b * p.zsb + n * p.zsn + c * p.zsc + hit]);
    const float xh = (z - mean) * invstd;
    const float gr = bf16_to_f32(p.dV[b * p.vsb + n * p.vsn + c * p.vsc]) * act_grad(fmaf(g, xh, bt), p.act, p.slope);
    s1 += gr;
    s2 = fmaf(gr, xh, s2);
    p.s[((int64_t)b * p.Nb + n) * p.Co + c] = gr;          // scaled by a below
  }
  s1 = wave_sum(s1);
  s2 = wave_sum(s2);
  const float a = g * invstd;
  const float m = (float)p.Nb * (float)p.L;
  const float bias = p.bias ? bf16_to_f32(p.bias[k]) : 0.f;
  for (int n = lane; n < p.Nb; n += 64) p.s[((int64_t)b * p.Nb + n) * p.Co + c] *= a;
  if (lane == 0) {
    p.dbeta[k] = s1;
    p.dgamma[k] = s2;
    if (p.dbias) p.dbias[k] = 0.f;                          // a bias in front of a BatchNorm: gradient exactly zero
    p.chan[k] = CbpChan{a, s1, s2, invstd, mean, bias};
    p.p1[k] = a * invstd * s2 / m;
    p.p0[k] = a * (s1 + invstd * s2 * (bias - mean)) / m;
  }
}

// ---- XX[b] = sum over (n, l) of x x^T, the Gram matrix of the layer input ------------------------
// One workgroup accumulates the whole Ci x Ci matrix (Ci <= 128) over its share of 128-point tiles:
// the tile is loaded ONCE (8-byte pieces, points contiguous = the contraction index), parked in one
// of two LDS buffers, and serves as both operands of the matrix instruction; the next tile is in
// flight in registers meanwhile.  Per-workgroup partial matrices are added in a fixed order by
// gram_reduce_kernel.  HBM-bound: x read once.
struct GramArgs {
  const bf16_raw* X; float* partial; float* XX;
  int64_t xsb, xsn, xsc;
  int Nb, Ci, L, tiles_k, chunks;
  uint32_t x_extent;
  InNorm in;          // X given as the previous block's stored pre-activation (gamma == nullptr: X as it is)
  bf16_raw* Xact;     // with `in`: where the values formed on load are also written (nullptr: nowhere)
  int64_t asb, asn, asc;
};

__global__ __launch_bounds__(GEMM_THREADS, 2) void gram_kernel(GramArgs p) {
  constexpr int GPTS = 128;                              // points per tile: 256-byte row segments (64 points moved at 2.6 TB/s)
  constexpr int GP = GPTS * 2 + 16;                      // bytes per LDS row: the tile's points + pad
  __shared__ __attribute__((aligned(16))) unsigned char smem[2][128 * GP];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int b = blockIdx.y, chunk = blockIdx.x;
  const int total = p.Nb * p.tiles_k;
  const int t0 = (int)((int64_t)total * chunk / p.chunks), t1 = (int)((int64_t)total * (chunk + 1) / p.chunks);
  const int row = t >> 5, piece = t & 31;                // 8 rows x 32 pieces per pass, 16 passes
  __shared__ float4 icn[128];                            // the input block's BatchNorm constants, if X is a pre-activation
  const bool xin = p.in.gamma != nullptr;
  if (xin) {
    if (t < 128) icn[t] = t < p.Ci ? in_norm_consts(p.in, (int64_t)b * p.Ci + t) : make_float4(0.f, 0.f, 0.f, 0.f);
    __syncthreads();
  }
  uint2 q[16];
  auto load = [&](int tile) {
    const int n = tile / p.tiles_k, l = (tile - n * p.tiles_k) * GPTS + piece * 4;
    const __amdgpu_buffer_rsrc_t rx = pf_rsrc(p.X + b * p.xsb + n * p.xsn, p.x_extent);
#pragma unroll
    for (int h = 0; h < 16; ++h) {
      const int ci = row + 8 * h;
      const bool ok = tile < t1 && ci < p.Ci && l + 4 <= p.L;
      const pf_u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rx, (int)(ok ? (uint32_t)ci * (uint32_t)(p.xsc * 2) + (uint32_t)l * 2u : PF_OOB), 0, 0);
      q[h] = make_uint2(v.x, v.y);
    }
  };
  f32x16_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  const int r = lane & 31, gsel = lane >> 5;
  load(t0);
  for (int tile = t0; tile < t1; ++tile) {
    unsigned char* buf = smem[(tile - t0) & 1];
    if (xin) {
      const int nn = tile / p.tiles_k;
      const bool ok = (tile - nn * p.tiles_k) * GPTS + piece * 4 + 4 <= p.L;
#pragma unroll
      for (int h = 0; h < 16; ++h) q[h] = in_norm_apply4(q[h], icn[row + 8 * h], ok, p.in.act, p.in.slope);
      if (p.Xact && ok) {                                  // every element of X passes through exactly one workgroup
        bf16_raw* o = p.Xact + b * p.asb + nn * p.asn + (tile - nn * p.tiles_k) * GPTS + piece * 4;
#pragma unroll
        for (int h = 0; h < 16; ++h)
          if (row + 8 * h < p.Ci) *reinterpret_cast<uint2*>(o + (row + 8 * h) * p.asc) = q[h];
      }
    }
#pragma unroll
    for (int h = 0; h < 16; ++h) *reinterpret_cast<uint2*>(buf + (row + 8 * h) * GP + piece * 8) = q[h];
    __syncthreads();                                     // the other buffer was last read one step ago
    load(tile + 1);
#pragma unroll
    for (int s = 0; s < GPTS / 16; ++s) {
      bf16x8_t a[2], bb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        a[i] = *reinterpret_cast<const bf16x8_t*>(buf + (wm * 64 + i * 32 + r) * GP + (2 * s + gsel) * 16);
        bb[i] = *reinterpret_cast<const bf16x8_t*>(buf + (wn * 64 + i * 32 + r) * GP + (2 * s + gsel) * 16);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bb[j], a[i], acc[i][j], 0, 0, 0);
    }
  }
  // acc[i][j][4q+e]: column (from the first operand) wn*64 + j*32 + 8q + 4*gsel + e, row (second operand) wm*64 + i*32 + r
  float* out = p.partial + ((int64_t)chunk * gridDim.y + b) * p.Ci * p.Ci;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int ci = wm * 64 + i * 32 + r;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int cj = wn * 64 + j * 32 + 8 * (v >> 2) + 4 * gsel + (v & 3);
        if (ci < p.Ci && cj < p.Ci) out[(int64_t)ci * p.Ci + cj] = acc[i][j][v];
      }
  }
}

__global__ __launch_bounds__(256) void gram_reduce_kernel(const float* __restrict__ partial, float* __restrict__ XX,
                                                          int64_t count, int chunks) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;          // four interleaved sums, then (0+1)+(2+3): a fixed order
  int k = 0;
  for (; k + 4 <= chunks; k += 4) {
    s0 += partial[(int64_t)k * count + i];
    s1 += partial[(int64_t)(k + 1) * count + i];
    s2 += partial[(int64_t)(k + 2) * count + i];
    s3 += partial[(int64_t)(k + 3) * count + i];
  }
  for (; k < chunks; ++k) s0 += partial[(int64_t)k * count + i];
  XX[i] = (s0 + s1) + (s2 + s3);
}

int gram_chunks(int B, int Nb, int L) {
  const int total = Nb * ((L + 127) / 128);
  int c = (512 + B - 1) / B;
  if (c > total) c = total;
  return c < 1 ? 1 : c;
}
size_t gram_partial_bytes(int B, int Nb, int Ci, int L) { return (size_t)gram_chunks(B, Nb, L) * B * Ci * Ci * 4; }

// XX[b][ci][cj] for all models; `partial` holds gram_partial_bytes
int gram_launch(int B, int Nb, int Ci, int L, const void* X, const int64_t xs[4], float* XX, float* partial,
                uint32_t x_extent, const InNorm& in, void* Xact, const int64_t xas[4], hipStream_t st) {
  GramArgs g{(const bf16_raw*)X, partial, XX, xs[0], xs[1], xs[2], Nb, Ci, L, (L + 127) / 128, gram_chunks(B, Nb, L), x_extent, in,
             (bf16_raw*)Xact, Xact ? xas[0] : 0, Xact ? xas[1] : 0, Xact ? xas[2] : 0};
  hipLaunchKernelGGL(gram_kernel, dim3((unsigned)g.chunks, (unsigned)B), dim3(GEMM_THREADS), 0, st, g);
  if (launch_status() != HFTA_OK) return HFTA_ELAUNCH;
  const int64_t count = (int64_t)B * Ci * Ci;
  hipLaunchKernelGGL(gram_reduce_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, (const float*)partial, XX,
                     count, g.chunks);
  return launch_status();
}

// ---- argmax positions of one (model, sample) sorted by point, ties in channel order ------------
// key = point << 10 | channel (Co <= 1024, L < 2^21: checked on the host); bitonic sort in LDS.
// toff[tile] = first sorted position whose point lies in 128-point tile `tile` or later.
__global__ __launch_bounds__(512) void cbp_sort_kernel(CbpArgs p, int P, int tiles) {
  __shared__ uint32_t key[1024];
  const int n = blockIdx.x, b = blockIdx.y, t = threadIdx.x;
  for (int c = t; c < P; c += 512) {
    uint32_t k = 0xffffffffu;
    if (c < p.Co) {
      const int hit = min(max(p.idx[b * p.vsb + n * p.vsn + c * p.vsc], 0), p.L - 1);
      k = ((uint32_t)hit << 10) | (uint32_t)c;
    }
    key[c] = k;
  }
  for (int k = 2; k <= P; k <<= 1)
    for (int j = k >> 1; j > 0; j >>= 1) {
      __syncthreads();
      for (int i = t; i < P / 2; i += 512) {
        const int lo = 2 * (i & ~(j - 1)) + (i & (j - 1)), hi = lo + j;
        const uint32_t x = key[lo], y = key[hi];
        if ((x > y) == ((lo & k) == 0)) { key[lo] = y; key[hi] = x; }
      }
    }
  __syncthreads();
  const int64_t base = ((int64_t)b * p.Nb + n) * p.Co;
  for (int c = t; c < p.Co; c += 512) {
    const uint32_t k = key[c];
    p.skey[base + c] = k;
    p.sval[base + c] = p.s[base + (k & 1023u)];
  }
  int* toff = p.toff + ((int64_t)b * p.Nb + n) * (tiles + 1);
  for (int k = t; k <= p.Co; k += 512) {
    const int cur = k < p.Co ? (int)(key[k] >> 17) : tiles;
    const int prev = k > 0 ? (int)(key[k - 1] >> 17) : -1;
    for (int tl = prev + 1; tl <= cur; ++tl) toff[tl] = k;
  }
}

// ---- G = sum_c p1[c] W[c,:]^T W[c,:] (stored negated, bf16) and v = sum_c p0[c] W[c,:] --------
// One workgroup per 32 x 32 tile of G and model, fp32 matrix instructions (the operands are exact
// in fp32); the eight wavefronts take an eighth of the channels each and are added in order.
constexpr int GW_WAVES = 8;
__global__ __launch_bounds__(GW_WAVES * 64) void cbp_gram_w_kernel(CbpArgs p) {
  __shared__ float red[GW_WAVES][16][64];
  __shared__ float vred[GW_WAVES][32];
  const int T = (p.Ci + 31) / 32;
  const int ti = blockIdx.x / T, tj = blockIdx.x % T, b = blockIdx.y;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int i = lane & 31, kh = lane >> 5;
  const int ca = ti * 32 + i, cb = tj * 32 + i;
  const float ma = ca < p.Ci ? 1.f : 0.f, mb = cb < p.Ci ? 1.f : 0.f;
  const bf16_raw* Wa = p.W + (int64_t)b * p.Co * p.Ci + min(ca, p.Ci - 1);
  const bf16_raw* Wc = p.W + (int64_t)b * p.Co * p.Ci + min(cb, p.Ci - 1);
  const float* P1 = p.p1 + b * p.Co;
  const float* P0 = p.p0 + b * p.Co;
  const int per = ((p.Co + 2 * GW_WAVES - 1) / (2 * GW_WAVES)) * 2;      // channels per wavefront, even
  const int c_lo = wave * per, c_hi = min(p.Co, c_lo + per);
  f32x16_t acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  float vacc = 0.f;
  for (int c2 = c_lo; c2 < c_hi; c2 += 16) {
    float wa[8], wb[8], q1[8], q0[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {                        // unconditional loads at a clamped channel, masked below
      const int c = c2 + 2 * u + kh;
      const int cc = min(c, c_hi - 1);
      const float live = c < c_hi ? 1.f : 0.f;
      wa[u] = bf16_to_f32(Wa[(int64_t)cc * p.Ci]) * (ma * live);
      wb[u] = bf16_to_f32(Wc[(int64_t)cc * p.Ci]) * mb;
      q1[u] = P1[cc];
      q0[u] = P0[cc];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(q1[u] * wa[u], wb[u], acc, 0, 0, 0);
      vacc = fmaf(q0[u], wa[u], vacc);
    }
  }
  vacc += __shfl_xor(vacc, 32, 64);
#pragma unroll
  for (int v = 0; v < 16; ++v) red[wave][v][lane] = acc[v];
  if (lane < 32) vred[wave][lane] = vacc;
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 16 * 64 / (GW_WAVES * 64); ++r) {
    const int o = t + GW_WAVES * 64 * r, v = o >> 6, ln = o & 63;
    float g = 0.f;
#pragma unroll
    for (int w = 0; w < GW_WAVES; ++w) g += red[w][v][ln];
    const int ci = ti * 32 + 8 * (v >> 2) + 4 * (ln >> 5) + (v & 3), cj = tj * 32 + (ln & 31);
    if (ci < p.Ci && cj < p.Ci) p.negG[((int64_t)b * p.Ci + ci) * p.Ci + cj] = f32_to_bf16(-g);
  }
  if (tj == 0 && t < 32 && ti * 32 + t < p.Ci) {
    float vs = 0.f;
#pragma unroll
    for (int w = 0; w < GW_WAVES; ++w) vs += vred[w][t];
    p.v[(int64_t)b * p.Ci + ti * 32 + t] = vs;
  }
}

// ---- dX tile = -(G x) - v + argmax columns.  Also emits, for the weight gradient, the input
// ---- column x[:, idx] of every argmax that falls in the tile and the tile's row sums of x. ----
template <int KT>
__global__ __launch_bounds__(GEMM_THREADS) void cbp_dx_kernel(CbpArgs p) {
  constexpr int PITCH = KT * 2 + 16;
  constexpr int TILE = 128 * PITCH;
  constexpr int STAGE = 64 * EPI_PITCH4;                 // fp32 staging of 64 rows
  constexpr int GREG = TILE > STAGE ? TILE : STAGE;
  constexpr int SUB = KT / 32;
  constexpr int WP = KT * 2;                             // pitch of a staged W row
  constexpr int HC = TILE / WP;                          // W rows that fit where the X tile was
  constexpr int PRE = 16;                                // W rows per wavefront fetched ahead into registers
  __shared__ __attribute__((aligned(16))) unsigned char smem[TILE + GREG];
  __shared__ unsigned short hit_c[1024];               // this tile's argmax hits (Co <= 1024 on the host):
  __shared__ unsigned char hit_q[1024];                // channel, column inside the tile, gradient value;
  __shared__ float hit_s[1024];                        // sorted by column, channel order inside a column
  __shared__ float sxs[256];
  __shared__ float4 icn[KT];                           // the input block's BatchNorm constants, if X is a pre-activation
  unsigned char* Xs = smem;
  unsigned char* Gs = smem + TILE;

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  int bx = blockIdx.x, bz = blockIdx.z;
  {  // XCD-aware renumbering (see gemm_kernel)
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
  const __amdgpu_buffer_rsrc_t rx = pf_rsrc(p.X + b * p.xsb + n * p.xsn, p.x_extent);
  const __amdgpu_buffer_rsrc_t rg = pf_rsrc(p.negG + (int64_t)b * p.Ci * p.Ci, p.g_extent);
  const int* toff = p.toff + (int64_t)bz * (gridDim.x + 1);
  const int k0 = toff[bx], nh = toff[bx + 1] - k0;
  const uint32_t* skey = p.skey + (int64_t)bz * p.Co + k0;
  const float* sval = p.sval + (int64_t)bz * p.Co + k0;
  const bf16_raw* Wb = p.W + (int64_t)b * p.Co * p.Ci;

  {  // X tile, transposed in registers into [point][ci]
    const int kq = t % 8, ng = t / 8;
    const int c = l0 + ng * 4;
    const uint32_t ldb = (uint32_t)(p.xsc * 2);
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
    if (p.in.gamma) {                    // X is a stored pre-activation: the block's activated output is formed here
      for (int k = t; k < KT; k += GEMM_THREADS)
        icn[k] = k < p.Ci ? in_norm_consts(p.in, (int64_t)b * p.Ci + k) : make_float4(0.f, 0.f, 0.f, 0.f);
      __syncthreads();
#pragma unroll
      for (int s = 0; s < SUB; ++s)
#pragma unroll
        for (int j = 0; j < 4; ++j) q[s][j] = in_norm_apply4(q[s][j], icn[s * 32 + 4 * kq + j], c + 4 <= p.L, p.in.act, p.in.slope);
    }
    // the tile's hit list rides along with the tile loads
    const uint32_t key0 = t < nh ? skey[t] : 0u;
    const float sv0 = t < nh ? sval[t] : 0.f;
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
    if (t < nh) {
      hit_c[t] = (unsigned short)(key0 & 1023u); hit_q[t] = (unsigned char)((int)(key0 >> 10) - l0); hit_s[t] = sv0;
    }
    for (int i = t + GEMM_THREADS; i < nh; i += GEMM_THREADS) {
      const uint32_t k = skey[i];
      hit_c[i] = (unsigned short)(k & 1023u); hit_q[i] = (unsigned char)((int)(k >> 10) - l0); hit_s[i] = sval[i];
    }
  }
  {  // -G rows (k-contiguous)
    const int wr = t >> 2, wg = (t & 3) * 8;
#pragma unroll
    for (int s = 0; s < SUB; ++s)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int row = wr + 64 * h, k = s * 32 + wg;
        const bool ok = row < p.Ci && k + 8 <= p.Ci;
        const pf_u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rg, (int)(ok ? ((uint32_t)row * (uint32_t)p.Ci + (uint32_t)k) * 2u : PF_OOB), 0, 0);
        *reinterpret_cast<uint4*>(Gs + row * PITCH + k * 2) = make_uint4(v.x, v.y, v.z, v.w);
      }
  }
  __syncthreads();

  // W rows of the first hits: fetched now, parked in LDS once the X tile is dead
  uint32_t wpre[PRE];
#pragma unroll
  for (int r = 0; r < PRE; ++r) {
    const int i = wave + 4 * r;
    wpre[r] = 0u;
    if (i < nh && 2 * lane < p.Ci) wpre[r] = reinterpret_cast<const uint32_t*>(Wb + (int64_t)hit_c[i] * p.Ci)[lane];
  }

  f32x16_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  const int r = lane & 31, gsel = lane >> 5;
#pragma unroll
  for (int s = 0; s < KT / 16; ++s) {
    bf16x8_t a[2], bb[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      a[i] = *reinterpret_cast<const bf16x8_t*>(Gs + (wm * 64 + i * 32 + r) * PITCH + (2 * s + gsel) * 16);
      bb[i] = *reinterpret_cast<const bf16x8_t*>(Xs + (wn * 64 + i * 32 + r) * PITCH + (2 * s + gsel) * 16);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bb[j], a[i], acc[i][j], 0, 0, 0);
  }

  {  // this tile's part of sum_l x: thread (ci, half) adds 64 points in order
    const int ci = t & 127, half = t >> 7;
    float sx = 0.f;
    if (ci < KT) {
      const unsigned char* col = Xs + (half * 64) * PITCH + ci * 2;
#pragma unroll 8
      for (int q = 0; q < 64; ++q) sx += bf16_to_f32(*reinterpret_cast<const bf16_raw*>(col + q * PITCH));
    }
    sxs[t] = sx;
  }
  // input columns at the argmax points, for the weight gradient's gather term
#pragma unroll 4
  for (int h = wave; h < nh; h += 4) {
    const uint32_t* xrow = reinterpret_cast<const uint32_t*>(Xs + hit_q[h] * PITCH);
    uint32_t* dst = reinterpret_cast<uint32_t*>(p.xg + ((int64_t)bz * p.Co + hit_c[h]) * p.Ci);
    if (2 * lane < p.Ci) dst[lane] = xrow[lane];
  }
  __syncthreads();                                       // both tiles are dead from here on

  if (p.SXpart && t < 128 && t < p.Ci) p.SXpart[((int64_t)bz * gridDim.x + bx) * p.Ci + t] = sxs[t] + sxs[t + 128];
  bf16_raw* dXb = p.dX + b * p.dxsb + n * p.dxsn;
  float* stage = reinterpret_cast<float*>(Gs);
  unsigned char* Wh = Xs;
  constexpr int SP = EPI_PITCH4 / 4;                     // staging pitch in floats
  const int ml = lane & 31, nq = (lane >> 5) * 4;

  // W rows kc .. kc+kn of the hit list into LDS (row i of the chunk at Wh + i * WP); lanes past Ci write zeros
  auto load_rows = [&](int kc, int kn, int first) {
    for (int i = wave + 4 * first; i < kn; i += 4) {
      uint32_t w = 0u;
      if (2 * lane < p.Ci) w = reinterpret_cast<const uint32_t*>(Wb + (int64_t)hit_c[kc + i] * p.Ci)[lane];
      if (4 * lane < WP) *reinterpret_cast<uint32_t*>(Wh + i * WP + lane * 4) = w;
    }
  };
#pragma unroll
  for (int r2 = 0; r2 < PRE; ++r2) {
    const int i = wave + 4 * r2;
    if (i < nh && i < HC && 4 * lane < WP) *reinterpret_cast<uint32_t*>(Wh + i * WP + lane * 4) = wpre[r2];
  }
  load_rows(0, min(nh, HC), PRE);
  int resident = 0;                                      // first hit of the chunk that sits in Wh

  // ---- two passes of 64 output rows: stage fp32 (dense part), add the columns, store as bf16
#pragma unroll 1
  for (int pass = 0; pass < 2; ++pass) {
    if (wm == pass) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int rl = i * 32 + ml;
        const int m = pass * 64 + rl;
        const float vm = m < p.Ci ? p.v[(int64_t)b * p.Ci + m] : 0.f;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int nl = wn * 64 + j * 32 + 8 * q + nq;
            *reinterpret_cast<float4*>(stage + rl * SP + nl) =
                make_float4(acc[i][j][4 * q] - vm, acc[i][j][4 * q + 1] - vm, acc[i][j][4 * q + 2] - vm,
                            acc[i][j][4 * q + 3] - vm);
          }
      }
    }
    __syncthreads();                                     // staged rows and W rows in place
    if (pass * 64 < p.Ci) {
#pragma unroll 1
      for (int kc = 0; kc < nh; kc += HC) {
        const int kn = min(HC, nh - kc);
        if (kc != resident) {
          load_rows(kc, kn, 0);
          resident = kc;
          __syncthreads();
        }
        // the wavefronts split the chunk at column boundaries; one lane per output row walks its
        // share in order: a column's hits in channel order, then one update of the staged cell
        int ka = kc + (kn * wave) / 4, ke = kc + (kn * (wave + 1)) / 4;
        while (ka > kc && ka < kc + kn && hit_q[ka] == hit_q[ka - 1]) ++ka;
        while (ke > kc && ke < kc + kn && hit_q[ke] == hit_q[ke - 1]) ++ke;
        const unsigned char* wcol = Wh + (pass * 64 + lane) * 2 - kc * WP;
        if (ka < ke) {
          int col = hit_q[ka];
          float val = 0.f;
#pragma unroll 4
          for (int k = ka; k < ke; ++k) {                // the loads of several hits are in flight together
            const int q = hit_q[k];
            const float sv = hit_s[k];
            const float w = bf16_to_f32(*reinterpret_cast<const bf16_raw*>(wcol + k * WP));
            if (q != col) {
              stage[lane * SP + col] += val;
              val = 0.f;
              col = q;
            }
            val = fmaf(sv, w, val);
          }
          stage[lane * SP + col] += val;
        }
        __syncthreads();
      }
    }
    // 64 rows x 128 columns out as bf16: 4-column (8-byte) pieces, consecutive lanes on consecutive pieces
#pragma unroll
    for (int it = 0; it < 64 * 32 / GEMM_THREADS; ++it) {
      const int id = t + GEMM_THREADS * it;
      const int rr = id >> 5, cp = id & 31;
      const int m = pass * 64 + rr, l = l0 + cp * 4;
      const float4 f = *reinterpret_cast<const float4*>(stage + rr * SP + cp * 4);
      if (m < p.Ci && l < p.L) {
        bf16_raw* d = dXb + (int64_t)m * p.dxsc + l;
        if (p.c_vec >= 8 && l + 4 <= p.L) {
          *reinterpret_cast<uint2*>(d) = make_uint2(pack_bf16x2(f.x, f.y), pack_bf16x2(f.z, f.w));
        } else {
          const float e[4] = {f.x, f.y, f.z, f.w};
#pragma unroll
          for (int k = 0; k < 4; ++k)
            if (l + k < p.L) d[k] = f32_to_bf16(e[k]);
        }
      }
    }
    __syncthreads();
  }
}

// ---- SX[b][ci] = sum over (n, l) of x, from the per-tile sums, in a fixed order -----------------
__global__ __launch_bounds__(1024) void cbp_sx_kernel(const float* part, float* SX, int Ci, int parts) {
  __shared__ float red[64][16];
  const int b = blockIdx.y, cl = threadIdx.x & 15, g = threadIdx.x >> 4;
  const int ci = blockIdx.x * 16 + cl;
  const float* src = part + (int64_t)b * parts * Ci;
  float s = 0.f;
  if (ci < Ci) {
#pragma unroll 4
    for (int q = g; q < parts; q += 64) s += src[(int64_t)q * Ci + ci];
  }
  red[g][cl] = s;
  __syncthreads();
  if (g == 0 && ci < Ci) {
    float tot = 0.f;
    for (int k = 0; k < 64; ++k) tot += red[k][cl];
    SX[(int64_t)b * Ci + ci] = tot;
  }
}

// ---- dW[c][:] = gather term - a (dbeta E[x] + invstd dgamma Cov(z_c, x)), 8 channels per workgroup ----
// One thread per (channel of the eight, input channel): the sums over ci and over the Nb argmax rows are
// short dependent chains of loads, so the kernel is bound by their latency and wants threads, not work
// per thread (128 threads walking the eight channels one after the other took 33 us on config 1).
__global__ __launch_bounds__(1024) void cbp_dw_kernel(CbpArgs p) {
  constexpr int CB = 8;
  __shared__ float wrow[CB][128];
  const int c0 = blockIdx.x * CB, b = blockIdx.y, cj = threadIdx.x & 127, e = threadIdx.x >> 7;
  for (int i = threadIdx.x; i < CB * p.Ci; i += 1024) {
    const int cc = i / p.Ci, k = i - cc * p.Ci;
    wrow[cc][k] = c0 + cc < p.Co ? bf16_to_f32(p.W[((int64_t)b * p.Co + c0 + cc) * p.Ci + k]) : 0.f;
  }
  __syncthreads();
  const int c = c0 + e;
  if (cj >= p.Ci || c >= p.Co) return;
  float T = 0.f;
  if (p.Tin) {
    T = p.Tin[((int64_t)b * p.Co + c) * p.Ci + cj];
  } else {
    const float* XXb = p.XX + (int64_t)b * p.Ci * p.Ci;
#pragma unroll 8
    for (int ci = 0; ci < p.Ci; ++ci) T = fmaf(wrow[e][ci], XXb[(int64_t)ci * p.Ci + cj], T);   // Ci is a multiple of 8 (host)
  }
  const double m = (double)p.Nb * (double)p.L;
  const double sx = (double)p.SX[(int64_t)b * p.Ci + cj], ex = sx / m;
  float sp = 0.f;
#pragma unroll 8
  for (int n = 0; n < p.Nb; ++n) {
    const int64_t row = ((int64_t)b * p.Nb + n) * p.Co + c;
    sp = fmaf(p.s[row], bf16_to_f32(p.xg[row * p.Ci + cj]), sp);
  }
  const CbpChan ch = p.chan[b * p.Co + c];
  const double ezx = ((double)T + (double)ch.bias * sx) / m;
  const double dense = (double)ch.a * ((double)ch.dbeta * ex + (double)ch.invstd * (double)ch.dgamma * (ezx - (double)ch.mean * ex));
  p.dW[((int64_t)b * p.Co + c) * p.Ci + cj] = (float)((double)sp - dense);
}

size_t a256(size_t v) { return (v + 255) & ~(size_t)255; }

// =====================================================================================================
// Forward of the same operator:  pooled = max_l act(BatchNorm(W x + bias)),  its argmax, the
// BatchNorm statistics -- without forming the [Nb, B*Co, L] convolution output.
//   * statistics from the input's moments: mean_c = (W_c SX)/m + bias_c,
//     var_c = (W_c XX W_c^T)/m - ((W_c SX)/m)^2, with XX, SX as in the backward (fp32 Gram matrix,
//     combined in double);
//   * the activations handled here (none, ReLU, LeakyReLU with slope >= 0) are non-decreasing and
//     BatchNorm is increasing in z where gamma > 0 and decreasing where gamma < 0, so the argmax of
//     the activated value is the argmax of  sign(gamma_c) (W_c x):  one pass of the matrix product
//     with sign-folded weights, a running (max, first argmax) per channel and tile, nothing stored.
// =====================================================================================================
// max of three without the quieting moves of fmaxf (inputs are matrix-instruction results)
__device__ __forceinline__ float fmax3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

struct FbpArgs {
  const bf16_raw* X; const bf16_raw* W; const bf16_raw* bias;
  const float* gamma; const float* beta;
  float* running_mean; float* running_var; float* save_mean; float* save_invstd;
  bf16_raw* V; int32_t* idx; float* zhit;
  int64_t xsb, xsn, xsc, vsb, vsn, vsc;
  int B, Nb, Ci, Co, L, act, tiles_co;
  float slope, eps, momentum;
  float* XX; float* SX; float* T;          // [B][Ci][Ci], [B][Ci], [B][Co][Ci]
  float* SXpart;                           // [B][Nb][tiles][2][Ci]
  float* pmax; int* pidx;                  // [B][Nb][tiles][Co]
  uint32_t x_extent, w_extent;
  InNorm in;                               // X given as the previous block's stored pre-activation (gamma == nullptr: X as it is)
};

// One workgroup owns a 128-point slice of one sample; each wavefront keeps its half of the X tile
// as matrix-instruction fragments in registers, the loop walks the RT-row tiles of W through two
// LDS buffers (tile ct+1 parked, tile ct+2 in flight in registers while tile ct is multiplied: one
// barrier per step), and the epilogue of a step is a per-lane search of the accumulators for
// (max, first argmax) instead of a store.  RT = 64: 32 accumulators and 16 in-flight W registers
// per lane (140 registers) and 36 KB of LDS, so three workgroups share a compute unit and cover each
// other's phases (128-row tiles: 201 registers, two workgroups, 10 % slower).
constexpr int FBP_RT = 64;     // rows of a W tile
constexpr int FBP_OCC = 3;     // workgroups per compute unit the register budget is set for
template <int KT, int RT>
__global__ __launch_bounds__(GEMM_THREADS, FBP_OCC) void fbp_main_kernel(FbpArgs p) {
  constexpr int PITCH = KT * 2 + 16;
  constexpr int XTILE = 128 * PITCH;
  constexpr int WTILE = RT * PITCH;
  constexpr int SUB = KT / 32;
  constexpr int H = RT / 64;                            // 64-row passes of the W tile load; 32-row blocks per wavefront
  __shared__ __attribute__((aligned(16))) unsigned char smem[XTILE > 2 * WTILE ? XTILE : 2 * WTILE];
  __shared__ float pm_v[2][2][RT];                     // [step parity][point half][channel]
  __shared__ int pm_p[2][2][RT];
  __shared__ float4 icn[KT];                           // the input block's BatchNorm constants, if X is a pre-activation

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  int bx = blockIdx.x, bz = blockIdx.z;
  {  // XCD-aware renumbering (see gemm_kernel)
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
  const __amdgpu_buffer_rsrc_t rx = pf_rsrc(p.X + b * p.xsb + n * p.xsn, p.x_extent);
  const __amdgpu_buffer_rsrc_t rgam = pf_rsrc(p.gamma + (int64_t)b * p.Co, (uint32_t)p.Co * 4u);

  // W tiles: rows t/4 (+64), 16-byte group t%4 of every 32-wide k block; a row whose gamma is
  // negative gets the sign bit of every element flipped (exact), so that every channel looks for a maximum
  const int wr = t >> 2, wg = (t & 3) * 8;
  uint4 wq[SUB][H];
  uint32_t gq[H];                        // the rows' gamma, raw bits: looked at only when the tile is parked
  auto load_w = [&](int ct) {
#pragma unroll
    for (int h = 0; h < H; ++h) {
      const int row = ct * RT + wr + 64 * h;
      gq[h] = __builtin_amdgcn_raw_buffer_load_b32(rgam, (int)(row < p.Co ? (uint32_t)row * 4u : PF_OOB), 0, 0);
#pragma unroll
      for (int s = 0; s < SUB; ++s) {
        const int k = s * 32 + wg;
        const bool ok = row < p.Co && k + 8 <= p.Ci;
        const pf_u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rw, (int)(ok ? ((uint32_t)row * (uint32_t)p.Ci + (uint32_t)k) * 2u : PF_OOB), 0, 0);
        wq[s][h] = make_uint4(v.x, v.y, v.z, v.w);
      }
    }
  };
  load_w(0);

  {  // X tile, transposed in registers into [point][ci]
    const int kq = t % 8, ng = t / 8;
    const int c = l0 + ng * 4;
    const uint32_t ldb = (uint32_t)(p.xsc * 2);
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
    if (p.in.gamma) {                    // X is a stored pre-activation: the block's activated output is formed here
      for (int k = t; k < KT; k += GEMM_THREADS)
        icn[k] = k < p.Ci ? in_norm_consts(p.in, (int64_t)b * p.Ci + k) : make_float4(0.f, 0.f, 0.f, 0.f);
      __syncthreads();
#pragma unroll
      for (int s = 0; s < SUB; ++s)
#pragma unroll
        for (int j = 0; j < 4; ++j) q[s][j] = in_norm_apply4(q[s][j], icn[s * 32 + 4 * kq + j], c + 4 <= p.L, p.in.act, p.in.slope);
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
        *reinterpret_cast<uint2*>(smem + (ng * 4 + i) * PITCH + s * 64 + kq * 8) = o[i];
    }
  }

  const int r = lane & 31, gsel = lane >> 5;
  const int tiles = gridDim.x;
  float* pmax = p.pmax + ((int64_t)bz * tiles + bx) * p.Co;
  int* pidx = p.pidx + ((int64_t)bz * tiles + bx) * p.Co;
  const int lim = p.L - l0;                              // points of this slice that exist (>= 1)
  auto publish = [&](int ct) {                           // step ct's per-channel result, both point halves merged
    if (t < RT && ct * RT + t < p.Co) {
      const int pb = ct & 1;
      const float v0 = pm_v[pb][0][t], v1 = pm_v[pb][1][t];
      const bool hi = v1 > v0;                           // a tie goes to the lower points
      pmax[ct * RT + t] = hi ? v1 : v0;
      pidx[ct * RT + t] = l0 + (hi ? pm_p[pb][1][t] : pm_p[pb][0][t]);
    }
  };
  auto park_w = [&](unsigned char* dst) {                // the W tile in registers -> LDS, sign-folded
#pragma unroll
    for (int s = 0; s < SUB; ++s)
#pragma unroll
      for (int h = 0; h < H; ++h) {
        const uint4 w = wq[s][h];
        const uint32_t flip = __uint_as_float(gq[h]) < 0.f ? 0x80008000u : 0u;
        *reinterpret_cast<uint4*>(dst + (wr + 64 * h) * PITCH + (s * 32 + wg) * 2) =
            make_uint4(w.x ^ flip, w.y ^ flip, w.z ^ flip, w.w ^ flip);
      }
  };

  // The X operand of this wavefront never changes: its matrix-instruction fragments move from LDS
  // into registers once, and the X tile's LDS becomes the two W buffers.
  __syncthreads();
  bf16x8_t xf[2][KT / 16];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int s = 0; s < KT / 16; ++s)
      xf[j][s] = *reinterpret_cast<const bf16x8_t*>(smem + (wn * 64 + j * 32 + r) * PITCH + (2 * s + gsel) * 16);
  {  // this slice's part of sum_l x: thread (ci, half) adds 64 points in order
    const int ci = t & 127, half = t >> 7;
    if (ci < p.Ci) {
      float sx = 0.f;
      const unsigned char* col = smem + (half * 64) * PITCH + ci * 2;
#pragma unroll 8
      for (int q = 0; q < 64; ++q) sx += bf16_to_f32(*reinterpret_cast<const bf16_raw*>(col + q * PITCH));
      p.SXpart[(((int64_t)bz * tiles + bx) * 2 + half) * p.Ci + ci] = sx;
    }
  }
  __syncthreads();                       // the X tile is dead
  park_w(smem);
  load_w(1);
  __syncthreads();

  for (int ct = 0; ct < p.tiles_co; ++ct) {
    const unsigned char* cur = smem + (ct & 1) * WTILE;
    park_w(smem + ((ct + 1) & 1) * WTILE);   // tile ct+1; that buffer was last read in step ct-1
    load_w(ct + 2);                      // past the last tile: rows >= Co, zeros, no traffic
    if (ct > 0) publish(ct - 1);

    f32x16_t acc[H][2];
#pragma unroll
    for (int i = 0; i < H; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
#pragma unroll
    for (int s = 0; s < KT / 16; ++s) {
      bf16x8_t a[H];
#pragma unroll
      for (int i = 0; i < H; ++i)
        a[i] = *reinterpret_cast<const bf16x8_t*>(cur + (wm * (RT / 2) + i * 32 + r) * PITCH + (2 * s + gsel) * 16);
#pragma unroll
      for (int i = 0; i < H; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf[j][s], a[i], acc[i][j], 0, 0, 0);
    }
    // lane = channel wm*(RT/2) + i*32 + (lane & 31); its 32 points wn*64 + j*32 + 8q + 4(lane>>5) + e in rising order.
    // Two passes per channel: the maximum of the lane's 32 values (no index carried), then the
    // first position that holds it, walking the positions downwards so the lowest one is kept.
    float bv[H];
    int bp[H];
    const int pt0 = wn * 64 + 4 * gsel;
    if (lim < 128) {                       // the last slice: points past L do not take part
      int room = lim - pt0;                // opaque to the optimizer: 64 loop-invariant lane masks
      asm volatile("" : "+v"(room));       // would otherwise be kept (and spilled) across the loop
#pragma unroll
      for (int i = 0; i < H; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            if (j * 32 + 8 * (v >> 2) + (v & 3) >= room) acc[i][j][v] = -INFINITY;
    }
#pragma unroll
    for (int i = 0; i < H; ++i) {
      float m[8];
#pragma unroll
      for (int q = 0; q < 8; ++q)
        m[q] = fmax3(acc[i][q >> 2][4 * (q & 3)], acc[i][q >> 2][4 * (q & 3) + 1],
                     fmax3(acc[i][q >> 2][4 * (q & 3) + 2], acc[i][q >> 2][4 * (q & 3) + 3], -INFINITY));
      bv[i] = fmax3(fmax3(m[0], m[1], m[2]), fmax3(m[3], m[4], m[5]), fmax3(m[6], m[7], -INFINITY));
    }
#pragma unroll
    for (int i = 0; i < H; ++i) {
      int rel = 0;
#pragma unroll
      for (int j = 1; j >= 0; --j)
#pragma unroll
        for (int v = 15; v >= 0; --v)
          rel = acc[i][j][v] == bv[i] ? j * 32 + 8 * (v >> 2) + (v & 3) : rel;
      bp[i] = pt0 + rel;
    }
#pragma unroll
    for (int i = 0; i < H; ++i) {        // the two lane halves hold interleaved groups of four points
      const float ov = __shfl_xor(bv[i], 32, 64);
      const int op = __shfl_xor(bp[i], 32, 64);
      if (ov > bv[i] || (ov == bv[i] && op < bp[i])) { bv[i] = ov; bp[i] = op; }
      if (lane < 32) {
        pm_v[ct & 1][wn][wm * (RT / 2) + i * 32 + lane] = bv[i];
        pm_p[ct & 1][wn][wm * (RT / 2) + i * 32 + lane] = bp[i];
      }
    }
    __syncthreads();                     // tile ct+1 is in LDS, tile ct is free, step ct's maxima are published next
  }
  publish(p.tiles_co - 1);
}

// ---- statistics from the moments; T = W XX kept for the backward operator --------------------------
__global__ __launch_bounds__(128) void fbp_stats_kernel(FbpArgs p) {
  constexpr int CB = 8;
  __shared__ double wrow[CB][128];                       // widened once: the loop below is bound by fp64 issue
  __shared__ double red[2][CB][2];
  const int c0 = blockIdx.x * CB, b = blockIdx.y, cj = threadIdx.x;
  for (int e = cj; e < CB * p.Ci; e += 128) {
    const int cc = e / p.Ci, k = e - cc * p.Ci;
    wrow[cc][k] = c0 + cc < p.Co ? (double)bf16_to_f32(p.W[((int64_t)b * p.Co + c0 + cc) * p.Ci + k]) : 0.0;
  }
  __syncthreads();
  const bool live = cj < p.Ci;
  const float* XXb = p.XX + (int64_t)b * p.Ci * p.Ci;
  double T[CB];
#pragma unroll
  for (int e = 0; e < CB; ++e) T[e] = 0.0;
  if (live) {
#pragma unroll 16
    for (int ci = 0; ci < p.Ci; ++ci) {                  // a chain of loads: sixteen in flight
      const double x = (double)XXb[(int64_t)ci * p.Ci + cj];
#pragma unroll
      for (int e = 0; e < CB; ++e) T[e] = fma(wrow[e][ci], x, T[e]);
    }
  }
  const double sxj = live ? (double)p.SX[(int64_t)b * p.Ci + cj] : 0.0;
#pragma unroll
  for (int e = 0; e < CB; ++e) {
    if (live && c0 + e < p.Co) p.T[((int64_t)b * p.Co + c0 + e) * p.Ci + cj] = (float)T[e];
    const double w = live ? wrow[e][cj] : 0.0;
    double q = T[e] * w, s1 = w * sxj;                   // terms of W_c XX W_c^T and of W_c SX
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { q += __shfl_xor(q, o, 64); s1 += __shfl_xor(s1, o, 64); }
    if ((cj & 63) == 0) { red[cj >> 6][e][0] = q; red[cj >> 6][e][1] = s1; }
  }
  __syncthreads();
  if (cj < CB && c0 + cj < p.Co) {
    const int k = b * p.Co + c0 + cj;
    const double m = (double)p.Nb * (double)p.L;
    const double quad = red[0][cj][0] + red[1][cj][0], ws = red[0][cj][1] + red[1][cj][1];
    const double mz = ws / m;                            // mean of W x (the bias shifts the mean only)
    double var = quad / m - mz * mz;
    var = var < 0.0 ? 0.0 : var;
    const float mean = (float)(mz + (p.bias ? (double)bf16_to_f32(p.bias[k]) : 0.0));
    const float varf = (float)var;
    p.save_mean[k] = mean;
    p.save_invstd[k] = (float)(1.0 / sqrt(var + (double)p.eps));
    if (p.running_mean) {
      const float mf = (float)m;
      const float unb = mf > 1.f ? varf * (mf / (mf - 1.f)) : varf;
      p.running_mean[k] = (1.f - p.momentum) * p.running_mean[k] + p.momentum * mean;
      p.running_var[k] = (1.f - p.momentum) * p.running_var[k] + p.momentum * unb;
    }
  }
}

// ---- per (model, sample, channel): first maximum over the slices, then BatchNorm + activation ------
__global__ __launch_bounds__(256) void fbp_finish_kernel(FbpArgs p, int tiles) {
  const int c = blockIdx.x * 256 + threadIdx.x, n = blockIdx.y, b = blockIdx.z;
  if (c >= p.Co) return;
  const int64_t bn = (int64_t)b * p.Nb + n;
  const float* pv = p.pmax + bn * tiles * p.Co + c;
  const int* pi = p.pidx + bn * tiles * p.Co + c;
  float best = pv[0];
  int at = pi[0];
  for (int q = 1; q < tiles; ++q) {
    const float v = pv[(int64_t)q * p.Co];
    if (v > best) { best = v; at = pi[(int64_t)q * p.Co]; }
  }
  const int k = b * p.Co + c;
  const float g = p.gamma[k];
  const float bias = p.bias ? bf16_to_f32(p.bias[k]) : 0.f;
  const float scale = g * p.save_invstd[k], mean = p.save_mean[k], beta = p.beta[k];
  float z = (g < 0.f ? -best : best) + bias;
  float pre = fmaf(scale, z - mean, beta);
  // Equal activated values: the maximum is taken over act(BatchNorm(z)), so where the activation
  // is flat (ReLU, or LeakyReLU with slope 0, at a maximum that is not positive) or the channel's
  // scale is zero, every point of the row holds the same value and the lowest index, 0, is the
  // argmax.  z at point 0 is recomputed here (Ci products) since no slice kept it.
  const bool flat = g == 0.f || ((p.act == HFTA_ACT_RELU || (p.act == HFTA_ACT_LEAKY && p.slope == 0.f)) && !(pre > 0.f));
  if (flat && at != 0) {
    const bf16_raw* x0 = p.X + b * p.xsb + n * p.xsn;
    const bf16_raw* w = p.W + (int64_t)k * p.Ci;
    float acc = 0.f;
    for (int ci = 0; ci < p.Ci; ++ci) {
      float xv = bf16_to_f32(x0[ci * p.xsc]);
      if (p.in.gamma) xv = bf16_to_f32(f32_to_bf16(in_norm_one(xv, in_norm_consts(p.in, (int64_t)b * p.Ci + ci), p.in.act, p.in.slope)));
      acc = fmaf(bf16_to_f32(w[ci]), xv, acc);
    }
    at = 0;
    z = acc + bias;
    pre = fmaf(scale, z - mean, beta);
    if ((p.act == HFTA_ACT_RELU || (p.act == HFTA_ACT_LEAKY && p.slope == 0.f)) && pre > 0.f) pre = 0.f;   // the row's maximum was not positive
  }
  const float y = apply_act(pre, p.act, p.slope);
  p.V[b * p.vsb + n * p.vsn + c * p.vsc] = f32_to_bf16(y);
  p.idx[b * p.vsb + n * p.vsn + c * p.vsc] = at;
  p.zhit[bn * p.Co + c] = z;
}

struct FbpLayout { size_t SXpart, pmax, pidx, moments, part, total; };

size_t saved_floats(int B, int Ci, int Co) { return (size_t)B * ((size_t)Ci * Ci + Ci + (size_t)Co * Ci); }


struct CbpLayout { size_t chan, p0, p1, s, XX, SX, negG, v, xg, SXpart, skey, sval, toff, part, total; };

FbpLayout fbp_layout(int B, int Nb, int Ci, int Co, int L, bool own_moments) {
  FbpLayout w{};
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t o = off; off += a256(bytes); return o; };
  const size_t tiles = (size_t)(L + 127) / 128;
  w.SXpart = take((size_t)B * Nb * tiles * 2 * Ci * 4);
  w.pmax = take((size_t)B * Nb * tiles * Co * 4);
  w.pidx = take((size_t)B * Nb * tiles * Co * 4);
  w.moments = take(own_moments ? saved_floats(B, Ci, Co) * 4 : 0);
  w.part = take(gram_partial_bytes(B, Nb, Ci, L));
  w.total = off;
  return w;
}

CbpLayout cbp_layout(int B, int Nb, int Ci, int Co, int L) {
  CbpLayout w{};
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t o = off; off += a256(bytes); return o; };
  w.chan = take((size_t)B * Co * sizeof(CbpChan));
  w.p0 = take((size_t)B * Co * 4);
  w.p1 = take((size_t)B * Co * 4);
  w.s = take((size_t)B * Nb * Co * 4);
  w.XX = take((size_t)B * Ci * Ci * 4);
  w.SX = take((size_t)B * Ci * 4);
  w.negG = take((size_t)B * Ci * Ci * 2);
  w.v = take((size_t)B * Ci * 4);
  w.xg = take((size_t)B * Nb * Co * Ci * 2);
  w.SXpart = take((size_t)B * Nb * ((L + 127) / 128) * Ci * 4);
  w.skey = take((size_t)B * Nb * Co * 4);
  w.sval = take((size_t)B * Nb * Co * 4);
  w.toff = take((size_t)B * Nb * ((L + 127) / 128 + 1) * 4);
  w.part = take(gram_partial_bytes(B, Nb, Ci, L));
  w.total = off;
  return w;
}

bool cbp_supported(int B, int Nb, int Ci, int Co, int L, int dtype) {
  return dtype == HFTA_BF16 && B > 0 && Nb > 0 && Ci > 0 && Co > 0 && L > 0 && Ci <= 128 && Ci % 8 == 0 && Co <= 1024 &&
         L % 4 == 0 && L < (1 << 21) && Nb <= 65535 && B <= 65535 && (int64_t)B * Nb <= 65535;
}

}  // namespace

extern "C" {

size_t hfta_conv1x1_bn_maxpool_bwd_workspace_bytes(int B, int Nb, int Ci, int Co, int L, int dtype) {
  if (!cbp_supported(B, Nb, Ci, Co, L, dtype)) return 0;
  return cbp_layout(B, Nb, Ci, Co, L).total;
}

static int cbp_run(int B, int Nb, int Ci, int Co, int L, int dtype, const void* X, const int64_t xs[4],
                   const void* W, const void* bias, const void* Z, const int64_t zs[4], const float* zhit,
                   const float* saved_moments, const void* dV, const int32_t* idx, const int64_t vs[3],
                   const float* gamma, const float* beta, const float* save_mean, const float* save_invstd,
                   void* dX, const int64_t dxs[4], float* dW, float* dbias, float* dgamma, float* dbeta,
                   int act, float act_slope, void* workspace, size_t ws_bytes, void* stream, const InNorm& in) {
  if (B <= 0 || Nb <= 0 || Ci <= 0 || Co <= 0 || L <= 0 || !valid_dtype(dtype) || !X || !xs || !W || !dV ||
      !idx || !vs || !gamma || !beta || !save_mean || !save_invstd || !dX || !dxs || !dW || !dgamma || !dbeta)
    return HFTA_EINVAL;
  if ((Z == nullptr) == (zhit == nullptr) || (Z && !zs)) return HFTA_EINVAL;     // exactly one source of z at the argmax
  if (!(act == HFTA_ACT_NONE || act == HFTA_ACT_RELU || act == HFTA_ACT_LEAKY)) return HFTA_EUNSUPPORTED;
  if (!cbp_supported(B, Nb, Ci, Co, L, dtype) || xs[3] != 1 || (Z && zs[3] != 1) || dxs[3] != 1) return HFTA_EUNSUPPORTED;
  auto al = [](const void* q, size_t a) { return (reinterpret_cast<uintptr_t>(q) % a) == 0; };
  if (!al(X, 8) || xs[0] % 4 || xs[1] % 4 || xs[2] % 4 || xs[2] <= 0 || !al(W, 4)) return HFTA_EUNSUPPORTED;
  const int64_t x_ext = ((int64_t)(Ci - 1) * xs[2] + L) * 2;
  if (x_ext >= (int64_t)1 << 31) return HFTA_EUNSUPPORTED;
  const CbpLayout lay = cbp_layout(B, Nb, Ci, Co, L);
  if (!workspace || !al(workspace, 256) || ws_bytes < lay.total) return HFTA_EWORKSPACE;
  unsigned char* ws = reinterpret_cast<unsigned char*>(workspace);
  hipStream_t st = as_stream(stream);

  CbpArgs a{};
  a.in = in;
  a.X = (const bf16_raw*)X; a.W = (const bf16_raw*)W; a.bias = (const bf16_raw*)bias; a.Z = (const bf16_raw*)Z;
  a.dV = (const bf16_raw*)dV; a.idx = idx; a.zhit = zhit;
  a.gamma = gamma; a.beta = beta; a.save_mean = save_mean; a.save_invstd = save_invstd;
  a.dX = (bf16_raw*)dX; a.dW = dW; a.dbias = dbias; a.dgamma = dgamma; a.dbeta = dbeta;
  a.xsb = xs[0]; a.xsn = xs[1]; a.xsc = xs[2];
  if (Z) { a.zsb = zs[0]; a.zsn = zs[1]; a.zsc = zs[2]; }
  a.vsb = vs[0]; a.vsn = vs[1]; a.vsc = vs[2]; a.dxsb = dxs[0]; a.dxsn = dxs[1]; a.dxsc = dxs[2];
  a.B = B; a.Nb = Nb; a.Ci = Ci; a.Co = Co; a.L = L; a.act = act; a.slope = act_slope;
  a.chan = (CbpChan*)(ws + lay.chan); a.p0 = (float*)(ws + lay.p0); a.p1 = (float*)(ws + lay.p1);
  a.s = (float*)(ws + lay.s); a.XX = (float*)(ws + lay.XX); a.SX = (float*)(ws + lay.SX);
  a.negG = (bf16_raw*)(ws + lay.negG); a.v = (float*)(ws + lay.v); a.xg = (bf16_raw*)(ws + lay.xg); a.SXpart = (float*)(ws + lay.SXpart);
  a.skey = (uint32_t*)(ws + lay.skey); a.sval = (float*)(ws + lay.sval); a.toff = (int*)(ws + lay.toff);
  a.c_vec = (al(dX, 8) && dxs[0] % 4 == 0 && dxs[1] % 4 == 0 && dxs[2] % 4 == 0) ? 8 : 0;
  a.x_extent = (uint32_t)x_ext; a.g_extent = (uint32_t)((int64_t)Ci * Ci * 2);

  if (saved_moments) {           // XX, SX and T = W XX as the forward operator left them
    a.XX = const_cast<float*>(saved_moments);
    a.SX = a.XX + (size_t)B * Ci * Ci;
    a.Tin = a.SX + (size_t)B * Ci;
    a.SXpart = nullptr;
  }
  hipLaunchKernelGGL(cbp_coef_kernel, dim3((unsigned)Co, (unsigned)B), dim3(64), 0, st, a);
  if (launch_status() != HFTA_OK) return HFTA_ELAUNCH;
  if (!saved_moments) {          // Gram matrix of the layer input: XX[b] = sum_{n,l} x x^T
    const int rc = gram_launch(B, Nb, Ci, L, X, xs, a.XX, (float*)(ws + lay.part), a.x_extent, in, nullptr, nullptr, st);
    if (rc != HFTA_OK) return rc;
  }
  const int T32 = (Ci + 31) / 32;
  hipLaunchKernelGGL(cbp_gram_w_kernel, dim3((unsigned)(T32 * T32), (unsigned)B), dim3(GW_WAVES * 64), 0, st, a);
  if (launch_status() != HFTA_OK) return HFTA_ELAUNCH;
  dim3 grid((unsigned)((L + 127) / 128), 1, (unsigned)(B * Nb));
  int P = 2;
  while (P < Co) P <<= 1;
  hipLaunchKernelGGL(cbp_sort_kernel, dim3((unsigned)Nb, (unsigned)B), dim3(512), 0, st, a, P, (int)grid.x);
  if (Ci <= 64) hipLaunchKernelGGL(cbp_dx_kernel<64>, grid, dim3(GEMM_THREADS), 0, st, a);
  else hipLaunchKernelGGL(cbp_dx_kernel<128>, grid, dim3(GEMM_THREADS), 0, st, a);
  if (launch_status() != HFTA_OK) return HFTA_ELAUNCH;
  if (!saved_moments)
    hipLaunchKernelGGL(cbp_sx_kernel, dim3((unsigned)((Ci + 15) / 16), (unsigned)B), dim3(1024), 0, st, a.SXpart, a.SX, Ci,
                       Nb * (int)grid.x);
  hipLaunchKernelGGL(cbp_dw_kernel, dim3((unsigned)((Co + 7) / 8), (unsigned)B), dim3(1024), 0, st, a);
  return launch_status();
}

size_t hfta_conv1x1_bn_maxpool_saved_floats(int B, int Ci, int Co) {
  if (B <= 0 || Ci <= 0 || Co <= 0) return 0;
  return saved_floats(B, Ci, Co);
}

size_t hfta_conv1x1_bn_maxpool_fwd_workspace_bytes(int B, int Nb, int Ci, int Co, int L, int dtype) {
  if (!cbp_supported(B, Nb, Ci, Co, L, dtype)) return 0;
  return fbp_layout(B, Nb, Ci, Co, L, true).total;
}

static int fbp_run(int B, int Nb, int Ci, int Co, int L, int dtype, const void* X, const int64_t xs[4],
                   const void* W, const void* bias, const float* gamma, const float* beta, float eps,
                   float momentum, float* running_mean, float* running_var, float* save_mean,
                   float* save_invstd, void* V, int32_t* idx, const int64_t vs[3], float* zhit,
                   float* saved_moments, int act, float act_slope, void* workspace, size_t ws_bytes,
                   void* stream, const InNorm& in, void* Xact = nullptr, const int64_t* xas = nullptr) {
  if (B <= 0 || Nb <= 0 || Ci <= 0 || Co <= 0 || L <= 0 || !valid_dtype(dtype) || !X || !xs || !W || !gamma || !beta ||
      !save_mean || !save_invstd || !V || !idx || !vs || !zhit || !(eps >= 0.f) || (Xact && !xas))
    return HFTA_EINVAL;
  if ((running_mean == nullptr) != (running_var == nullptr)) return HFTA_EINVAL;
  // the argmax is taken on sign(gamma) z: needs a non-decreasing activation
  if (!(act == HFTA_ACT_NONE || act == HFTA_ACT_RELU || (act == HFTA_ACT_LEAKY && act_slope >= 0.f))) return HFTA_EUNSUPPORTED;
  if (!cbp_supported(B, Nb, Ci, Co, L, dtype) || xs[3] != 1) return HFTA_EUNSUPPORTED;
  auto al = [](const void* q, size_t a) { return (reinterpret_cast<uintptr_t>(q) % a) == 0; };
  if (!al(X, 8) || xs[0] % 4 || xs[1] % 4 || xs[2] % 4 || xs[2] <= 0 || !al(W, 16)) return HFTA_EUNSUPPORTED;
  const int64_t x_ext = ((int64_t)(Ci - 1) * xs[2] + L) * 2, w_ext = (int64_t)Co * Ci * 2;
  if (x_ext >= (int64_t)1 << 31 || w_ext >= (int64_t)1 << 31) return HFTA_EUNSUPPORTED;
  const int64_t xa_ext = Xact ? ((int64_t)(Ci - 1) * xas[2] + L) * 2 : 0;
  if (Xact && (!al(Xact, 8) || xas[3] != 1 || xas[0] % 4 || xas[1] % 4 || xas[2] % 4 || xas[2] <= 0 || xa_ext >= (int64_t)1 << 31))
    return HFTA_EUNSUPPORTED;
  const FbpLayout lay = fbp_layout(B, Nb, Ci, Co, L, true);
  if (!workspace || !al(workspace, 256) || ws_bytes < lay.total) return HFTA_EWORKSPACE;
  unsigned char* ws = reinterpret_cast<unsigned char*>(workspace);
  hipStream_t st = as_stream(stream);

  FbpArgs a{};
  a.in = in;
  a.X = (const bf16_raw*)X; a.W = (const bf16_raw*)W; a.bias = (const bf16_raw*)bias; a.gamma = gamma; a.beta = beta;
  a.running_mean = running_mean; a.running_var = running_var; a.save_mean = save_mean; a.save_invstd = save_invstd;
  a.V = (bf16_raw*)V; a.idx = idx; a.zhit = zhit;
  a.xsb = xs[0]; a.xsn = xs[1]; a.xsc = xs[2]; a.vsb = vs[0]; a.vsn = vs[1]; a.vsc = vs[2];
  a.B = B; a.Nb = Nb; a.Ci = Ci; a.Co = Co; a.L = L; a.act = act; a.tiles_co = (Co + FBP_RT - 1) / FBP_RT;
  a.slope = act_slope; a.eps = eps; a.momentum = momentum;
  a.XX = saved_moments ? saved_moments : (float*)(ws + lay.moments);
  a.SX = a.XX + (size_t)B * Ci * Ci;
  a.T = a.SX + (size_t)B * Ci;
  a.SXpart = (float*)(ws + lay.SXpart); a.pmax = (float*)(ws + lay.pmax); a.pidx = (int*)(ws + lay.pidx);
  a.x_extent = (uint32_t)x_ext; a.w_extent = (uint32_t)w_ext;

  const int rc = gram_launch(B, Nb, Ci, L, X, xs, a.XX, (float*)(ws + lay.part), a.x_extent, in, Xact, xas, st);
  if (rc != HFTA_OK) return rc;
  if (Xact) {                    // the first kernel wrote the activated input out: the others read that, as it is
    a.in = InNorm{};
    a.X = (const bf16_raw*)Xact; a.xsb = xas[0]; a.xsn = xas[1]; a.xsc = xas[2]; a.x_extent = (uint32_t)xa_ext;
  }
  dim3 grid((unsigned)((L + 127) / 128), 1, (unsigned)(B * Nb));
  if (Ci <= 64) hipLaunchKernelGGL((fbp_main_kernel<64, FBP_RT>), grid, dim3(GEMM_THREADS), 0, st, a);
  else hipLaunchKernelGGL((fbp_main_kernel<128, FBP_RT>), grid, dim3(GEMM_THREADS), 0, st, a);
  if (launch_status() != HFTA_OK) return HFTA_ELAUNCH;
  hipLaunchKernelGGL(cbp_sx_kernel, dim3((unsigned)((Ci + 15) / 16), (unsigned)B), dim3(1024), 0, st, a.SXpart, a.SX, Ci,
                     Nb * (int)grid.x * 2);
  hipLaunchKernelGGL(fbp_stats_kernel, dim3((unsigned)((Co + 7) / 8), (unsigned)B), dim3(128), 0, st, a);
  if (launch_status() != HFTA_OK) return HFTA_ELAUNCH;
  hipLaunchKernelGGL(fbp_finish_kernel, dim3((unsigned)((Co + 255) / 256), (unsigned)Nb, (unsigned)B), dim3(256), 0, st, a,
                     (int)grid.x);
  return launch_status();
}


int hfta_conv1x1_bn_maxpool_fwd(int B, int Nb, int Ci, int Co, int L, int dtype, const void* X, const int64_t xs[4],
                                const void* W, const void* bias, const float* gamma, const float* beta, float eps,
                                float momentum, float* running_mean, float* running_var, float* save_mean,
                                float* save_invstd, void* V, int32_t* idx, const int64_t vs[3], float* zhit,
                                float* saved_moments, int act, float act_slope, void* workspace, size_t ws_bytes,
                                void* stream) {
  return fbp_run(B, Nb, Ci, Co, L, dtype, X, xs, W, bias, gamma, beta, eps, momentum, running_mean, running_var, save_mean,
                 save_invstd, V, idx, vs, zhit, saved_moments, act, act_slope, workspace, ws_bytes, stream, InNorm{});
}

int hfta_conv1x1_bn_maxpool_bwd(int B, int Nb, int Ci, int Co, int L, int dtype, const void* X, const int64_t xs[4],
                                const void* W, const void* bias, const void* Z, const int64_t zs[4], const float* zhit,
                                const float* saved_moments, const void* dV, const int32_t* idx, const int64_t vs[3],
                                const float* gamma, const float* beta, const float* save_mean, const float* save_invstd,
                                void* dX, const int64_t dxs[4], float* dW, float* dbias, float* dgamma, float* dbeta,
                                int act, float act_slope, void* workspace, size_t ws_bytes, void* stream) {
  return cbp_run(B, Nb, Ci, Co, L, dtype, X, xs, W, bias, Z, zs, zhit, saved_moments, dV, idx, vs, gamma, beta, save_mean,
                 save_invstd, dX, dxs, dW, dbias, dgamma, dbeta, act, act_slope, workspace, ws_bytes, stream, InNorm{});
}

// The same operator with X given as the previous block's stored pre-activation and that block's BatchNorm
// constants: every kernel that reads X forms the block's activated output on load.
int hfta_conv1x1_bn_maxpool_prenorm_fwd(int B, int Nb, int Ci, int Co, int L, int dtype, const void* Xpre,
                                        const int64_t xs[4], const float* in_gamma, const float* in_beta,
                                        const float* in_mean, const float* in_invstd, int in_act, float in_slope,
                                        const void* W, const void* bias, const float* gamma, const float* beta, float eps,
                                        float momentum, float* running_mean, float* running_var, float* save_mean,
                                        float* save_invstd, void* V, int32_t* idx, const int64_t vs[3], float* zhit,
                                        float* saved_moments, int act, float act_slope, void* Xact, const int64_t xas[4],
                                        void* workspace, size_t ws_bytes, void* stream) {
  if (!in_gamma || !in_beta || !in_mean || !in_invstd) return HFTA_EINVAL;
  const InNorm in{in_gamma, in_beta, in_mean, in_invstd, in_act, in_slope};
  if (!in_norm_valid(in)) return HFTA_EUNSUPPORTED;
  return fbp_run(B, Nb, Ci, Co, L, dtype, Xpre, xs, W, bias, gamma, beta, eps, momentum, running_mean, running_var, save_mean,
                 save_invstd, V, idx, vs, zhit, saved_moments, act, act_slope, workspace, ws_bytes, stream, in, Xact, xas);
}

int hfta_conv1x1_bn_maxpool_prenorm_bwd(int B, int Nb, int Ci, int Co, int L, int dtype, const void* Xpre,
                                        const int64_t xs[4], const float* in_gamma, const float* in_beta,
                                        const float* in_mean, const float* in_invstd, int in_act, float in_slope,
                                        const void* W, const void* bias, const float* zhit, const float* saved_moments,
                                        const void* dV, const int32_t* idx, const int64_t vs[3], const float* gamma,
                                        const float* beta, const float* save_mean, const float* save_invstd, void* dX,
                                        const int64_t dxs[4], float* dW, float* dbias, float* dgamma, float* dbeta, int act,
                                        float act_slope, void* workspace, size_t ws_bytes, void* stream) {
  if (!in_gamma || !in_beta || !in_mean || !in_invstd) return HFTA_EINVAL;
  const InNorm in{in_gamma, in_beta, in_mean, in_invstd, in_act, in_slope};
  if (!in_norm_valid(in)) return HFTA_EUNSUPPORTED;
  return cbp_run(B, Nb, Ci, Co, L, dtype, Xpre, xs, W, bias, nullptr, nullptr, zhit, saved_moments, dV, idx, vs, gamma, beta,
                 save_mean, save_invstd, dX, dxs, dW, dbias, dgamma, dbeta, act, act_slope, workspace, ws_bytes, stream, in);
}

}  // extern "C"
