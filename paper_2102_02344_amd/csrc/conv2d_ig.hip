// Grouped Conv2d / ConvTranspose2d as an implicit GEMM whose columns run over (sample, output pixel)
// of one model (fusion rules table, rows "Conv2d" and "ConvTranspose2d": one grouped operator with
// G = B; here the model is grid.z and never mixes with the channels).
//
// No column buffer exists in memory.  Per 32-element k-tile a workgroup (128 x 128 output tile, four
// wavefronts of 64 x 64) brings the raw input patch its 128 columns need -- whole image rows, 16-byte
// loads -- into LDS, builds the k-contiguous column tile [128 columns][32 k] from it there (LDS reads
// of single elements, 16-byte writes), and runs the matrix instructions of the batched GEMM core on
// it; the weight tile is an ordinary k-contiguous operand.  Folding the sample index into the columns
// keeps the tiles full for 8x8 and 4x4 images, where a GEMM per sample has 64 or 16 columns.
//
//   forward (and the data gradient of a transposed convolution):
//       Y[o][(n, y, x)] = sum_{(c, ky, kx)} W[o][(c, ky, kx)] X[n][c][s y + ky - p][s x + kx - p]
//   data gradient (and the forward of a transposed convolution), per output-parity class (py, px):
//       dX[c][(n, qy, qx)] = sum_{(o, jy, jx)} Wp[class][c][(o, jy, jx)] dY[n][o][qy + py - 1 + jy][qx + px - 1 + jx]
//     a stride-1 correlation with a 2x2 window and the weights regrouped per class (the taps a class
//     does not see are never multiplied); results land at (2 qy + py, 2 qx + px).
//   weight gradient: conv_ig_dw_kernel below, dW[o][(c, ky, kx)] = sum_{(n, y, x)} dY[n][o][y][x] X[n][c][...].
//
// bf16 only; output grids whose width and height are powers of two; see ig_*_supported.
#include <mutex>
#include <vector>
#include "gemm_pf.h"

namespace hfta {

namespace {

constexpr int IG_MARGIN = 8;            // zero columns left of a patch row (keeps the data 16-byte aligned)

// Workgroups are dispatched to the 8 XCDs (each with its own L2) round-robin by their linear id.
// The kernels are launched on a 1-D grid and turn the id into a logical (x, y, z) block such that
// consecutive logical blocks -- the column tiles that share a weight slab, then the row tiles that
// share a patch -- run on the SAME XCD at about the same time, instead of each XCD fetching every
// slab for itself (the 8x8 layer's forward went from a 32 % L2 hit rate to sharing).
struct IgGrid { int gx, gy, gz; };
__device__ __forceinline__ void ig_block(const IgGrid& g, int& bx, int& by, int& bz) {
  const int total = g.gx * g.gy * g.gz, id = blockIdx.x;
  int logical = id;
  if (total % 8 == 0) logical = (id & 7) * (total >> 3) + (id >> 3);
  bx = logical % g.gx;
  const int r = logical / g.gx;
  by = r % g.gy;
  bz = r / g.gy;
}

struct IgClass {
  int oy, ox;                           // patch row / column of tap (0, 0) for output (0, 0), before the margin
  int out_y0, out_x0;                   // where the class's outputs start in the output image
  int64_t a_off;                        // offset of the class's weights inside a model's block
};

struct IgArgs {
  const bf16_raw* X; const bf16_raw* A; bf16_raw* Out; const bf16_raw* bias;
  int64_t x_img, x_model;               // element strides of the view operand: sample, model (channel stride = H * W)
  int64_t a_model;                      // weights: [b][..][m][K], K contiguous
  int64_t o_img, o_model, o_m;          // output element strides: sample, model, GEMM row (channel)
  int Nb, Cx, H, W;                     // view operand: channels per model, image size
  int M, K, N;                          // GEMM sizes per model: rows, reduction, columns = Nb * Ho * Wo
  int Ho, Wo, lgWo, lgP;                // logical output grid per sample (powers of two)
  int OW, oys, oxs;                     // output image width in memory, output step per grid step
  int tap_step;                         // 1 (patch elements between the taps of a window row; see the column-tile build)
  int NI, TR, PR, PW, SP;               // samples per tile, grid rows per tile and sample, patch rows, row pitch, sample pitch (elements)
  int nchunk, chunk_el;                 // 16- or 8-byte pieces of patch rows per k-tile, elements per piece
  uint32_t x_bytes, a_bytes;            // extent of one model's slice of the view operand / of its weights
  IgGrid grid;                          // logical grid: x = tiles, y = class / k split, z = model
  int ksplit, kt_per_split;             // k range split over the grid's y (> 1: fp32 partial slices instead of Out)
  float* part; int64_t part_split;      // partial slices [split][same indexing as Out]
  int tiles_n, act;
  float slope;
  IgClass cls[4];
};

constexpr int IG_EPI_PITCH = 128 * 2 + 16;   // bytes per staged output row (64 rows at a time)

// accumulators of a wavefront (64 rows x 32 FN columns from column col0) -> staging tile [64][128]
template <int FN>
__device__ __forceinline__ void ig_stage64(f32x16_t (&acc)[2][FN], unsigned char* lds, int M, int mrow0, const bf16_raw* bias,
                                           int act, float slope, int lane, int col0) {
  const int ml = lane & 31, nq = (lane >> 5) * 4;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int rl = i * 32 + ml, m = mrow0 + rl;
    const float bm = (bias && m < M) ? bf16_to_f32(bias[m]) : 0.f;
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int nl = col0 + j * 32 + 8 * q + nq;
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = cheap_act(acc[i][j][4 * q + e] + bm, act, slope);
        *reinterpret_cast<uint2*>(lds + rl * IG_EPI_PITCH + nl * 2) = make_uint2(pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]));
      }
  }
}

// Four wavefronts; each computes 64 rows x 64 columns of a TM = 128 row tile, or 64 rows x 32 columns
// of a TM = 64 row tile (layers with at most 64 output rows).
// PAIR (data gradient): the tile's 128 columns are 64 pixels of the parity class px = 0 followed by
// the same 64 pixels of px = 1 (the grid's y = py); the weight tile holds both classes' rows, a
// wavefront works on the class its columns belong to, and the epilogue interleaves the two classes
// into whole 16-byte pieces of the output rows.
//
// Weight tile, column tile and patch are double-buffered and there is one barrier per k-tile.  In
// iteration kt a thread
//   issues the LDS reads that gather its part of column tile kt+1 from patch kt+1,
//   parks the weights of k-tile kt+1 and the patch of k-tile kt+2 (registers -> LDS),
//   issues the loads of the weights of kt+2 and of the patch of kt+3,
//   runs the matrix instructions on k-tile kt (the gather's reads return meanwhile),
//   writes its part of column tile kt+1, and meets the others at the barrier.
// Every load is a raw buffer load whose offset is inside the model's slice or the fixed out-of-range
// value (the hardware returns zeros): no load sits under control flow, so the compiler's wait
// counters let the loads of later k-tiles stay in flight across iterations.  Nothing in the loop
// depends on the k-tile index: loads past the last k-tile are out of range, and what is parked or
// built from them lands in buffers nobody reads any more.
template <int KH, int KW, int S, bool PAIR, int TM, bool CH8>
__global__ __launch_bounds__(256) void conv_ig_fwd_kernel(IgArgs p) {
  static_assert(TM == 128 || TM == 64, "row tiles of 128 or 64");
  constexpr int TK = KH * KW, CPT = 32 / TK;             // taps per channel, channels per k-tile
  constexpr int NT = 256;
  constexpr int AROWS = TM;                              // rows of the weight tile (PAIR: none, see below)
  constexpr int NA = AROWS * 4 / NT;                     // 16-byte weight pieces per thread
  // Weights as matrix-instruction fragments straight from memory: only where they are stored in
  // fragment order (PAIR).  From the forward's row-major weights a wavefront's fragment load touches
  // 32 rows of 64 bytes, and the kernel measured 1.3-1.5x slower than with the LDS tile.
  constexpr bool AFRAG = PAIR;
  constexpr int A_BYTES = AFRAG ? 0 : AROWS * GEMM_PITCH;
  constexpr int KPT = 16;                                // k per thread of the column tile
  constexpr int COLS = PAIR ? 64 : 128;                  // pixel columns per tile
  constexpr int FN = TM == 128 ? 2 : 1;                  // 32-column blocks per wavefront
  constexpr int CH = CH8 ? 8 : 4;                        // elements per patch piece
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  auto As = [&](int buf) { return smem + buf * A_BYTES; };
  auto Cb = [&](int buf) { return smem + 2 * A_BYTES + buf * GEMM_TILE_BYTES; };
  const int chan_el = p.NI * p.SP;
  const int patch_el = CPT * chan_el;
  auto Pt = [&](int buf) { return reinterpret_cast<bf16_raw*>(smem + 2 * A_BYTES + 2 * GEMM_TILE_BYTES) + buf * patch_el; };
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  int bx, by, b;
  ig_block(p.grid, bx, by, b);
  const int tile_m = bx / p.tiles_n, tile_n = bx % p.tiles_n;
  const int m0 = tile_m * TM, n0 = tile_n * COLS;
  // grid y: PAIR py + 2 * (k split), else the k split
  const int py2 = PAIR ? 2 * (by & 1) : 0;
  const int split = PAIR ? by >> 1 : by;
  const IgClass cl0 = p.cls[py2];
  const int P = 1 << p.lgP;
  const int img0 = n0 >> p.lgP;                          // first sample of the tile
  const int y0 = (n0 & (P - 1)) >> p.lgWo;               // first grid row (tiles inside one sample)
  const int HW = p.H * p.W;
  const int rmin = cl0.oy;                               // first patch row's image row for grid row 0 (the same for both classes of a pair)
  const int row_base = y0 * S + rmin;
  const int ktiles = (p.K + 31) / 32;
  const int kt0 = split * p.kt_per_split, kt1 = min(ktiles, kt0 + p.kt_per_split);

  // position of the wavefront's block of the tile
  const int wm = TM == 128 ? wave >> 1 : 0;
  const int col0 = TM == 128 ? (wave & 1) * 64 : wave * 32;
  const int a_row0 = wm * 64;

  const __amdgpu_buffer_rsrc_t rx = pf_rsrc(p.X + (int64_t)b * p.x_model, p.x_bytes);
  const __amdgpu_buffer_rsrc_t rw = pf_rsrc(p.A + (int64_t)b * p.a_model, p.a_bytes);
  // ---- patch pieces: fixed over the k-loop up to the channel, which advances CPT per k-tile.
  // Pieces outside the image or past the batch load zeros; threads without a piece park nothing.
  uint32_t pxo[2];                                        // byte offset of the piece at its channel of k-tile 0, or PF_OOB
  int pl[2], pcl[2];                                      // LDS element offset, channel inside the k-tile
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int q = t + NT * i;
    pxo[i] = PF_OOB; pl[i] = -1; pcl[i] = 0;
    if (q < p.nchunk) {
      const int cpr = p.W / CH;                           // pieces per image row
      const int xc = q % cpr;
      int r = q / cpr;
      const int pr = r % p.PR; r /= p.PR;
      const int il = r % p.NI, c_l = r / p.NI;
      const int iy = row_base + pr, img = img0 + il;
      pcl[i] = c_l;
      pl[i] = (c_l * p.NI + il) * p.SP + pr * p.PW + IG_MARGIN + xc * CH;
      if (iy >= 0 && iy < p.H && img < p.Nb)
        pxo[i] = (uint32_t)(((int64_t)img * p.x_img + (int64_t)c_l * HW + (int64_t)iy * p.W + xc * CH) * 2);
    }
  }
  const uint32_t px_step = (uint32_t)(CPT * HW * 2);
  // ---- column of the tile being built: KPT consecutive k of column t % 128
  const int bcol = t & 127, bhalf = t >> 7;
  int boff;                                               // patch element of tap (0, 0), first channel of this half
  {
    const IgClass cl = PAIR ? p.cls[py2 + (bcol >> 6)] : cl0;
    const int n = n0 + (PAIR ? (bcol & 63) : bcol);
    const int il = (n >> p.lgP) - img0;
    const int y = (n & (P - 1)) >> p.lgWo, x = n & (p.Wo - 1);
    boff = il * p.SP + ((y - y0) * S + (cl.oy - rmin)) * p.PW + x * S + cl.ox + IG_MARGIN;
    boff += ((bhalf * KPT) / TK) * chan_el;
  }
  // ---- weights.  Forward: rows ra + 64 h of the weight tile, 8 k at ga, through LDS.
  // PAIR: the regrouped weights are stored in the order the matrix instructions consume them
  // ([class][row tile][k-tile][32-row block][k-step][lane][8 k], ig_pack_class_w_kernel), so a
  // wavefront loads its own fragments -- 64 rows of its class, four 16-byte loads per lane, each a
  // contiguous 1 KB per wavefront -- straight into registers: no LDS write, no LDS fragment read.
  const int ga = t & 3, ra = t >> 2;
  uint32_t wo[NA];
  uint32_t fo = 0;                                        // PAIR: byte offset of this lane's first fragment of k-tile 0
  if constexpr (PAIR) {
    const int64_t tile_el = (int64_t)ktiles * TM * 32;    // one (class, row tile): every k-tile's TM x 32 block
    fo = (uint32_t)((p.cls[py2 + (col0 >> 6)].a_off + (int64_t)tile_m * tile_el) * 2) + (uint32_t)((wm * 4 * 64 + lane) * 16);
#pragma unroll
    for (int h = 0; h < NA; ++h) wo[h] = PF_OOB;
  } else {
#pragma unroll
    for (int h = 0; h < NA; ++h) {
      const int r = ra + (NT / 4) * h;
      const int m = m0 + r;
      wo[h] = m < p.M ? (uint32_t)((cl0.a_off + (int64_t)m * p.K + ga * 8) * 2) : PF_OOB;
    }
  }
  pf_u32x4 qa[NA], qp[2];
  pf_u32x4 fa_cur[2][2], fa_nxt[2][2];                    // PAIR: fragments [32-row block][k-step] of this and the next k-tile
  auto issue_a = [&](int kt) {
    if constexpr (PAIR) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
          fa_nxt[i][s2] = __builtin_amdgcn_raw_buffer_load_b128(
              rw, (int)(kt < ktiles ? fo + (uint32_t)kt * (uint32_t)(TM * 64) + (uint32_t)((i * 2 + s2) * 1024) : PF_OOB), 0, 0);
    } else {
      const bool in_k = kt * 32 + ga * 8 + 8 <= p.K;
#pragma unroll
      for (int h = 0; h < NA; ++h)
        qa[h] = __builtin_amdgcn_raw_buffer_load_b128(rw, (int)((in_k && wo[h] != PF_OOB) ? wo[h] + (uint32_t)kt * 64u : PF_OOB), 0, 0);
    }
  };
  auto issue_p = [&](int kt) {
    const int c0 = kt * CPT;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const uint32_t off = (c0 + pcl[i] < p.Cx && pxo[i] != PF_OOB) ? pxo[i] + (uint32_t)kt * px_step : PF_OOB;
      if constexpr (CH8) {
        qp[i] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)off, 0, 0);
      } else {
        const pf_u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rx, (int)off, 0, 0);
        qp[i].x = v.x; qp[i].y = v.y;
      }
    }
  };
  auto park_a = [&](int buf) {
    if constexpr (AFRAG) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) fa_cur[i][s2] = fa_nxt[i][s2];
    } else {
#pragma unroll
      for (int h = 0; h < NA; ++h) *reinterpret_cast<pf_u32x4*>(As(buf) + (ra + (NT / 4) * h) * GEMM_PITCH + ga * 16) = qa[h];
    }
  };
  auto park_p = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      if (pl[i] >= 0) {                                   // a store under a branch; the loads stay branch-free
        if constexpr (CH8) *reinterpret_cast<pf_u32x4*>(Pt(buf) + pl[i]) = qp[i];
        else *reinterpret_cast<uint2*>(Pt(buf) + pl[i]) = make_uint2(qp[i].x, qp[i].y);
      }
    }
  };
  // column tile from the patch: this thread's 16 consecutive k (the taps of 16 / TK channels) of its column
  // (p.tap_step is 1, passed at run time: with a constant step the compiler merges the KW adjacent
  // elements of a window row into one 2-byte-aligned wide LDS read, which the hardware executes
  // several times slower than the separate 2-byte reads.)
  uint32_t bv[KPT];
  auto build_read = [&](int buf) {
    const bf16_raw* src = Pt(buf) + boff;
#pragma unroll
    for (int kk = 0; kk < KPT; ++kk) {
      const int c_l = kk / TK, tap = kk % TK, ty = tap / KW, tx = tap % KW;
      bv[kk] = src[c_l * chan_el + ty * p.PW + tx * p.tap_step];
    }
  };
  auto build_write = [&](int buf) {
    uint32_t w[KPT / 2];
#pragma unroll
    for (int e = 0; e < KPT / 2; ++e) w[e] = bv[2 * e] | (bv[2 * e + 1] << 16);
    unsigned char* dst = Cb(buf) + bcol * GEMM_PITCH + bhalf * KPT * 2;
    *reinterpret_cast<uint4*>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
    *reinterpret_cast<uint4*>(dst + 16) = make_uint4(w[4], w[5], w[6], w[7]);
  };
  const int r = lane & 31, gsel = lane >> 5;
  f32x16_t acc[2][FN];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  auto mma = [&](int buf) {
    const unsigned char* Ab = As(buf) + (a_row0 + r) * GEMM_PITCH + gsel * 16;
    const unsigned char* Bb = Cb(buf) + (col0 + r) * GEMM_PITCH + gsel * 16;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      bf16x8_t a[2], bq[FN];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        if constexpr (AFRAG) a[i] = __builtin_bit_cast(bf16x8_t, fa_cur[i][s]);
        else a[i] = *reinterpret_cast<const bf16x8_t*>(Ab + i * 32 * GEMM_PITCH + s * 32);
      }
#pragma unroll
      for (int j = 0; j < FN; ++j) bq[j] = *reinterpret_cast<const bf16x8_t*>(Bb + j * 32 * GEMM_PITCH + s * 32);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bq[j], a[i], acc[i][j], 0, 0, 0);
    }
  };

  issue_a(kt0);
  issue_p(kt0);
  // zero both patch buffers once: the margins stay zero
  for (int i = t; i < 2 * patch_el / 2; i += NT) reinterpret_cast<uint32_t*>(Pt(0))[i] = 0u;
  __syncthreads();
  park_a(0);
  park_p(0);
  issue_a(kt0 + 1);
  issue_p(kt0 + 1);
  __syncthreads();
  build_read(0);
  park_p(1);
  issue_p(kt0 + 2);
  build_write(0);
  __syncthreads();
  for (int kt = kt0; kt < kt1; ++kt) {
    const int buf = (kt - kt0) & 1;
    build_read(buf ^ 1);                                  // gather of column tile kt + 1 (patch kt + 1 was parked an iteration ago)
    if constexpr (!AFRAG) { park_a(buf ^ 1); issue_a(kt + 2); }  // weights kt + 1 -> LDS, kt + 2 requested
    park_p(buf);                                          // patch kt + 2
    issue_p(kt + 3);
    mma(buf);
    if constexpr (AFRAG) { park_a(0); issue_a(kt + 2); }  // fragments kt + 1 become current, kt + 2 requested
    build_write(buf ^ 1);
    __syncthreads();
  }

  if (p.ksplit > 1) {
    // ---- split k: this workgroup's fp32 partial tile goes to its slice, indexed like the output;
    // bias, activation and the conversion happen in ig_split_finish_kernel
    float* lds_f = reinterpret_cast<float*>(smem);
    float* ob = p.part + (int64_t)split * p.part_split + (int64_t)b * p.o_model;
    constexpr int FP = 132;                               // floats per staged row
#pragma unroll 1
    for (int pass = 0; pass < TM / 64; ++pass) {
      const int mp = m0 + 64 * pass;
      if (wm == pass) {
        const int ml = lane & 31, nq = (lane >> 5) * 4;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q)
              *reinterpret_cast<float4*>(lds_f + (i * 32 + ml) * FP + col0 + j * 32 + 8 * q + nq) =
                  make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
      }
      __syncthreads();
#pragma unroll
      for (int id = t; id < 64 * 32; id += NT) {
        const int rr = id >> 5, pc = id & 31;
        const int m = mp + rr;
        if (!PAIR) {
          const int n = n0 + pc * 4;
          if (m >= p.M || n >= p.N) continue;
          const int img = n >> p.lgP, pix = n & (P - 1);
          *reinterpret_cast<float4*>(ob + (int64_t)img * p.o_img + (int64_t)m * p.o_m + pix) =
              *reinterpret_cast<const float4*>(lds_f + rr * FP + pc * 4);
        } else {
          const int n = n0 + pc * 2;                      // 2 pixels x 2 classes = 4 consecutive output elements
          if (m >= p.M || n >= p.N) continue;
          const int img = n >> p.lgP, y = (n & (P - 1)) >> p.lgWo, x = n & (p.Wo - 1);
          const float2 e = *reinterpret_cast<const float2*>(lds_f + rr * FP + pc * 2);
          const float2 o = *reinterpret_cast<const float2*>(lds_f + rr * FP + 64 + pc * 2);
          *reinterpret_cast<float4*>(ob + (int64_t)img * p.o_img + (int64_t)m * p.o_m + (int64_t)(y * p.oys + cl0.out_y0) * p.OW + x * p.oxs) =
              make_float4(e.x, o.x, e.y, o.y);
        }
      }
      if (pass + 1 < TM / 64) __syncthreads();
    }
    return;
  }

  // ---- epilogue: bias + activation, 64 rows at a time through an LDS staging tile, then whole
  // 16-byte pieces of the output rows
  unsigned char* lds = smem;
  const bf16_raw* bias = p.bias ? p.bias + (int64_t)b * p.M : nullptr;
  bf16_raw* ob = p.Out + (int64_t)b * p.o_model;
#pragma unroll 1
  for (int pass = 0; pass < TM / 64; ++pass) {
    const int mp = m0 + 64 * pass;
    if (wm == pass) ig_stage64<FN>(acc, lds, p.M, mp, bias, p.act, p.slope, lane, col0);
    __syncthreads();
    if (!PAIR) {
      // 8 consecutive columns = 8 consecutive pixels of one sample: one 16-byte piece
#pragma unroll
      for (int id = t; id < 64 * 16; id += NT) {
        const int rr = id >> 4, pc = id & 15;
        const int m = mp + rr, n = n0 + pc * 8;
        if (m >= p.M || n >= p.N) continue;
        const int img = n >> p.lgP, pix = n & (P - 1);
        *reinterpret_cast<uint4*>(ob + (int64_t)img * p.o_img + (int64_t)m * p.o_m + pix) =
            *reinterpret_cast<const uint4*>(lds + rr * IG_EPI_PITCH + pc * 16);
      }
    } else {
      // 4 consecutive pixels x 2 classes = 8 consecutive output elements
#pragma unroll
      for (int id = t; id < 64 * 16; id += NT) {
        const int rr = id >> 4, pc = id & 15;
        const int m = mp + rr, n = n0 + pc * 4;
        if (m >= p.M || n >= p.N) continue;
        const int img = n >> p.lgP, y = (n & (P - 1)) >> p.lgWo, x = n & (p.Wo - 1);
        const uint2 e = *reinterpret_cast<const uint2*>(lds + rr * IG_EPI_PITCH + pc * 8);          // px = 0
        const uint2 o = *reinterpret_cast<const uint2*>(lds + rr * IG_EPI_PITCH + 128 + pc * 8);    // px = 1
        const uint4 v = make_uint4((e.x & 0xffffu) | (o.x << 16), (e.x >> 16) | (o.x & 0xffff0000u),
                                   (e.y & 0xffffu) | (o.y << 16), (e.y >> 16) | (o.y & 0xffff0000u));
        *reinterpret_cast<uint4*>(ob + (int64_t)img * p.o_img + (int64_t)m * p.o_m + (int64_t)(y * p.oys + cl0.out_y0) * p.OW + x * p.oxs) = v;
      }
    }
    if (pass + 1 < TM / 64) __syncthreads();
  }
}

int ilog2(int v) { int l = 0; while ((1 << l) < v) ++l; return l; }
bool pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

// patch geometry shared by the host-side checks and the launch
// Patch geometry.  The gather reads 2-byte elements: the LDS serves 32 lanes per clock from 32
// banks of 4 bytes (lanes on the same word are served together; measured: 2 clocks for a
// conflict-free 64-lane read, 2n for an n-way conflict), and the 32 lanes of a half wavefront are 32
// consecutive columns, i.e. several image rows (and samples) of small images.  With the natural row
// pitch the four rows of an 8x8 layer that a half wavefront touches fall on the same banks (4-way,
// 8 clocks per read).  Row pitch and sample pitch are therefore searched (multiples of 8 elements,
// so that 16-byte pieces stay aligned) for the fewest conflicts over all taps of a window row.
// (The search is a pure function of the layer geometry; its results are memoised, a call costs the
// host ~100 us otherwise.)
struct IgPitchKey { int KW, S, Ho, Wo, W, cols, pair, PW, SP; };
std::mutex ig_pitch_mutex;
std::vector<IgPitchKey> ig_pitch_cache;

bool ig_geometry(IgArgs& a, int KW, int KH, int S, int Ho, int Wo, int W, int cols, bool pair) {
  a.Ho = Ho; a.Wo = Wo; a.lgWo = ilog2(Wo); a.lgP = ilog2(Ho * Wo);
  const int P = Ho * Wo;
  if (P >= cols) { a.NI = 1; a.TR = cols / Wo; } else { a.NI = cols / P; a.TR = Ho; }
  a.PR = (a.TR - 1) * S + KH;
  a.chunk_el = W % 8 == 0 ? 8 : 4;
  const int pw0 = W % 8 == 0 ? W + 16 : W + 12;
  {
    std::lock_guard<std::mutex> lock(ig_pitch_mutex);
    for (const IgPitchKey& k : ig_pitch_cache)
      if (k.KW == KW && k.S == S && k.Ho == Ho && k.Wo == Wo && k.W == W && k.cols == cols && k.pair == (int)pair) {
        a.PW = k.PW; a.SP = k.SP;
        return true;
      }
  }
  const int floor_cost = (pair ? 2 : 1) * KW * (cols / 32);   // one pass per half wavefront and tap
  int64_t best = -1;
  for (int i = 0; i < 6 && best / (1 << 20) != floor_cost; ++i)
    for (int j = 0; j < 8 && best / (1 << 20) != floor_cost; ++j) {
      const int pw = pw0 + 8 * i, sp = a.PR * pw + 8 * j;
      int cost = 0;
      for (int cls = 0; cls < (pair ? 2 : 1); ++cls)
        for (int tx = 0; tx < KW; ++tx)
          for (int h = 0; h < cols; h += 32) {            // one half wavefront's columns
            int words[32], nw = 0, per_bank[32] = {0}, worst = 0;
            for (int l = 0; l < 32; ++l) {
              const int n = h + l, il = n >> a.lgP, y = (n & (P - 1)) >> a.lgWo, x = n & (Wo - 1);
              const int word = (il * sp + y * S * pw + x * S + (pair ? cls - 1 : -1) + IG_MARGIN + tx) >> 1;
              bool seen = false;
              for (int q = 0; q < nw; ++q) seen = seen || words[q] == word;
              if (!seen) { words[nw++] = word; worst = ++per_bank[word & 31] > worst ? per_bank[word & 31] : worst; }
            }
            cost += worst;
          }
      const int64_t key = (int64_t)cost * (1 << 20) + (int64_t)a.NI * sp;   // fewest conflicts first, then the smallest patch
      if (best < 0 || key < best) { best = key; a.PW = pw; a.SP = sp; }
    }
  std::lock_guard<std::mutex> lock(ig_pitch_mutex);
  if (ig_pitch_cache.size() < 256) ig_pitch_cache.push_back(IgPitchKey{KW, S, Ho, Wo, W, cols, (int)pair, a.PW, a.SP});
  return true;
}

// byte extents of one model's slices (buffer-load range checks); false when they do not fit 31 bits
bool ig_extents(IgArgs& a) {
  const int64_t xb = ((int64_t)(a.Nb - 1) * a.x_img + (int64_t)a.Cx * a.H * a.W) * 2, ab = a.a_model * 2;
  if (xb >= ((int64_t)1 << 31) || ab >= ((int64_t)1 << 31)) return false;
  a.x_bytes = (uint32_t)xb; a.a_bytes = (uint32_t)ab;
  return true;
}

size_t ig_lds_bytes(const IgArgs& a, int cpt, int a_rows) {
  const size_t k_loop = 2 * (size_t)a_rows * GEMM_PITCH + 2 * GEMM_TILE_BYTES + 2 * (size_t)cpt * a.NI * a.SP * 2;
  const size_t staging = a.ksplit > 1 ? 64 * (size_t)132 * 4 : 64 * (size_t)IG_EPI_PITCH;
  return k_loop > staging ? k_loop : staging;
}

// Weights regrouped per output-parity class for the data gradient of a 4x4 / stride 2 / pad 1
// convolution, Wc[class = 2 py + px][c][k = (o, jy, jx)] = W[o][c][ry + 2 (1 - jy)][rx + 2 (1 - jx)] with
// ry = (py + 1) % 2 (the two taps per axis that reach pixels of that parity, in the order in which
// the gradient rows / columns qy + py - 1 + jy they multiply ascend), and stored in the order the
// matrix instructions consume them:
//   Wp[b][class][row tile][k-tile][32-row block][k-step (16 k)][lane][8 k],
//   lane = 32 (k half) + row inside the block; rows past Ci and k past 4 Co are zeros.
// One thread per 16-byte fragment piece: 8 k = the class's 2x2 taps of two output channels of one
// input channel, read as two 32-byte windows; consecutive lanes read consecutive channels and
// write consecutive pieces.
__global__ __launch_bounds__(256) void ig_pack_class_w_kernel(const bf16_raw* __restrict__ Wt, bf16_raw* __restrict__ Wp, int Ci,
                                                              int Co, int tm, int tiles_m, int ktiles, int64_t count) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  const int lane = (int)(i & 63), s2 = (int)((i >> 6) & 1);
  int64_t r = i >> 7;
  const int rbs = tm / 32;
  const int rb = (int)(r % rbs); r /= rbs;
  const int kt = (int)(r % ktiles); r /= ktiles;
  const int tile_m = (int)(r % tiles_m); r /= tiles_m;
  const int cls = (int)(r & 3);
  const int64_t b = r >> 2;
  const int c = tile_m * tm + rb * 32 + (lane & 31);
  const int o0 = (kt * 32 + s2 * 16 + (lane >> 5) * 8) >> 2;       // two output channels: o0, o0 + 1
  const int py = cls >> 1, px = cls & 1;
  const int ry = (py + 1) & 1, rx = (px + 1) & 1;
  uint32_t out[4] = {0u, 0u, 0u, 0u};
  if (c < Ci) {
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      if (o0 + q < Co) {
        const uint4* src = reinterpret_cast<const uint4*>(Wt + ((b * Co + o0 + q) * Ci + c) * 16);
        const uint4 lo = src[0], hi = src[1];              // rows ky = 0, 1 | 2, 3; two taps per 32-bit word
        const uint32_t w[4][2] = {{lo.x, lo.y}, {lo.z, lo.w}, {hi.x, hi.y}, {hi.z, hi.w}};
        auto tap = [&](int ky, int kx) { return (w[ky][kx >> 1] >> (16 * (kx & 1))) & 0xffffu; };
        out[2 * q] = tap(ry + 2, rx + 2) | (tap(ry + 2, rx) << 16);      // (jy, jx) = (0, 0), (0, 1)
        out[2 * q + 1] = tap(ry, rx + 2) | (tap(ry, rx) << 16);          // (1, 0), (1, 1)
      }
    }
  }
  *reinterpret_cast<uint4*>(Wp + i * 8) = make_uint4(out[0], out[1], out[2], out[3]);
}


// ---- weight gradient ---------------------------------------------------------------------------
//   dW[o][j = (c, ky, kx)] = sum over k = (n, y, x) of dY[n][o][y][x] X[n][c][2 y + ky - 1][2 x + kx - 1]
// Rows are output channels (dY is k-contiguous inside a sample), columns the 128 taps of 8 input
// channels, and a k-tile is 32 consecutive output pixels (of one sample, or of two 4x4 samples).
// The column tile [128 j][32 k] is built from the patch of the 8 channels' input rows those pixels
// touch.  The grid's y splits the k range; partial sums go to fp32 slices reduced afterwards.
struct IgDwArgs {
  const bf16_raw* X; const bf16_raw* dY; float* Out;
  int64_t x_img, x_model, y_img, y_model;                // element strides: sample, model
  int64_t o_model, o_split;                              // output strides: model, k split
  int Nb, Ci, Co, H, W, Ho, Wo, lgWo, lgP;
  int NI, PR, PW, SP, nchunk;                            // samples per k-tile, patch rows, row pitch, sample pitch (elements)
  int tiles_n, kt_total, kt_per_split;
  IgGrid grid;                                           // logical grid: x = tiles, y = k split, z = model
  uint32_t x_bytes, y_bytes;                             // extents of one model's slices of X and dY
};

__global__ __launch_bounds__(256) void conv_ig_dw_kernel(IgDwArgs p) {
  constexpr int NT = 256;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  auto As = [&](int buf) { return smem + buf * GEMM_TILE_BYTES; };
  auto Cb = [&](int buf) { return smem + 2 * GEMM_TILE_BYTES + buf * GEMM_TILE_BYTES; };
  bf16_raw* const Pt = reinterpret_cast<bf16_raw*>(smem + 4 * GEMM_TILE_BYTES);
  const int chan_el = p.NI * p.SP, patch_el = 8 * chan_el;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  int bx, by, b;
  ig_block(p.grid, bx, by, b);
  const int tile_m = bx / p.tiles_n, tile_n = bx % p.tiles_n;
  const int m0 = tile_m * 128, c0 = tile_n * 8;
  const int P = 1 << p.lgP, HW = p.H * p.W;
  const int kt_begin = by * p.kt_per_split;
  const int kt_end = min(p.kt_total, kt_begin + p.kt_per_split);

  for (int i = t; i < patch_el / 2; i += NT) reinterpret_cast<uint32_t*>(Pt)[i] = 0u;   // margins stay zero

  // Raw buffer loads, in range or at the fixed out-of-range offset (zeros): no load under control flow.
  const __amdgpu_buffer_rsrc_t rx = pf_rsrc(p.X + (int64_t)b * p.x_model, p.x_bytes);
  const __amdgpu_buffer_rsrc_t ry = pf_rsrc(p.dY + (int64_t)b * p.y_model, p.y_bytes);
  // this thread's patch piece: channel, sample, patch row and position in the row are fixed; the image row moves with the k-tile
  int p_row = 0, p_il = 0, p_lds = -1;
  uint32_t p_off = PF_OOB;                                // byte offset at sample 0, image row 0
  if (t < p.nchunk) {
    const int cpr = p.W / 8;
    const int xc = t % cpr;
    int r = t / cpr;
    p_row = r % p.PR; r /= p.PR;
    p_il = r % p.NI;
    const int c_l = r / p.NI;
    p_lds = (c_l * p.NI + p_il) * p.SP + p_row * p.PW + IG_MARGIN + xc * 8;
    if (c0 + c_l < p.Ci) p_off = (uint32_t)(((int64_t)(c0 + c_l) * HW + xc * 8) * 2);
  }
  // this thread's part of the column tile: row j = t % 128, 16 consecutive k (pixels) as four groups of 4 in a row
  const int bj = t & 127, bhalf = t >> 7;
  int boff[4];
  {
    const int c_l = bj >> 4, ky = (bj >> 2) & 3, kx = bj & 3;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int kl = bhalf * 16 + 4 * g;
      const int il = kl >> p.lgP, y_l = (kl & (P - 1)) >> p.lgWo, x = kl & (p.Wo - 1);
      boff[g] = (c_l * p.NI + il) * p.SP + (2 * y_l + ky) * p.PW + 2 * x + kx - 1 + IG_MARGIN;
    }
  }
  const int ga = t & 3, ra = t >> 2;
  uint32_t a_off[2];                                      // byte offset of the row's pixel 0 in sample 0
#pragma unroll
  for (int h = 0; h < 2; ++h) a_off[h] = m0 + ra + 64 * h < p.Co ? (uint32_t)((int64_t)(m0 + ra + 64 * h) * P * 2) : PF_OOB;
  pf_u32x4 qa[2], qp;
  auto issue = [&](int kt) {
    const int kk = kt * 32 + ga * 8;                      // global pixel index of this 16-byte piece
    const int n = kk >> p.lgP, pix = kk & (P - 1);
    const uint32_t ab = (uint32_t)n * (uint32_t)(p.y_img * 2) + (uint32_t)pix * 2u;
#pragma unroll
    for (int h = 0; h < 2; ++h)
      qa[h] = __builtin_amdgcn_raw_buffer_load_b128(ry, (int)((n < p.Nb && a_off[h] != PF_OOB) ? a_off[h] + ab : PF_OOB), 0, 0);
    const int kk0 = kt * 32;
    const int img = (kk0 >> p.lgP) + p_il;
    const int iy = 2 * ((kk0 & (P - 1)) >> p.lgWo) - 1 + p_row;
    const bool ok = p_off != PF_OOB && img < p.Nb && iy >= 0 && iy < p.H;
    qp = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)(ok ? p_off + (uint32_t)img * (uint32_t)(p.x_img * 2) + (uint32_t)(iy * p.W * 2) : PF_OOB), 0, 0);
  };
  auto park = [&](int buf) {
#pragma unroll
    for (int h = 0; h < 2; ++h) *reinterpret_cast<pf_u32x4*>(As(buf) + (ra + 64 * h) * GEMM_PITCH + ga * 16) = qa[h];
    if (p_lds >= 0) *reinterpret_cast<pf_u32x4*>(Pt + p_lds) = qp;
  };
  auto build = [&](int buf) {
    uint32_t w[8];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const bf16_raw* src = Pt + boff[g];
      const uint32_t v0 = src[0], v1 = src[2], v2 = src[4], v3 = src[6];
      w[2 * g] = v0 | (v1 << 16);
      w[2 * g + 1] = v2 | (v3 << 16);
    }
    unsigned char* dst = Cb(buf) + bj * GEMM_PITCH + bhalf * 32;
    *reinterpret_cast<uint4*>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
    *reinterpret_cast<uint4*>(dst + 16) = make_uint4(w[4], w[5], w[6], w[7]);
  };

  f32x16_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // nothing below depends on the k-tile index: tiles past the end of the split are loaded (or read as
  // zeros past the batch) and parked where nobody reads them any more
  issue(kt_begin);
  __syncthreads();
  park(0);
  issue(kt_begin + 1);
  __syncthreads();
  build(0);
  __syncthreads();
  int buf = 0;
  for (int kt = kt_begin; kt < kt_end; ++kt) {
    park(buf ^ 1);
    issue(kt + 2);
    mma_tile<bf16_raw>(acc, As(buf), Cb(buf), wm, wn, lane);
    __syncthreads();
    build(buf ^ 1);
    __syncthreads();
    buf ^= 1;
  }
  const int N = p.Ci * 16;
  float* ob = p.Out + (int64_t)by * p.o_split + (int64_t)b * p.o_model;
  store_tile<float, float, false>(acc, smem, ob, N, p.Co, N, m0, c0 * 16, (const float*)nullptr, 0, HFTA_ACT_NONE, 0.f, 16, t);
}

// out[i] = bf16(act(sum of the k splits' partials + bias of i's channel)); 8 consecutive elements per thread
__global__ __launch_bounds__(256) void ig_split_finish_kernel(const float* __restrict__ part, bf16_raw* __restrict__ out,
                                                              const bf16_raw* __restrict__ bias, int64_t count8, int64_t slice,
                                                              int splits, int64_t o_m, int channels, int act, float slope) {
  const int64_t i8 = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i8 >= count8) return;
  const int64_t i = i8 * 8;
  float v[8];
  {
    const float4 a = *reinterpret_cast<const float4*>(part + i), c = *reinterpret_cast<const float4*>(part + i + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = c.x; v[5] = c.y; v[6] = c.z; v[7] = c.w;
  }
  for (int s = 1; s < splits; ++s) {
    const float4 a = *reinterpret_cast<const float4*>(part + s * slice + i), c = *reinterpret_cast<const float4*>(part + s * slice + i + 4);
    v[0] += a.x; v[1] += a.y; v[2] += a.z; v[3] += a.w; v[4] += c.x; v[5] += c.y; v[6] += c.z; v[7] += c.w;
  }
  const float bm = bias ? bf16_to_f32(bias[(i / o_m) % channels]) : 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = cheap_act(v[e] + bm, act, slope);
  *reinterpret_cast<uint4*>(out + i) = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
}

// k split of the forward kernel: taken when the tiles alone leave most compute units with a single
// workgroup and the reduction is long (the 8x8 layers: 320 tiles, 128 k-tiles: 101 -> 90 us).  With
// 640 tiles and more, and for the class-pair data gradient, the split measured no gain or a loss.
int ig_pick_ksplit(int64_t blocks, int ktiles, bool pair) {
  if (pair || blocks >= 384 || ktiles < 64) return 1;
  return ktiles >= 128 ? 4 : 2;
}

__global__ __launch_bounds__(256) void ig_split_reduce_kernel(const float4* __restrict__ partial, float4* __restrict__ out, int64_t count4, int splits) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count4) return;
  float4 s = partial[i];
  for (int k = 1; k < splits; ++k) {
    const float4 v = partial[(int64_t)k * count4 + i];
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  out[i] = s;
}

constexpr size_t IG_MAX_LDS = 96 * 1024;

// Kernels here take more dynamic LDS than the default limit allows: the limit of each instantiation
// is raised before its launches (an idempotent attribute of the loaded kernel, not library state).
template <typename K>
void ig_launch(K kernel, dim3 grid, int threads, size_t lds, hipStream_t st, IgArgs a) {
  if (lds > 48 * 1024) (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)IG_MAX_LDS);
  a.grid = IgGrid{(int)grid.x, (int)grid.y, (int)grid.z};
  hipLaunchKernelGGL(kernel, dim3(grid.x * grid.y * grid.z), dim3((unsigned)threads), lds, st, a);
}

}  // namespace

// Forward of the grouped convolution (also the data gradient of the transposed convolution).
// HFTA_EUNSUPPORTED when the shape is outside what the kernel handles (the caller falls back).
// fp32 partial slices the forward wants for its k split (0: no split).  Without that much workspace it runs unsplit.
size_t conv_ig_fwd_split_bytes(int B, int Nb, int Ci, int Co, int H, int W) {
  const int Ho = H / 2, Wo = W / 2, tm = Co <= 64 ? 64 : 128;
  if (Ho <= 0 || Wo <= 0) return 0;
  const int64_t blocks = (int64_t)((Co + tm - 1) / tm) * (((int64_t)Nb * Ho * Wo + 127) / 128) * B;
  const int ks = ig_pick_ksplit(blocks, (Ci * 16 + 31) / 32, false);
  return ks > 1 ? (size_t)ks * Nb * B * Co * Ho * Wo * sizeof(float) : 0;
}

int conv_ig_forward(int B, int Nb, int Ci, int Co, int H, int W, int kh, int kw, int stride, int pad, const void* X,
                    const void* Wt, const void* bias, void* Y, int act, float slope, void* ws, size_t ws_bytes,
                    hipStream_t st) {
  const int Ho = (H + 2 * pad - kh) / stride + 1, Wo = (W + 2 * pad - kw) / stride + 1;
  if (kh != 4 || kw != 4 || stride != 2 || pad != 1) return HFTA_EUNSUPPORTED;
  if (!pow2(Ho) || !pow2(Wo) || Wo < 4 || Ho * Wo < 16 || W % 8 != 0 || (128 % (Ho * Wo) != 0 && (Ho * Wo) % 128 != 0)) return HFTA_EUNSUPPORTED;
  if ((Ho * Wo >= 128 && 128 % Wo != 0) || (int64_t)Nb * Ho * Wo > 0x7fffffff) return HFTA_EUNSUPPORTED;
  if (act != HFTA_ACT_NONE && act != HFTA_ACT_RELU && act != HFTA_ACT_LEAKY) return HFTA_EUNSUPPORTED;
  if (reinterpret_cast<uintptr_t>(X) % 16 || reinterpret_cast<uintptr_t>(Wt) % 16 || reinterpret_cast<uintptr_t>(Y) % 16) return HFTA_EUNSUPPORTED;
  IgArgs a{};
  a.X = (const bf16_raw*)X; a.A = (const bf16_raw*)Wt; a.Out = (bf16_raw*)Y; a.bias = (const bf16_raw*)bias;
  a.x_img = (int64_t)B * Ci * H * W; a.x_model = (int64_t)Ci * H * W;
  a.a_model = (int64_t)Co * Ci * 16;
  a.o_img = (int64_t)B * Co * Ho * Wo; a.o_model = (int64_t)Co * Ho * Wo; a.o_m = (int64_t)Ho * Wo;
  a.Nb = Nb; a.Cx = Ci; a.H = H; a.W = W;
  a.M = Co; a.K = Ci * 16; a.N = Nb * Ho * Wo;
  if (!ig_extents(a)) return HFTA_EUNSUPPORTED;
  a.OW = Wo; a.oys = 1; a.oxs = 1; a.tap_step = 1;
  ig_geometry(a, 4, 4, 2, Ho, Wo, W, 128, false);
  const int tm = Co <= 64 ? 64 : 128;
  a.nchunk = 2 * a.NI * a.PR * (W / a.chunk_el);
  if (a.nchunk > 512) return HFTA_EUNSUPPORTED;
  a.tiles_n = (a.N + 127) / 128;
  a.act = act; a.slope = slope;
  a.cls[0] = IgClass{-pad, -pad, 0, 0, 0};
  const size_t lds = ig_lds_bytes(a, 2, tm);
  if (lds > IG_MAX_LDS) return HFTA_EUNSUPPORTED;
  const int tiles_m = (Co + tm - 1) / tm;
  if ((int64_t)tiles_m * a.tiles_n > 0x7fffffff || B > 65535) return HFTA_EUNSUPPORTED;
  const int ktiles = (a.K + 31) / 32;
  const size_t need = conv_ig_fwd_split_bytes(B, Nb, Ci, Co, H, W);
  a.ksplit = (need && ws && ws_bytes >= need && reinterpret_cast<uintptr_t>(ws) % 16 == 0) ? ig_pick_ksplit((int64_t)tiles_m * a.tiles_n * B, ktiles, false) : 1;
  a.kt_per_split = (ktiles + a.ksplit - 1) / a.ksplit;
  a.part = reinterpret_cast<float*>(ws);
  a.part_split = (int64_t)Nb * a.o_img;
  const size_t lds2 = ig_lds_bytes(a, 2, tm);
  dim3 grid((unsigned)(tiles_m * a.tiles_n), (unsigned)a.ksplit, (unsigned)B);
  if (tm == 64) ig_launch(conv_ig_fwd_kernel<4, 4, 2, false, 64, true>, grid, 256, lds2, st, a);
  else ig_launch(conv_ig_fwd_kernel<4, 4, 2, false, 128, true>, grid, 256, lds2, st, a);
  if (a.ksplit > 1) {
    if (launch_status() != HFTA_OK) return HFTA_ELAUNCH;
    const int64_t count8 = a.part_split / 8;
    hipLaunchKernelGGL(ig_split_finish_kernel, dim3((unsigned)((count8 + 255) / 256)), dim3(256), 0, st, (const float*)a.part,
                       a.Out, a.bias, count8, a.part_split, a.ksplit, a.o_m, B * Co, act, slope);
  }
  return launch_status();
}

}  // namespace hfta

namespace hfta {

// Data gradient of the 4x4 / stride 2 / pad 1 grouped convolution (= forward of the transposed one):
// four parity classes (grid.y = py, the two px of a tile side by side), each a stride-1 2x2 correlation
// over dY with its regrouped weights.
// `pack` receives the regrouped weights: conv_ig_dx_pack_bytes(...) bytes, 16-byte aligned.
size_t conv_ig_dx_pack_bytes(int B, int Ci, int Co) {                  // whole row tiles and k-tiles; a multiple of 256 bytes
  const int tm = Ci <= 64 ? 64 : 128, tiles_m = (Ci + tm - 1) / tm, ktiles = (Co * 4 + 31) / 32;
  return (size_t)B * 4 * tiles_m * tm * ktiles * 32 * sizeof(bf16_raw);
}

bool conv_ig_dx_supported(int Nb, int Ci, int Co, int H, int W, int kh, int kw, int stride, int pad) {
  if (kh != 4 || kw != 4 || stride != 2 || pad != 1 || H % 2 || W % 2) return false;
  const int Hq = H / 2, Wq = W / 2;
  if (!pow2(Hq) || !pow2(Wq) || Wq < 4 || Wq > 64 || Hq * Wq < 16) return false;
  if ((int64_t)Nb * Hq * Wq > 0x7fffffff || Ci < 32 || Co % 2 != 0) return false;
  return true;
}

// fp32 partial slices the data gradient wants for its k split (0: no split)
size_t conv_ig_dx_split_bytes(int B, int Nb, int Ci, int Co, int H, int W) {
  const int Hq = H / 2, Wq = W / 2, tm = Ci <= 64 ? 64 : 128;
  if (Hq <= 0 || Wq <= 0) return 0;
  const int64_t blocks = (int64_t)((Ci + tm - 1) / tm) * (((int64_t)Nb * Hq * Wq + 63) / 64) * 2 * B;
  const int ks = ig_pick_ksplit(blocks, (Co * 4 + 31) / 32, true);
  return ks > 1 ? (size_t)ks * Nb * B * Ci * H * W * sizeof(float) : 0;
}

int conv_ig_dx(int B, int Nb, int Ci, int Co, int H, int W, int kh, int kw, int stride, int pad, const void* Wt,
               const void* dY, void* dX, void* pack, void* split_ws, hipStream_t st) {
  if (!conv_ig_dx_supported(Nb, Ci, Co, H, W, kh, kw, stride, pad)) return HFTA_EUNSUPPORTED;
  if (reinterpret_cast<uintptr_t>(dY) % 16 || reinterpret_cast<uintptr_t>(Wt) % 16 || reinterpret_cast<uintptr_t>(dX) % 16 ||
      reinterpret_cast<uintptr_t>(pack) % 16 || B > 65535)
    return HFTA_EUNSUPPORTED;
  const int Hq = H / 2, Wq = W / 2;                      // class grid = the gradient's own grid (Ho x Wo)
  IgArgs a{};
  a.X = (const bf16_raw*)dY; a.A = (const bf16_raw*)pack; a.Out = (bf16_raw*)dX; a.bias = nullptr;
  a.x_img = (int64_t)B * Co * Hq * Wq; a.x_model = (int64_t)Co * Hq * Wq;
  const int tm = Ci <= 64 ? 64 : 128, tiles_m = (Ci + tm - 1) / tm, ktiles = (Co * 4 + 31) / 32;
  const int64_t cls_el = (int64_t)tiles_m * tm * ktiles * 32;          // one class of one model, fragment order
  a.a_model = 4 * cls_el;
  a.o_img = (int64_t)B * Ci * H * W; a.o_model = (int64_t)Ci * H * W; a.o_m = (int64_t)H * W;
  a.Nb = Nb; a.Cx = Co; a.H = Hq; a.W = Wq;
  a.M = Ci; a.K = Co * 4; a.N = Nb * Hq * Wq;
  if (!ig_extents(a)) return HFTA_EUNSUPPORTED;
  a.OW = W; a.oys = 2; a.oxs = 2; a.tap_step = 1;
  ig_geometry(a, 2, 2, 1, Hq, Wq, Wq, 64, true);
  a.nchunk = 8 * a.NI * a.PR * (Wq / a.chunk_el);
  if (a.nchunk > 512) return HFTA_EUNSUPPORTED;
  a.tiles_n = (a.N + 63) / 64;
  a.act = HFTA_ACT_NONE; a.slope = 0.f;
  for (int cls = 0; cls < 4; ++cls) {
    const int py = cls >> 1, px = cls & 1;
    a.cls[cls] = IgClass{py - 1, px - 1, py, px, cls * cls_el};          // window rows qy + py - 1, qy + py
  }
  const size_t lds = ig_lds_bytes(a, 8, 0);
  if (lds > IG_MAX_LDS) return HFTA_EUNSUPPORTED;
  if ((int64_t)tiles_m * a.tiles_n > 0x7fffffff) return HFTA_EUNSUPPORTED;
  const int64_t count = (int64_t)B * 4 * cls_el / 8;                   // 16-byte fragment pieces
  hipLaunchKernelGGL(ig_pack_class_w_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, (const bf16_raw*)Wt,
                     (bf16_raw*)pack, Ci, Co, tm, tiles_m, ktiles, count);
  a.ksplit = (split_ws && reinterpret_cast<uintptr_t>(split_ws) % 16 == 0) ? ig_pick_ksplit((int64_t)tiles_m * a.tiles_n * 2 * B, ktiles, true) : 1;
  a.kt_per_split = (ktiles + a.ksplit - 1) / a.ksplit;
  a.part = reinterpret_cast<float*>(split_ws);
  a.part_split = (int64_t)Nb * a.o_img;
  const size_t lds2 = ig_lds_bytes(a, 8, 0);
  if (lds2 > IG_MAX_LDS) return HFTA_EUNSUPPORTED;
  dim3 grid((unsigned)(tiles_m * a.tiles_n), (unsigned)(2 * a.ksplit), (unsigned)B);
  if (a.chunk_el == 8) {
    if (tm == 64) ig_launch(conv_ig_fwd_kernel<2, 2, 1, true, 64, true>, grid, 256, lds2, st, a);
    else ig_launch(conv_ig_fwd_kernel<2, 2, 1, true, 128, true>, grid, 256, lds2, st, a);
  } else {
    if (tm == 64) ig_launch(conv_ig_fwd_kernel<2, 2, 1, true, 64, false>, grid, 256, lds2, st, a);
    else ig_launch(conv_ig_fwd_kernel<2, 2, 1, true, 128, false>, grid, 256, lds2, st, a);
  }
  if (a.ksplit > 1) {
    if (launch_status() != HFTA_OK) return HFTA_ELAUNCH;
    const int64_t count8 = a.part_split / 8;
    hipLaunchKernelGGL(ig_split_finish_kernel, dim3((unsigned)((count8 + 255) / 256)), dim3(256), 0, st, (const float*)a.part,
                       a.Out, (const bf16_raw*)nullptr, count8, a.part_split, a.ksplit, a.o_m, B * Ci, HFTA_ACT_NONE, 0.f);
  }
  return launch_status();
}

}  // namespace hfta

namespace hfta {

// Weight gradient of the 4x4 / stride 2 / pad 1 grouped convolution.  `partial` holds the k splits'
// fp32 slices when conv_ig_dw_splits(...) > 1 (that many times B * Co * Ci * 16 floats).
bool conv_ig_dw_supported(int Nb, int Ci, int Co, int H, int W, int kh, int kw, int stride, int pad) {
  if (kh != 4 || kw != 4 || stride != 2 || pad != 1 || H % 2 || W % 2) return false;
  const int Ho = H / 2, Wo = W / 2;
  if (!pow2(Ho) || !pow2(Wo) || Wo < 4 || Wo > 32 || Ho * Wo < 16) return false;
  if ((int64_t)Nb * Ho * Wo > 0x7fffffff || Co < 32) return false;   // fewer than 8 input channels: the missing columns are zeros
  return true;                                           // a k-tile's second 4x4 sample past the batch reads as zeros
}

int conv_ig_dw_splits(int B, int Nb, int Ci, int Co, int H, int W) {
  const int64_t kt_total = ((int64_t)Nb * (H / 2) * (W / 2) + 31) / 32;
  const int64_t tiles = (int64_t)((Co + 127) / 128) * ((Ci + 7) / 8) * B;
  if (tiles >= 512 || kt_total < 32) return 1;
  // two workgroups per compute unit: more splits only add partial-slice traffic (measured 512 .. 1536)
  int64_t want = (512 + tiles - 1) / tiles, cap = kt_total / 16;
  if (want > cap) want = cap;
  if (want > 64) want = 64;
  return want < 1 ? 1 : (int)want;
}

int conv_ig_dw(int B, int Nb, int Ci, int Co, int H, int W, int kh, int kw, int stride, int pad, const void* X,
               const void* dY, float* dW, float* partial, hipStream_t st) {
  if (!conv_ig_dw_supported(Nb, Ci, Co, H, W, kh, kw, stride, pad)) return HFTA_EUNSUPPORTED;
  if (reinterpret_cast<uintptr_t>(X) % 16 || reinterpret_cast<uintptr_t>(dY) % 16 || reinterpret_cast<uintptr_t>(dW) % 16 ||
      reinterpret_cast<uintptr_t>(partial) % 16 || B > 65535)
    return HFTA_EUNSUPPORTED;
  const int Ho = H / 2, Wo = W / 2, P = Ho * Wo;
  IgDwArgs a{};
  a.X = (const bf16_raw*)X; a.dY = (const bf16_raw*)dY;
  a.x_img = (int64_t)B * Ci * H * W; a.x_model = (int64_t)Ci * H * W;
  a.y_img = (int64_t)B * Co * P; a.y_model = (int64_t)Co * P;
  a.o_model = (int64_t)Co * Ci * 16;
  a.Nb = Nb; a.Ci = Ci; a.Co = Co; a.H = H; a.W = W; a.Ho = Ho; a.Wo = Wo;
  a.lgWo = ilog2(Wo); a.lgP = ilog2(P);
  a.NI = P >= 32 ? 1 : 2;
  const int TR = P >= 32 ? 32 / Wo : Ho;
  a.PR = (TR - 1) * 2 + 4;
  {
    // Row and sample pitch of the patch with the fewest LDS bank conflicts in the gather (32 banks of
    // 4 bytes, 32 lanes per clock): the lanes of a half wavefront read the 16 taps of two channels.
    int64_t best = -1;
    for (int i = 0; i < 6; ++i)
      for (int j = 0; j < 8; ++j) {
        const int pw = W + 16 + 8 * i, sp = a.PR * pw + 8 * j;
        int cost = 0;
        for (int h = 0; h < 2; ++h) {
          int words[32], nw = 0, per_bank[32] = {0}, worst = 0;
          for (int l = 0; l < 32; ++l) {
            const int bj = h * 32 + l, c_l = bj >> 4, ky = (bj >> 2) & 3, kx = bj & 3;
            const int word = (c_l * a.NI * sp + ky * pw + kx + IG_MARGIN - 1) >> 1;
            bool seen = false;
            for (int q = 0; q < nw; ++q) seen = seen || words[q] == word;
            if (!seen) { words[nw++] = word; worst = ++per_bank[word & 31] > worst ? per_bank[word & 31] : worst; }
          }
          cost += worst;
        }
        const int64_t key = (int64_t)cost * (1 << 20) + (int64_t)a.NI * sp;
        if (best < 0 || key < best) { best = key; a.PW = pw; a.SP = sp; }
      }
  }
  a.nchunk = 8 * a.NI * a.PR * (W / 8);
  if (a.nchunk > 256 || W % 8 != 0) return HFTA_EUNSUPPORTED;
  const int64_t xb = ((int64_t)(Nb - 1) * a.x_img + (int64_t)Ci * H * W) * 2, yb = ((int64_t)(Nb - 1) * a.y_img + (int64_t)Co * P) * 2;
  if (xb >= ((int64_t)1 << 31) || yb >= ((int64_t)1 << 31)) return HFTA_EUNSUPPORTED;
  a.x_bytes = (uint32_t)xb; a.y_bytes = (uint32_t)yb;
  a.tiles_n = (Ci + 7) / 8;
  a.kt_total = (int)(((int64_t)Nb * P + 31) / 32);
  const int splits = conv_ig_dw_splits(B, Nb, Ci, Co, H, W);
  if (splits > 1 && !partial) return HFTA_EWORKSPACE;
  a.kt_per_split = (a.kt_total + splits - 1) / splits;
  a.o_split = (int64_t)B * a.o_model;
  a.Out = splits > 1 ? partial : dW;
  const size_t k_loop = 4 * (size_t)GEMM_TILE_BYTES + (size_t)8 * a.NI * a.SP * 2;
  const size_t staging = 64 * (size_t)EPI_PITCH4;
  const size_t lds = k_loop > staging ? k_loop : staging;
  if (lds > IG_MAX_LDS) return HFTA_EUNSUPPORTED;
  const int tiles_m = (Co + 127) / 128;
  if (lds > 48 * 1024)
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(conv_ig_dw_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)IG_MAX_LDS);
  a.grid = IgGrid{tiles_m * a.tiles_n, splits, B};
  if ((int64_t)a.grid.gx * splits * B > 0x7fffffff) return HFTA_EUNSUPPORTED;
  hipLaunchKernelGGL(conv_ig_dw_kernel, dim3((unsigned)(a.grid.gx * splits * B)), dim3(256), lds, st, a);
  if (launch_status() != HFTA_OK) return HFTA_ELAUNCH;
  if (splits > 1) {
    const int64_t count4 = (int64_t)B * a.o_model / 4;
    hipLaunchKernelGGL(ig_split_reduce_kernel, dim3((unsigned)((count4 + 255) / 256)), dim3(256), 0, st, (const float4*)partial,
                       (float4*)dW, count4, splits);
  }
  return launch_status();
}

}  // namespace hfta
