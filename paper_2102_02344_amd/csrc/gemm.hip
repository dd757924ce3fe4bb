// Host side of the batched GEMM core: split selection, alignment checks, dispatch.
#include "gemm.h"
#include "gemm_pf.h"

namespace hfta {

// Sum split-K partials in a fixed order: out[i] = sum_s partial[s][i].
// out[i] = sum over the splits of partial[k][i] in a fixed order: thread (i, q) adds the splits
// k = q, q+4, ... (several loads in flight), the four quarter sums are combined as (0+1)+(2+3).
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, float* __restrict__ out,
                                                            int64_t count, int splits) {
  __shared__ float sh[4][64];
  const int q = threadIdx.x >> 6, li = threadIdx.x & 63;
  const int64_t i = (int64_t)blockIdx.x * 64 + li;
  float s = 0.f;
  if (i < count) {
#pragma unroll 8
    for (int k = q; k < splits; k += 4) s += partial[(int64_t)k * count + i];
  }
  sh[q][li] = s;
  __syncthreads();
  if (q == 0 && i < count) out[i] = (sh[0][li] + sh[1][li]) + (sh[2][li] + sh[3][li]);
}

int gemm_big_launch(const GemmDesc& d, const GemmArgs& a, bool v16, bool n16, dim3 grid, hipStream_t st);

static inline bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

static int total_tiles(const GemmDesc& d) {
  const int BK = d.dtype == HFTA_BF16 ? GemmT<bf16_raw>::BK : GemmT<float>::BK;
  return d.S * ((d.K + BK - 1) / BK);
}

// 256x256-tile kernel: one workgroup per compute unit at a time, so a launch runs in rounds of 256
// workgroups.  Cost model per split count s: rounds * (k-tiles per workgroup + a fixed prologue /
// epilogue, in k-tile units) + the partial buffer's write and read; the cheapest s wins.
// shortest reduction (per split) the 256x256-tile kernel is used for
constexpr int BIG_MIN_K = 256;
static int pick_splits_big(const GemmDesc& d) {
  if (d.dtype != HFTA_BF16 || d.M < 192 || d.N < 192 || d.K < 256) return 0;
  const int64_t t256 = (int64_t)((d.M + 255) / 256) * ((d.N + 255) / 256) * d.G0 * d.G1;
  const int64_t tt = (int64_t)d.S * ((d.K + 63) / 64);
  if (tt < 32) return 0;
  const double fixed = 4.0;                                   // prologue + epilogue, in k-tiles
  const double per_split = 0.2 * (double)t256 / 256.0;        // partial traffic of one more split
  int best = 0;
  double best_cost = 0.0;
  for (int s = 1; s <= 32 && tt / s >= 16; ++s) {
    if (t256 * s < 192) continue;
    const double rounds = (double)((t256 * s + 255) / 256);
    const double cost = rounds * ((double)tt / s + fixed) + (s > 1 ? per_split * s : 0.0);
    if (best == 0 || cost < best_cost) { best = s; best_cost = cost; }
  }
  return best;
}

// Enough workgroups to fill 256 compute units a few times over, without cutting
// the reduction into pieces shorter than 8 k-tiles.
int gemm_pick_splits(const GemmDesc& d) {
  const int big = pick_splits_big(d);
  if (big > 0) return big;
  const int64_t tiles = (int64_t)((d.M + GEMM_BM - 1) / GEMM_BM) * ((d.N + GEMM_BN - 1) / GEMM_BN) * d.G0 * d.G1;
  const int tt = total_tiles(d);
  if (tiles >= 512 || tt < 16) return 1;
  int64_t want = (512 + tiles - 1) / tiles;       // two workgroups per compute unit (measured best: 256-1536 swept)
  int64_t cap = tt / 8;
  if (want > cap) want = cap;
  if (want > 256) want = 256;
  return want < 1 ? 1 : (int)want;
}

size_t gemm_partial_bytes(const GemmDesc& d, int splits) {
  if (splits <= 1) return 0;
  return (size_t)splits * d.G0 * d.G1 * (size_t)d.M * d.N * sizeof(float);
}

template <typename T, bool A_KC, bool B_KC>
static void launch_typed(const GemmDesc& d, const GemmArgs& a, dim3 grid, hipStream_t st) {
  if (d.out_f32 || d.splits > 1)
    hipLaunchKernelGGL((gemm_kernel<T, A_KC, B_KC, float>), grid, dim3(GEMM_THREADS), 0, st, a);
  else
    hipLaunchKernelGGL((gemm_kernel<T, A_KC, B_KC, T>), grid, dim3(GEMM_THREADS), 0, st, a);
}

template <typename T>
static int launch_layout(const GemmDesc& d, const GemmArgs& a, dim3 grid, hipStream_t st) {
  if (d.a_kc && !d.b_kc) launch_typed<T, true, false>(d, a, grid, st);
  else if (d.a_kc && d.b_kc) launch_typed<T, true, true>(d, a, grid, st);
  else if (!d.a_kc && !d.b_kc) launch_typed<T, false, false>(d, a, grid, st);
  else return HFTA_EUNSUPPORTED;
  return launch_status();
}

static int reduce_partials(const GemmDesc& d, int64_t G, int splits, hipStream_t st) {
  const int64_t count = G * (int64_t)d.M * d.N;
  hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((count + 63) / 64)), dim3(256), 0, st,
                     d.partial, reinterpret_cast<float*>(d.C), count, splits);
  return launch_status();
}

int gemm_launch(const GemmDesc& d, hipStream_t st) {
  if (d.M <= 0 || d.N <= 0 || d.K <= 0 || d.S <= 0 || d.G0 <= 0 || d.G1 <= 0) return HFTA_EINVAL;
  const int64_t G = (int64_t)d.G0 * d.G1;
  const int splits = d.splits < 1 ? 1 : d.splits;
  if (G * splits > 65535) return HFTA_EUNSUPPORTED;
  if (splits > 1 && (!d.partial || !d.out_f32 || d.bias || d.act != HFTA_ACT_NONE)) return HFTA_EINVAL;
  if (d.dtype == HFTA_BF16 && d.out_f32 &&
      ((d.bias && d.bias_mode == 2) || d.act == HFTA_ACT_TANH || d.act == HFTA_ACT_GELU))
    return HFTA_EUNSUPPORTED;

  GemmArgs a;
  a.A = d.A; a.Bm = d.Bm; a.C = d.C; a.bias = d.bias; a.partial = d.partial;
  a.a_ld = d.a_ld; a.a_ss = d.a_ss; a.a_g0 = d.a_g0; a.a_g1 = d.a_g1;
  a.b_ld = d.b_ld; a.b_ss = d.b_ss; a.b_g0 = d.b_g0; a.b_g1 = d.b_g1;
  a.c_ld = d.c_ld; a.c_g0 = d.c_g0; a.c_g1 = d.c_g1;
  a.bias_g0 = d.bias_g0; a.bias_g1 = d.bias_g1;
  a.M = d.M; a.N = d.N; a.K = d.K; a.S = d.S; a.G1 = d.G1;
  a.tiles_n = (d.N + GEMM_BN - 1) / GEMM_BN;
  a.tiles_m = (d.M + GEMM_BM - 1) / GEMM_BM;
  const int BK = d.dtype == HFTA_BF16 ? GemmT<bf16_raw>::BK : GemmT<float>::BK;
  a.tiles_per_seg = (d.K + BK - 1) / BK;
  a.total_tiles = d.S * a.tiles_per_seg;
  a.splits = splits;
  a.bias_mode = d.bias ? d.bias_mode : 0;
  a.act = d.act; a.slope = d.slope;
  a.a_extent = a.b_extent = 0;
  a.c_seg = d.c_seg; a.c_seg_stride = d.c_seg_stride;
  a.stat_part = d.stat_part;
  if (d.stat_done) *d.stat_done = false;

  // vector-load eligibility: every address the fast path forms must be aligned
  const int es = (int)dtype_size(d.dtype);
  const int kg = 16 / es, nv = 8 / es;
  // 0: element-wise; 1: 8-byte loads; 2 (k-contiguous operands only): 16-byte loads
  auto ok = [&](const void* p, int64_t ld, int64_t ss, int64_t s0, int64_t s1, bool kc) {
    auto al = [&](int q, size_t bytes) {
      return aligned_to(p, bytes) && ld % q == 0 && ss % q == 0 && s0 % q == 0 && s1 % q == 0;
    };
    if (kc && al(kg, 16)) return 2;
    return al(nv, 8) ? 1 : 0;
  };
  a.a_vec = ok(d.A, d.a_ld, d.a_ss, d.a_g0, d.a_g1, d.a_kc);
  a.b_vec = ok(d.Bm, d.b_ld, d.b_ss, d.b_g0, d.b_g1, d.b_kc);
  // widest store (bytes) every row start of C / of the partial buffer is aligned to
  const int oes = (d.out_f32 || splits > 1) ? 4 : es;
  auto store_bytes = [&](const void* p, int64_t ld, int64_t s0, int64_t s1) {
    for (int w = 16; w >= 8; w >>= 1) {
      const int q = w / oes;
      if (aligned_to(p, w) && ld % q == 0 && s0 % q == 0 && s1 % q == 0) return w;
    }
    return 0;
  };
  a.c_vec = store_bytes(d.C, d.c_ld, d.c_g0, d.c_g1);
  if (d.c_seg > 0) {                 // a store piece must not straddle two column segments
    if (splits > 1) return HFTA_EUNSUPPORTED;
    while (a.c_vec >= 8 && (d.c_seg % (a.c_vec / oes) != 0 || d.c_seg_stride % (a.c_vec / oes) != 0)) a.c_vec >>= 1;
    if (a.c_vec < 8) a.c_vec = 0;
  }
  a.p_vec = splits > 1 ? store_bytes(d.partial, d.N, (int64_t)d.M * d.N, 0) : 0;

  // operand slice extents for the buffer-load kernels
  const int64_t a_ext = ((d.a_kc ? (int64_t)(d.M - 1) * d.a_ld + d.K : (int64_t)(d.K - 1) * d.a_ld + d.M)) * es;
  const int64_t b_ext = ((d.b_kc ? (int64_t)(d.N - 1) * d.b_ld + d.K : (int64_t)(d.K - 1) * d.b_ld + d.N)) * es;
  const bool buffers_ok = d.dtype == HFTA_BF16 && a_ext < (int64_t)1 << 31 && b_ext < (int64_t)1 << 31 &&
                          d.a_ld > 0 && d.b_ld > 0 && (d.a_kc || !d.b_kc);
  auto whole_pieces = [&](int vec, bool kc, int extent_mn, bool v16) {
    if (vec == 0 || (v16 && kc && vec != 2)) return false;
    if (kc) return d.K % (v16 ? 8 : 4) == 0;
    return extent_mn % 4 == 0;
  };
  const bool v16 = buffers_ok && (d.a_kc || d.b_kc) && whole_pieces(a.a_vec, d.a_kc, d.M, true) &&
                   whole_pieces(a.b_vec, d.b_kc, d.N, true);
  const bool v8 = buffers_ok && whole_pieces(a.a_vec, d.a_kc, d.M, false) && whole_pieces(a.b_vec, d.b_kc, d.N, false);
  if (buffers_ok) {
    a.a_extent = (uint32_t)a_ext;
    a.b_extent = (uint32_t)b_ext;
  }
  {
    const int64_t last = d.N - 1;
    const int64_t c_cols = d.c_seg > 0 ? (last / d.c_seg) * d.c_seg_stride + last % d.c_seg + 1 : (int64_t)d.N;
    const int64_t c_ext = ((int64_t)(d.M - 1) * d.c_ld + c_cols) * oes;
    a.c_extent = c_ext > 0 && c_ext < (int64_t)1 << 31 ? (uint32_t)c_ext : 0u;
  }

  // operands contiguous along m / n: 16-byte pieces when every row start and the extent allow it
  auto n16ok = [&](const void* q, int64_t ld, int64_t ss, int64_t s0, int64_t s1, bool kc, int extent) {
    return kc || (aligned_to(q, 16) && ld % 8 == 0 && ss % 8 == 0 && s0 % 8 == 0 && s1 % 8 == 0 && extent % 8 == 0);
  };
  const bool n16 = n16ok(d.A, d.a_ld, d.a_ss, d.a_g0, d.a_g1, d.a_kc, d.M) &&
                   n16ok(d.Bm, d.b_ld, d.b_ss, d.b_g0, d.b_g1, d.b_kc, d.N);

  // Compute-bound problems (MLP-sized bf16 GEMMs) take the 256x256 kernel: it needs 16-byte
  // loadable operands, no split, a long reduction, and enough tiles to give every compute unit
  // at least one.
  if ((v16 || (v8 && d.a_kc == d.b_kc)) && d.M >= 192 && d.N >= 192 && d.K >= 256 && (int64_t)d.K * d.S >= BIG_MIN_K * (int64_t)splits &&
      (d.c_seg == 0 || a.c_vec >= 8)) {
    const int64_t t256 = (int64_t)((d.M + 255) / 256) * ((d.N + 255) / 256) * G;
    if (t256 * splits >= 192) {
      GemmArgs b = a;
      b.tiles_m = (d.M + 255) / 256;
      b.tiles_n = (d.N + 255) / 256;
      b.tiles_per_seg = (d.K + 63) / 64;
      b.total_tiles = d.S * b.tiles_per_seg;
      dim3 grid((unsigned)(b.tiles_m * b.tiles_n), 1, (unsigned)(G * splits));
      const int rc = gemm_big_launch(d, b, v16 || !(d.a_kc || d.b_kc), n16, grid, st);
      if (rc == HFTA_OK && splits > 1 && !d.keep_partials) return reduce_partials(d, G, splits, st);
      if (rc != HFTA_EUNSUPPORTED) return rc;
    }
  }

  const int tiles_m = (d.M + GEMM_BM - 1) / GEMM_BM;
  dim3 grid((unsigned)(tiles_m * a.tiles_n), 1, (unsigned)(G * splits));
  int rc;
  // bf16 problems whose operands can be fetched in whole 8/16-byte pieces take the deep-prefetch
  // kernel (branch-free buffer loads, several k-tiles in flight).
  const bool pf = v16 || v8;
  if (pf) {
    rc = gemm_pf_launch(d, a, v16, n16, grid, st);
  } else {
    rc = d.dtype == HFTA_BF16 ? launch_layout<bf16_raw>(d, a, grid, st) : launch_layout<float>(d, a, grid, st);
  }
  if (rc != HFTA_OK) return rc;
  if (splits > 1 && !d.keep_partials) return reduce_partials(d, G, splits, st);
  return HFTA_OK;
}

}  // namespace hfta
