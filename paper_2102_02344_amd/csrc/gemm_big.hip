// Instantiations and launcher of the 256x256 compute-bound GEMM kernel.
#include "gemm_big.h"

namespace hfta {

// n16: the m/n-contiguous operands (if any) load in 16-byte pieces; a launch without such an operand
// has one instantiation only.
template <bool A_KC, bool B_KC, typename OutT, bool COLB, int ACT>
static void launch_big(const GemmArgs& a, bool n16, dim3 grid, hipStream_t st) {
  if (n16 && !(A_KC && B_KC))
    hipLaunchKernelGGL((gemm_big_kernel<A_KC, B_KC, OutT, true, COLB, ACT, true>), grid, dim3(BIG_THREADS), 0, st, a);
  else
    hipLaunchKernelGGL((gemm_big_kernel<A_KC, B_KC, OutT, true, COLB, ACT, false>), grid, dim3(BIG_THREADS), 0, st, a);
}

// Persistent form: as many workgroups as compute units (a multiple of 8, one per XCD slot), each
// walking several output tiles.  Taken when a launch has more tiles than that, the epilogue is the
// select kind, every operand loads in 16-byte pieces, and output rows take whole 16-byte stores.
static int persistent_blocks() {
  static const int n = [] {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
      return 0;
    return cus / 8 * 8;
  }();
  return n;
}

template <bool A_KC, bool B_KC, typename OutT, bool COLB, bool V16, bool N16>
static void launch_bigp2(const GemmArgs& a, bool ident, dim3 grid, int blocks, hipStream_t st) {
  if constexpr (A_KC && !B_KC && std::is_same<OutT, bf16_raw>::value && !COLB && V16) {
    if (ident && a.stat_part) {          // k=1 convolution forward with the statistics epilogue
      hipLaunchKernelGGL((gemm_bigp_kernel<A_KC, B_KC, OutT, COLB, BIG_NONE, V16, N16, true>), dim3((unsigned)blocks), dim3(BIG_THREADS), 0,
                         st, a, (int)grid.x, (int)(grid.x * grid.z));
      return;
    }
  }
  if (ident)
    hipLaunchKernelGGL((gemm_bigp_kernel<A_KC, B_KC, OutT, COLB, BIG_NONE, V16, N16>), dim3((unsigned)blocks), dim3(BIG_THREADS), 0, st, a,
                       (int)grid.x, (int)(grid.x * grid.z));
  else
    hipLaunchKernelGGL((gemm_bigp_kernel<A_KC, B_KC, OutT, COLB, BIG_SEL, V16, N16>), dim3((unsigned)blocks), dim3(BIG_THREADS), 0, st, a,
                       (int)grid.x, (int)(grid.x * grid.z));
}

// One load-width flag matters per operand pair: v16 for two k-contiguous operands, n16 otherwise
// (a k-contiguous operand next to an m/n-contiguous one always loads 16-byte pieces here).
template <bool A_KC, bool B_KC, typename OutT, bool COLB>
static void launch_bigp(const GemmArgs& a, bool ident, bool v16, bool n16, dim3 grid, int blocks, hipStream_t st) {
  if constexpr (A_KC && B_KC) {
    if (v16) launch_bigp2<A_KC, B_KC, OutT, COLB, true, false>(a, ident, grid, blocks, st);
    else launch_bigp2<A_KC, B_KC, OutT, COLB, false, false>(a, ident, grid, blocks, st);
  } else {
    if (n16) launch_bigp2<A_KC, B_KC, OutT, COLB, true, true>(a, ident, grid, blocks, st);
    else launch_bigp2<A_KC, B_KC, OutT, COLB, true, false>(a, ident, grid, blocks, st);
  }
}

static bool persistent_ok(const GemmDesc& d, const GemmArgs& a, bool v16, bool sel, dim3 grid, int blocks) {
  if (blocks < 8 || (int64_t)grid.x * grid.z <= blocks || !sel) return false;
  if (!v16 && !(d.a_kc && d.b_kc)) return false;       // 8-byte k-contiguous loads: both operands only
  const bool partial = a.splits > 1;
  const int oes = (d.out_f32 || partial) ? 4 : 2;
  const int vb = partial ? a.p_vec : a.c_vec;
  if ((vb != 16 && vb != 8) || d.N % (vb / oes) != 0) return false;
  if (partial) return (int64_t)d.M * d.N * 4 < (int64_t)1 << 31;
  return a.c_extent != 0;
}

// `a` must carry tile counts for 256x256 tiles and 64-element k-tiles and operand extents.
// `v16`: k-contiguous operands are loadable in 16-byte pieces; otherwise (rows only 8-byte aligned,
// e.g. 2500 points per sample) only the weight-gradient form (both operands k-contiguous, fp32
// output) is built, on 8-byte loads.  `n16`: operands contiguous along m / n load in 16-byte pieces
// (else 8-byte).  HFTA_EUNSUPPORTED: not a combination this kernel is built for.
int gemm_big_launch(const GemmDesc& d, const GemmArgs& a0, bool v16, bool n16, dim3 grid, hipStream_t st) {
  GemmArgs a = a0;
  const bool colb = d.bias && d.bias_mode == 2;
  const bool sel = d.act == HFTA_ACT_NONE || d.act == HFTA_ACT_RELU || d.act == HFTA_ACT_LEAKY;
  a.slope = d.act == HFTA_ACT_NONE ? 1.f : d.act == HFTA_ACT_RELU ? 0.f : d.slope;
  if (colb && (reinterpret_cast<uintptr_t>(d.bias) % 8 != 0 || d.bias_g0 % 4 != 0 || d.bias_g1 % 4 != 0 || d.N % 4 != 0))
    return HFTA_EUNSUPPORTED;
  const int blocks = persistent_blocks();
  if (persistent_ok(d, a, v16, sel, grid, blocks)) {
    const bool f32 = d.out_f32 || a.splits > 1;
    const bool ident = d.act == HFTA_ACT_NONE;
    if (f32 && !colb) {
      if (d.a_kc && !d.b_kc) { launch_bigp<true, false, float, false>(a, ident, v16, n16, grid, blocks, st); return launch_status(); }
      if (d.a_kc && d.b_kc) { launch_bigp<true, true, float, false>(a, ident, v16, n16, grid, blocks, st); return launch_status(); }
      if (!d.a_kc && !d.b_kc) { launch_bigp<false, false, float, false>(a, ident, v16, n16, grid, blocks, st); return launch_status(); }
    } else if (!f32) {
      if (d.a_kc && !d.b_kc) {
        if (colb) launch_bigp<true, false, bf16_raw, true>(a, ident, v16, n16, grid, blocks, st);
        else launch_bigp<true, false, bf16_raw, false>(a, ident, v16, n16, grid, blocks, st);
        const int rc = launch_status();
        if (rc == HFTA_OK && !colb && ident && a.stat_part && a.splits == 1 && d.stat_done) *d.stat_done = true;
        return rc;
      }
      if (!colb && d.a_kc && d.b_kc) { launch_bigp<true, true, bf16_raw, false>(a, ident, v16, n16, grid, blocks, st); return launch_status(); }
      if (!colb && !d.a_kc && !d.b_kc) { launch_bigp<false, false, bf16_raw, false>(a, ident, v16, n16, grid, blocks, st); return launch_status(); }
    }
  }
  if (!v16) {
    if (!(d.out_f32 && d.a_kc && d.b_kc) || colb || !sel) return HFTA_EUNSUPPORTED;
    hipLaunchKernelGGL((gemm_big_kernel<true, true, float, false, false, BIG_SEL>), grid, dim3(BIG_THREADS), 0, st, a);
    return launch_status();
  }
  if (d.out_f32) {
    if (colb || !sel) return HFTA_EUNSUPPORTED;
    if (d.a_kc && !d.b_kc) launch_big<true, false, float, false, BIG_SEL>(a, n16, grid, st);
    else if (d.a_kc && d.b_kc) launch_big<true, true, float, false, BIG_SEL>(a, n16, grid, st);
    else if (!d.a_kc && !d.b_kc) launch_big<false, false, float, false, BIG_SEL>(a, n16, grid, st);
    else return HFTA_EUNSUPPORTED;
    return launch_status();
  }
  if (d.a_kc && !d.b_kc) {
    if (colb) {
      if (sel) launch_big<true, false, bf16_raw, true, BIG_SEL>(a, n16, grid, st);
      else if (d.act == HFTA_ACT_GELU) launch_big<true, false, bf16_raw, true, BIG_GELU>(a, n16, grid, st);
      else launch_big<true, false, bf16_raw, true, BIG_TANH>(a, n16, grid, st);
    } else {
      if (sel) launch_big<true, false, bf16_raw, false, BIG_SEL>(a, n16, grid, st);
      else if (d.act == HFTA_ACT_GELU) launch_big<true, false, bf16_raw, false, BIG_GELU>(a, n16, grid, st);
      else launch_big<true, false, bf16_raw, false, BIG_TANH>(a, n16, grid, st);
    }
  } else {
    if (colb || !sel) return HFTA_EUNSUPPORTED;
    if (d.a_kc && d.b_kc) launch_big<true, true, bf16_raw, false, BIG_SEL>(a, n16, grid, st);
    else if (!d.a_kc && !d.b_kc) launch_big<false, false, bf16_raw, false, BIG_SEL>(a, n16, grid, st);
    else return HFTA_EUNSUPPORTED;
  }
  return launch_status();
}

}  // namespace hfta
