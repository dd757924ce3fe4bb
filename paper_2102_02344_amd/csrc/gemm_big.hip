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
