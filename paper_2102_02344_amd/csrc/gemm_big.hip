// Instantiations and launcher of the 256x256 compute-bound GEMM kernel.
#include "gemm_big.h"

namespace hfta {

template <bool A_KC, bool B_KC>
static void launch_big(const GemmDesc& d, const GemmArgs& a, bool slow, dim3 grid, hipStream_t st) {
  if (d.out_f32) {
    if (slow) hipLaunchKernelGGL((gemm_big_kernel<A_KC, B_KC, float, true>), grid, dim3(BIG_THREADS), 0, st, a);
    else hipLaunchKernelGGL((gemm_big_kernel<A_KC, B_KC, float, false>), grid, dim3(BIG_THREADS), 0, st, a);
  } else {
    if (slow) hipLaunchKernelGGL((gemm_big_kernel<A_KC, B_KC, bf16_raw, true>), grid, dim3(BIG_THREADS), 0, st, a);
    else hipLaunchKernelGGL((gemm_big_kernel<A_KC, B_KC, bf16_raw, false>), grid, dim3(BIG_THREADS), 0, st, a);
  }
}

// `a` must carry tile counts for 256x256 tiles and 64-element k-tiles.
int gemm_big_launch(const GemmDesc& d, const GemmArgs& a, dim3 grid, hipStream_t st) {
  const bool slow = d.act == HFTA_ACT_TANH || d.act == HFTA_ACT_GELU || (d.bias && d.bias_mode == 2);
  if (d.a_kc && !d.b_kc) launch_big<true, false>(d, a, slow, grid, st);
  else if (d.a_kc && d.b_kc) launch_big<true, true>(d, a, slow, grid, st);
  else if (!d.a_kc && !d.b_kc) launch_big<false, false>(d, a, slow, grid, st);
  else return HFTA_EUNSUPPORTED;
  return launch_status();
}

}  // namespace hfta
