// Instantiations and launcher of the deep-prefetch 128x128 bf16 GEMM kernel.
#include "gemm_pf.h"

namespace hfta {

#ifndef HFTA_GEMM_PF_DEPTH
#define HFTA_GEMM_PF_DEPTH 2
#endif
constexpr int PF_DEPTH = HFTA_GEMM_PF_DEPTH;

// V16: k-contiguous operands load in 16-byte pieces; N16: the same for operands contiguous along m / n
template <bool A_KC, bool B_KC, bool V16, bool N16>
static void launch_pf(const GemmDesc& d, const GemmArgs& a, dim3 grid, hipStream_t st) {
  if (d.out_f32 || d.splits > 1)
    hipLaunchKernelGGL((gemm_pf_kernel<A_KC, B_KC, float, V16, PF_DEPTH, N16>), grid, dim3(GEMM_THREADS), 0, st, a);
  else
    hipLaunchKernelGGL((gemm_pf_kernel<A_KC, B_KC, bf16_raw, V16, PF_DEPTH, N16>), grid, dim3(GEMM_THREADS), 0, st, a);
}

int gemm_pf_launch(const GemmDesc& d, const GemmArgs& a, bool v16, bool n16, dim3 grid, hipStream_t st) {
  if (d.a_kc && !d.b_kc) {
    if (v16 && n16) launch_pf<true, false, true, true>(d, a, grid, st);
    else if (v16) launch_pf<true, false, true, false>(d, a, grid, st);
    else if (n16) launch_pf<true, false, false, true>(d, a, grid, st);
    else launch_pf<true, false, false, false>(d, a, grid, st);
  } else if (d.a_kc && d.b_kc) {
    if (v16) launch_pf<true, true, true, false>(d, a, grid, st); else launch_pf<true, true, false, false>(d, a, grid, st);
  } else if (!d.a_kc && !d.b_kc) {
    if (n16) launch_pf<false, false, false, true>(d, a, grid, st); else launch_pf<false, false, false, false>(d, a, grid, st);
  } else return HFTA_EUNSUPPORTED;
  return launch_status();
}

}  // namespace hfta
