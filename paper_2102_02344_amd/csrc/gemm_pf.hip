// Instantiations and launcher of the deep-prefetch 128x128 bf16 GEMM kernel.
#include "gemm_pf.h"

namespace hfta {

#ifndef HFTA_GEMM_PF_DEPTH
#define HFTA_GEMM_PF_DEPTH 2
#endif
constexpr int PF_DEPTH = HFTA_GEMM_PF_DEPTH;

template <bool A_KC, bool B_KC, bool V16>
static void launch_pf(const GemmDesc& d, const GemmArgs& a, dim3 grid, hipStream_t st) {
  if (d.out_f32 || d.splits > 1)
    hipLaunchKernelGGL((gemm_pf_kernel<A_KC, B_KC, float, V16, PF_DEPTH>), grid, dim3(GEMM_THREADS), 0, st, a);
  else
    hipLaunchKernelGGL((gemm_pf_kernel<A_KC, B_KC, bf16_raw, V16, PF_DEPTH>), grid, dim3(GEMM_THREADS), 0, st, a);
}

int gemm_pf_launch(const GemmDesc& d, const GemmArgs& a, bool v16, dim3 grid, hipStream_t st) {
  if (d.a_kc && !d.b_kc) { if (v16) launch_pf<true, false, true>(d, a, grid, st); else launch_pf<true, false, false>(d, a, grid, st); }
  else if (d.a_kc && d.b_kc) { if (v16) launch_pf<true, true, true>(d, a, grid, st); else launch_pf<true, true, false>(d, a, grid, st); }
  else if (!d.a_kc && !d.b_kc) launch_pf<false, false, false>(d, a, grid, st);
  else return HFTA_EUNSUPPORTED;
  return launch_status();
}

}  // namespace hfta
