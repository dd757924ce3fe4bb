// Fused Conv2d with groups = B (placeholder until the implicit-GEMM kernel lands).
#include "common.h"
using namespace hfta;
extern "C" {
int hfta_conv2d_grouped_fwd(int, int, int, int, int, int, int, int, int, int, int, const void*, const void*, const void*,
                            void*, int, float, void*) { return HFTA_EUNSUPPORTED; }
size_t hfta_conv2d_grouped_bwd_workspace_bytes(int, int, int, int, int, int, int, int, int, int, int) { return 0; }
int hfta_conv2d_grouped_bwd(int, int, int, int, int, int, int, int, int, int, int, const void*, const void*, const void*,
                            void*, float*, float*, void*, size_t, void*) { return HFTA_EUNSUPPORTED; }
}
