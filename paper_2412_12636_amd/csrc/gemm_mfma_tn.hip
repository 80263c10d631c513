// MFMA GEMM kernels for one operand layout (see gemm_mfma_impl.h).
#include "gemm_mfma_impl.h"

namespace tmk {
TM_GEMM_INSTANTIATE(false, false, 1)
TM_GEMM_INSTANTIATE(false, false, 2)
TM_GEMM_INSTANTIATE(false, false, 3)
int gemm_mfma_tn(const GemmArgs &g, int config, hipStream_t s) {
  if (g.c_mode == 3) {
    if (g.K % GEMM_BK != 0) return fail(TM_ESIZE, "gemm_mfma: the fused update needs a reduction length that is a multiple of 64");
    return launch_layout<false, false, 3>(g, config, s);
  }
  return g.c_mode == 2 ? launch_layout<false, false, 2>(g, config, s) : launch_layout<false, false, 1>(g, config, s);
}
}  // namespace tmk
