// MFMA GEMM kernels for one operand layout (see gemm_mfma_impl.h).
#include "gemm_mfma_impl.h"

namespace tmk {
TM_GEMM_INSTANTIATE(true, true, 0)
int gemm_mfma_nt(const GemmArgs &g, int config, hipStream_t s) { return launch_layout<true, true, 0>(g, config, s); }
}  // namespace tmk
