// MFMA GEMM kernels for one operand layout (see gemm_mfma_impl.h).
#include "gemm_mfma_impl.h"

namespace tmk {
TM_GEMM_INSTANTIATE(true, false, 0)
TM_GEMM_INSTANTIATE_ONE(128, 192, 2, 2, true, false, 2)  // fp32 partial results of a split reduction
int gemm_mfma_nn(const GemmArgs &g, int config, hipStream_t s) { return launch_layout<true, false, 0>(g, config, s); }
int gemm_mfma_nn_partial(const GemmArgs &g, hipStream_t s) { return launch_pipe<128, 192, 2, 2, true, false, 2>(g, s); }
}  // namespace tmk
