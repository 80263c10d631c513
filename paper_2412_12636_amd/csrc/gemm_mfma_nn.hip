// MFMA GEMM kernels for one operand layout (see gemm_mfma_impl.h).
#include "gemm_mfma_impl.h"

namespace tmk {
TM_GEMM_INSTANTIATE(true, false, 0)
TM_GEMM_INSTANTIATE_ONE(128, 192, 2, 2, true, false, 2)  // fp32 partial results of a split reduction
template __global__ void gemm_ldw_kernel<256, 192, GEMM_BK, 4, 2, 4, true, false, 2>(const MfmaGemmParams);
int gemm_mfma_nn(const GemmArgs &g, int config, hipStream_t s) { return launch_layout<true, false, 0>(g, config, s); }
// large: 256x192 tiles of the kernel with loader waves (one block per compute unit), else 128x192 tiles, two per unit
int gemm_mfma_nn_partial(const GemmArgs &g, bool large, hipStream_t s) {
  return large ? launch_ldw<256, 192, 4, 2, 4, true, false, 2>(g, s) : launch_pipe<128, 192, 2, 2, true, false, 2>(g, s);
}
}  // namespace tmk
