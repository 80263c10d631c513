// The three products of a linear map y = x W^T + b, dispatched to the MFMA kernels (bf16) or the
// plain-ALU kernel (fp32, and bf16 shapes the MFMA path does not take).
#include "gemm.h"
#include "../../include/tm_ops.h"

using namespace tmk;

static int check_linear(const char *what, int dtype, int64_t T, int64_t N, int64_t K) {
  if (dtype != TM_DTYPE_FP32 && dtype != TM_DTYPE_BF16) return fail(TM_EINVAL, "%s: unknown dtype %d", what, dtype);
  if (T <= 0 || N <= 0 || K <= 0)
    return fail(TM_EINVAL, "%s: empty shape T=%lld N=%lld K=%lld", what, (long long)T, (long long)N, (long long)K);
  if (N % 8 || K % 8) return fail(TM_ESIZE, "%s: N=%lld and K=%lld must be multiples of 8", what, (long long)N, (long long)K);
  if (T > 0x7fffffffLL || N > 0x7fffffffLL || K > 0x7fffffffLL) return fail(TM_ESIZE, "%s: dimension above 2^31", what);
  return TM_OK;
}

static int run(int dtype, const GemmArgs &g, hipStream_t s) {
  if (dtype == TM_DTYPE_BF16 && gemm_mfma_supported(g)) return gemm_mfma(g, s);
  return gemm_generic(dtype, g, s);
}

extern "C" int tm_op_linear_fwd(int dtype, int64_t T, int64_t N, int64_t K, const void *x, const void *w,
                                const void *bias, const void *residual, void *y, void *stream) {
  if (int e = check_linear("linear_fwd", dtype, T, N, K)) return e;
  if (!x || !w || !y) return fail(TM_EINVAL, "linear_fwd: NULL pointer");
  GemmArgs g{T, N, K, x, K, 1, w, K, 1, y, N, bias, residual, 0};
  return run(dtype, g, (hipStream_t)stream);
}

extern "C" int tm_op_linear_dgrad(int dtype, int64_t T, int64_t N, int64_t K, const void *dy, const void *w, void *dx,
                                  void *stream) {
  if (int e = check_linear("linear_dgrad", dtype, T, N, K)) return e;
  if (!dy || !w || !dx) return fail(TM_EINVAL, "linear_dgrad: NULL pointer");
  // dx[t,k] = sum_n dy[t,n] w[n,k]: reduction over n; w is read along its strided axis
  GemmArgs g{T, K, N, dy, N, 1, w, 1, K, dx, K, nullptr, nullptr, 0};
  return run(dtype, g, (hipStream_t)stream);
}

extern "C" int64_t tm_op_linear_dgrad_scratch_bytes(int dtype, int64_t T, int64_t N, int64_t K) {
  if (int e = check_linear("linear_dgrad_scratch_bytes", dtype, T, N, K)) return e;
  if (dtype != TM_DTYPE_BF16) return 0;
  GemmArgs g{T, K, N, nullptr, N, 1, nullptr, 1, K, nullptr, K, nullptr, nullptr, 0};
  return gemm_mfma_splitk_bytes(g);
}

extern "C" int tm_op_linear_dgrad_ws(int dtype, int64_t T, int64_t N, int64_t K, const void *dy, const void *w,
                                     void *dx, void *scratch, int64_t scratch_bytes, void *stream) {
  if (int e = check_linear("linear_dgrad", dtype, T, N, K)) return e;
  if (!dy || !w || !dx) return fail(TM_EINVAL, "linear_dgrad: NULL pointer");
  GemmArgs g{T, K, N, dy, N, 1, w, 1, K, dx, K, nullptr, nullptr, 0};
  g.splitk_scratch = scratch;
  g.splitk_bytes = scratch ? scratch_bytes : 0;
  return run(dtype, g, (hipStream_t)stream);
}

extern "C" int tm_op_linear_wgrad(int dtype, int64_t T, int64_t N, int64_t K, const void *dy, const void *x, float *dw,
                                  int accumulate, void *stream) {
  if (int e = check_linear("linear_wgrad", dtype, T, N, K)) return e;
  if (!dy || !x || !dw) return fail(TM_EINVAL, "linear_wgrad: NULL pointer");
  // dw[n,k] (+)= sum_t dy[t,n] x[t,k]: reduction over tokens, both operands read along their strided axis
  GemmArgs g{N, K, T, dy, 1, N, x, 1, K, dw, K, nullptr, nullptr, accumulate ? 1 : 2};
  return run(dtype, g, (hipStream_t)stream);
}

namespace tmk {
bool linear_wgrad_adam_supported(int64_t T, int64_t N, int64_t K, const void *dy, const void *x, const float *dw) {
  if (T <= 0 || N <= 0 || K <= 0 || T % 64 != 0) return false;
  GemmArgs g{N, K, T, dy, 1, N, x, 1, K, const_cast<float *>(dw), K, nullptr, nullptr, 3};
  return gemm_mfma_supported(g);
}
int linear_wgrad_adam(int64_t T, int64_t N, int64_t K, const void *dy, const void *x, float *dw, const AdamTarget &target,
                      hipStream_t s) {
  if (!linear_wgrad_adam_supported(T, N, K, dy, x, dw)) return fail(TM_ESIZE, "linear_wgrad_adam: shape not supported");
  GemmArgs g{N, K, T, dy, 1, N, x, 1, K, dw, K, nullptr, nullptr, 3};
  g.adam = &target;
  return gemm_mfma(g, s);
}
}  // namespace tmk

extern "C" int tm_gemm_config_count(void) { return gemm_mfma_config_count(); }
extern "C" int tm_gemm_force_config(int index) { return gemm_mfma_force_config(index); }
