// Internal GEMM interface shared by the plain-ALU and the MFMA kernels.
#pragma once
#include "adam.h"
#include "common.h"

namespace tmk {

// C[m,n] = sum_k A(m,k) * B(n,k) with A(m,k) = A[m*a_rs + k*a_cs], B(n,k) = B[n*b_rs + k*b_cs].
// c_mode 0: C (stage dtype, row stride ldc) = result (+ bias[n]) (+ residual[m*ldc + n])
// c_mode 1: C is fp32 and the result is added to it (weight gradients, accumulating)
// c_mode 2: C is fp32 and is overwritten with the result (first micro-batch of an iteration)
// c_mode 3: as 2, and the epilogue applies the Adam update of `adam` with the result as the gradient (the gradient is
//           still stored; what is saved is reading it back, and the update overlaps the products of other blocks)
struct GemmArgs {
  int64_t M, N, K;
  const void *A;
  int64_t a_rs, a_cs;
  const void *B;
  int64_t b_rs, b_cs;
  void *C;
  int64_t ldc;
  const void *bias;
  const void *residual;
  int c_mode;
  // Split reduction (dx = dy W with few output tiles).  Caller side: scratch for the fp32 partial results;
  // gemm_mfma() decides from the shape whether to use it (gemm_mfma_splitk_bytes says how much it wants).
  void *splitk_scratch = nullptr;
  int64_t splitk_bytes = 0;
  // Kernel side: block row y of the grid reduces over the y-th of k_splits equal parts of K and writes the
  // y-th of k_splits results [M, ldc] behind C (c_mode 2).
  int k_splits = 1;
  const AdamTarget *adam = nullptr;  // c_mode 3
};

int gemm_generic(int dtype, const GemmArgs &g, hipStream_t s);

// bf16 operands through the matrix cores.  Needs: one of each operand's strides equal to 1, the
// other a multiple of 8; the extent along each operand's contiguous axis a multiple of 8;
// 16-byte aligned base pointers.
bool gemm_mfma_supported(const GemmArgs &g);
int gemm_mfma(const GemmArgs &g, hipStream_t s);
// Bytes of scratch with which gemm_mfma() would split this product's reduction (0: it would not).
int64_t gemm_mfma_splitk_bytes(const GemmArgs &g);
// Measures the tile configurations for one layout and shape, on n instances of the product that live
// in different memory (the launches cycle through them), and makes later gemm_mfma() calls of that layout
// and shape use the fastest.  Overwrites every C; waits for the stream.  Without it a cost model picks.
int gemm_mfma_tune(const GemmArgs *variants, int n, hipStream_t s);
// Number of tile configurations, and a process-wide override (index, or -1 for the automatic choice).
// dw[N,K] = dy[T,N]^T x[T,K] (bf16 operands) with the Adam update of those N*K parameters in the product's
// epilogue.  `supported` says whether the shapes and pointers allow it (matrix-core path, T a multiple of 64).
bool linear_wgrad_adam_supported(int64_t T, int64_t N, int64_t K, const void *dy, const void *x, const float *dw);
int linear_wgrad_adam(int64_t T, int64_t N, int64_t K, const void *dy, const void *x, float *dw, const AdamTarget &target,
                      hipStream_t s);
int gemm_mfma_config_count();
int gemm_mfma_force_config(int index);

}  // namespace tmk
