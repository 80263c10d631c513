// Internal GEMM interface shared by the plain-ALU and the MFMA kernels.
#pragma once
#include "common.h"

namespace tmk {

// C[m,n] = sum_k A(m,k) * B(n,k) with A(m,k) = A[m*a_rs + k*a_cs], B(n,k) = B[n*b_rs + k*b_cs].
// accumulate_f32 == false: C (stage dtype, row stride ldc) = result (+ bias[n]) (+ residual[m*ldc + n])
// accumulate_f32 == true : C is fp32 and the result is added to it (weight gradients)
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
  bool accumulate_f32;
};

int gemm_generic(int dtype, const GemmArgs &g, hipStream_t s);

// bf16 operands through the matrix cores.  Needs: one of each operand's strides equal to 1, the
// other a multiple of 8; the extent along each operand's contiguous axis a multiple of 8;
// 16-byte aligned base pointers.
bool gemm_mfma_supported(const GemmArgs &g);
int gemm_mfma(const GemmArgs &g, hipStream_t s);
void gemm_pick_tile(int64_t M, int64_t N, int &bm, int &bn);

}  // namespace tmk
