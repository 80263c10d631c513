// Plain-ALU tiled GEMM with arbitrary strides: the fp32 stage dtype and bf16 shapes the MFMA
// kernels do not take.  64x64 output tile per 256-thread block, 4x4 outputs per thread,
// fp32 fused multiply-adds, operands staged through LDS 16 reduction steps at a time.
#include "gemm.h"

namespace tmk {

constexpr int GT = 64, GK = 16;

// C[m,n] = sum_k A(m,k) B(n,k), A(m,k) = A[m*a_rs + k*a_cs], B(n,k) = B[n*b_rs + k*b_cs]
// EPI 0: C = acc (+bias[n]) (+residual[m,n]) stored as TC ; EPI 1: C(fp32) += acc ; EPI 2: C(fp32) = acc
template <typename TA, typename TC, int EPI>
__global__ __launch_bounds__(256) void gemm_generic_kernel(int M, int N, int K, const TA *__restrict__ A,
                                                          int64_t a_rs, int64_t a_cs, const TA *__restrict__ B,
                                                          int64_t b_rs, int64_t b_cs, TC *C, int64_t ldc,
                                                          const TA *__restrict__ bias, const TA *residual) {
  __shared__ float As[GK][GT + 4], Bs[GK][GT + 4];
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  const int m0 = blockIdx.y * GT, n0 = blockIdx.x * GT;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += GK) {
    // 64 x 16 elements per operand, 4 per thread
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = threadIdx.x + i * 256;
      int r, kk;
      if (a_cs == 1) { kk = e % GK; r = e / GK; } else { r = e % GT; kk = e / GT; }
      float v = 0.f;
      if (m0 + r < M && k0 + kk < K) v = to_f32(A[(int64_t)(m0 + r) * a_rs + (int64_t)(k0 + kk) * a_cs]);
      As[kk][r] = v;
      if (b_cs == 1) { kk = e % GK; r = e / GK; } else { r = e % GT; kk = e / GT; }
      v = 0.f;
      if (n0 + r < N && k0 + kk < K) v = to_f32(B[(int64_t)(n0 + r) * b_rs + (int64_t)(k0 + kk) * b_cs]);
      Bs[kk][r] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < GK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[i] = As[kk][ty * 4 + i];
        b[i] = Bs[kk][tx * 4 + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      float v = acc[i][j];
      if (EPI == 0) {
        if (bias) v += to_f32(bias[n]);
        if (residual) v += to_f32(residual[(int64_t)m * ldc + n]);
        C[(int64_t)m * ldc + n] = from_f32<TC>(v);
      } else if (EPI == 1) {
        C[(int64_t)m * ldc + n] = from_f32<TC>(to_f32(C[(int64_t)m * ldc + n]) + v);
      } else {
        C[(int64_t)m * ldc + n] = from_f32<TC>(v);
      }
    }
  }
}

template <typename T>
static int launch_generic(const GemmArgs &g, hipStream_t s) {
  dim3 grid((unsigned)ceil_div(g.N, GT), (unsigned)ceil_div(g.M, GT));
  g_last_kernel = "gemm_generic_kernel";
  if (g.c_mode == 1)
    gemm_generic_kernel<T, float, 1><<<grid, 256, 0, s>>>((int)g.M, (int)g.N, (int)g.K, (const T *)g.A, g.a_rs, g.a_cs,
                                                          (const T *)g.B, g.b_rs, g.b_cs, (float *)g.C, g.ldc, nullptr,
                                                          nullptr);
  else if (g.c_mode == 2)
    gemm_generic_kernel<T, float, 2><<<grid, 256, 0, s>>>((int)g.M, (int)g.N, (int)g.K, (const T *)g.A, g.a_rs, g.a_cs,
                                                          (const T *)g.B, g.b_rs, g.b_cs, (float *)g.C, g.ldc, nullptr,
                                                          nullptr);
  else
    gemm_generic_kernel<T, T, 0><<<grid, 256, 0, s>>>((int)g.M, (int)g.N, (int)g.K, (const T *)g.A, g.a_rs, g.a_cs,
                                                      (const T *)g.B, g.b_rs, g.b_cs, (T *)g.C, g.ldc,
                                                      (const T *)g.bias, (const T *)g.residual);
  return check_launch("gemm_generic");
}

int gemm_generic(int dtype, const GemmArgs &g, hipStream_t s) {
  return dtype == TM_DTYPE_BF16 ? launch_generic<bf16>(g, s) : launch_generic<float>(g, s);
}

}  // namespace tmk
