// Internal attention interface: plain-ALU kernels and the MFMA flash-style kernels.
#pragma once
#include "common.h"

namespace tmk {

int attn_generic_max_seq();
int attn_fwd_generic_launch(int dtype, int64_t seq, int64_t batch, int64_t nq, int64_t nkv, int64_t d,
                            const void *qkv, void *ctx, float *lse, hipStream_t s);
int attn_dvec_launch(int dtype, int64_t seq, int64_t batch, int64_t nq, int64_t nkv, int64_t d, const void *ctx,
                     const void *dctx, float *dvec, hipStream_t s);
int attn_bwd_generic_launch(int dtype, int64_t seq, int64_t batch, int64_t nq, int64_t nkv, int64_t d,
                            const void *qkv, const void *dctx, const float *lse, const float *dvec, void *dqkv,
                            hipStream_t s);

// bf16, head size 128
bool attn_mfma_supported(int dtype, int64_t d);
int attn_fwd_mfma_launch(int64_t seq, int64_t batch, int64_t nq, int64_t nkv, int64_t d, const void *qkv, void *ctx,
                         float *lse, hipStream_t s);
// fp32 elements of the partial buffer the backward kernels need (0 unless query heads share kv heads)
int64_t attn_bwd_mfma_partial_floats(int64_t seq, int64_t batch, int64_t nq, int64_t nkv);
int attn_bwd_mfma_launch(int64_t seq, int64_t batch, int64_t nq, int64_t nkv, int64_t d, const void *qkv,
                         const void *dctx, const float *lse, const float *dvec, float *part, void *dqkv,
                         hipStream_t s);

}  // namespace tmk
