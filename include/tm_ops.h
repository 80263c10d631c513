/*
 * tm_ops.h - the individual steps of the stage-shard iteration, one C entry
 * point per step, as the stage functions of tm_stage.h enqueue them.
 *
 * The shadow iteration of TrainMover's sandbox (arXiv 2412.12636, section 4.2)
 * is, for a middle pipeline stage (section 6.1), a chain of these operations
 * per transformer block.  They are exported separately so that each can be
 * checked and timed on its own at the real shard shapes.
 *
 * Common rules: every pointer is a DEVICE pointer, caller-owned, 16-byte
 * aligned; matrices are dense row-major; `dtype` is TM_DTYPE_FP32 or
 * TM_DTYPE_BF16 and names the storage type of every `void*` tensor (gradient
 * accumulators, statistics and scratch are always fp32); `stream` is a
 * hipStream_t.  Nothing is allocated and the device is never synchronised.
 * Return value: tm_status_t.  Row widths must be multiples of 8.
 */
#ifndef TM_OPS_H
#define TM_OPS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The bf16 products choose among tm_gemm_config_count() tile configurations (by a cost model, or by measurement after
 * tm_stage_tune); every configuration adds the terms of an output element in the same order, so the choice changes
 * speed only.  tm_gemm_force_config(i) makes every later product of the process use configuration i (products whose
 * reduction length is not a multiple of 64 keep their own kernel); -1 restores the automatic choice.  A testing and
 * tuning aid; not thread-safe. */
int tm_gemm_config_count(void);
int tm_gemm_force_config(int index);

/* y[T,N] = x[T,K] w[N,K]^T (+ bias[N]) (+ residual[T,N]).  bias, residual may be NULL;
 * residual may alias y.  (Linear maps of the block; the residual form is the row-parallel
 * projection whose all-reduce is the identity.) */
int tm_op_linear_fwd(int dtype, int64_t T, int64_t N, int64_t K, const void *x, const void *w,
                     const void *bias, const void *residual, void *y, void *stream);

/* dx[T,K] = dy[T,N] w[N,K]   (input gradient of the linear map) */
int tm_op_linear_dgrad(int dtype, int64_t T, int64_t N, int64_t K, const void *dy, const void *w,
                       void *dx, void *stream);

/* The same product with scratch: where the output has few tiles and the reduction is long (the
 * out-projection's input gradient at a tensor-parallel shard) the reduction is split into parts that fill
 * the chip, their fp32 results are added in part order and rounded once.  Whether it splits depends on
 * the shape only (tm_op_linear_dgrad_scratch_bytes > 0); with less scratch than that, or NULL, this is
 * tm_op_linear_dgrad.  The two differ by fp32 summation order where it splits. */
int64_t tm_op_linear_dgrad_scratch_bytes(int dtype, int64_t T, int64_t N, int64_t K);
int tm_op_linear_dgrad_ws(int dtype, int64_t T, int64_t N, int64_t K, const void *dy, const void *w,
                          void *dx, void *scratch, int64_t scratch_bytes, void *stream);

/* Weight gradient in fp32: dw[N,K] += dy[T,N]^T x[T,K] when accumulate != 0, dw = ... otherwise
 * (the old contents are then not read). */
int tm_op_linear_wgrad(int dtype, int64_t T, int64_t N, int64_t K, const void *dy, const void *x,
                       float *dw, int accumulate, void *stream);

/* Bytes of fp32 scratch the reductions below need for a [T, width] input. */
int64_t tm_op_reduce_scratch_bytes(int64_t T, int64_t width);

/* db[N] (+)= sum over rows of dy[T,N]; fixed summation order (bit-reproducible); accumulate as above. */
int tm_op_bias_grad(int dtype, int64_t T, int64_t N, const void *dy, float *db, void *scratch,
                    int accumulate, void *stream);

/* LayerNorm / RMSNorm over rows of x[T,h]: out = gain*xhat (+ offset); writes mean[T]
 * (LayerNorm only, may be NULL for RMSNorm) and rstd[T]. */
int tm_op_norm_fwd(int dtype, int kind, int64_t T, int64_t h, double eps, const void *x,
                   const void *gain, const void *offset, void *out, float *mean, float *rstd,
                   void *stream);

/* dx[T,h] = (dres or 0) + gradient of the norm w.r.t. x for output gradient dout; dgain[h] (+)=,
 * doffset[h] (+)= (LayerNorm), accumulate as above.  dres may be NULL and may alias dx.
 * scratch: see above with width 3h. */
int tm_op_norm_bwd(int dtype, int kind, int64_t T, int64_t h, const void *dout, const void *x,
                   const float *mean, const float *rstd, const void *gain, const void *dres,
                   void *dx, float *dgain, float *doffset, void *scratch, int accumulate, void *stream);

/* As tm_op_norm_bwd, and dx_colsum[h] (+)= column sums of dx as stored: when dx is the output gradient of a linear map
 * with a bias (dres = that map's output gradient path), this is the bias gradient, without another pass over dx. */
int tm_op_norm_bwd_colsum(int dtype, int kind, int64_t T, int64_t h, const void *dout, const void *x,
                          const float *mean, const float *rstd, const void *gain, const void *dres,
                          void *dx, float *dgain, float *doffset, float *dx_colsum, void *scratch, int accumulate,
                          void *stream);

/* g[T,f] = gelu(u[T,f])  or  silu(u[T,0:f]) * u[T,f:2f]  for TM_ACT_SWIGLU (u is [T,2f]). */
int tm_op_act_fwd(int dtype, int act, int64_t T, int64_t f, const void *u, void *g, void *stream);

/* du = gradient of the activation; du has u's shape; du may alias dg only for the GeLU forms. */
int tm_op_act_bwd(int dtype, int act, int64_t T, int64_t f, const void *dg, const void *u, void *du,
                  void *stream);

/* Rotates, in place, the first n_heads heads of width d in every row of buf[seq*batch, row_width]
 * (token row = position*batch + entry) by angle position * theta^(-2j/d) for pair (j, j+d/2);
 * inverse != 0 rotates by the negative angle (the backward map). */
int tm_op_rotary(int dtype, int64_t seq, int64_t batch, int64_t n_heads, int64_t d, int64_t row_width,
                 double theta, int inverse, void *buf, void *stream);

/* Causal softmax attention.  qkv[T, (nq+2nkv)*d] holds Q heads, K heads, V heads side by side
 * (already rotated); query head g reads kv head g / (nq/nkv).  ctx[T, nq*d];
 * lse[batch, nq, seq] = log-sum-exp of the scaled scores of each query row. */
int tm_op_attn_fwd(int dtype, int64_t seq, int64_t batch, int64_t nq, int64_t nkv, int64_t d,
                   const void *qkv, void *ctx, float *lse, void *stream);

/* Bytes of scratch tm_op_attn_bwd needs: the row statistics D = rowsum(dctx * ctx) [batch, nq, seq] fp32
 * and, when query heads share kv heads, one fp32 partial of dK and dV per query head.  Negative: status. */
int64_t tm_op_attn_bwd_scratch_bytes(int dtype, int64_t seq, int64_t batch, int64_t nq, int64_t nkv,
                                     int64_t d);

/* dqkv (same layout as qkv) from dctx; scratch: see above, 16-byte aligned, contents undefined afterwards. */
int tm_op_attn_bwd(int dtype, int64_t seq, int64_t batch, int64_t nq, int64_t nkv, int64_t d,
                   const void *qkv, const void *ctx, const void *dctx, const float *lse, void *scratch,
                   void *dqkv, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TM_OPS_H */
