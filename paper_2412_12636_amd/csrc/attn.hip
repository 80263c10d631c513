// Causal attention entry points: argument checks and dispatch between the MFMA flash-style
// kernels (bf16, head size 128) and the plain-ALU kernels (everything else).
#include "attn.h"
#include "../../include/tm_ops.h"

using namespace tmk;

static int check_attn(const char *what, int dtype, int64_t seq, int64_t batch, int64_t nq, int64_t nkv, int64_t d) {
  if (dtype != TM_DTYPE_FP32 && dtype != TM_DTYPE_BF16) return fail(TM_EINVAL, "%s: unknown dtype %d", what, dtype);
  if (seq <= 0 || batch <= 0 || nq <= 0 || nkv <= 0 || d <= 0) return fail(TM_EINVAL, "%s: empty shape", what);
  if (nq % nkv) return fail(TM_ESIZE, "%s: %lld query heads are not a multiple of %lld kv heads", what, (long long)nq, (long long)nkv);
  if (d % 8 || d > 256) return fail(TM_ESIZE, "%s: head size %lld must be a multiple of 8, at most 256", what, (long long)d);
  if (nq > 65535 || batch > 65535) return fail(TM_ESIZE, "%s: more than 65535 heads or batch entries", what);
  if (seq * batch * (nq + 2 * nkv) * d >= (1LL << 40)) return fail(TM_ESIZE, "%s: tensor too large", what);
  if (!attn_mfma_supported(dtype, d) && seq > attn_generic_max_seq())
    return fail(TM_ESIZE, "%s: sequences above %d need bf16 with head size 128", what, attn_generic_max_seq());
  return TM_OK;
}

extern "C" int tm_op_attn_fwd(int dtype, int64_t seq, int64_t batch, int64_t nq, int64_t nkv, int64_t d,
                              const void *qkv, void *ctx, float *lse, void *stream) {
  if (int e = check_attn("attn_fwd", dtype, seq, batch, nq, nkv, d)) return e;
  if (!qkv || !ctx || !lse) return fail(TM_EINVAL, "attn_fwd: NULL pointer");
  hipStream_t s = (hipStream_t)stream;
  if (attn_mfma_supported(dtype, d)) return attn_fwd_mfma_launch(seq, batch, nq, nkv, d, qkv, ctx, lse, s);
  return attn_fwd_generic_launch(dtype, seq, batch, nq, nkv, d, qkv, ctx, lse, s);
}

extern "C" int64_t tm_op_attn_bwd_scratch_bytes(int dtype, int64_t seq, int64_t batch, int64_t nq, int64_t nkv,
                                                int64_t d) {
  if (int e = check_attn("attn_bwd_scratch_bytes", dtype, seq, batch, nq, nkv, d)) return e;
  const int64_t dvec = (batch * nq * seq + 63) / 64 * 64;  // the row statistics D, padded to 256 bytes
  const int64_t part = attn_mfma_supported(dtype, d) ? attn_bwd_mfma_partial_floats(seq, batch, nq, nkv) : 0;
  return (dvec + part) * (int64_t)sizeof(float);
}

extern "C" int tm_op_attn_bwd(int dtype, int64_t seq, int64_t batch, int64_t nq, int64_t nkv, int64_t d,
                              const void *qkv, const void *ctx, const void *dctx, const float *lse, void *scratch,
                              void *dqkv, void *stream) {
  if (int e = check_attn("attn_bwd", dtype, seq, batch, nq, nkv, d)) return e;
  if (!qkv || !ctx || !dctx || !lse || !scratch || !dqkv) return fail(TM_EINVAL, "attn_bwd: NULL pointer");
  if (((uintptr_t)scratch) & 15) return fail(TM_EALIGN, "attn_bwd: scratch must be 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  float *dvec = (float *)scratch;
  float *part = dvec + (batch * nq * seq + 63) / 64 * 64;
  if (int e = attn_dvec_launch(dtype, seq, batch, nq, nkv, d, ctx, dctx, dvec, s)) return e;
  if (attn_mfma_supported(dtype, d))
    return attn_bwd_mfma_launch(seq, batch, nq, nkv, d, qkv, dctx, lse, dvec, part, dqkv, s);
  return attn_bwd_generic_launch(dtype, seq, batch, nq, nkv, d, qkv, dctx, lse, dvec, dqkv, s);
}
