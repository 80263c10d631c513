/*
 * tm_roles.h - the layers that only the first and the last pipeline stage have.
 *
 * TrainMover's general standby (arXiv 2412.12636, section 6.2) warms up all three
 * pipeline roles; section 6.1 names what sets the first and the last stage apart
 * from the middle stages of tm_stage.h: the word-embedding layer and the output
 * layer, of one shape (weight tying).  These entry points are those layers in the
 * tensor-parallel form one rank runs inside the sandbox of section 4.2, i.e. with
 * every collective served locally (the identity):
 *
 *   first stage   x0[t] = W[token[t] - v0] if the token lies in this rank's rows
 *                 [v0, v0 + v_local) of the vocabulary, else 0; plus P[position]
 *                 where the model has learned positions.  Feed x0 to tm_stage_fwd.
 *   last stage    final norm -> logits = hn W^T over the rank's v_local rows ->
 *                 cross-entropy over that shard: loss_t = log sum exp(logits[t,:])
 *                 - (logits[t, target - v0] if the target is local, else 0);
 *                 loss = mean over tokens.  Take tm_stage_fwd's y, hand dy to
 *                 tm_stage_bwd.
 *
 * Common rules as in tm_ops.h: DEVICE pointers, caller-owned, 16-byte aligned
 * (workspace 256); `dtype` names the storage type of every void* tensor;
 * gradients of parameters are fp32 and are added to when accumulate != 0,
 * overwritten otherwise; tokens and targets are int32 [seq*batch] in token-row
 * order (row = position*batch + entry), global vocabulary ids; nothing is
 * allocated, the device is never synchronised; return value tm_status_t.
 */
#ifndef TM_ROLES_H
#define TM_ROLES_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* x0[seq*batch, h] from w[v_local, h] and, if not NULL, pos_emb[>= seq, h]. */
int tm_op_embed_fwd(int dtype, int64_t seq, int64_t batch, int64_t h, int64_t v_local, int64_t v0,
                    const int32_t *tokens, const void *w, const void *pos_emb, void *x0, void *stream);

/* dw[v_local, h] (+)= rows of dx0 gathered by token, added in token order (reproducible; rows no token
 * names get zero).  dpos[n_pos, h] (+)= sums over batch entries, rows >= seq get zero; dpos may be NULL.
 * h at most 16384 (bf16) / 8192 (fp32). */
int tm_op_embed_bwd(int dtype, int64_t seq, int64_t batch, int64_t h, int64_t v_local, int64_t v0,
                    const int32_t *tokens, const void *dx0, float *dw, float *dpos, int64_t n_pos,
                    int accumulate, void *stream);

/* Cross-entropy over the shard: loss_t[T] and loss[0] = mean(loss_t) (fp32), and IN PLACE of logits[T, v_local]
 * their gradient dloss/T * (softmax - one-hot where the target is local).  v_local a multiple of 8. */
int tm_op_xent(int dtype, int64_t T, int64_t v_local, int64_t v0, void *logits, const int32_t *targets,
               double dloss, float *loss_t, float *loss, void *stream);

/* Last stage, forward and backward in one call: y[seq*batch, h] -> loss[0]; dy (gradient handed to the
 * blocks), dgain[h], doffset[h] (LayerNorm; NULL for RMSNorm), dw[v_local, h].  norm: TM_NORM_*.
 * workspace: tm_head_workspace_bytes() bytes, checked against workspace_bytes (TM_ESIZE). */
int64_t tm_head_workspace_bytes(int dtype, int64_t seq, int64_t batch, int64_t h, int64_t v_local);
int tm_head_fwd_bwd(int dtype, int norm, double eps, int64_t seq, int64_t batch, int64_t h, int64_t v_local,
                    int64_t v0, const void *y, const int32_t *targets, const void *gain, const void *offset,
                    const void *w, double dloss, void *workspace, int64_t workspace_bytes, float *loss, void *dy,
                    float *dgain, float *doffset, float *dw, int accumulate, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TM_ROLES_H */
