/*
 * tm_moe.h - one rank's mixture-of-experts MLP shard.
 *
 * TrainMover's largest workloads (arXiv 2412.12636, Table 3: 960B to 5.12T parameters, expert parallelism 2 to 16)
 * are mixture-of-experts GPT models.  Section 4.2 observes that token routing depends on the input, but that the
 * frameworks pre-allocate fixed-size expert buffers whatever the routing decides, so the memory layout and the
 * communication structure stay static and the sandboxed shadow iteration covers them.  This is that layer, in the
 * form a rank runs inside the sandbox: every collective is served locally (the token all-to-all is the identity).
 * It takes the place of the dense MLP of tm_stage.h: input c[T, h] (the normalised residual stream), output
 * out[T, h] (what is added to the residual stream).
 *
 *   router    logits[t, e] = c[t] . Wr[e] in fp32, E = n_experts global experts; the top_k largest logits of a token
 *             are chosen (ties: lower expert index first); gate = softmax over the chosen logits (fp32)
 *   dispatch  expert e owns a buffer of `capacity` rows; assignments are taken in token order (within a token in
 *             order of decreasing logit) and get the next free row of their expert's buffer; an assignment that
 *             finds the buffer full is dropped; unused rows are zero
 *   exchange  identity: the rank processes all E buffers, buffer e with its local expert e mod E_local, where
 *             E_local = n_experts / ep (global expert e is local expert e mod E_local of rank e div E_local)
 *   expert    o = gelu(buf W1^T + b1) W2^T + b2, one pass per local expert over its ep * capacity rows
 *   combine   out[t] = sum over the token's kept assignments of gate * o[its row], fp32, one rounding
 * Backward: the routing decision gets no gradient, the gates do.  Everything is reproducible bit for bit (no
 * atomics; every sum has a fixed order).
 *
 * Parameters (flat, dtype elements, every tensor 16-byte aligned): w_router [E, h]; then per local expert j:
 * w_fc1.j [f, h], b_fc1.j [f], w_fc2.j [h, f], b_fc2.j [h] (biases only with has_bias).  Gradients: fp32, same
 * element order.  The optimizer step is tm_adam_step_flat over the flat buffers.
 *
 * Common rules as in tm_ops.h: DEVICE pointers, caller-owned, 256-byte aligned; nothing is allocated, the device is
 * never synchronised; tm_status_t return values.
 */
#ifndef TM_MOE_H
#define TM_MOE_H

#include <stdint.h>

#include "tm_stage.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Constraints (TM_ESIZE / TM_EINVAL otherwise): hidden and ffn multiples of 8; 1 <= n_experts <= 64, a multiple of
 * ep; 1 <= top_k <= min(n_experts, 8); capacity >= 1; act TM_ACT_GELU_TANH or TM_ACT_GELU_ERF;
 * n_experts * capacity * max(hidden, ffn) elements below 2^31. */
typedef struct {
  int32_t tokens;     /* T = seq * micro_batch */
  int32_t hidden;
  int32_t ffn;        /* local width f of an expert's MLP (after the tensor-parallel slice) */
  int32_t n_experts;  /* E, global */
  int32_t ep;         /* expert-parallel size; the rank holds E / ep experts */
  int32_t top_k;
  int32_t capacity;   /* rows of one expert's buffer, e.g. ceil(capacity_factor * T * top_k / E) */
  int32_t dtype;      /* TM_DTYPE_* */
  int32_t act;
  int32_t has_bias;
} tm_moe_config_t;

int64_t tm_moe_param_count(const tm_moe_config_t *cfg);
/* index -1: number of tensors.  Names stay valid for the life of the calling thread. */
int tm_moe_param_layout(const tm_moe_config_t *cfg, int index, const char **name, int64_t *offset_elems, int64_t shape[2]);
int64_t tm_moe_workspace_bytes(const tm_moe_config_t *cfg);

/* Where tm_moe_fwd leaves its routing in the workspace (byte offset returned, size in *bytes), for inspection:
 * LOGITS fp32 [T, E]; TOP_IDX int32 [T, top_k]; GATES fp32 [T, top_k]; SLOT_ROW int32 [T, top_k] = row in the
 * library's buffer order or -1 when dropped, the buffer of global expert e starting at row
 * ((e mod E_local) * ep + e div E_local) * capacity. */
enum { TM_MOE_WS_LOGITS = 0, TM_MOE_WS_TOP_IDX = 1, TM_MOE_WS_GATES = 2, TM_MOE_WS_SLOT_ROW = 3 };
int64_t tm_moe_workspace_offset(const tm_moe_config_t *cfg, int region, int64_t *bytes);

/* out[T, h] from c[T, h]; the workspace keeps what the backward pass needs. */
int tm_moe_fwd(const tm_moe_config_t *cfg, const void *params, const void *c, void *out, void *workspace,
               int64_t workspace_bytes, void *stream);
/* dc[T, h] and grads (+)= from dout[T, h], after tm_moe_fwd on the same workspace with the same params and c.
 * accumulate == 0 overwrites grads. */
int tm_moe_bwd(const tm_moe_config_t *cfg, const void *params, const void *c, const void *dout, void *dc, float *grads,
               int accumulate, void *workspace, int64_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TM_MOE_H */
