/*
 * tm_sandbox.h - the record / replay layer of the communication-free sandbox.
 *
 * TrainMover (arXiv 2412.12636, section 4.2) puts a hook between the training
 * framework and the collective library.  Pre-record step: on designated ranks
 * the hook stores the OUTPUT tensor of every collective call to persistent
 * storage once the call has completed.  Replay step: a joiner runs its shadow
 * iteration alone; a call that would reach outside the sandbox is answered with
 * the stored tensor, `send` and `barrier` are skipped (they do not change the
 * caller's state).  Section 4.3 narrows the scope to the communication edges
 * that cross the sandbox boundary: intra-machine tensor-parallel traffic runs
 * natively and is not recorded, and on replay only the boundary's entries are
 * loaded.
 *
 * Here the hook is a `tm_comm_t` that a stage calls at each of its collective
 * call sites (tm_stage_attach_comm).  On this one-GPU library "natively" means
 * what tm_stage.h already does: the call returns the rank's own tensor.
 *
 *   mode             scope in `scopes`                      scope not in `scopes`
 *   TM_COMM_PASS     native                                  native
 *   TM_COMM_RECORD   native, then the result is appended     native, nothing stored
 *                    to the tape file (recv, all-reduce)
 *   TM_COMM_REPLAY   recv / all-reduce: the tensor is        native; the tape's entries of
 *                    overwritten with the tape's next        such scopes are never loaded
 *                    entry; send / barrier: skipped
 *
 * A replayed call must match the tape's next entry in kind, scope, site and
 * byte count (the deterministic collective order the paper relies on);
 * otherwise TM_ESTATE and nothing is written.
 *
 * Call sites of a stage, in call order (tensors in the stage dtype, [seq*micro_batch, hidden]):
 *   tm_stage_fwd    recv x (pipeline); per layer all-reduce of ctx Wout^T and of g W2^T (tensor; the
 *                   map's bias and the residual are added afterwards); send y (pipeline)
 *   tm_stage_bwd    recv dy (pipeline); per layer all-reduce of du W1 and of dqkv Wqkv (tensor);
 *                   send dx (pipeline)
 *   tm_stage_grad_sync   all-reduce of the flat fp32 gradient buffer (data), then a barrier
 * With the tensor scope intercepted (recorded or replayed) the two forward products run without
 * their fused bias / residual epilogue and a separate kernel adds both after the hook, so the
 * partial sum is rounded to the stage dtype once more than in the fused form, as it would be
 * before a real all-reduce.
 *
 * Tape file (little endian): 16-byte header "TMTAPE01" + uint64 entry count (rewritten on close), then
 * per entry a 64-byte record {uint32 kind, scope, site, dtype; uint64 bytes, checksum; 32 bytes zero}
 * followed by the payload padded to a multiple of 64 bytes.  checksum: over the payload's 64-bit
 * words w_i (tail zero-padded), c = (c XOR w_i) * 0x100000001b3 mod 2^64 starting from
 * 0xcbf29ce484222325.  A tape whose checksum does not match its payload is refused at open.
 *
 * Device memory: none is allocated.  Host memory: recording stages through a pinned buffer of at most
 * 64 MiB; replay holds the boundary's entries in pinned host memory from open to close.  Recording
 * synchronises the stream at every stored call (the tensor must be complete before it is written:
 * the pre-record step runs once, at the start of a job); replay only enqueues host-to-device copies.
 * Return values and tm_last_error() as in tm_stage.h.
 */
#ifndef TM_SANDBOX_H
#define TM_SANDBOX_H

#include <stdint.h>

#include "tm_stage.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tm_comm tm_comm_t; /* opaque, host memory */

enum { TM_COMM_PASS = 0, TM_COMM_RECORD = 1, TM_COMM_REPLAY = 2 };
enum { TM_SCOPE_TP = 1, TM_SCOPE_PP = 2, TM_SCOPE_DP = 4 }; /* bit mask */
enum { TM_COLL_ALL_REDUCE = 0, TM_COLL_RECV = 1, TM_COLL_SEND = 2, TM_COLL_BARRIER = 3 };
enum {
  TM_SITE_X = 0, TM_SITE_Y = 1, TM_SITE_DY = 2, TM_SITE_DX = 3, TM_SITE_ATTN_OUT = 4, TM_SITE_MLP_OUT = 5,
  TM_SITE_D_MLP_IN = 6, TM_SITE_D_ATTN_IN = 7, TM_SITE_GRADS = 8, TM_SITE_STEP_END = 9
};

typedef struct {
  int64_t calls;          /* all calls seen */
  int64_t stored;         /* record: entries written; replay: entries served */
  int64_t stored_bytes;
  int64_t skipped;        /* replay: send / barrier calls on the boundary */
  int64_t native;         /* calls left to run natively */
  int64_t tape_entries;   /* replay: entries loaded (boundary scopes only); record: entries so far */
  int64_t tape_bytes;     /* payload bytes of those */
} tm_comm_stats_t;

/* path: the tape file (host string; ignored for TM_COMM_PASS, may then be NULL).  RECORD creates / truncates it,
 * REPLAY reads it.  scopes: TM_SCOPE_* bits to record, or the scopes on the sandbox boundary. */
int tm_comm_open(const char *path, int mode, int scopes, tm_comm_t **out);

/* One collective call on `buf` (DEVICE pointer, in place; NULL with bytes 0 for a barrier), `bytes` long, elements
 * of TM_DTYPE_* `dtype`, enqueued on `stream`.  The stage calls this at its call sites; it is exported so that the
 * other collectives of a training loop can go through the same tape. */
int tm_comm_call(tm_comm_t *c, int kind, int scope, int site, int dtype, void *buf, int64_t bytes, void *stream);

/* Replay: start again from the tape's first entry (one more shadow iteration). */
int tm_comm_rewind(tm_comm_t *c);
int tm_comm_stats(const tm_comm_t *c, tm_comm_stats_t *out);
/* Record: writes the entry count and closes the file.  Replay: every copy enqueued from the pinned copies must have
 * completed (synchronise the streams first).  Detach the object from every stage before closing it. */
int tm_comm_close(tm_comm_t *c);

/* The stage calls `c` at its call sites from now on; NULL detaches.  tm_stage_bwd_adam refuses to run while a hook
 * that intercepts the data scope is attached (the update must follow tm_stage_grad_sync). */
int tm_stage_attach_comm(tm_stage_t *st, tm_comm_t *c);
/* The data-parallel reduction of the gradient buffer and the barrier that ends the step. */
int tm_stage_grad_sync(tm_stage_t *st, void *stream);

/* out[T, h] = residual[T, h] + part[T, h] + bias[h] (bias may be NULL), fp32 arithmetic, one rounding: what follows an
 * intercepted all-reduce of a row-parallel map's partial product.  DEVICE pointers, 16-byte aligned, h a multiple of 8. */
int tm_op_bias_residual_add(int dtype, int64_t T, int64_t h, const void *part, const void *bias, const void *residual,
                            void *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TM_SANDBOX_H */
