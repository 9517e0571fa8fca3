/*
 * hpsgd.h -- C ABI of the HPSGD hot path on one MI355X (gfx950).
 *
 * HPSGD (Hierarchical Parallel SGD): every worker trains a replica of the global
 * model while the previous round's changes are being synchronised; the average
 * change of the replicas is then merged into the global model (Abstract; Sec. 3).
 * K workers are simulated on one GPU as a group dimension: every buffer that a
 * worker owns is an array of K equally strided slices.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers unless a parameter says HOST.
 *   - The caller owns every device buffer, the workspace included.  The library never
 *     allocates or frees device memory and never creates or destroys a stream.
 *   - What the library owns besides host memory: HIP events.  A context creates two when an
 *     auxiliary stream is set (hpsgd_set_aux_stream) and pairs of them while timing is enabled
 *     (hpsgd_timer_enable, hpsgd_kernel_timer_enable); hpsgd_destroy frees them.  One more
 *     event per device lives as long as the process: it is recorded behind the most recent
 *     resident-weight recurrence launch (hpsgd_set_recurrence) and is, with the stream that
 *     launch went to and a mutex, the library's only per-process state.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls
 *     enqueue work and return without waiting for the device; ordering between streams is the
 *     caller's job.  Two entry points wait by design and say so: hpsgd_recurrence_gave_up and
 *     hpsgd_timer_read / hpsgd_kernel_timer_read (they read results back).
 *   - Return value: HPSGD_OK or an error code.  Arguments are validated before
 *     anything is enqueued; on error nothing has been written.
 *   - Parameter buffers (global, snapshot, replicas) must be 16-byte aligned and replica
 *     strides multiples of 4 floats; batch inputs and labels need 4-byte alignment only.
 *   - Results are deterministic: fixed reduction orders, no floating-point atomics.
 */
#ifndef HPSGD_H
#define HPSGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hpsgd_ctx hpsgd_ctx; /* opaque: shapes, layout table, launch plan (host memory), HIP events */

enum hpsgd_status {
  HPSGD_OK = 0,
  HPSGD_EINVAL = 1,       /* null pointer, K < 1, negative size, unknown enum */
  HPSGD_ESHAPE = 2,       /* model description inconsistent or out of supported range */
  HPSGD_EALIGN = 3,       /* pointer not 16-byte aligned or stride not a multiple of 4 floats */
  HPSGD_EALIAS = 4,       /* output overlaps an input it must not overlap */
  HPSGD_EWORKSPACE = 5,   /* workspace null or misaligned */
  HPSGD_EUNSUPPORTED = 6, /* valid request the library does not implement */
  HPSGD_EHIP = 7          /* a HIP call or launch failed */
};

enum hpsgd_model_kind {
  HPSGD_GRU_CLASSIFIER = 0, /* GRU stack, linear + softmax head on the last hidden state */
  HPSGD_GRU_LM = 1,         /* embedding, GRU stack, linear + softmax head at every step */
  HPSGD_MLP = 2             /* ReLU multilayer perceptron with a softmax head */
};

enum hpsgd_precision {
  HPSGD_FP32 = 0,     /* fp32 operands on the fp32 matrix cores */
  HPSGD_BF16_MFMA = 1 /* GEMM operands rounded to bf16 (nearest-even), fp32 accumulate;
                         parameters, gate math, softmax and gradients stay fp32 */
};

#define HPSGD_MAX_WORKERS 32
#define HPSGD_MAX_MLP_DIMS 8

typedef struct hpsgd_model_desc {
  int kind;      /* enum hpsgd_model_kind */
  int prec;      /* enum hpsgd_precision */
  int layers;    /* GRU layers (GRU kinds) */
  int input;     /* input width I (classifier) */
  int hidden;    /* hidden width H */
  int seq_len;   /* T */
  int batch;     /* B, per worker */
  int classes;   /* C (classifier); the LM's class count is `vocab` */
  int vocab;     /* V (LM) */
  int embed;     /* E (LM) */
  int n_mlp_dims;                   /* MLP: number of layer widths, input and output included */
  int mlp_dims[HPSGD_MAX_MLP_DIMS]; /* MLP: widths d0, d1, ..., d_last */
} hpsgd_model_desc;

/* ---- context --------------------------------------------------------------------------
 * Describes the model every worker trains (Sec. 3.1: each worker runs the same local
 * training phase on its own sub-dataset) and the number of workers K.  No device memory. */
int hpsgd_create(const hpsgd_model_desc *desc, int K, hpsgd_ctx **out);
int hpsgd_destroy(hpsgd_ctx *ctx);

/* Number of fp32 parameters P of one replica. */
size_t hpsgd_param_count(const hpsgd_ctx *ctx);
/* Number of parameter tensors in the flat layout. */
int hpsgd_param_entries(const hpsgd_ctx *ctx);
/* i-th tensor of the flat layout: name (owned by ctx), offset in floats, rows, cols
 * (cols = 1 for vectors).  Matrices are row-major [out, in]; the three GRU gates are
 * stacked r, z, n along `out`.  Returns HPSGD_EINVAL if i is out of range. */
int hpsgd_param_entry(const hpsgd_ctx *ctx, int i, const char **name, size_t *offset,
                      int *rows, int *cols);
/* Bytes of device workspace hpsgd_local_step_all needs for all K workers
 * (activations saved for the backward pass, gradients, per-row losses). */
size_t hpsgd_workspace_bytes(const hpsgd_ctx *ctx);

/* ---- local training step (Alg. 2: compute the local gradients on the replica, then
 *      "update replica" r_i <- r_i - mu * grad) ------------------------------------------
 * One step for all K workers as grouped launches.  Worker k reads its parameters at
 * replicas_in + k*replica_stride and writes the updated ones at replicas_out +
 * k*replica_stride (replicas_out == replicas_in is allowed: in-place; any other overlap
 * is HPSGD_EALIAS).  replica_stride >= P, in floats.
 *   x: GRU classifier  fp32  [K][T][B][I]   (time-major batch)
 *      GRU LM          int32 [K][T][B]      token ids in [0, V)
 *      MLP             fp32  [K][B][d0]
 *   y: int32 labels [K][B]; for the LM the next-token ids [K][T][B].
 *      Labels outside [0, classes) are not checked on the device: caller's duty.
 *   loss_out: device, K floats (mean cross-entropy of each worker's batch), or NULL.
 *   workspace: hpsgd_workspace_bytes(ctx) bytes, 256-byte aligned, contents undefined
 *      on entry and on exit; two calls that may run concurrently need two workspaces. */
int hpsgd_local_step_all(hpsgd_ctx *ctx, const float *replicas_in, float *replicas_out,
                         size_t replica_stride, const void *x, const int32_t *y, float lr,
                         float *loss_out, void *workspace, void *hip_stream);

/* Alg. 2 "make replica" and the local step behind it as one call: every worker's replica is a
 * clone of `source` (DEVICE, P floats, 16-byte aligned: the global model, or the copy of it taken
 * when the round began) that has not been written out.  The step reads every parameter from
 * `source` and writes every parameter of every worker's updated replica to replicas_out
 * [K][replica_stride]: the same bits as hpsgd_sync_all(source -> replicas) followed by
 * hpsgd_local_step_all in place, without the K copies of the model ever being written and read
 * back (4 (K + 1) bytes per parameter of traffic less per round).  What hpsgd_merge needs
 * afterwards - the replicas and the model they were cloned from - is there: replicas_out and
 * `source`.  `source` must not overlap replicas_out or the workspace (HPSGD_EALIAS); other
 * arguments and errors as for hpsgd_local_step_all.  hpsgd_prepare_clones(source, replicas_out,
 * ..) before the call is honoured as for a step on written-out clones. */
int hpsgd_local_step_all_cloned(hpsgd_ctx *ctx, const float *source, float *replicas_out,
                                size_t replica_stride, const void *x, const int32_t *y, float lr,
                                float *loss_out, void *workspace, void *hip_stream);

/* hpsgd_local_step_all for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * workspace is a fixed array of HPSGD_STATIC_WORKSPACE_BYTES in the library's own device image
 * (every GPU the library runs on holds one copy until the process ends); its address on the
 * current device is looked up on the first call there.  The call allocates nothing, and computes
 * exactly what hpsgd_local_step_all computes (same kernels, same bits).
 * HPSGD_EWORKSPACE if hpsgd_workspace_bytes(ctx) exceeds HPSGD_STATIC_WORKSPACE_BYTES (checked
 * first, before any device is touched); otherwise errors as for hpsgd_local_step_all.
 * All calls on one GPU share that GPU's array, whatever their context: two calls that may run
 * concurrently on one GPU race (order them on one stream or with events).  The array keeps the
 * last call's contents; a step clears what it needs to start from zero itself.
 * hpsgd_recurrence_gave_up does not apply (it reads a caller's workspace): a given-up wait still
 * shows as NaN in loss_out and in the first parameter of every output replica. */
#define HPSGD_STATIC_WORKSPACE_BYTES (32u << 20)
int hpsgd_local_step_all_static(hpsgd_ctx *ctx, const float *replicas_in, float *replicas_out,
                                size_t replica_stride, const void *x, const int32_t *y, float lr,
                                float *loss_out, void *hip_stream);

/* Optional, between "make replica" and the local step (Alg. 2): makes, on hip_stream, the
 * operand copies that the next hpsgd_local_step_all(_acc) on (replicas, replica_stride,
 * workspace) would otherwise make at its start - in the bf16 configurations the rounded and the
 * transposed bf16 copies of every weight matrix; nothing in the others - so that they can
 * be made on the synchronising side, behind hpsgd_sync_all, while the training stream is busy
 * with another generation of replicas.  The context remembers (replicas, replica_stride,
 * workspace), one such mark per workspace; the next local step on that workspace skips its own
 * copies if it is given exactly these, and forgets the workspace's mark either way (it changes
 * the weights).  The caller must not write the replicas
 * between this call and that step, must order the two streams (the step after this call's
 * work), and must not use the workspace for another step in between.
 * Errors as for hpsgd_local_step_all's replicas_in and workspace arguments. */
int hpsgd_prepare_replicas(hpsgd_ctx *ctx, const float *replicas, size_t replica_stride,
                           void *workspace, void *hip_stream);

/* The same for replicas that are clones of the global model (Alg. 2 "make replica": the caller has
 * called, or will have called by the time of the local step, hpsgd_sync_all(global, replicas ...)
 * and nothing has written them since): ONE set of operand copies is made from `global` and the
 * marked local step hands it to all K workers (the K sets would hold the same bits; one set is an
 * eighth of the bytes to write at K = 8 and is fetched once by the products of all workers).  The
 * caller vouches for the equality: a step whose replicas differ from `global` would multiply with
 * the wrong weights.
 * `replicas` / replica_stride / workspace are those of the local step meant (they name the mark, as
 * for hpsgd_prepare_replicas; the replicas are not read here).  A context keeps one mark per
 * workspace (up to four), so a schedule with two generations of buffers may prepare one
 * generation, on its synchronising stream, while the other one steps.  The copies of the GRU
 * layers' matrices are made by this call; those of the head's matrix too if with_head != 0, else by
 * the marked local step itself, from `global`, right before its logits product: `global` must then
 * stay unchanged until that step has run (a snapshot of the clone's source does).  Errors as above. */
int hpsgd_prepare_clones(hpsgd_ctx *ctx, const float *global, const float *replicas, size_t replica_stride,
                         void *workspace, int with_head, void *hip_stream);

/* The same for ONE worker (`worker` in [0, K) selects nothing but the workspace slice,
 * so that different workers may be stepped on different streams).  loss_out: 1 float. */
int hpsgd_local_step(hpsgd_ctx *ctx, int worker, const float *replica_in, float *replica_out,
                     const void *x, const int32_t *y, float lr, float *loss_out,
                     void *workspace, void *hip_stream);

/* Optional second stream (hipStream_t as void*, NULL = none, the default).  When set,
 * hpsgd_local_step(_all) runs the weight-gradient GEMMs of time steps that backpropagation
 * through time has already passed on this stream, beside the rest of the recurrence -- the
 * same idea as the paper's hierarchy (Sec. 3.1: work that does not depend on the training
 * loop runs beside it), applied inside one local step.  The library orders the two streams
 * with two HIP events owned by the context and joins before the local step's remaining work,
 * so the caller still sees everything complete in order on the stream it passed.  The stream
 * must belong to the same device and must not be the stream passed to the local step.
 * Results are deterministic but differ in the last bits from the single-stream order (the
 * gradients are summed chunk by chunk). */
int hpsgd_set_aux_stream(hpsgd_ctx *ctx, void *hip_stream);

/* How the GRU recurrence of a local step (Alg. 2 "compute local gradients") is launched.
 * resident != 0 (the default): where the shape allows it (the workgroups of one launch must
 * all fit the device at once, and a workgroup's slice of W_hh must fit its LDS or, with bf16
 * operands, its registers), all time steps of a layer run as one launch per direction whose
 * workgroups keep their weights on the chip and wait for each other through flag words in
 * the workspace; such a launch may also take over the input projection of a narrow layer
 * input, the recurrent weight gradient and the bias gradients.  Otherwise, and with
 * resident == 0, one launch per time step.  Both forms compute the same quantities; the fp32
 * sums inside a dot product are taken in a different order.  The workgroups of such a launch
 * exchange h_t (forward) and the gate gradients (backward) through the L2 of the XCD they share
 * when the launch fills the chip and can seat each group of workgroups on one XCD, else, and always with
 * resident == 2, through memory at device scope; the results are the same bits.  spin_limit
 * bounds every such wait
 * (polls of the flags; 0 makes every wait fail at once, for testing).  A wait that is given up
 * ends the launch early on every workgroup, and the local step then delivers NaN in loss_out
 * and in the first parameter of every output replica; hpsgd_recurrence_gave_up reports it too.
 * Launches of this kind need the whole chip and must not run side by side.  The library orders
 * them itself, across streams, contexts and host threads: a local step holds a per-device lock
 * while it issues them, and when the previous ones went to another stream it lets its stream
 * wait (hipStreamWaitEvent, the host does not block) for the event recorded behind them. */
int hpsgd_set_recurrence(hpsgd_ctx *ctx, int resident, unsigned spin_limit);

/* *gave_up = 1 if a wait of the last local step(s) that used `workspace` was given up, else 0.
 * Synchronises hip_stream.  workspace: device, as passed to the local step. */
int hpsgd_recurrence_gave_up(const hpsgd_ctx *ctx, const void *workspace, void *hip_stream,
                             int *gave_up);

/* ---- batch gather (Sec. 3.2: every worker samples its own sub-dataset) ----------------
 * Time-major gather of n_idx samples: for b < n_idx, c < n_chunks
 *     out[(c*n_idx + b)*chunk_bytes ...] = shard[idx[b]*row_bytes + c*chunk_bytes ...]
 * n_chunks = 1 is a plain row gather.  chunk_bytes and row_bytes are multiples of 4,
 * n_chunks*chunk_bytes <= row_bytes.  Bit-exact.  idx values are the caller's duty. */
int hpsgd_gather_batch(const void *shard, const int32_t *idx, int n_idx, size_t row_bytes,
                       int n_chunks, size_t chunk_bytes, void *out, void *hip_stream);

/* The same gather for K workers in one launch: shards, idx and outs are HOST arrays of K
 * DEVICE pointers (worker k: shards[k], idx[k] with n_idx entries, outs[k]). */
int hpsgd_gather_batch_all(const void *const *shards, const int32_t *const *idx, int K, int n_idx,
                           size_t row_bytes, int n_chunks, size_t chunk_bytes, void *const *outs,
                           void *hip_stream);

/* ---- merge (Eq. 1; Alg. 3 "update global model" with the all-reduce taken as the mean
 *      over the K workers): global[j] += (1/K) * sum_k (replicas[k][j] - snapshot[j]) ----
 * replicas: HOST array of K DEVICE pointers (1 <= K <= HPSGD_MAX_WORKERS).
 * snapshot: the global model as it was when the replicas were cloned; may equal `global`.
 * The sum runs over k in increasing order in fp32.  P == 0 is a successful no-op.
 * `global` must not overlap any replica (HPSGD_EALIAS). */
int hpsgd_merge(float *global, const float *const *replicas, const float *snapshot, int K,
                size_t P, void *hip_stream);

/* ---- synchronisation in gradient form (Eq. 1 as printed; Alg. 2 "accumulate gradients") ----
 * hpsgd_local_step_all_acc is hpsgd_local_step_all that also adds the step's gradient of
 * worker k to grad_acc[k * acc_stride .. + P) (DEVICE fp32, 16-byte aligned, acc_stride >= P and
 * a multiple of 4 when K > 1; must not overlap the replicas, else HPSGD_EALIAS).  The caller
 * zeroes the accumulators at the start of a round.  In this form every gradient passes through
 * the gradient buffer (no update in a GEMM epilogue), so a step moves more bytes.
 * hpsgd_merge_grad: global[j] -= lr * (1/K) * sum_k grad_accs[k][j], the sum taken in worker
 * order in fp32.  grad_accs: HOST array of K DEVICE pointers, none overlapping `global`.
 * For a learning rate that is constant over the round this is hpsgd_merge up to rounding. */
int hpsgd_local_step_all_acc(hpsgd_ctx *ctx, const float *replicas_in, float *replicas_out,
                             size_t replica_stride, const void *x, const int32_t *y, float lr,
                             float *loss_out, float *grad_acc, size_t acc_stride, void *workspace,
                             void *hip_stream);
int hpsgd_merge_grad(float *global, const float *const *grad_accs, float lr, int K, size_t P,
                     void *hip_stream);

/* ---- sync (Alg. 2 "make replica": r_i = clone(w)) -------------------------------------
 * replica <- global, bit-exact. */
int hpsgd_sync_replica(const float *global, float *replica, size_t P, void *hip_stream);
/* One pass over `global` that writes all K replicas (HOST array of DEVICE pointers) and,
 * if not NULL, the snapshot.  0 <= K <= HPSGD_MAX_WORKERS; K = 0 writes the snapshot alone
 * (what a round needs when its local step is hpsgd_local_step_all_cloned). */
int hpsgd_sync_all(const float *global, float *const *replicas, int K, float *snapshot,
                   size_t P, void *hip_stream);

/* ---- merge and sync of one generation in one pass (Eq. 1 / Alg. 3 "update global model", then
 *      Alg. 2 "make replica" for the same workers) ---------------------------------------------
 * Exactly hpsgd_merge(global, replicas, snapshot, K, P) followed by hpsgd_sync_all(global, replicas,
 * K, snapshot, P), bit for bit, with every buffer read once and written once: 4 (2K + 4) bytes per
 * parameter instead of 4 (2K + 5).  For the synchronising side of the overlapped schedule, where
 * the replicas whose changes were just merged are the ones cloned next.  All K + 2 buffers are
 * written: none may overlap another (HPSGD_EALIAS; `snapshot` may therefore not be `global` here). */
int hpsgd_merge_sync(float *global, float *const *replicas, float *snapshot, int K, size_t P,
                     void *hip_stream);

/* hpsgd_merge(global, replicas, snapshot, ..) followed by snapshot = global (hpsgd_sync_all with K = 0),
 * bit for bit, in one pass: 4 (K + 4) bytes per parameter instead of 4 (K + 5).  The synchronising side
 * of a round whose local step is hpsgd_local_step_all_cloned: the replicas are only read.  `global` and
 * `snapshot` are written and may overlap neither each other nor a replica (HPSGD_EALIAS). */
int hpsgd_merge_snapshot(float *global, const float *const *replicas, float *snapshot, int K, size_t P,
                         void *hip_stream);

/* ---- kernel timing for benchmarks (not part of the method) ------------------------------
 * The launches of one local step fall into roles.  While a role's bit is set in the mask,
 * hpsgd_local_step(_all) records a HIP event pair on the caller's stream around every launch
 * group of that role (hpsgd_destroy frees the events).  hpsgd_timer_read waits for the recorded events, returns the number of timed
 * launch groups of `role` and their summed duration in milliseconds, and clears that role.
 * With an auxiliary stream set (hpsgd_set_aux_stream) some launches run beside others: the
 * bf16 head's two backward GEMMs share one pair (counted as two launches), and a launch
 * that the library issues on the auxiliary stream alone (a layer's input-gradient GEMM beside
 * its weight-gradient GEMMs) is not timed. */
enum hpsgd_role {
  HPSGD_ROLE_OTHER = 0,        /* zero fills */
  HPSGD_ROLE_GEMM_INPUT = 1,   /* time-batched input projection  X W_ih^T */
  HPSGD_ROLE_GEMM_REC_FWD = 2, /* per-step recurrent GEMM        h W_hh^T */
  HPSGD_ROLE_GEMM_REC_BWD = 3, /* per-step BPTT GEMM             dGh W_hh */
  HPSGD_ROLE_GEMM_WGRAD = 4,   /* time-batched weight gradients and bias column sums */
  HPSGD_ROLE_GEMM_DX = 5,      /* gradient to the layer below    dGx W_ih */
  HPSGD_ROLE_GEMM_HEAD = 6,    /* head forward and backward GEMMs */
  HPSGD_ROLE_CELL_FWD = 7,     /* gate nonlinearities and cell update */
  HPSGD_ROLE_CELL_BWD = 8,     /* BPTT gate gradients */
  HPSGD_ROLE_LOSS = 9,         /* softmax cross-entropy and loss mean */
  HPSGD_ROLE_EMBED = 10,       /* embedding lookup and its gradient */
  HPSGD_ROLE_COMMIT = 11,      /* SGD commit to the replica */
  HPSGD_ROLE_MLP_FWD = 12,     /* MLP forward GEMMs */
  HPSGD_ROLE_MLP_BWD = 13,     /* MLP backward GEMMs and bias column sums */
  HPSGD_ROLE_COUNT = 14
};
int hpsgd_timer_enable(hpsgd_ctx *ctx, unsigned role_mask);
int hpsgd_timer_read(hpsgd_ctx *ctx, int role, long *launches, double *total_ms);
const char *hpsgd_role_name(int role); /* static string, NULL if out of range */
/* How many parameters per worker went through the gradient buffer and the commit kernel in
 * the last local step of this context (Alg. 2 "update replica" as a separate streaming pass).
 * The other weight matrices were updated by the epilogue of their own gradient GEMM.  0
 * before the first step.  For the byte accounting of the HPSGD_ROLE_COMMIT timings. */
size_t hpsgd_commit_kernel_params(const hpsgd_ctx *ctx);

/* The same per KERNEL instead of per role: while a kernel's bit is set in the mask, every launch
 * of that kernel inside hpsgd_local_step(_all)(_acc) is bracketed by a HIP event pair on the
 * stream the launch goes to (the auxiliary stream included), and the launch's algorithmic work
 * is added up: flops (2 M N Kd per group; a recurrence launch 2 B 3H H per time step, plus the
 * products it fuses) for the contractions, bytes (each operand once) for the streaming kernels.
 * hpsgd_kernel_timer_read waits for the recorded events, returns the number of timed launches of
 * `kernel`, their summed duration in milliseconds and their summed work, and clears that kernel.
 * Names are those a kernel trace shows (template arguments included where they tell forms apart). */
enum hpsgd_kernel {
  HPSGD_KERNEL_NONE = 0,
  HPSGD_KERNEL_GRU_FWD_PERSIST = 1,
  HPSGD_KERNEL_GRU_BWD_PERSIST = 2,
  HPSGD_KERNEL_GRU_FWD_PERSIST_BF16 = 3,
  HPSGD_KERNEL_GRU_BWD_PERSIST_BF16 = 4,
  HPSGD_KERNEL_GEMM_BF16_DL = 5,
  HPSGD_KERNEL_GEMM_BF16_DL_COMMIT = 6,
  HPSGD_KERNEL_GEMM_BF16_DLX128 = 7,
  HPSGD_KERNEL_GEMM_BF16_DLX128_COMMIT = 8,
  HPSGD_KERNEL_GEMM_BF16_DLX192 = 9,
  HPSGD_KERNEL_GEMM_BF16_DLX192_COMMIT = 10,
  HPSGD_KERNEL_GEMM_BF16_DLX256 = 11,
  HPSGD_KERNEL_GEMM_BF16_DLX256_COMMIT = 12,
  HPSGD_KERNEL_GEMM_BF16_NT = 13,
  HPSGD_KERNEL_GEMM_F32_FAST = 14,
  HPSGD_KERNEL_GEMM_F32 = 15,
  HPSGD_KERNEL_CVT2 = 16,           /* streaming: bytes */
  HPSGD_KERNEL_SOFTMAX_CE_BF16 = 17, /* streaming: bytes */
  HPSGD_KERNEL_GRU_STEP = 18,
  HPSGD_KERNEL_COMMIT_ACC = 19,     /* streaming: bytes */
  HPSGD_KERNEL_COMMIT = 20,         /* streaming: bytes */
  HPSGD_KERNEL_CVT2_PACK = 21,      /* streaming: bytes */
  HPSGD_KERNEL_COUNT = 22
};
int hpsgd_kernel_timer_enable(hpsgd_ctx *ctx, unsigned kernel_mask);
int hpsgd_kernel_timer_read(hpsgd_ctx *ctx, int kernel, long *launches, double *total_ms, double *work);
const char *hpsgd_kernel_name(int kernel); /* static string, NULL if out of range */

/* What the recurrence launches of the last local step included (benchmarks: which role the
 * work of a fused part is accounted to).  Each count is a number of GRU layers:
 *   resident_layers: layers whose recurrence ran as resident-weight launches,
 *   xproj_layers:    of those, layers whose forward launch did the input projection itself,
 *   dw_layers:       of those, layers whose backward launch accumulated dW_hh and the bias
 *                    gradients itself.
 * Any pointer may be NULL. */
int hpsgd_recurrence_info(const hpsgd_ctx *ctx, int *resident_layers, int *xproj_layers, int *dw_layers);

/* ---- synthetic synchronisation latency (measurement / test aid) ---------------------------
 * Occupies `hip_stream` for about `microseconds` (one wave that sleeps until the 100 MHz wall
 * clock has advanced that far; at most 1 000 000, else HPSGD_EINVAL).  Stands in for a slow
 * interconnect on the synchronising side (Sec. 3.2: t_sync = k * t_train), so that the
 * asynchronous schedule of Alg. 2 / Alg. 3 can be driven into rounds of several local steps. */
int hpsgd_delay_us(unsigned microseconds, void *hip_stream);

/* ---- the bf16 product of the local step, on its own --------------------------------------
 * Every matrix product of the gradient computation (Alg. 2, the local training step) runs, in
 * the bf16 configurations, as  C[g] = A[g] * B[g]^T  (M x N, fp32) for g < groups, or, where
 * the product is a weight gradient, directly as the SGD update  C[g] = win[g] - lr * A[g] * B[g]^T
 * (win != NULL; win may be C).  This entry point runs that one kernel family on caller data.
 * A: [M][Kd], B: [N][Kd], bf16 bit patterns (DEVICE), row pitches lda / ldb and group strides
 * strideA / strideB in elements; C and win: fp32 (DEVICE), row pitch ldc, group strides strideC
 * / strideWin in elements.  Products are exact, accumulation is fp32 in the order of k
 * (v_mfma_f32_32x32x16_bf16).  form: 0 lets the library choose the tile by shape; 1 .. 4
 * force 128 x 128, 128 x 256, 192 x 256, 256 x 256 (the results do not depend on the form).
 * Asynchronous on hip_stream; the caller owns all buffers.
 * HPSGD_EINVAL: null pointer, size < 1, Kd not a multiple of 8, form out of range;
 * HPSGD_EALIGN: A or B not 16-byte aligned, or a pitch / stride of A or B not a multiple of 8. */
int hpsgd_gemm_bf16_nt(const void *A, long lda, long strideA, const void *B, long ldb, long strideB,
                       float *C, long ldc, long strideC, const float *win, long strideWin, float lr,
                       int M, int N, int Kd, int groups, int form, void *hip_stream);

/* ---- matrix-core rate probe (measurement aid, not part of the method) --------------------
 * Runs a loop of independent MFMAs with no memory traffic on every CU: `precision` picks
 * v_mfma_f32_32x32x16_bf16 (HPSGD_BF16_MFMA) or v_mfma_f32_32x32x2_f32 (HPSGD_FP32);
 * operand registers are filled from `operands` (DEVICE pointer, at least 16 KiB: zeros, ones
 * or random values: the data decides how much power the matrix cores draw and with it the
 * clock the chip sustains).  `result` (DEVICE, 4 doubles, written asynchronously):
 * [0] shader clock ticks and [1] 100 MHz wall-clock ticks of workgroup 0, [2] MFMA
 * instructions per wave, [3] flops per MFMA instruction.  256 workgroups of 4 waves: one wave
 * per SIMD, so the chip's rate is 1024 waves x [2] x [3] / ([1] / 100 MHz). */
int hpsgd_probe_mfma_rate(int precision, const void *operands, int iterations, double *result,
                          float *sink /* DEVICE, 256*256 floats */, void *hip_stream);

/* Human-readable name of a status code (static string). */
const char *hpsgd_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* HPSGD_H */
