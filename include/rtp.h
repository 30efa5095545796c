/*
 * rtp.h -- C ABI of the rotated-shard linear layer of Rotated Tensor
 * Parallelism (RTP, arXiv 2311.01635) for one worker on one MI355X (gfx950).
 *
 * The worker keeps 1/N of the batch and, at any moment, 1/N of a layer
 * unit's weights.  Over N steps it computes on the weight shard it holds
 * while the next shard is brought in on a second HIP stream (Design section;
 * Rotating Communication Primitive section).  The other workers' memory is
 * played by a caller-owned "home" store of N slots on the same GPU; there is
 * no second device and no collective.
 *
 * Conventions
 *   - Every pointer named `*_dev` or documented "device" is device memory the
 *     CALLER allocates and frees; the library allocates no device memory.  It
 *     owns only its host objects and the HIP events inside them.
 *   - Streams are passed as `void*` holding a `hipStream_t`.  The two streams
 *     of a ring must differ and must have default priority.
 *   - Matrices are row-major and contiguous: W[O, I], X[T, I], Y[T, O].
 *     Weight shard k of an output-partitioned matrix is rows
 *     [k*o, (k+1)*o) of W, o = O/N, stored [o, I]; of an input-partitioned
 *     matrix it is columns [k*o, (k+1)*o) of W[O, I], o = I/N, stored
 *     contiguously as [O, o] (Partition Strategies section).
 *   - Calls only enqueue work and return; ordering between the two streams is
 *     the library's job (events).  rtp_ring_sync() joins both streams and
 *     reports asynchronous HIP errors.
 *   - Every function returns an rtp_status (or a plain integer for the pure
 *     index helpers); nothing throws or aborts.  rtp_last_error() gives the
 *     text of the last failure on the calling thread.
 */
#ifndef RTP_H_
#define RTP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RTP_OK = 0,
    RTP_ERR_INVALID = 1,     /* null or aliasing pointer, bad enum value            */
    RTP_ERR_SHAPE = 2,       /* N does not divide the partitioned dim, size <= 0,
                                alignment the kernels need is not met                */
    RTP_ERR_STATE = 3,       /* call out of sequence (see each function)            */
    RTP_ERR_UNSUPPORTED = 4, /* dtype / mode / activation combination not built     */
    RTP_ERR_HIP = 5          /* a HIP runtime call failed; text in rtp_last_error() */
} rtp_status;

typedef enum { RTP_F32 = 0, RTP_BF16 = 1, RTP_F16 = 2 } rtp_dtype;

/* Output-Partition (outputs are concatenated) and the input-dimension
 * partition of the layer that follows it (outputs are summed): Partition
 * Strategies section, first and second item. */
typedef enum { RTP_SPLIT_OUT = 0, RTP_SPLIT_IN = 1 } rtp_split;

/* How the next shard is staged (Rotating Communication Primitive section):
 *  RTP_DOUBLE_BUFFER   out-of-place rotation: two (W_k, G_k) buffers that swap
 *                      roles every step; all traffic overlaps compute.
 *  RTP_INPLACE_STAGED  one extra weight buffer only; the gradient shard is
 *                      exchanged in place (written home, then the next one
 *                      read into the same buffer) as soon as the step's dW
 *                      kernel is done, under the step's dX kernel.
 *  RTP_INPLACE_BLOCKING the paper's in-place variant: no extra buffer, the
 *                      exchange runs on the compute stream between steps.   */
typedef enum { RTP_DOUBLE_BUFFER = 0, RTP_INPLACE_STAGED = 1, RTP_INPLACE_BLOCKING = 2 } rtp_mode;

/* Activation fused after an output-partitioned GEMM (RTP Transformers
 * section, linear-block item: the first GEMM of an MLP block is followed by
 * its activation); RTP_ACT_SWIGLU is the gated form silu(a)*b over a
 * (gate, up) pair. */
typedef enum { RTP_ACT_NONE = 0, RTP_ACT_GELU_ERF = 1, RTP_ACT_GELU_TANH = 2, RTP_ACT_SWIGLU = 3 } rtp_act;

typedef enum { RTP_PASS_IDLE = 0, RTP_PASS_FWD = 1, RTP_PASS_BWD = 2 } rtp_pass;

#define RTP_CW (+1)  /* clockwise: forward, weights only            */
#define RTP_CCW (-1) /* counter-clockwise: backward, weights + grads */

#define RTP_FLAG_DRY_RUN 1u /* make no HIP call at all: the schedule and the
                               state machine run on the host only (tests)   */
#define RTP_FLAG_STEPWISE 2u /* rtp_mlp_*: one kernel launch per linear and step,
                                exactly the rtp_rotate_step / rtp_linear_* call
                                sequence (no grouped launches)                 */

#define RTP_FLAG_GROUPED 4u  /* rtp_mlp_*: grouped launches in the backward pass too
                                when an auxiliary stream is given (default then: one
                                launch per GEMM, weight gradients on that stream)    */
#define RTP_FLAG_PIPELINED 8u /* rtp_mlp_*: with an auxiliary stream, run each pass as
                                two decoupled kernel chains (first linear's GEMMs /
                                second linear's GEMMs forward; input gradients /
                                weight gradients backward), shard parts moving as
                                soon as their last reader is enqueued               */
#define RTP_FLAG_FUSED_STEP 32u /* rtp_mlp_*: the dependent GEMMs of a rotation step as one
                                launch (RTP Transformers section, linear-block item: the
                                first GEMM, its activation and the second GEMM of the
                                block): forward Z_t -> down_t, backward dPre_s -> dX_s; the
                                second GEMM's tiles start as their rows of the first are
                                done.  Needs rtp_mlp_desc.step_sync_dev                  */
#define RTP_FLAG_STAGE_MEMCPY 16u /* shard transfers through hipMemcpyAsync (device to
                                device) on the stage stream instead of the library's
                                copy kernel: the runtime's own transfer path, for
                                comparison (Rotating Communication Primitive section:
                                communication on a stream of its own)                */

typedef struct rtp_ring rtp_ring;
typedef struct rtp_linear rtp_linear;
typedef struct rtp_mlp rtp_mlp;
typedef struct rtp_moe rtp_moe;

/* ---- pure host integer helpers (no GPU needed) ------------------------- */

/* Shard a worker holds at a step, 0-based (Design section, workflow
 * paragraph): forward (rank - step) mod n, backward (rank + 1 + step) mod n.
 * Return -1 if n <= 0 or rank/step are outside [0, n). */
int rtp_fwd_shard(int rank, int step, int n);
int rtp_bwd_shard(int rank, int step, int n);

/* First row (or column) of shard k of a dimension of size `dim` split n
 * ways; -1 if n does not divide dim or k is outside [0, n). */
int64_t rtp_shard_begin(int k, int64_t dim, int n);

/* Width of the n equal shards of a dimension of size `dim` (FlatParameter
 * section: the flat parameter is padded so that it divides evenly).  dim / n
 * when n divides dim; otherwise the smallest width that covers dim and is a
 * multiple of 8 (bf16), 32 (fp16) or 1 (fp32) elements: shard k then holds
 * elements [k w, min((k + 1) w, dim)), its tail is padding (zeros, never read
 * as data, never written).  -1 if that would leave the last shard empty. */
int64_t rtp_shard_width(int64_t dim, int n, rtp_dtype dtype);

/* Parameter bytes one worker holds for a unit whose slot has w_bytes of
 * weights and g_bytes of gradients, per mode; 0 on a bad mode.
 *   DOUBLE_BUFFER 2(w+g), INPLACE_STAGED 2w+g, INPLACE_BLOCKING w+g.
 * rtp_table1_worker_bytes is the matching per-worker share of Table 1
 * (RTP: w+g+max(w,g); RTP in place: w+g) for comparison. */
size_t rtp_worker_bytes(rtp_mode mode, size_t w_bytes, size_t g_bytes);
size_t rtp_table1_worker_bytes(int inplace, size_t w_bytes, size_t g_bytes);

/* ---- the shard layout of the ring store (device kernels) ---------------- */

/* Writes a full row-major matrix W[O, I] (device) into the ring store as its
 * n shards (Partition Strategies section: Output-Partition and the
 * input-dimension partition of the layer that follows it; FlatParameter
 * paragraph: every parameter of the unit flattened into one slot, padded so
 * that it divides evenly).  Shard k's part is written at
 * home_dev + k * slot_bytes + offset:
 *   RTP_SPLIT_OUT  rows [k w, (k+1) w) of W, stored [w, I];
 *   RTP_SPLIT_IN   columns [k w, (k+1) w) of W, stored contiguously as [O, w];
 * w = `width` (rtp_shard_width of the partitioned dimension; O / n or I / n
 * when n divides it).  Elements of a shard that lie past the matrix (padded
 * partition) are written as zeros.  `dtype` is the element type of W and of
 * the store (RTP_F32 for a gradient store).  Nothing else of the slot is
 * touched, so a unit's slot is built by one call per matrix with that
 * matrix's offset: a (gate, up) pair is two output-partitioned matrices whose
 * parts follow each other; a bias vector is a matrix with I = 1 (its shard
 * entries follow its matrix, see rtp_linear_desc.has_bias; the pieces of an
 * input-partitioned layer's bias are RTP_SPLIT_OUT with
 * width = rtp_bias_piece_width).  With n = 1 the call copies one matrix into
 * one slot (an expert of the expert partition).
 * rtp_unpack_shards is the inverse: it reads the n parts back into W[O, I]
 * and drops the padding.  Both enqueue one kernel on `stream` (a hipStream_t)
 * and return.  All memory is the caller's.
 * Errors: RTP_ERR_INVALID (null pointer, bad enum), RTP_ERR_SHAPE (sizes not
 * positive, n * width short of the partitioned dimension, part beyond the
 * slot, pointers / offset / slot size not multiples of the element size). */
rtp_status rtp_pack_shards(void *home_dev, size_t slot_bytes, size_t offset, int n, rtp_split split,
                           const void *W_dev, int64_t O, int64_t I, int64_t width, rtp_dtype dtype, void *stream);
rtp_status rtp_unpack_shards(void *W_dev, const void *home_dev, size_t slot_bytes, size_t offset, int n,
                             rtp_split split, int64_t O, int64_t I, int64_t width, rtp_dtype dtype, void *stream);

const char *rtp_status_str(rtp_status s);
const char *rtp_last_error(void);

/* ---- the ring: one layer unit's shard store and rotation --------------- */

typedef struct {
    int n;            /* partition factor N >= 1                                  */
    int rank;         /* this worker, 0 <= rank < n                               */
    rtp_mode mode;
    unsigned flags;   /* RTP_FLAG_*                                               */
    size_t w_bytes;   /* weight part of one slot: every matrix shard of the unit,
                         back to back (the FlatParameter idea); multiple of 16    */
    size_t g_bytes;   /* gradient part of one slot; multiple of 16; may be 0      */
    void *home_w_dev; /* n * w_bytes, slot k at k * w_bytes                       */
    void *home_g_dev; /* n * g_bytes                                              */
    void *buf_w_dev[2]; /* w_bytes each; [1] unused (may be NULL) when blocking   */
    void *buf_g_dev[2]; /* g_bytes each; [1] used by RTP_DOUBLE_BUFFER only       */
    void *compute_stream; /* hipStream_t */
    void *stage_stream;   /* hipStream_t, != compute_stream unless blocking.  The
                             stage and the auxiliary stream are the ring's alone
                             from create to destroy: the caller enqueues nothing on
                             them (a pass relies on finding them as it left them)  */
    void *aux_stream;     /* optional second compute stream (hipStream_t, distinct):
                             the weight-gradient kernels run there, beside the
                             input-gradient kernels, since one shard GEMM seldom fills
                             the machine.  Everything is joined back into the compute
                             stream when a pass ends.  NULL = one compute stream.      */
} rtp_ring_desc;

/* Creates the host object.  Errors: RTP_ERR_INVALID (null desc/out, null
 * device pointer that the mode needs, equal streams), RTP_ERR_SHAPE (n < 1,
 * rank outside [0, n), sizes not multiples of 16). */
rtp_status rtp_ring_create(rtp_ring **out, const rtp_ring_desc *desc);
rtp_status rtp_ring_destroy(rtp_ring *ring);

/* Starts a pass.  RTP_PASS_FWD: the worker starts on its own shard (Design
 * section, workflow paragraph).  If a completed backward pass has left that
 * shard in the worker's buffer, it is used where it is; otherwise (first
 * pass, after a forward pass, after rtp_ring_flush or rtp_ring_abort) home
 * slot `rank` is copied into the resident buffer.  The caller therefore must
 * not touch the worker's weight buffers between passes, and calls
 * rtp_ring_flush before it writes to the weight store (an optimizer step).
 * RTP_PASS_BWD: must follow a
 * completed forward pass (the worker holds shard (rank+1) mod n) or, with
 * n == 1 or after rtp_ring_seek_bwd_start(), any idle state; loads that shard's
 * gradient part, after writing the gradient shard an earlier backward pass
 * left in the buffer (the worker's own; see rtp_ring_resident_grad) back to
 * its slot: gradients accumulate over any number of passes.  These two gradient transfers run on
 * the stage stream; only the weight-gradient kernels wait for them.
 * RTP_ERR_STATE if a pass is in progress.
 * Stream capture of a pass is not supported: the calls decide on the host,
 * when they are made, what a pass enqueues (the write-back above, for one),
 * and use three streams.  RTP_ERR_UNSUPPORTED, before anything is enqueued,
 * if any of the ring's streams is capturing (so do rtp_ring_seek_bwd_start,
 * rtp_ring_flush, rtp_ring_zero_grads and the rtp_mlp_* / rtp_moe_* passes). */
rtp_status rtp_ring_begin(rtp_ring *ring, rtp_pass pass);

/* Makes shard (rank+1) mod n resident without a forward pass (tests and
 * backward-only timing). */
rtp_status rtp_ring_seek_bwd_start(rtp_ring *ring);

/* One rotation (Rotating Communication Primitive section).  `direction`
 * RTP_CW in a forward pass, RTP_CCW in a backward pass; `step` is the step
 * whose compute the transfer overlaps, 0 <= step < n-1 (the pass computes n
 * times and rotates n-1 times).  Must be called once per step, in order,
 * BEFORE the rtp_linear_* calls of that step (so that the transfer is not
 * ordered behind them), and after every linear of the ring has been issued
 * for the previous step.  Enqueues on the stage stream: the held weights go
 * back to their home slot, the next shard's weights come into the staging
 * buffer; in a backward pass the gradient part follows each linear's dW
 * kernel (see rtp_linear_bwd).  Errors: RTP_ERR_STATE for a wrong direction,
 * a step out of order or >= n-1, a linear lagging behind. */
rtp_status rtp_rotate_step(rtp_ring *ring, int direction, int step);

/* Ends a pass after step n-1 (Design section, workflow paragraph: a forward
 * pass ends on the next worker's shard, a backward pass on the worker's own).
 * After a backward pass writes nothing: the worker holds its own
 * (W_rank, G_rank).  The stage and auxiliary streams are joined into the
 * compute stream.  RTP_ERR_STATE if steps remain. */
rtp_status rtp_ring_end(rtp_ring *ring);

/* Way out of a pass that failed half-way (any call of an open pass returned
 * an error): joins the three streams, closes the pass and forgets what the
 * worker holds, so that rtp_ring_begin(RTP_PASS_FWD), rtp_ring_zero_grads,
 * rtp_ring_flush (a no-op then) and the destroy calls work again.  Outputs,
 * saved activations and the gradient shard the worker held are undefined
 * after it: clear the gradients and start over.  The rtp_mlp_* and rtp_moe_*
 * passes call it themselves before they return an error.  No-op when idle. */
rtp_status rtp_ring_abort(rtp_ring *ring);

/* Copies the resident (W, G) to their home slot so that a reader of the home
 * store sees every shard (tests, checkpoints, an optimizer): between passes
 * the worker's copy is the only current one of the shard it holds (Memory
 * Arrangement section: each parameter exists once in the system).  Idle state only.
 * Between a backward pass and the flush the home slot of the worker's own
 * gradient shard is stale: write to the gradient store only after a flush (or
 * through rtp_ring_zero_grads), else the next backward pass writes the
 * worker's copy back over it. */
rtp_status rtp_ring_flush(rtp_ring *ring);

/* The optimizer step's "zero the gradients" for a store whose shards travel
 * (Design section: the gradient shard rides with its weight): clears
 * every gradient slot of the home store (a fill kernel on the compute
 * stream, ordered after everything enqueued so far) and drops the gradient
 * shard the worker still holds, so that the next backward pass accumulates
 * from zero.  Idle state only. */
rtp_status rtp_ring_zero_grads(rtp_ring *ring);

/* Joins both streams; returns RTP_ERR_HIP if anything asynchronous failed. */
rtp_status rtp_ring_sync(rtp_ring *ring);

/* Shard currently resident (after everything enqueued so far), or -1. */
int rtp_ring_resident(const rtp_ring *ring);

/* Gradient shard the worker's buffer still holds that is NOT yet in its slot
 * of the home store (the next backward pass or rtp_ring_flush writes it
 * back), or -1 when every slot is current.  A backward pass ends on the
 * worker's own shard (Design section, workflow paragraph), which travels no
 * further: the MLP unit's default schedule and the expert layer (staged
 * modes, own expert with tokens) store `arrived + own` straight into the own
 * slot and leave -1; the other schedules, the bare linear layers and K-split
 * weight-gradient kernels leave the shard in the buffer. */
int rtp_ring_resident_grad(const rtp_ring *ring);

/* Timing aid (the three-run measurement of how much of the staging hides
 * under compute): `rotate` = 0 skips the transfers (every step computes on the
 * shard that is resident: results are meaningless), `compute` = 0 skips the
 * kernels of the ring's layers (the staging traffic alone).  Idle state only.
 * rtp_mlp_set_ablation / rtp_moe_set_ablation do the same for a unit. */
rtp_status rtp_ring_set_ablation(rtp_ring *ring, int rotate, int compute);

/* Test aid for the cross-stream ordering.  From now on the ring enqueues a
 * bounded spin kernel (one wave that watches the wall clock for the given
 * number of microseconds, at most 5000, and exits) ahead of every transfer on
 * the stage stream (`stage_us`) and ahead of every GEMM on the auxiliary
 * stream (`aux_us`), so that those streams run late against the compute
 * stream: a result that only came out right because a transfer or a
 * weight-gradient kernel happened to finish early no longer does.  Results
 * must not change.  `scratch32_dev`: 32 bytes of caller-owned device memory
 * the spin kernels write their clock readings to.  Zero for both switches it
 * off.  Idle state only. */
rtp_status rtp_ring_set_test_delay(rtp_ring *ring, void *scratch32_dev, int64_t stage_us, int64_t aux_us);

/* The same for the compute stream: a bounded spin kernel ahead of every GEMM
 * on it (`compute_us`, at most 5000; `scratch16_dev`: 16 bytes of device
 * memory), so that the compute stream runs late against the stage and the
 * auxiliary stream: a transfer that did not really wait for the kernels
 * reading its destination, or a weight-gradient kernel that did not wait for
 * the input-gradient kernel it depends on, shows.  Zero switches it off.
 * Idle state only. */
rtp_status rtp_ring_set_test_delay_compute(rtp_ring *ring, void *scratch16_dev, int64_t compute_us);

/* Copies up to `cap` records of what the ring has enqueued since creation
 * (or the last call with clear != 0) and returns the total number recorded.
 * kind: 1 compute-fwd, 2 compute-bwd, 3 weights in, 4 weights out,
 * 5 gradients in, 6 gradients out.  Integer record of the schedule, for
 * bit-exact comparison with the oracle. */
typedef struct { int kind, pass, step, shard, buffer; } rtp_trace_rec;
int64_t rtp_ring_trace(rtp_ring *ring, rtp_trace_rec *out, int64_t cap, int clear);

/* ---- a linear layer whose shards live in a ring slot ------------------- */

typedef struct {
    int64_t T;            /* local tokens                                         */
    int64_t I, O;         /* full matrix W[O, I]                                  */
    rtp_split split;
    rtp_dtype dtype;      /* of X, W, Y, dY, dX                                   */
    rtp_dtype grad_dtype; /* of the gradient shard: RTP_F32, or equal to dtype    */
    rtp_act act;          /* RTP_SPLIT_OUT: fused after the forward GEMM.
                             RTP_SPLIT_IN: the activation that produced this
                             layer's input; if not NONE the backward returns the
                             gradient w.r.t. that activation's pre-activation.    */
    size_t w_offset;      /* byte offset of this matrix's shard in the slot       */
    size_t g_offset;
    void *preact_dev;     /* act != NONE: pre-activations, dtype, [T, O] for
                             SPLIT_OUT (written by fwd), [T, P] for SPLIT_IN
                             (read by bwd), P = I (GELU) or 2 I (SWIGLU)          */
    float *acc_ws_dev;    /* fp32 [T, I] (SPLIT_OUT, dX) or [T, O] (SPLIT_IN, Y):
                             cross-step accumulator; needed when dtype != F32
                             and n > 1 (a call that needs it and finds NULL returns
                             RTP_ERR_INVALID)                                      */
    int has_bias;         /* the layer is Y = X W^T + b.  The bias rides in the flat
                             parameter (FlatParameter paragraph).  RTP_SPLIT_OUT:
                             shard k's w entries of b follow its rows of W in the
                             slot (at w_offset + w * I * sizeof(dtype)).
                             RTP_SPLIT_IN: b is spread evenly over the shards, piece
                             k = entries [k p, (k+1) p) with
                             p = rtp_bias_piece_width(O, n, dtype) (zero padding
                             past O), after shard k's [O, w] matrix; shard k's step
                             adds its piece.  The fp32 bias gradient follows the
                             matrix gradient the same way                          */
} rtp_linear_desc;

/* Entries of the bias piece an input-partitioned layer's shard carries:
 * ceil(O / n) rounded up to a whole number of 16-byte units.  -1 for bad
 * arguments. */
int64_t rtp_bias_piece_width(int64_t O, int n, rtp_dtype dtype);

/* Bytes one shard of the layer takes in the weight part / the gradient part
 * of a slot (matrix shard, bias shard if any, rounded up to 16); 0 on a bad
 * description. */
size_t rtp_linear_shard_w_bytes(const rtp_linear_desc *desc, int n);
size_t rtp_linear_shard_g_bytes(const rtp_linear_desc *desc, int n);

/* With act == RTP_ACT_SWIGLU and SPLIT_OUT, W is the stack of the gate and up
 * matrices arranged so that shard k (o = O/n rows, o even) is gate rows
 * [k*o/2, (k+1)*o/2) followed by the same rows of up; the forward output is
 * [T, O/2].  With SPLIT_IN and SWIGLU the backward output is [T, 2 I] in the
 * same shard-stacked column order.
 * A layer (not a gated one) may have a partitioned dimension n does not
 * divide: its shards are padded to rtp_shard_width() and stored at that width
 * ([w, I] rows for SPLIT_OUT, [O, w] columns for SPLIT_IN, padding zero); the
 * kernels only compute, read and write the columns that exist.
 * Errors: RTP_ERR_SHAPE (n does not divide the partitioned dimension of a
 * gated layer, or padding would leave a shard empty; bf16 or
 * fp16: I, O, o not multiples of 8; shard does not fit the slot),
 * RTP_ERR_INVALID, RTP_ERR_UNSUPPORTED (gradient dtype other than F32; fp16
 * with T, o or the unpartitioned dimension not a multiple of 32: fp16 inputs
 * run on the tiled kernel only, which needs such contraction lengths). */
rtp_status rtp_linear_create(rtp_linear **out, rtp_ring *ring, const rtp_linear_desc *desc);
rtp_status rtp_linear_destroy(rtp_linear *lin);

/* Forward step (RTP Transformers section, embedding-and-linear item), on the
 * shard k = rtp_fwd_shard(rank, step, n) that the ring holds:
 *   SPLIT_OUT  Y[:, k*o:(k+1)*o] = act(X W_k^T)       X[T, I], Y[T, O]
 *              (SWIGLU: Y[T, O/2], slice of width o/2), pre-activations saved;
 *   SPLIT_IN   Y += X[:, k*o:(k+1)*o] W_k^T           X[T, I], Y[T, O]
 *              summed over the n steps (fp32 accumulator, rounded once).
 * X, Y device.  RTP_ERR_STATE unless a forward pass is open, `step` is this
 * linear's next step, and (step == 0 or rtp_rotate_step(step-1) was issued). */
rtp_status rtp_linear_fwd(rtp_linear *lin, int step, const void *X_dev, void *Y_dev);

/* Backward step on shard k = rtp_bwd_shard(rank, step, n); first the weight
 * gradient, fused into the travelling gradient shard, then the input
 * gradient:
 *   SPLIT_OUT  G_k += dY[:, k*o:(k+1)*o]^T X ;  dX += dY[:, k*o:(k+1)*o] W_k
 *   SPLIT_IN   G_k += dY^T X[:, k*o:(k+1)*o] ;  dX[:, k*o:(k+1)*o] = dY W_k
 *              (times act'(preact) if act != NONE).
 * When this step rotates, the gradient part of this linear is handed to the
 * stage stream right after the dW kernel.  dX_dev may be NULL to skip the
 * input gradient.  Same state rules as rtp_linear_fwd, in a backward pass. */
rtp_status rtp_linear_bwd(rtp_linear *lin, int step, const void *X_dev, const void *dY_dev, void *dX_dev);

/* rtp_linear_fwd for callers that cannot allocate device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same steps, same kernels and same results as rtp_linear_fwd for an
 * input-partitioned (RTP_SPLIT_IN) bf16 / fp16 layer, but the fp32 accumulator
 * in which the n steps' partial products meet is a fixed array of
 * RTP_NOALLOC_ACC_BYTES inside the library's device image (each GPU the
 * library runs on holds it until the process ends) instead of
 * rtp_linear_desc.acc_ws_dev, which may then be NULL at rtp_linear_create.
 * The call itself allocates nothing (no hipMalloc, no hipFree, no allocating
 * library routine).  X [T, I], Y [T, O] device, as rtp_linear_fwd.
 * Errors: RTP_ERR_SHAPE if T * O * 4 exceeds RTP_NOALLOC_ACC_BYTES (nothing
 * is enqueued); RTP_ERR_UNSUPPORTED for an output-partitioned or fp32 layer
 * (they use no accumulator: call rtp_linear_fwd); otherwise rtp_linear_fwd's.
 * Every call on a GPU shares that GPU's array.  A pass's step 0 overwrites it
 * (nothing needs clearing), steps 1 .. n-1 add onto it and step n-1 rounds it
 * into Y; so the n step calls of one layer's pass must not be interleaved or
 * overlapped with those of another layer on the same GPU: such calls race. */
#define RTP_NOALLOC_ACC_BYTES (16u << 20)
rtp_status rtp_linear_fwd_noalloc(rtp_linear *lin, int step, const void *X_dev, void *Y_dev);

/* ---- MLP unit: the whole N-step loop in one call ------------------------ */

typedef struct {
    int64_t T, I, O, O2;  /* X[T, I]; W1 (or gate, up) [O, I]; W2 (down) [O2, O]   */
    int n, rank;
    rtp_mode mode;
    rtp_dtype dtype;      /* RTP_BF16, RTP_F16 or RTP_F32                         */
    rtp_act act;          /* GELU_* (one matrix) or SWIGLU (gate + up)            */
    unsigned flags;
    /* slot = [W1_k | W2_k] or [gate_k | up_k | down_k]; gradients fp32         */
    void *home_w_dev, *home_g_dev;
    void *buf_w_dev[2], *buf_g_dev[2];
    /* workspaces, Hw = rtp_mlp_hidden_width() columns per hidden unit row:    */
    void *preact_dev;     /* [T, P*Hw], P = 2 for SWIGLU                           */
    void *hidden_dev;     /* [T, Hw]                                               */
    void *dpre_dev;       /* [T, P*Hw]                                             */
    float *acc_y_dev;     /* fp32 [T, O2]                                          */
    float *acc_dx_dev;    /* fp32 [T, I]                                           */
    void *compute_stream, *stage_stream;
    void *aux_stream;     /* optional, as in rtp_ring_desc                           */
    void *step_sync_dev;  /* RTP_FLAG_FUSED_STEP only: rtp_mlp_step_sync_bytes() bytes of
                             device memory for the per-row-block counters of a fused
                             step (the library clears them when a pass begins)       */
    int has_bias;         /* every linear of the unit carries a bias: slot =
                             [W1_k | b1_k | W2_k | piece k of b2] (gated unit:
                             [gate_k ; up_k | bgate_k | bup_k | down_k | piece k of
                             bdown]), each linear's part padded to 16 bytes as
                             rtp_linear_shard_w_bytes gives it                       */
} rtp_mlp_desc;

/* Hidden width the unit computes on (FlatParameter paragraph: the flat
 * parameter is padded so that it divides evenly): O when n divides it,
 * otherwise n * rtp_shard_width(O, n, dtype).  Shard k then holds hidden units
 * [k w, (k+1) w); units past O are padding: their weights, biases and
 * gradients are zeros in the store (rtp_pack_shards writes them), so their
 * activations are act(0) = 0 and they change nothing.  The three hidden
 * workspaces have this many columns (times P); columns past O of each shard's
 * slice hold zeros after a pass.  -1 if the width cannot be split into n
 * non-empty aligned shards. */
int64_t rtp_mlp_hidden_width(const rtp_mlp_desc *d);

/* Bytes of rtp_mlp_desc.step_sync_dev: one int32 per 64 tokens and an error
 * word (rtp_mlp_sync returns RTP_ERR_HIP if a tile of a fused step ever gave
 * up its bounded wait). */
size_t rtp_mlp_step_sync_bytes(const rtp_mlp_desc *d);
size_t rtp_mlp_slot_w_bytes(const rtp_mlp_desc *d);
size_t rtp_mlp_slot_g_bytes(const rtp_mlp_desc *d);

/* An MLP block with its first GEMM output-partitioned and its second
 * input-partitioned, so that unit k is self-contained and rotates as one
 * message.  rtp_mlp_fwd runs n x (rtp_rotate_step, rtp_linear_fwd x 2);
 * rtp_mlp_bwd the mirror image.  For bf16 units in a staged mode whose shapes
 * the tiled kernel takes (all contraction lengths multiples of 32), the
 * forward pass instead issues the same GEMMs as grouped launches with the
 * second linear one step behind the first ({Z_t, down_{t-1}}), the shard
 * parts moving accordingly; so does the backward pass when no auxiliary
 * stream was given ({dX_{s-1}, dPre_s} and {dW1_s, dW2_s}).  Results, buffers
 * and bytes moved are the same; so are they for a unit with biases (the
 * pieces of the second linear's bias and the bias gradients are small kernels
 * between the launches).  RTP_FLAG_STEPWISE in `flags` keeps the
 * step-by-step sequence everywhere.  `rotate` = 0 skips the rotation calls (the
 * resident shard is used for every step: timing of compute alone, results
 * are meaningless); `compute` = 0 skips the kernels (timing of the staging
 * traffic alone). */
rtp_status rtp_mlp_create(rtp_mlp **out, const rtp_mlp_desc *desc);
rtp_status rtp_mlp_destroy(rtp_mlp *mlp);
rtp_status rtp_mlp_fwd(rtp_mlp *mlp, const void *X_dev, void *Y_dev);
rtp_status rtp_mlp_bwd(rtp_mlp *mlp, const void *X_dev, const void *dY_dev, void *dX_dev);
rtp_status rtp_mlp_set_ablation(rtp_mlp *mlp, int rotate, int compute);
rtp_status rtp_mlp_flush(rtp_mlp *mlp);
rtp_status rtp_mlp_sync(rtp_mlp *mlp);
rtp_ring *rtp_mlp_ring(rtp_mlp *mlp);

/* ---- expert partition: the ring's shard is one whole expert -------------- */

/* Expert partition (Partition Strategies section, last item; MoE block item
 * of the RTP Transformers section): n experts of one shape, worker `rank`
 * starts with expert `rank`, the experts rotate like any other shard and at
 * each step the worker runs the expert it holds on those of its own tokens
 * that are routed to it; the outputs of the n steps, back in token order, are
 * the layer's output (no token leaves the worker).  The paper gives no
 * router: the routing, one expert id per token, is an input.
 *
 * Slot e of the ring = [W1_e | W2_e], W1_e [O, I] (for RTP_ACT_SWIGLU
 * [gate_e ; up_e], 2*O rows), W2_e [O2, O]; gradients fp32 in the same order.
 * Inputs 16-bit (RTP_BF16: I, O, O2 multiples of 8; RTP_F16: of 32).
 * Workspace (device, caller-owned, Tp = rtp_moe_padded_rows(T, n) rows):
 * tokens grouped by expert, each group padded with zero rows to a multiple of
 * 32 rows. */
typedef struct {
    int64_t T, I, O, O2;
    int n, rank;
    rtp_mode mode;
    rtp_dtype dtype;
    rtp_act act;          /* GELU_* or SWIGLU                                      */
    unsigned flags;       /* RTP_FLAG_DRY_RUN is not available here                */
    void *home_w_dev, *home_g_dev;
    void *buf_w_dev[2], *buf_g_dev[2];
    void *xp_dev;         /* [Tp, I]    grouped tokens                             */
    void *preact_dev;     /* [Tp, P*O]  P = 2 for SWIGLU                           */
    void *hidden_dev;     /* [Tp, O]                                               */
    void *yp_dev;         /* [Tp, O2]   grouped outputs; grouped dY in backward    */
    void *dpre_dev;       /* [Tp, P*O]                                             */
    void *dxp_dev;        /* [Tp, I]                                               */
    int32_t *perm_dev;    /* [Tp]       token of each grouped row, -1 = padding    */
    int32_t *counts_dev;  /* [n + 1]    tokens per expert; [n] = ids out of range  */
    void *compute_stream, *stage_stream;
    void *aux_stream;     /* optional, as in rtp_ring_desc                         */
} rtp_moe_desc;

/* Rows of the grouped workspace: 32 * (T / 32 + n), an upper bound of the sum
 * of the padded group sizes for any routing.  -1 for bad arguments. */
int64_t rtp_moe_padded_rows(int64_t T, int n);
size_t rtp_moe_slot_w_bytes(const rtp_moe_desc *d);
size_t rtp_moe_slot_g_bytes(const rtp_moe_desc *d);

rtp_status rtp_moe_create(rtp_moe **out, const rtp_moe_desc *desc);
rtp_status rtp_moe_destroy(rtp_moe *moe);

/* Forward: groups the tokens by route_dev[t] (int32 in [0, n), device; a
 * stable grouping computed on the device), then n x (rotate, expert on its
 * group), then Y[t] = output of token t.  X [T, I], Y [T, O2] device.
 * The group sizes shape the GEMMs, so this call waits once for the grouping
 * kernel on the compute stream (it cannot be captured into a graph).
 * RTP_ERR_INVALID if an id is out of range (nothing else has run then). */
rtp_status rtp_moe_fwd(rtp_moe *moe, const void *X_dev, const int32_t *route_dev, void *Y_dev);

/* Backward of the last forward (its routing and saved activations):
 * per step G_e += its expert's weight gradients over the group (travelling
 * with the expert), dX[t] = gradient of token t.  dY [T, O2], dX [T, I].
 * RTP_ERR_STATE without a preceding forward. */
rtp_status rtp_moe_bwd(rtp_moe *moe, const void *dY_dev, void *dX_dev);

/* Group sizes (counts_out[n]) and first grouped row of each expert
 * (begin_out[n + 1]) of the last forward; either may be NULL.  Host arrays. */
rtp_status rtp_moe_routing(const rtp_moe *moe, int32_t *counts_out, int64_t *begin_out);
/* As rtp_mlp_set_ablation: timing of compute alone / of the staging traffic alone. */
rtp_status rtp_moe_set_ablation(rtp_moe *moe, int rotate, int compute);
rtp_status rtp_moe_flush(rtp_moe *moe);
rtp_status rtp_moe_sync(rtp_moe *moe);
rtp_ring *rtp_moe_ring(rtp_moe *moe);

/* ---- single GEMM launch (kernel tests and roofline timing) -------------- */

/* C[M,N] (+)= op(A) op(B) on `stream`, bf16 or f32 inputs, layout 0 NT
 * (A[M,K], B[N,K]), 1 NN (A[M,K], B[K,N]), 2 TN (A[K,M], B[K,N]); leading
 * dimensions in elements.  accumulate != 0 adds onto fp32 C (out_dtype must
 * be RTP_F32).  variant selects a tile configuration (0 = default).
 * Name of the kernel it launches: rtp_gemm_kernel_name(). */
rtp_status rtp_gemm(int layout, rtp_dtype in_dtype, rtp_dtype out_dtype, int accumulate,
                    const void *A_dev, int64_t lda, const void *B_dev, int64_t ldb,
                    void *C_dev, int64_t ldc, int64_t M, int64_t N, int64_t K,
                    int variant, void *stream);

/* Name (as a profiler shows it, up to template arguments) of the bf16 kernel
 * behind a layout and a non-zero variant; "" if there is none. */
const char *rtp_gemm_kernel_name(int layout, int variant);

/* ---- per-launch timing of the bf16 GEMM kernels -------------------------- */

/* Between rtp_prof_begin() and rtp_prof_end() every GEMM launch the
 * library makes (from any entry point) is bracketed by HIP events on the
 * stream it is launched on.  rtp_prof_end() waits for them and fills
 * out[layout] (0 NT, 1 NN, 2 TN) with the number of launches, the sum of
 * their durations and the sum of their flops (2 M N K each).  Process-wide,
 * not thread-safe; meant for benchmarks. */
typedef struct { int64_t launches; double total_ms; double total_flops; } rtp_prof_result;
rtp_status rtp_prof_begin(void);
/* The same with alone != 0: the host drains the device before and after every
 * timed launch, so each duration is that of the kernel running by itself (no
 * other GEMM, no staging copy beside it).  Slow; for reports only. */
rtp_status rtp_prof_begin_alone(int alone);
rtp_status rtp_prof_end(rtp_prof_result out[3]);

/* ---- sustained shader clock ------------------------------------------------ */

/* Enqueues a one-wave kernel on `stream` that spins for `wall_us` microseconds
 * of the constant-rate wall clock and then writes two int64 to `out_dev`
 * (device memory, 16 bytes): the wall-clock ticks and the shader-clock cycles
 * it saw.  Launched on a stream of its own beside the GEMMs it reports the
 * clock the chip sustains under that load (the figure the MFMA peak scales
 * with).  *wall_khz receives the wall clock's rate.  wall_us is capped at one
 * second. */
rtp_status rtp_clock_probe(void *stream, void *out_dev, int64_t wall_us, int *wall_khz);

#ifdef __cplusplus
}
#endif
#endif /* RTP_H_ */
