/* pbd.h - C ABI of the MI355X blockwise-distillation library (libpbd.so).
 *
 * One GPU runs the whole step of blockwise distillation (Sec. II-A): the frozen
 * teacher is evaluated once, block by block, and every activation
 * A_0 = x, A_i = T_i(A_{i-1}) stays resident in device memory ("internal
 * relaying", Sec. VII-A; the one-device form of teacher relaying, Sec. IV-A).
 * Student block S_i then reads A_{i-1}, is compared with A_i by a mean squared
 * error, is back-propagated and is updated at once with SGD-momentum
 * (Algorithm 1: load, T.forward, S.forward, S.backward(L), update_weight; the
 * update needs no barrier because blocks share no parameters, Sec. IV-B).
 *
 * Conventions
 *  - Every function returns PBD_OK (0) or a negative pbd_status; nothing throws
 *    or aborts.  pbd_last_error() gives the text of the last failure of a context.
 *    Arguments are validated on the host before any kernel is launched.
 *  - "host" pointers are ordinary CPU memory; "device" pointers are HIP device
 *    memory owned by the caller.  The library never allocates device memory: the
 *    caller hands it one workspace (pbd_bind) that must outlive the context's use.
 *  - All kernels are enqueued on the stream given to pbd_bind; calls return
 *    without waiting unless stated.  Kernel faults surface in pbd_sync.
 *  - Blocks are numbered as in the paper for the step calls (i = 1..B) and from
 *    0 (b = i-1) where a single tensor of a block is addressed.
 *  - Host-side tensors are float32 in the textbook layouts: activations NCHW,
 *    convolution weights [C_out][C_in/groups][k][k].  Device activations are
 *    channel-last (NHWC) with the channel count padded to a multiple of 8.
 */
#ifndef PBD_H_
#define PBD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  PBD_OK = 0,
  PBD_EINVAL = -1,   /* null pointer, index out of range, non-finite scalar */
  PBD_ESHAPE = -2,   /* descriptor inconsistent, tensor size or view mismatch */
  PBD_ENOMEM_WS = -3,/* workspace missing, too small or misaligned */
  PBD_ESTATE = -4,   /* call out of order (not bound, no relay yet) */
  PBD_EHIP = -5      /* a HIP runtime call failed */
} pbd_status;

enum { PBD_F32 = 0, PBD_BF16 = 1 };                       /* arithmetic / storage type */
enum { PBD_TEACHER = 0, PBD_STUDENT = 1 };                /* net */
enum { PBD_WEIGHT = 0, PBD_GAMMA = 1, PBD_BETA = 2, PBD_RMEAN = 3, PBD_RVAR = 4 }; /* slot */
enum { PBD_PARAM = 0, PBD_GRAD = 1, PBD_MOMENTUM = 2, PBD_PROB = 3 };   /* kind (PBD_PROB: pbd_read_alpha only) */

typedef struct pbd_ctx pbd_ctx;

typedef struct {
  int32_t batch;        /* N, samples per step */
  int32_t precision;    /* PBD_F32: everything float32.  PBD_BF16: bf16 tensors and MFMA
                           operands, fp32 accumulation, statistics, gradients of
                           parameters, master weights and optimiser state */
  float momentum;       /* mu of  v <- mu v + g ; w <- w - lr v */
  float bn_eps;         /* added to the variance inside batch normalisation */
  float bn_momentum;    /* rate of the student's running statistics */
  int32_t force_direct; /* nonzero: run every convolution with the plain direct kernels
                           (testing aid; the MFMA kernels are the default for bf16) */
  int32_t no_graph;     /* nonzero: pbd_distill_step launches its kernels one by one instead of
                           replaying a captured HIP graph (for callers that capture the call
                           themselves, and for per-kernel hardware counters) */
} pbd_opts;

/* A borrowed view of an activation inside the workspace. */
typedef struct {
  void* ptr;            /* device; element (n,h,w,c) at ((n*h_ + h)*w_ + w)*c_phys + c */
  int32_t n, c, h, w;
  int32_t c_phys;       /* channels per pixel in memory, >= c, multiple of 8; pads are 0 */
  int32_t dtype;        /* PBD_F32 or PBD_BF16 */
} pbd_tensor;

/* One timed kernel launch (see pbd_set_profile). */
typedef struct {
  char name[32];        /* kernel class, e.g. "igemm_fwd_128x128_affine", "bn_apply" */
  float ms;             /* HIP-event time of this launch on the bound stream */
  double bytes;         /* algorithmic bytes: tensors the operation must touch once */
  double flops;         /* algorithmic flops: 2 x MACs of the unpadded problem, else 0 */
  int32_t net, block, op;
} pbd_prof_entry;

/* Build a context from a packed descriptor (host).  words/pool: the int32 record
 * stream and float64 pool that list the teacher blocks T_i and student blocks S_i
 * (Sec. II-A: both map A_{i-1} to tensors of one shape; create checks it).  Header
 * MAGIC 0x50424431, version 1, B, C0, H0, W0; then per net (teacher, student) and
 * block: n_ops and n_ops records of 20 words
 * [type, n_in, in0..in7, c_out, k, stride, pad, groups, act, pool_offset, 0,0,0];
 * type 1 conv+BN+activation, 2 max-pool, 3 add(+activation), 4 weighted sum.  Pure
 * host work, no GPU needed.  *out is owned by the caller until pbd_destroy. */
int pbd_create(const int32_t* words, int32_t nwords, const double* pool, int32_t npool,
               const pbd_opts* opts, pbd_ctx** out);
void pbd_destroy(pbd_ctx* ctx);

/* Text of the last error of ctx (host, owned by ctx; valid until the next call).
 * With ctx == NULL: why the last pbd_create on this thread failed. */
const char* pbd_last_error(const pbd_ctx* ctx);

int32_t pbd_num_blocks(const pbd_ctx* ctx);

/* Bytes of device workspace the context needs (relay store A_0..A_B, parameters,
 * optimiser state, saved activations, gradients, reduction scratch). */
size_t pbd_workspace_bytes(const pbd_ctx* ctx);

/* Adopt dev_ws (device, 256-byte aligned, >= pbd_workspace_bytes) and hip_stream
 * (a hipStream_t, may be null for the default stream).  Zero-fills parameters and
 * optimiser state, sets BN to the identity.  The caller keeps ownership. */
int pbd_bind(pbd_ctx* ctx, void* dev_ws, size_t bytes, void* hip_stream);

/* Copy one parameter tensor from host float32 (textbook layout) into the workspace,
 * or one parameter / gradient / momentum tensor back.  n = element count of the
 * textbook shape.  Both wait for the stream.  Slots RMEAN/RVAR exist for PBD_PARAM only. */
int pbd_load_param(pbd_ctx* ctx, int32_t net, int32_t b, int32_t op, int32_t slot,
                   const float* host, size_t n);
int pbd_read_tensor(pbd_ctx* ctx, int32_t kind, int32_t net, int32_t b, int32_t op,
                    int32_t slot, float* host, size_t n);

/* Copy A_i (i = 0..B) of the last relay to host as float32 NCHW; waits. */
int pbd_read_act(pbd_ctx* ctx, int32_t i, float* host, size_t n);
/* Copy value v of student block b (0 = its input, j+1 = output of op j) as saved by
 * the last step of that block, float32 NCHW.  When the blocks' scratch does not fit side by
 * side in the workspace they share one region and the values are valid only until another
 * block is stepped (PBD_ESTATE afterwards).  The output of a layer without activation whose only reader is
 * a two-input add is never written (the add is fused into the layer's normalisation pass; PBD_ESTATE);
 * read the add's output instead.  Likewise the output of a layer whose only reader is a max-pool (the pool
 * normalises the convolution output as it reads it).  Testing aid; waits. */
int pbd_read_value(pbd_ctx* ctx, int32_t b, int32_t v, float* host, size_t n);

/* More of what the last pbd_student_step of student block b (from 0) left behind, for checking one layer at a
 * time (testing aids like pbd_read_value; float32 NCHW; same validity rules; all wait):
 *  - pbd_read_conv_out: the output of the convolution of conv+BN op `op`, before normalisation.
 *  - pbd_read_batch_stats: that op's batch mean and 1 / sqrt(biased batch variance + eps), n = its channels.
 *  - pbd_read_grad_value: the stored gradient that belongs to value v (v >= 1).  For the output of a conv+BN op
 *    this is the gradient of loss_i (Sec. II-A) with respect to the CONVOLUTION output, i.e. already taken back
 *    through the activation and the normalisation (the tensor the op's weight gradient and backward-data are
 *    formed from); for the output of a pool, add or weighted-sum op it is the gradient with respect to the value
 *    itself.  Unspecified for values no gradient reached (e.g. after pbd_arch_step).  Not stored (PBD_ESTATE) for
 *    the block's output when the block ends in a two-input add that is fused into the normalisation pass of the
 *    layer before it: that layer's backward reduction forms 2 (S_i - A_i) / M_i itself. */
int pbd_read_conv_out(pbd_ctx* ctx, int32_t b, int32_t op, float* host, size_t n);
int pbd_read_batch_stats(pbd_ctx* ctx, int32_t b, int32_t op, float* mean_host, float* invstd_host, size_t n);
int pbd_read_grad_value(pbd_ctx* ctx, int32_t b, int32_t v, float* host, size_t n);

/* Teacher relay (Algorithm 1, load + T.forward; Sec. IV-A, Sec. VII-A).  x_dev:
 * device float32 NCHW [batch][C0][H0][W0].  Runs T_1..T_B once each in inference
 * mode and keeps every activation.  A (host array of B+1 views, may be null) gets
 * A_0..A_B, borrowed from the workspace and valid until the next relay. */
int pbd_teacher_relay(pbd_ctx* ctx, const float* x_dev, pbd_tensor* A);

/* The teacher WITHOUT relaying (Sec. III, Fig. 1: in the baseline every worker re-runs the
 * teacher from the input up to its own block): runs T_1..T_upto from x, upto in 1..B, and
 * leaves A_0..A_upto in the workspace; A (host array of upto+1 views, may be null) as in
 * pbd_teacher_relay.  Later activations are stale afterwards: pbd_student_step(i) and
 * pbd_read_act(i) need i <= upto (PBD_ESTATE otherwise).  Exists so that the cost of the
 * redundant teacher passes can be timed next to the relay on the same kernels. */
int pbd_teacher_prefix(pbd_ctx* ctx, const float* x_dev, int32_t upto, pbd_tensor* A);

/* One student block (Algorithm 1, S.forward, S.backward(L), update_weight; Sec. II-A
 * for L; Sec. IV-B for the immediate update).  i in 1..B.  A_prev, A_i: views returned
 * by the last relay for A_{i-1} and A_i (checked).  Forward with batch statistics,
 * loss_i = mean((S_i(A_{i-1}) - A_i)^2), backward through S_i only, then
 * v <- mu v + g, w <- w - lr v on S_i's parameters and the running-statistics
 * update.  loss_dev: device float32 scalar written by the stream (no host wait).
 * Any order of i gives the same results. */
int pbd_student_step(pbd_ctx* ctx, int32_t i, const pbd_tensor* A_prev, const pbd_tensor* A_i,
                     float lr, float* loss_dev);

/* pbd_student_step for callers that cannot allocate device memory and do not want a workspace region to be
 * written as scratch: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same results bit for bit.  The block's reduction scratch (partial sums of the loss, of the
 * batch-norm statistics and of the weight gradients, split-K partial tiles) is a 16 MiB static device array
 * inside the library instead of the workspace's scratch region; a block that needs more returns
 * PBD_ENOMEM_WS and launches nothing (pbd_student_step has no such limit).  The call allocates nothing on the
 * device or through HIP (no hipMalloc / hipFree, no events, no graph): it only launches kernels on the bound
 * stream; profiling must be off (PBD_ESTATE otherwise).  Each GPU holds one copy of the array until the
 * process ends and every call on that GPU shares it: calls that may overlap on one GPU (two contexts, two
 * streams) race, so order them.  Nothing in it has to start at zero (every partial result is written before
 * it is read), so the contents a previous call left behind are harmless. */
int pbd_student_step_static(pbd_ctx* ctx, int32_t i, const pbd_tensor* A_prev, const pbd_tensor* A_i,
                            float lr, float* loss_dev);

/* The whole step: relay, then every student block; no teacher block runs twice.
 * losses_dev: device float32[B].  Same results as the two calls above.  When the bound
 * stream is a real (non-null) stream and profiling is off, the body of the step is
 * captured once into a HIP graph and replayed on later calls (it only touches
 * workspace addresses; x_dev, lr and losses_dev stay outside the graph). */
int pbd_distill_step(pbd_ctx* ctx, const float* x_dev, float lr, float* losses_dev);

/* Architecture round of a supernet student (Sec. VI-A, neural architecture search: every step has a
 * second forward/backward round that trains the architecture parameters, and that round is an
 * ordinary training step of the block).  A type-4 op of the student computes z = sum_k p_k y_k over its
 * candidates with p = softmax(alpha).  The round runs the same forward (batch statistics, running
 * statistics updated) and the same loss as pbd_student_step, back-propagates to every mix op, forms
 *   g_k = <dL/dz, y_k>,   dL/dalpha_j = p_j (g_j - sum_k p_k g_k)
 * and applies v <- mu v + dL/dalpha, alpha <- alpha - lr_alpha v, p <- softmax(alpha).  Weights, gamma
 * and beta are frozen: their values and momenta are untouched (their gradient tensors are unspecified
 * afterwards), and layers with no mix op above them are not back-propagated at all.  Later weight
 * rounds mix with the new p.  Until alpha is loaded or first trained a mix uses the descriptor's
 * weights unchanged; the first round then starts from alpha_k = ln p_k, which requires those weights
 * to be positive and to sum to 1 (PBD_ESTATE otherwise: load alpha first).  Arguments as for
 * pbd_student_step.  A block without mix ops only gets its forward pass and loss. */
int pbd_arch_step(pbd_ctx* ctx, int32_t i, const pbd_tensor* A_prev, const pbd_tensor* A_i,
                  float lr_alpha, float* loss_dev);

/* Relay, then the architecture round of every block; arguments and graph capture as for
 * pbd_distill_step (the two rounds are captured separately). */
int pbd_distill_arch_step(pbd_ctx* ctx, const float* x_dev, float lr_alpha, float* losses_dev);

/* The whole step as one stage of a pipeline over batches (Sec. IV-A, teacher relaying, and Sec. IV-B,
 * decoupled updates: no student waits for another, so the teacher may go on to the next batch while
 * the students still train on the last one; Fig. 2d shows the schedule over devices, this is its
 * one-device form).  The call hands in batch k: the teacher relays it into the spare copy of the
 * activation store while, next to it, every student block trains on batch k-1 from the other copy, with
 * the learning rate that was passed along with batch k-1.  losses_dev (device float32[B]) receives the
 * losses of batch k-1; the first call after pbd_bind or pbd_pipeline_flush only runs the teacher and
 * leaves losses_dev alone.  pbd_pipeline_flush trains the students on the batch still waiting (nothing
 * if none) and writes its losses.  K calls and a flush leave the same parameters, statistics and losses,
 * bit for bit, as K calls of pbd_distill_step on the same batches.  x_dev is consumed by the call (it is
 * cast into the store).  Graph capture as for pbd_distill_step (one graph per copy).  While a batch waits,
 * the one-step calls (relay, prefix, student, architecture and whole steps) return PBD_ESTATE, the views
 * and pbd_read_act show the waiting batch, and pbd_read_value has nothing to show until the flush.
 * Parameters loaded while a batch waits are the ones its students then train from.
 * Which learning rate trains which batch: the one handed in WITH that batch, one call later.
 *     pbd_pipeline_step(ctx, x0, lr0, L);   // relays x0; no student work; L untouched
 *     pbd_pipeline_step(ctx, x1, lr1, L);   // relays x1; students train on x0 with lr0; L = losses of x0
 *     pbd_pipeline_flush(ctx, L);           // students train on x1 with lr1; L = losses of x1 */
int pbd_pipeline_step(pbd_ctx* ctx, const float* x_dev, float lr, float* losses_dev);
int pbd_pipeline_flush(pbd_ctx* ctx, float* losses_dev);

/* Order in which pbd_pipeline_step captures its B+1 independent branches into the graph: a permutation of
 * 0..B, where b < B is student block b (from 0) and B is the teacher's relay (Sec. IV-B: no block depends
 * on another, so every order computes the same bits).  The order decides how the replayed branches share
 * the GPU's hardware queues and moves the step time by a few per cent; the best one depends on the
 * workload, so a caller times a few and keeps the fastest.  Default: 0, 1, .., B.  n must be B+1
 * (PBD_EINVAL otherwise, also for a non-permutation); PBD_ESTATE while a batch waits.  Host-only apart
 * from a wait for the stream when a captured graph has to go. */
int pbd_set_pipeline_order(pbd_ctx* ctx, const int32_t* order, int32_t n);

/* Architecture parameters of student block b (from 0), op index op (a type-4 op with n inputs).
 * pbd_load_alpha copies n float32 from host and sets p = softmax(alpha); momentum is kept.
 * pbd_read_alpha copies alpha (PBD_PARAM), its last gradient (PBD_GRAD), its momentum (PBD_MOMENTUM)
 * or the weights p in use (PBD_PROB) to host; all but PBD_PROB need alpha to be defined (PBD_ESTATE).
 * Both wait for the stream. */
int pbd_load_alpha(pbd_ctx* ctx, int32_t b, int32_t op, const float* host, size_t n);
int pbd_read_alpha(pbd_ctx* ctx, int32_t kind, int32_t b, int32_t op, float* host, size_t n);

/* 1 if pbd_distill_step, pbd_distill_arch_step or pbd_pipeline_step currently replays a captured HIP
 * graph, 0 if they launch directly. */
int pbd_uses_graph(const pbd_ctx* ctx);

/* Wait for the bound stream; reports asynchronous failures. */
int pbd_sync(pbd_ctx* ctx);

/* Profiling: when on, every kernel launch is bracketed by HIP events on the bound
 * stream.  pbd_get_profile waits, then copies up to max entries of the launches
 * recorded since the last pbd_reset_profile and returns how many there were. */
int pbd_set_profile(pbd_ctx* ctx, int32_t on);
int pbd_reset_profile(pbd_ctx* ctx);
int pbd_get_profile(pbd_ctx* ctx, pbd_prof_entry* out, int32_t max);

#ifdef __cplusplus
}
#endif
#endif /* PBD_H_ */
