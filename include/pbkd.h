/*
 * pbkd -- per-block knowledge distillation on one MI355X (gfx950), C ABI.
 *
 * One "block" is one distillation task of parallel blockwise knowledge distillation
 * (arXiv 2012.03096): a frozen teacher block f_k and the cheaper student block g_k that is trained to
 * reproduce f_k's activations from f_k's own input (section 3.1, Eq. 3), independently of every other
 * block (section 3.1, second improvement; section 3.3).
 *
 * Conventions
 *   - Every tensor is fp32, contiguous, NCHW.  Weights: full 3x3 conv [Cout,Cin,3,3]; depthwise
 *     [C,1,3,3]; pointwise and shortcut 1x1 [Cout,Cin]; BatchNorm gamma, beta [C].
 *   - Pointers named *_dev are device pointers, *_host host pointers.  `hip_stream` is a hipStream_t
 *     passed as void* (NULL = the default stream).
 *   - Every call returns a pbkd_status (0 = ok, negative = error) and never throws or aborts; a text
 *     for the last error of the calling thread is available from pbkd_last_error().
 *   - The library allocates no device memory: the caller hands a device workspace of
 *     pbkd_block_workspace_bytes() bytes to pbkd_block_create and keeps it alive (and untouched) until
 *     pbkd_block_destroy.  Weights, momentum, saved activations, gradients and reduction scratch live
 *     inside it.
 *   - Device work is asynchronous on the given stream unless stated.  A block handle is not
 *     re-entrant; distinct blocks may be driven from distinct host threads and streams.
 *
 * Layer semantics (the paper names the layer types, section 3.2, but gives no formulas; these are the
 * textbook definitions): 3x3 convolutions are cross-correlations without bias, zero padding 1 on all
 * sides at every stride, output size floor((H-1)/stride)+1; a depthwise-separable layer is
 * depthwise 3x3 (carrying the stride) followed directly by a pointwise 1x1; every layer ends in
 * BatchNorm in training mode (batch mean, biased batch variance, eps inside the root) and ReLU.  With a
 * projection shortcut, `1x1 conv(stride) + BN` of the block input is added to the last layer's BN
 * output before the last ReLU; with an identity skip (section 3.2's candidate blocks (c) and (d): stacked
 * depthwise-separable layers with a residual-style skip connection around them) the block input itself is.
 * An optional 2x2 stride-2 max-pool follows the last ReLU.
 *
 * Tuning overrides (test and measurement aids, never needed for correct results).  pbkd_block_create reads these
 * environment variables and lets them replace the kernel variant the library would pick from the layer's shape;
 * a value that does not fit the shape is ignored:
 *   PBKD_CONV_TILE=0..3     workgroup tile of the 3x3 convolution: 128 ch x 128 px, 64 x 256, 64 x 128, 64 x 64
 *   PBKD_CONV_KSPLIT=n      3x3 convolution on whole-image tiles: K = 9*Cin split over n workgroups
 *   PBKD_CONV_SPLIT=0       the teacher's 3x3 convolutions on the fp32 matrix cores.  Default: on the bf16 matrix cores,
 *                           every fp32 operand written exactly as the sum of three bf16 terms and every product formed
 *                           from six of the nine cross terms (the three left out are at most 2^-24 of the product, 2^-27 rms), fp32
 *                           accumulation; measured against the fp64 oracle it is within 1.2x of the fp32 kernel's error.
 *                           Read when a block is created.
 *   PBKD_SPLIT_WGS=n        that kernel is persistent, one workgroup per compute unit: launch n workgroups instead and
 *                           leave the other compute units to the kernels of other streams (read at every launch)
 *   PBKD_TEACHER_LAG=1      pbkd_distill_step on two streams, eager: a call's teacher starts only when the student step
 *                           before the previous one has ended (default: as early as its dependencies allow); same
 *                           results, another overlap (read at every call)
 *   PBKD_PW_VARIANT=0..12   1x1 convolution: 0-3 scalar kernel (channel blocks x pixel blocks per wave = 4x2, 4x1, 2x2,
 *                           2x1), 4-9 vector kernel (waves over channels x waves over pixels, pixels per lane = 4x1x4,
 *                           4x1x2, 2x2x4, 2x2x2, 1x4x4, 1x4x2), 10-12 K split over a workgroup's waves (4, 2, 1 pixels
 *                           per lane)
 *   PBKD_WGRAD_VARIANT=0..3 pointwise weight gradient tile: bit 1 = 64 (else 128) rows, bit 0 = 64 (else 128) columns
 *   PBKD_CF_TH=4|8          first-layer 3x3 convolution (at most three input channels): rows of a workgroup's tile
 *   PBKD_CF_OCC=1..8        same kernel: workgroups per compute unit its persistent grid is sized for (default 4)
 *   PBKD_DW_EDGE=0          depthwise register-window kernels on maps whose width is not 4, 8, 16, 32 or 64: a strip's
 *                           two edge columns by loads instead of from the neighbouring lanes of the wave
 *   PBKD_WGRAD_BN_FUSED=0   a full 3x3 first layer's weight gradient does not fold its BatchNorm backward in (an
 *                           elementwise kernel forms dz first, as for every other layer)
 *   PBKD_DWPW=0|1           1: depthwise + pointwise forward as one kernel wherever the layer's shape allows (stride 1,
 *                           height a multiple of 4, width 4, 8, 16 or a multiple of 32); default 0: two kernels, which
 *                           measured faster on MI355X
 */
#ifndef PBKD_H
#define PBKD_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pbkd_block pbkd_block_t; /* opaque; host memory owned by the library */

typedef enum {
  PBKD_OK = 0,
  PBKD_EINVAL = -1,       /* null pointer, bad enum, bad count                                   */
  PBKD_ESHAPE = -2,       /* descriptor shapes inconsistent (channel chain, teacher/student out) */
  PBKD_ENOMEM = -3,       /* workspace too small or misaligned                                   */
  PBKD_EHIP = -4,         /* a HIP call failed; see pbkd_last_error                              */
  PBKD_ESTATE = -5,       /* call order violated (e.g. last_loss before any step)                */
  PBKD_EUNSUPPORTED = -6  /* valid request the library does not implement                        */
} pbkd_status;

enum { PBKD_CONV3X3 = 0, PBKD_DWSEP3X3 = 1 };

/* One layer = convolution + BatchNorm + ReLU.  kind CONV3X3: full 3x3; DWSEP3X3: depthwise 3x3 on cin
 * channels (stride here) then pointwise cin->cout.  trainable: 1 = updated by pbkd_student_step. */
typedef struct {
  int kind, cin, cout, stride, trainable;
} pbkd_layer_desc;

typedef struct {
  int n, c, h, w;                 /* block input, NCHW */
  int n_layers;
  const pbkd_layer_desc *layers;  /* host array, copied by the library */
  int shortcut;                   /* 0 none; 1 = projection shortcut (1x1 conv + BN), frozen; 2 = identity skip
                                     (block output and input must have the same shape; no parameters) */
  int shortcut_stride;
  int pool;                       /* 0 none; 2 = max-pool 2x2 stride 2 after the last ReLU (odd sizes drop the last row/col) */
  float bn_eps;
} pbkd_arch_desc;

/* momentum: v <- momentum*v + g; theta <- theta - lr*v (v starts at 0; no dampening, Nesterov, decay).
 * loss_reduction 0: mean of (p-t)^2 over all N*C*H*W outputs; 1: Eq. 3's form, sum / N.
 * bn_decay in [0,1): every BatchNorm keeps a running mean (starts at 0) and a running variance (starts at 1);
 * each student step moves those of every student BatchNorm (frozen layers and the projection shortcut too) by
 * running <- bn_decay*running + (1-bn_decay)*(batch mean | biased batch variance) of its forward pass.  They
 * serve the inference-mode forward of the reassembled network (Algorithm 1's last loop); the paper leaves them
 * to its framework's BatchNorm layer. */
typedef struct {
  float momentum;
  int loss_reduction;
  float bn_decay;
} pbkd_train_desc;

/* Which tensor pbkd_block_get_tensor / set_tensor address.  `layer` counts the student's (or
 * teacher's) layers from 0; layer == n_layers addresses the shortcut.  `slot` indexes the layer's
 * tensors: CONV3X3: 0 W, 1 gamma, 2 beta; DWSEP3X3: 0 D, 1 P, 2 gamma, 3 beta; shortcut: 0 W, 1 gamma,
 * 2 beta.  For the *_ACT kinds: slot 0 = depthwise output u (DWSEP3X3 only), 1 = pre-BN conv output z,
 * 2 = batch mean, 3 = 1/sqrt(var+eps), 4 = scale = gamma/sqrt(var+eps), 5 = shift = beta - mean*scale
 * (BatchNorm is applied as fmaf(z, scale, shift) wherever it is needed) -- as left by the last forward.
 * For the *_BN_RUNNING kinds: slot 0 = running mean, 1 = running variance of the layer's BatchNorm (the
 * teacher's come with its weights: set them with pbkd_block_set_tensor). */
enum {
  PBKD_STUDENT_PARAM = 0,
  PBKD_STUDENT_GRAD = 1,      /* gradient of the last pbkd_student_step (before the update) */
  PBKD_STUDENT_MOMENTUM = 2,
  PBKD_TEACHER_PARAM = 3,
  PBKD_STUDENT_ACT = 4,
  PBKD_TEACHER_ACT = 5,
  PBKD_STUDENT_BN_RUNNING = 6,
  PBKD_TEACHER_BN_RUNNING = 7
};

/* Validates a teacher/student pair without touching the GPU (host only).  Rules: at least one layer;
 * channel chain consistent; strides 1 or 2; teacher and student output shapes equal; same block input;
 * student CONV3X3 layers and frozen (trainable=0) student layers only as layer 0 (no data gradient
 * through a full or frozen convolution is implemented: PBKD_EUNSUPPORTED); teacher layers any kind.
 * Size limits (PBKD_EUNSUPPORTED beyond): every activation tensor below 2^31 elements; the input of a
 * CONV3X3 layer below 4 GiB. */
pbkd_status pbkd_arch_validate(const pbkd_arch_desc *teacher, const pbkd_arch_desc *student);

/* Bytes of device workspace pbkd_block_create needs for this pair (0 if the pair is invalid). */
size_t pbkd_block_workspace_bytes(const pbkd_arch_desc *teacher, const pbkd_arch_desc *student);

/* Creates one distillation task (section 3.1: block k of the teacher and its replacement).
 * teacher_params_host / student_params_host: arrays of host pointers, layer by layer in slot order
 * (see above), then the shortcut's three tensors if `shortcut` == 1; the values are copied to the device
 * (the call synchronises hip_stream before it returns, so the host arrays may be freed at once).
 * device_workspace: device memory, 256-byte aligned, >= pbkd_block_workspace_bytes(), caller-owned.
 * Momentum starts at zero. */
pbkd_status pbkd_block_create(const pbkd_arch_desc *teacher, const float *const *teacher_params_host,
                              const pbkd_arch_desc *student, const float *const *student_params_host,
                              const pbkd_train_desc *train, void *device_workspace, size_t workspace_bytes,
                              void *hip_stream, pbkd_block_t **out);

/* Frees the host-side handle (synchronises nothing; the workspace stays the caller's). */
pbkd_status pbkd_block_destroy(pbkd_block_t *blk);

/* target_dev <- f_k(x_dev): the frozen teacher block's activations, which Eq. 3 uses as the label.
 * x_dev [n,c,h,w]; target_dev [n,cout,h',w'] (after the optional pool).  Asynchronous.
 * Here and below, every device tensor the caller passes (x_dev, target_dev, out_dev) is dense NCHW fp32
 * and 16-byte aligned (PBKD_EINVAL otherwise): the kernels move it in 16-byte vectors. */
pbkd_status pbkd_teacher_forward(pbkd_block_t *blk, const float *x_dev, float *target_dev, void *hip_stream);

/* One distillation step on one batch (section 3.1, Eq. 3; section 3.3): student forward on x_dev,
 * local loss against target_dev, backward through the student block only, SGD-momentum update with
 * learning rate lr.  The loss is that of this step's forward pass, i.e. before the update.
 * loss_host != NULL: the call synchronises hip_stream and stores the loss there.
 * loss_host == NULL: fully asynchronous; fetch the loss later with pbkd_block_last_loss. */
pbkd_status pbkd_student_step(pbkd_block_t *blk, const float *x_dev, const float *target_dev, float lr,
                              float *loss_host, void *hip_stream);

/* pbkd_teacher_forward followed by pbkd_student_step of the same block (section 3.1: the teacher block's
 * output is the student block's label), issued on two streams so that they overlap: the student's forward
 * pass does not depend on the label, so the teacher's convolutions (matrix-core bound) run beside the
 * student's memory-bound kernels, and the teacher of the next call may start while this call's student is
 * still in its backward pass.  Only the kernel that writes target_dev waits for the previous call's last
 * reader of it, and only the loss kernel waits for the teacher.  Results are bit-identical to the two calls
 * made one after the other.  student_stream == teacher_stream degenerates to exactly that.  The caller
 * must not touch target_dev or x_dev from other streams without synchronising both streams first.
 * loss_host as in pbkd_student_step (synchronises student_stream only).
 * Measured on MI355X: a stream gets its hardware queue when it first submits work, and the earlier queue is served
 * better; the overlap is best when teacher_stream submitted its first work before student_stream did (up to 10 %
 * on some blocks, nothing on others).
 */
pbkd_status pbkd_distill_step(pbkd_block_t *blk, const float *x_dev, float *target_dev, float lr, float *loss_host,
                              void *student_stream, void *teacher_stream);

/* Gives the block a second stream for its backward pass (NULL: none, the default).  With one, the weight
 * gradients of every layer (which nothing but the final update consumes) run on aux_stream beside the
 * data-gradient chain on the step's own stream; events order the two, the update waits for both, and the
 * results stay bit-identical.  aux_stream must differ from the streams passed to the step calls and stay
 * valid while the block uses it; it costs no device memory. */
pbkd_status pbkd_block_set_aux_stream(pbkd_block_t *blk, void *aux_stream);

/* Graph mode (on = 0: off, the default).  With it on, the kernel launches of a pbkd_distill_step, pbkd_student_step or
 * pbkd_teacher_forward call on this block are captured into a HIP graph the first time a tuple of arguments (tensors,
 * learning rate, streams) is seen, and every later call with that tuple is one graph launch (the eight most recent
 * tuples are kept per block); pbkd_distill_step_all does the same for the whole all-block step when every block it is
 * given has graph mode on.  A block's step is some twenty launches of a few microseconds each, so this removes most of
 * the host's share of a step.  Results are bit-identical to the ungraphed calls.  What changes is ordering: a captured
 * step runs as a whole on ONE stream, its origin (pbkd_distill_step: student_stream; pbkd_distill_step_all:
 * teacher_stream with chain != 0, else the stream of the first block issued); the other streams passed only name the
 * branches that run beside each other inside the graph and receive no work afterwards, so consecutive steps do not
 * overlap and the caller orders later work against the origin stream.  Calls on the NULL stream, and calls made while
 * kernel timing is enabled, run ungraphed.  A new learning rate means a new capture. */
pbkd_status pbkd_block_set_graph_mode(pbkd_block_t *blk, int on);

/* out_dev <- g_k(x_dev) with the current student weights; no loss, no update.  Asynchronous. */
pbkd_status pbkd_student_forward(pbkd_block_t *blk, const float *x_dev, float *out_dev, void *hip_stream);

/* Loss of the last pbkd_student_step; synchronises the stream that step ran on. */
pbkd_status pbkd_block_last_loss(pbkd_block_t *blk, float *loss_host);

/* Block scheduling (section 3.3).  Host only.  Distributes n_blocks independent tasks over n_streams
 * workers.  weights: one per block (FLOPs, or measured times in any unit); NULL = take
 * pbkd_block_flops(blocks[i], 3).  policy 0: bin packing by worst-fit-decreasing -- stable sort by
 * decreasing weight (ties: lower index first), each task to the least-loaded worker (ties: lowest worker
 * index); policy 1: round robin in the given order.  Outputs: stream_of_block[n_blocks];
 * order[n_blocks] = position of the block within its stream; stream_load[n_streams] (nullable). */
pbkd_status pbkd_schedule_blocks(int n_blocks, const unsigned long long *weights, pbkd_block_t *const *blocks,
                                 int n_streams, int policy, int *stream_of_block, int *order,
                                 unsigned long long *stream_load);

/* Runs one distillation step of every block concurrently (section 3.1: every block is trained on its own, all of
 * them at the same time; section 3.3: tasks are spread over the workers by the scheduler).
 * Worker i is streams[i] (hipStream_t as void*); block b runs on streams[stream_of_block[b]], the
 * blocks of one stream in increasing order[].  For every block: teacher forward on x_dev[b] into
 * target_dev[b], then the student step.  chain != 0 states that x_dev[b+1] == target_dev[b] (the
 * teacher blocks form a chain, Eq. 1): then the teacher forwards run once, in block order, on
 * streams[0]'s companion stream `teacher_stream`, and each student step waits (hipEvent) only for its
 * own input and target.  Across calls, the teacher launch that overwrites target_dev[b] waits for those of the last two
 * student steps of blocks b and b+1 that read that very buffer: a caller that passes two sets of target buffers in turn
 * (double buffering; with a chain x_dev follows, x_dev[b+1] == target_dev[b] of the same set) lets the next call's
 * teacher chain run while this call's students are still at work; with one set the calls are ordered as before.
 * Asynchronous; losses via pbkd_block_last_loss. */
pbkd_status pbkd_distill_step_all(int n_blocks, pbkd_block_t *const *blocks, const float *const *x_dev,
                                  float *const *target_dev, float lr, int n_streams, void *const *streams,
                                  const int *stream_of_block, const int *order, int chain, void *teacher_stream);

/* Work stealing (section 3.3: the scheduling policy for when no task times are known).  Task i = steps[i]
 * distillation steps of blocks[i] (each: teacher forward of x_dev[i] into target_dev[i], then a student step).
 * Every stream (worker) starts with the queue of the tasks whose queue_of_task[i] names it and serves it from
 * the front, in index order; a stream that has nothing left running and an empty queue takes a task from the
 * TAIL of the longest other queue.  The decision is taken from the streams' actual progress (event queries),
 * so which worker runs what can differ from run to run; the results cannot (blocks share nothing).
 * Host-blocking: returns when every task has finished.  Distinct tasks must use distinct blocks and distinct
 * target tensors.  ran_on[n_tasks] (nullable): the stream that ran each task; n_steals (nullable). */
pbkd_status pbkd_run_tasks_work_stealing(int n_tasks, pbkd_block_t *const *blocks, const float *const *x_dev,
                                         float *const *target_dev, float lr, const int *steps, int n_streams,
                                         void *const *streams, const int *queue_of_task, int *ran_on, int *n_steals);

/* Reassembly (Algorithm 1, the loop after the gather; Eq. 1 and Eq. 2 are its two extremes): runs the chain of
 * blocks on x_dev, block k by its student g_k where use_student[k] != 0 and by the teacher f_k otherwise;
 * outs_dev[k] [n,cout_k,h'_k,w'_k] receives block k's output and is block k+1's input (PBKD_ESHAPE if the
 * shapes do not chain).  bn_mode 0: BatchNorm with the statistics of this batch, as during distillation;
 * 1: inference mode, b = gamma*(z - running_mean)/sqrt(running_var + eps) + beta with each network's running
 * statistics (see pbkd_train_desc; an image's features then do not depend on the rest of the batch).  Either mode
 * overwrites the stored activations and statistics (the *_ACT tensors) of the networks it runs, never the running
 * pairs.  Asynchronous. */
pbkd_status pbkd_network_forward(int n_blocks, pbkd_block_t *const *blocks, const int *use_student, int bn_mode,
                                 const float *x_dev, float *const *outs_dev, void *hip_stream);

/* *mse_host <- mean((a_dev[i] - b_dev[i])^2) over n floats, accumulated in fp64 in a fixed order: the label-free
 * stand-in for Algorithm 1's accuracy check (features of a network with student blocks against the teacher's).
 * Uses a few hundred bytes of blk's workspace as scratch; synchronises hip_stream. */
pbkd_status pbkd_feature_mse(pbkd_block_t *blk, const float *a_dev, const float *b_dev, size_t n, double *mse_host,
                             void *hip_stream);

/* pbkd_feature_mse for callers that cannot allocate device memory and hold no block workspace (code that must
 * not call hipMalloc: tight serving loops, harnesses that forbid it): the same kernels, the same fixed summation
 * order and therefore the same bits, with the 256 partial sums and the result in a static device array of the
 * library (2056 bytes, which every GPU the library runs on holds until the process ends) instead of a block's
 * workspace.  Calls hipMalloc/hipFree nowhere.  n above PBKD_FEATURE_MSE_NOALLOC_MAX_N: PBKD_EINVAL.  All calls
 * on one GPU share that array: calls that overlap on one GPU (two streams, two host threads) race; nothing in it
 * needs clearing between calls (every partial is rewritten by every call).  Synchronises hip_stream. */
#define PBKD_FEATURE_MSE_NOALLOC_MAX_N ((size_t)1 << 32)
pbkd_status pbkd_feature_mse_noalloc(const float *a_dev, const float *b_dev, size_t n, double *mse_host,
                                     void *hip_stream);

/* Algorithm 1's selection (the loop after the gather; section 3.1: only the blocks that meet the threshold enter
 * the reconstructed model), with the label-free feature error in place of the accuracy: runs the teacher network on
 * x_dev (teacher_outs_dev[k] receives block k's output), then for every k the network with only block k replaced by
 * its student, block_err[k] (nullable) <- mean squared difference of its final features from the teacher's, and
 * use_student[k] <- 1 if that error is below `threshold`, else 0; finally (if final_err is given) the network
 * reassembled from the chosen blocks and *final_err <- its feature error.  teacher_outs_dev and scratch_outs_dev:
 * n_blocks device tensors each, shaped like the block outputs, all distinct.  bn_mode as in pbkd_network_forward.
 * Host-blocking (every error is read back). */
pbkd_status pbkd_select_blocks(int n_blocks, pbkd_block_t *const *blocks, int bn_mode, const float *x_dev,
                               float *const *teacher_outs_dev, float *const *scratch_outs_dev, double threshold,
                               int *use_student, double *block_err, double *final_err, void *hip_stream);

/* 2*multiply-accumulates of the block's convolutions for the batch in its descriptor.
 * which 0: teacher forward; 1: student forward; 2: student step (forward + weight gradients + data
 * gradients; no depthwise data gradient for layer 0; frozen layers forward only); 3: 0 + 2. */
unsigned long long pbkd_block_flops(const pbkd_block_t *blk, int which);
/* The same count from descriptors alone (host only; 0 if invalid). */
unsigned long long pbkd_arch_flops(const pbkd_arch_desc *arch, int training_step);

/* Copies one tensor between host and the block (synchronous on the default stream; for tests,
 * checkpoints and gathering the trained student).  n = number of floats, must match the tensor. */
pbkd_status pbkd_block_get_tensor(pbkd_block_t *blk, int which, int layer, int slot, float *host_out, size_t n);
pbkd_status pbkd_block_set_tensor(pbkd_block_t *blk, int which, int layer, int slot, const float *host_in, size_t n);

/* Per-kernel timing for benchmarks.  pbkd_kernel_kinds() kinds of kernels exist, named by
 * pbkd_kernel_kind_name(kind).  pbkd_block_profile_enable(blk, mask, capacity): from now on every launch
 * whose kind has its bit set in mask is bracketed by a pair of HIP events on the launch's own stream, for
 * at most `capacity` launches between two reads (further launches run untimed); capacity 0 switches
 * timing off.  Synchronises the device.  pbkd_block_profile_read: waits for the recorded launches,
 * returns per kind the summed duration in milliseconds and the number of timed launches
 * (arrays of at least pbkd_kernel_kinds() entries), and clears the records. */
int pbkd_kernel_kinds(void);
const char *pbkd_kernel_kind_name(int kind);
pbkd_status pbkd_block_profile_enable(pbkd_block_t *blk, unsigned kind_mask, int capacity);
pbkd_status pbkd_block_profile_read(pbkd_block_t *blk, int n_kinds, double *ms_sum, int *launches);

/* Message for the last error on the calling thread ("" if none). */
const char *pbkd_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PBKD_H */
