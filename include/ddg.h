/*
 * ddg.h - C boundary of the MI355X DDG module-step library.
 *
 * The operations follow "Decoupled Parallel Backpropagation with Convergence
 * Guarantee" (arXiv 1804.10574):
 *   - a feed-forward network is cut into K modules G(1..K) (Section 3);
 *   - in iteration t every module runs its forward pass on minibatch t
 *     (Section 3.1; Section 2, Eq. 3);
 *   - module k then back-propagates the error gradient of iteration
 *     s = t-K+k, which the module above produced one iteration earlier
 *     (Section 3.1, Eq. 6-7; Figure 2), and computes no gradient while s < 0
 *     (Section 3.3, Eq. 8);
 *   - every module updates its own weights (Eq. 9, Algorithm 1), here with
 *     the momentum SGD of Section 5.2.
 * The paper does not say how a module obtains its inner activations of
 * iteration s. This library keeps the module INPUT of the last K-k iterations
 * in a ring of device buffers and re-runs the module's forward on the stored
 * input with the module's current weights before back-propagating (for a module
 * with a delay, ddg_forward(t) does this in the same launches as the forward pass
 * on minibatch t: same weights, two minibatches, separate batch statistics).
 * ddg_module_desc.stale_jacobian selects the literal reading of Eq. 6-7 instead.
 *
 * Environment (read when a module or pipeline is created; all optional)
 *   DDG_NO_GRAPH=1   the pipeline enqueues every kernel instead of replaying graphs
 *   DDG_NO_PAIR=1    forward(t) and the re-forward run as separate passes
 *   DDG_NO_DEFER=1   every residual block runs its own normalise-add-ReLU pass
 *   DDG_NO_BWD_PAIR=1  the weight gradient of a layer runs in a launch of its own (with the
 *                    batch-norm backward fused into it) instead of beside the next
 *                    input-gradient kernel
 *   DDG_NO_WIDE=1    wide bf16 layers (>= 128 channels, stride 1) run the generic kernels
 *   DDG_NO_WIDE_BELOW=1  the input-gradient kernel of a wide layer leaves the batch-norm
 *                    backward sums of the layer below to a reduction pass
 *   DDG_NO_WGRAD_XCD=1  the wide weight-gradient kernel keeps the launch order of its workgroups
 *   DDG_NO_PREMASK=1 readers of an error gradient that was stored already multiplied by a
 *                    ReLU mask load the mask tensor and apply it again (same values)
 *   DDG_NO_LDS32=1   fp32 3x3 stride-1 layers run the gather kernels and separate batch-norm
 *                    passes instead of the LDS-tiled kernels
 *   DDG_CHECK_ORDER=1  ddg_pipeline_step also runs its host-side model of the stream ordering
 *                    (always on in dry-run pipelines) and fails with DDG_ERR_STATE, naming the
 *                    tensor, if the events it issues leave two accesses of a tensor unordered
 *   DDG_TUNE_CONV_GRID_C16/_C32/_C64, DDG_TUNE_WGRAD_ROWS[_C16/_C32/_C64], DDG_TUNE_WGRAD_WIDE_WGS,
 *   DDG_TUNE_WGRAD_GENERIC_WGS, DDG_TUNE_CONV_GRID_F32, DDG_TUNE_WGRAD_ROWS_F32
 *                    workgroup counts of the LDS-tiled kernels (clamped to safe ranges)
 * None of them changes a result beyond the order of floating-point sums.
 *
 * Conventions for every call
 *   - All tensor pointers are DEVICE pointers unless the argument says "host".
 *   - Activations and error gradients are NHWC (channels innermost), element
 *     type = the module's `compute` type (float, or bfloat16 stored as
 *     uint16_t, round-to-nearest-even).
 *   - Master weights, velocity, gradients, BN statistics and the loss are fp32.
 *   - The caller owns every pointer it passes; the library owns everything it
 *     allocates in ddg_module_create and frees it in ddg_module_destroy.
 *   - Calls enqueue work on the module's stream and return without waiting,
 *     except where a call says it synchronises. Ordering between modules
 *     (stream waits on the tensors they exchange) is the caller's job, or
 *     ddg_pipeline_* does it.
 *   - Every call returns a ddg_status; ddg_last_error() gives the message of
 *     the last failure on the calling thread. Argument, shape and state errors
 *     are detected before any device work and leave the module unchanged.
 */
#ifndef DDG_H
#define DDG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ddg_module ddg_module;     /* opaque */
typedef struct ddg_pipeline ddg_pipeline; /* opaque */

typedef enum {
  DDG_OK = 0,
  DDG_ERR_INVALID_ARG = 1, /* null pointer, bad enum, bad K/k                     */
  DDG_ERR_SHAPE = 2,       /* block list inconsistent or a shape no kernel covers */
  DDG_ERR_STATE = 3,       /* calls out of order, wrong iteration index           */
  DDG_ERR_OOM = 4,         /* device allocation failed                            */
  DDG_ERR_DEVICE = 5       /* any other HIP error (sticky on the handle)          */
} ddg_status;

typedef enum { DDG_F32 = 0, DDG_BF16 = 1 } ddg_dtype;

typedef enum {
  DDG_BLOCK_STEM = 0,       /* conv3x3(cin->cout, stride) + BN + ReLU                        */
  DDG_BLOCK_BASIC = 1,      /* conv3x3+BN+ReLU, conv3x3+BN, shortcut, add, ReLU (Table 2)     */
  DDG_BLOCK_BOTTLENECK = 2, /* conv1x1(cin->cmid)+BN+ReLU, conv3x3+BN+ReLU, conv1x1+BN, add   */
  DDG_BLOCK_HEAD = 3        /* global average pool + linear + softmax cross-entropy (loss f)  */
} ddg_block_kind;

/* One block. `projection` != 0 puts conv1x1(cin->cout, stride)+BN on the shortcut;
 * it is required when stride != 1 or cin != cout. For DDG_BLOCK_HEAD only cin is read. */
typedef struct {
  int kind;
  int cin, cmid, cout;
  int stride;
  int projection;
} ddg_block_desc;

typedef struct {
  int K, k;                    /* number of modules, 1-based index of this one; delay = K-k   */
  int batch, in_c, in_h, in_w; /* logical shape of the module input (stored NHWC)             */
  int num_blocks;
  const ddg_block_desc* blocks; /* host; copied                                               */
  int num_classes;             /* > 0 iff the last block is DDG_BLOCK_HEAD (then k must be K) */
  int compute;                 /* ddg_dtype of activations, error gradients, conv operands    */
  float momentum, weight_decay, bn_eps;
  void* stream;                /* hipStream_t the module's work is enqueued on (0 = default)  */
  void* forward_stream;        /* optional second hipStream_t: when given (and the delay K-k is
                                  > 0) ddg_forward runs on it, concurrently with the delayed
                                  backward of the same iteration on `stream` (both read the same
                                  weights; the update waits for both). 0: everything on `stream` */
  int dry_run;                 /* != 0: no device memory, no launches; only the argument and
                                  state checks run (lets host logic be tested without a GPU) */
  int stale_jacobian;          /* != 0: Eq. 6-7 read literally. ddg_forward(t) keeps every saved
                                  activation of iteration t and a snapshot of the weights it used
                                  (K-k+1 of each), and ddg_backward_delayed(t) back-propagates the
                                  delayed error gradient through the activations and weights of
                                  iteration t-K+k: no re-forward, (K-k+1) times the activation
                                  memory. 0 (default): only the module input is kept and it is
                                  re-forwarded with the current weights. forward_stream is
                                  ignored in this mode. */
} ddg_module_desc;

/* Section 3: create module G(k). Allocates weights, velocity, gradients, the input ring of
 * K-k+1 slots, saved activations and workspaces on the current device. Weights start at
 * zero: set them with ddg_set_params before the first forward. */
ddg_status ddg_module_create(const ddg_module_desc* desc, ddg_module** out);
ddg_status ddg_module_destroy(ddg_module* m);

/* Number of fp32 parameters. Flat order, per block: conv1.W, bn1.gamma, bn1.beta, conv2.W,
 * ..., then the projection's conv and BN if present; conv W is [Cout][Cin][R][S]; the head
 * holds fc.W[classes][C] then fc.b. Velocity and gradient use the same order. */
size_t ddg_param_count(const ddg_module* m);
/* Logical output shape (channels, height, width) of the module; batch is the input's. */
ddg_status ddg_out_shape(const ddg_module* m, int* c, int* h, int* w);
/* Device bytes the module holds. */
size_t ddg_device_bytes(const ddg_module* m);

/* Copy parameters in (src: host if !is_device, else device; fp32, ddg_param_count values) and
 * refresh the packed conv operands. Enqueued on the module's stream; a host source is read
 * before the call returns. */
ddg_status ddg_set_params(ddg_module* m, const float* src, int is_device);
/* Same for the momentum buffer (resuming a run; v starts at zero after create). */
ddg_status ddg_set_velocity(ddg_module* m, const float* src, int is_device);
/* Copy parameters / velocity / last gradient to HOST memory; synchronises the stream.
 * ddg_get_grad sets *valid = 0 if the last backward call computed no gradient. */
ddg_status ddg_get_params(ddg_module* m, float* host_dst);
ddg_status ddg_get_velocity(ddg_module* m, float* host_dst);
ddg_status ddg_get_grad(ddg_module* m, float* host_dst, int* valid);

/* Section 3.1 / Eq. 3: forward of module k on the minibatch of iteration t with the current
 * weights (BN uses batch statistics). h_in [batch,in_h,in_w,in_c] is copied into ring slot
 * t mod (K-k+1) and kept for K-k iterations; h_out [batch,out_h,out_w,out_c] receives the
 * module output (may be NULL when the module ends in the head). t counts iterations from 0
 * and must increase by exactly 1 from one forward call to the next. */
ddg_status ddg_forward(ddg_module* m, long t, const void* h_in, void* h_out);

/* Section 3.1, Eq. 6-7 and Eq. 8: delayed backward of iteration s = t-K+k. If s < 0 nothing
 * is computed and *did_backward = 0. Otherwise the input stored at iteration s is re-forwarded
 * with the current weights (the last module reuses the forward of this same iteration), then
 * delta_in = df/dh at the module output [batch,out_h,out_w,out_c] is back-propagated:
 * parameter gradients g_k^t go to the module's gradient buffer, and df/dh at the module input
 * is written to delta_out [batch,in_h,in_w,in_c] (NULL allowed when k == 1: never computed).
 * For the head module delta_in must be NULL and labels (device int32 [batch], class of each
 * sample of minibatch s = t) non-NULL; the mean cross-entropy is written to loss_out (device
 * float, may be NULL). did_backward is a host int, may be NULL. Must follow ddg_forward(t). */
ddg_status ddg_backward_delayed(ddg_module* m, long t, const void* delta_in, const int32_t* labels,
                                void* delta_out, float* loss_out, int* did_backward);

/* Eq. 9 / Algorithm 1 with momentum (Section 5.2): v <- mu*v + (g + wd*w); w <- w - lr*v,
 * then the packed conv operands are refreshed. A no-op while the module has no gradient
 * (s < 0). Must follow ddg_backward_delayed(t). */
ddg_status ddg_update(ddg_module* m, long t, float lr);

/* Algorithm 2 (Adam with delayed gradients) in place of momentum SGD: with kind = DDG_OPT_ADAM,
 * ddg_update applies, to the delayed gradient g (plus wd*w),
 *   m <- b1*m + (1-b1)*g;  v <- b2*v + (1-b2)*g^2;
 *   w <- w - lr * (m/(1-b1^n)) / (sqrt(v/(1-b2^n)) + eps),
 * where n counts the updates this module has executed (its warm-up iterations execute none).
 * The first moment lives in the velocity buffer (ddg_set_velocity / ddg_get_velocity), the
 * second in a buffer of its own; both start at zero, n at 0. Switching the kind keeps the
 * buffers as they are. Paper's constants: b1 = 0.9, b2 = 0.999, eps = 1e-8. */
enum { DDG_OPT_SGD = 0, DDG_OPT_ADAM = 1 };
ddg_status ddg_set_optimizer(ddg_module* m, int kind, float beta1, float beta2, float eps);
/* Second-moment buffer in / out (fp32, ddg_param_count values; same conventions as the velocity
 * calls) and the executed-update count n (resuming a run). */
ddg_status ddg_set_moment2(ddg_module* m, const float* src, int is_device);
ddg_status ddg_get_moment2(ddg_module* m, float* host_dst);
ddg_status ddg_set_update_count(ddg_module* m, long n);
long ddg_get_update_count(const ddg_module* m);

/* Evaluation (the paper reports test error, Section 5; batch normalisation at test time is
 * left to its citations). Every BN layer keeps running estimates of mean and variance,
 *   r <- (1-rho)*r + rho*(batch statistic),  variance unbiased (batch variance * m/(m-1)),
 * starting from mean 0 / variance 1, moved by ddg_forward's pass on minibatch t only (never
 * by the re-forward of a stored input). rho defaults to 0.1; it can be changed before the
 * first iteration (0 switches the estimates off). The estimates are a flat fp32 vector of
 * ddg_running_count values: per conv unit in parameter order, mean[C] then variance[C]; get /
 * set use host pointers and synchronise. */
ddg_status ddg_set_bn_momentum(ddg_module* m, float rho);
size_t ddg_running_count(const ddg_module* m);
ddg_status ddg_get_running(ddg_module* m, float* host_dst);
ddg_status ddg_set_running(ddg_module* m, const float* host_src);
/* Evaluation forward of the module on h_in [batch,in_h,in_w,in_c]: the same layers with every
 * BN normalising by its running estimates, current weights. Without a head the output goes to
 * h_out [batch,out_h,out_w,out_c]. With a head h_out is ignored; logits_out (device fp32
 * [batch][classes], may be NULL) receives the logits and loss_out (device float, may be NULL;
 * needs labels, device int32 [batch]) the mean cross-entropy. Allowed between iterations only
 * (after ddg_update, before the next ddg_forward); it overwrites the module's forward buffers
 * and nothing else: weights, estimates, the input ring and the gradient mailbox are
 * untouched. Not available in stale-Jacobian mode (DDG_ERR_STATE), where every set of forward
 * buffers holds a tape that a later backward pass needs. Enqueues on the module's stream. */
ddg_status ddg_forward_eval(ddg_module* m, const void* h_in, void* h_out, const int32_t* labels,
                            float* loss_out, float* logits_out);

/* For callers that cannot allocate device memory when they evaluate (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): ddg_forward_eval with every
 * intermediate of the pass (conv outputs, statistics rows, activations, block outputs, the
 * head's per-sample vectors) in a static device array that is part of the library, 64 MiB per
 * GPU, held until the process ends, instead of the module's forward buffers. Same arguments,
 * same results (the same kernels run). It calls no hipMalloc / hipFree and leaves the module's
 * forward buffers alone, so it is also available in stale-Jacobian mode. A module whose pass
 * needs more than the 64 MiB (two block outputs plus two blocks' worth of conv outputs; e.g.
 * ResNet-110's first module up to batch 256 fits) is refused with DDG_ERR_SHAPE and a message
 * that names both sizes. Every call on one GPU, from any module or thread, uses the same array:
 * calls that overlap on one GPU (different streams, or threads) race, so keep them on one
 * stream or order them yourself. Between iterations only, like ddg_forward_eval. */
ddg_status ddg_forward_eval_static(ddg_module* m, const void* h_in, void* h_out, const int32_t* labels,
                                   float* loss_out, float* logits_out);

/* Wait for the module's stream. */
ddg_status ddg_module_sync(ddg_module* m);

/* Checkpoint of the delay ring (Section 3.1: a module keeps its inputs for K-k iterations, so a
 * checkpoint of weights and velocity alone would have to replay the warm-up of Eq. 8). The ring
 * has ddg_ring_slots() = K-k+1 slots of ddg_ring_slot_bytes() bytes each (the module input,
 * [batch,in_h,in_w,in_c] in the compute type); slot i holds the input of the iteration t with
 * t mod (K-k+1) == i. get copies a slot to host memory, set copies host memory into a slot; both
 * synchronise. ddg_set_time makes t the next iteration the module expects (ddg_get_time reads
 * it): with weights, velocity (second moment, update count, running estimates) and ring slots
 * restored and the time set, a new module continues a run exactly where the checkpoint was taken.
 * Between iterations only (DDG_ERR_STATE otherwise), t >= 0; not in stale-Jacobian mode, whose
 * kept forward passes are not part of a checkpoint (DDG_ERR_STATE). */
int ddg_ring_slots(const ddg_module* m);
size_t ddg_ring_slot_bytes(const ddg_module* m);
ddg_status ddg_get_ring_slot(ddg_module* m, int slot, void* host_dst);
ddg_status ddg_set_ring_slot(ddg_module* m, int slot, const void* host_src);
ddg_status ddg_set_time(ddg_module* m, long t);
long ddg_get_time(const ddg_module* m);

/* ---- K modules as concurrent streams (Algorithm 1, "for k = 1..K in parallel") -------------
 * The pipeline owns the K modules, the activations handed from module k to k+1 and the
 * double-buffered error-gradient mailboxes handed from k+1 to k, and orders the streams with
 * events: forward runs k = 1..K in turn; the K backward passes and updates of one iteration
 * overlap. streams: K hipStream_t handles (host array) or NULL to run everything on stream 0
 * (serialised; results are identical). descs[i] describes module i+1; descs[i].stream is
 * ignored; descs[i].forward_stream, if set, gives module i+1 a forward stream of its own. */
ddg_status ddg_pipeline_create(const ddg_module_desc* descs, int K, void* const* streams,
                               ddg_pipeline** out);
ddg_status ddg_pipeline_destroy(ddg_pipeline* p);
ddg_module* ddg_pipeline_module(ddg_pipeline* p, int k);
/* One iteration: x [batch,in_h,in_w,in_c] in module 1's compute type, labels int32 [batch],
 * both device pointers whose contents are complete when the call is made and stay valid until
 * the step's work has run (they are first copied to pipeline-owned buffers on the pipeline's
 * streams); loss_out: device float or NULL. Iterations are counted internally from 0. */
ddg_status ddg_pipeline_step(ddg_pipeline* p, const void* x, const int32_t* labels, float lr,
                             float* loss_out);
/* The pipeline replays each module's forward and backward+update launches as captured HIP graphs
 * once every module computes a gradient (iteration >= K); on = 0 enqueues every kernel
 * individually instead (same results). Also off when the environment has DDG_NO_GRAPH=1. */
ddg_status ddg_pipeline_set_graphs(ddg_pipeline* p, int on);
/* ddg_set_optimizer on every module of the pipeline. */
ddg_status ddg_pipeline_set_optimizer(ddg_pipeline* p, int kind, float beta1, float beta2, float eps);
/* Evaluation forward of the whole network (ddg_forward_eval of module 1..K in turn) on x
 * [batch,in_h,in_w,in_c]; labels / loss_out / logits_out as for ddg_forward_eval of the head
 * module. Between iterations only; synchronises. */
ddg_status ddg_pipeline_forward_eval(ddg_pipeline* p, const void* x, const int32_t* labels, float* loss_out,
                                     float* logits_out);
/* ddg_set_bn_momentum on every module (before the first iteration). */
ddg_status ddg_pipeline_set_bn_momentum(ddg_pipeline* p, float rho);
/* Copy module k's latest forward output / the error gradient last delivered to module k
 * (mailbox) to host memory as fp32 NHWC; synchronises. *iteration receives the iteration the
 * mailbox content belongs to (-1: none yet). */
ddg_status ddg_pipeline_get_h(ddg_pipeline* p, int k, float* host_dst);
ddg_status ddg_pipeline_get_delta(ddg_pipeline* p, int k, float* host_dst, long* iteration);
ddg_status ddg_pipeline_sync(ddg_pipeline* p);
/* Checkpoint of the pipeline's own state between two iterations (Fig. 2: the error gradient
 * module k+1 computed in the last iteration is in flight to module k). ddg_pipeline_time: the
 * next iteration. ddg_pipeline_get_mail: that gradient for edge k (1 <= k < K), raw, in module
 * k's compute type (ddg_pipeline_mail_bytes(p, k) bytes), and the iteration it belongs to (-1:
 * none, then nothing is copied); synchronises. To resume: create the pipeline, restore every
 * module (weights, velocity, ring slots, ...; not their time), then ddg_pipeline_set_time(p, t)
 * (sets the time of every module too), then ddg_pipeline_set_mail for every edge whose
 * iteration was >= 0. The run then continues bit for bit as the checkpointed one would have. */
long ddg_pipeline_time(const ddg_pipeline* p);
ddg_status ddg_pipeline_set_time(ddg_pipeline* p, long t);
size_t ddg_pipeline_mail_bytes(const ddg_pipeline* p, int k);
ddg_status ddg_pipeline_get_mail(ddg_pipeline* p, int k, void* host_dst, long* iteration);
ddg_status ddg_pipeline_set_mail(ddg_pipeline* p, int k, const void* host_src, long iteration);

/* ---- measurement ----------------------------------------------------------------------------
 * Per-kernel-family timing with HIP events on the module's stream. While enabled, every launch
 * of a kernel family is bracketed by two events; ddg_profile_read synchronises and returns, for
 * family `kind` (0 <= kind < ddg_profile_kinds()), since the last reset: the number of launches,
 * their summed duration in milliseconds, and their summed algorithmic work: bytes (each tensor a
 * launch must read, once, plus each tensor it must write, once, in its storage type) and flops
 * (2*M*N*K per convolution pass). Any output pointer may be NULL. */
int ddg_profile_kinds(void);
const char* ddg_profile_kind_name(int kind);
ddg_status ddg_profile_enable(ddg_module* m, int on);
ddg_status ddg_profile_read(ddg_module* m, int kind, long* launches, double* total_ms, double* bytes,
                            double* flops);
ddg_status ddg_profile_reset(ddg_module* m);

const char* ddg_last_error(void);
const char* ddg_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DDG_H */
