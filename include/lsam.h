/*
 * lsam.h -- C boundary of the K-replica LSAM step engine for AMD MI355X (gfx950).
 *
 * K worker replicas of one model live on one GPU.  `lsam_step` advances every replica by
 * one sharpness-aware local iteration; `lsam_sync` performs the center update for the
 * replicas whose communication period has elapsed.  The paper's asynchronous multi-worker
 * schedule (Algorithm 2, "Asynchronous Distributed LSAM") is replayed deterministically:
 * every call to `lsam_step` is one local iteration of every worker, and the period of each
 * worker comes from an explicit list or a seeded integer generator.
 *
 * Conventions
 *   - C linkage, no exceptions cross the boundary.  Every call returns 0 (or a count >= 0
 *     where stated) on success and a negative LSAM_E* code on failure;
 *     `lsam_last_error()` then returns a thread-local message.
 *   - Pointer arguments are marked [host] or [device].  The library never allocates or
 *     frees device memory: all device state lives in one caller-provided workspace
 *     (`lsam_workspace_bytes` tells its size) that must stay valid, and must not be
 *     touched by the caller, until `lsam_destroy`.  It must be 256-byte aligned.
 *   - All kernels are enqueued on the caller's stream (a hipStream_t passed as void*,
 *     NULL = the default stream).  `lsam_step` and `lsam_sync` do not block the host,
 *     allocate nothing and may be captured into a HIP graph (the host-side counters --
 *     periods, local counts, the noise step -- advance at capture, not at replay; see
 *     lsam_note_replay).  The
 *     read-out and restore calls synchronise the stream and move data through a pinned
 *     host staging buffer (64 MiB, allocated by the context on first use, freed by
 *     `lsam_destroy`).
 *   - A context is not thread-safe; use one per host thread.
 *
 * Flat parameter layout of one replica and of the center y (what `init_params` holds and
 * what `lsam_get_params` returns): for l = 1..L: W_l row-major [out_l, in_l], then
 * b_l [out_l].  In raw-vector mode (n_layers == 0) it is a plain vector of d_raw floats.
 *
 * Convolutional model (n_conv > 0; the paper's experiments train convolutional networks on
 * 32x32x3 images, Section "Experiments"): dims = C_0, ..., C_{n_conv}, F_1, ..., classes.
 * Layer l < n_conv maps C_l to C_{l+1} channels and stores its filters as W_l
 * [C_{l+1}, 3, 3, C_l] row-major, i.e. in_l = 9 C_l in the layout above; the first dense layer
 * reads the (pooled) image flattened in (row, column, channel) order, in_l = H' W' C_{n_conv}.
 * Images are [H, W, C] with the channel contiguous.  C_1..C_{n_conv} must be multiples of 8
 * and every pooled image must have even sides.  All tensors of this model, the input X
 * included, are fp32 in memory in both arithmetic modes: with LSAM_GEMM_BF16 every matrix
 * product (each convolution and dense layer, forward, dW and dX) rounds its two operands to
 * bfloat16 (nearest even) on their way into the matrix unit and accumulates in fp32; biases,
 * normalisation, pooling, the loss and the bias gradients (sums of the unrounded dZ) are fp32.
 * The pool's gradient goes to the first maximum of a window in row-major order.
 * A batch-normalised convolution (bn_mask) computes, per replica and channel over the B H W
 * positions of that replica's minibatch, Y = gamma (Z - mean) / sqrt(var + bn_eps) + beta before
 * the ReLU (training mode; the backward pass differentiates through mean and var; Appendix
 * "Batch Normalization": workers do not synchronise these statistics).  Its gamma [C_{l+1}]
 * and beta [C_{l+1}] follow b_l in the flat layout.  No running averages are kept.  The bias
 * b_l of such a layer cannot influence the loss; its gradient is reported as exactly zero.
 * LSAM_BUF_PERTURBED holds x~_i in both arithmetic modes of this model (no bf16 copy exists).
 * Residual networks (Section "Experiments" trains ResNet models; the blocks are the basic
 * blocks of He et al., "Deep Residual Learning for Image Recognition", in their CIFAR form):
 * stride_mask gives a convolution stride 2; skip_mask closes a block of two convolutions with a
 * shortcut from the block's input, which must be the ReLU output of a convolution (not a pool,
 * not the input image) and is taken as it is when the shapes agree and otherwise -- the block
 * halved the image and/or widened the channels -- as every second pixel in both directions with
 * zero channels appended (that paper's parameter-free shortcut).  The closing convolution must
 * be batch-normalised and must not be followed by a pool inside the block; channel counts of
 * the block input must be multiples of 4 and at most the block's output channels.
 * proj_mask (a subset of skip_mask) replaces the shortcut of a block by that paper's projection,
 * as its ResNet-18/34 use where a block changes shape: a 1x1 convolution of the block input
 * with the block's stride, C_{l-1} -> C_{l+1} channels, with bias, followed by a batch
 * normalisation of its own (same bn_eps, no ReLU).  Its parameters W_p [C_{l+1}, C_{l-1}],
 * b_p, gamma_p, beta_p [C_{l+1}] follow those of the closing convolution l in the flat layout;
 * b_p, like b_l, cannot influence the loss and its gradient is reported as exactly zero.  Any
 * channel counts (multiples of 8) are allowed on both sides of a projection.
 * preact = 1 reads the same layer list as the pre-activation blocks of wide residual networks
 * (Zagoruyko and Komodakis, "Wide Residual Networks"; Section "Experiments" trains WRN-16x10,
 * WRN-28x10 and WRN-40x10): a block's sum is taken on convolution outputs before any
 * normalisation, u_l = conv_l(a_{l-1}) + b_l [+ shortcut], a_l = relu(bn_l(u_l)); the shortcut of
 * the block closed by convolution l is u_{l-2} (same shape required) or, with bit l of proj_mask,
 * a 1x1 convolution (block stride, bias, no normalisation) of a_{l-2}, whose parameters are W_p
 * and b_p only.  Every convolution must be batch-normalised; then no convolution bias, b_p
 * included, influences the loss, and their gradients are reported as exactly zero.
 */
#ifndef LSAM_H
#define LSAM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LSAM_OK       0
#define LSAM_EINVAL  -1   /* bad argument or configuration                       */
#define LSAM_ENOMEM  -2   /* workspace too small / host allocation failed        */
#define LSAM_EHIP    -3   /* a HIP runtime call failed                           */
#define LSAM_ESTATE  -4   /* call not valid for this context (e.g. wrong mode)   */

#define LSAM_MAX_REPLICAS 64
#define LSAM_MAX_LAYERS   40

#define LSAM_GEMM_FP32 0  /* fp32 operands, fp32 accumulate                      */
#define LSAM_GEMM_BF16 1  /* bf16 operands, fp32 accumulate, fp32 master weights */

#define LSAM_SCHED_FIXED  0  /* periods drawn once at init                       */
#define LSAM_SCHED_REDRAW 1  /* a replica draws a new period at each of its syncs */

/* What the K replicas run.
 * LSAM_ALG_LSAM: Algorithm 2.  With rho = 0 the perturbed point is the point itself and the
 *   step makes one forward/backward pass instead of two (the ESGD / EASGD family of the
 *   "One-step LSAM / ESGD Update" algorithm; same results as the two-pass step).
 * LSAM_ALG_DATA_PARALLEL: the synchronous baseline of Section "Experiments" (DP-SAM; DP-SGD
 *   with rho = 0), communication interval 1: every step the K gradients are averaged, at the
 *   first pass and again at the perturbed point; the one perturbation and the one momentum
 *   step computed from the averages are applied to every replica.  No coupling term and no
 *   center: lambda, beta, lr_center and the periods are ignored, `lsam_sync` returns 0. */
#define LSAM_ALG_LSAM          0
#define LSAM_ALG_DATA_PARALLEL 1

typedef struct lsam_ctx lsam_ctx;

/* The fields follow the input list of Algorithm 2 (coupling strength, perturbation radius, the
 * two step sizes, communication period, look-ahead factor), plus the model shape. */
typedef struct {
  int32_t K;              /* number of replicas = the paper's n workers, 1..LSAM_MAX_REPLICAS */
  int32_t n_layers;       /* L dense layers; 0 selects raw-vector mode                */
  const int32_t* dims;    /* [host] L+1 entries in_0, out_1, ..., out_L (MLP mode);
                             channel counts for the convolution layers, see above     */
  int64_t d_raw;          /* parameters per replica, raw-vector mode only             */
  int32_t batch;          /* B samples per replica per step (MLP mode)                */
  int32_t gemm_dtype;     /* LSAM_GEMM_FP32 or LSAM_GEMM_BF16                         */
  float rho;              /* perturbation radius (Formulation, f_SAM)                 */
  float gamma;            /* stabiliser in rho*g/(||g||+gamma), >= 0                  */
  float lr;               /* eta: sampler step size                                   */
  float lr_center;        /* eta': center step size; the paper fixes 1.0              */
  float momentum;         /* mu of the momentum sampler (Section "Distributed Training") */
  float beta;             /* look-ahead factor of g = g' + beta (g' - g'_prev)        */
  float lambda0;          /* lambda_i = lambda0 / (lr * tau_i) (Appendix, Hyperparameter Search) */
  float lambda_abs;       /* if >= 0: fixed lambda for every replica instead          */
  int32_t nesterov;       /* 1: x -= lr (G + mu v);  0: x -= lr v                     */
  const int32_t* tau;     /* [host] K explicit periods >= 1, or NULL to draw them     */
  int32_t tau_min;        /* inclusive range of drawn periods                         */
  int32_t tau_max;
  uint64_t sched_seed;    /* s_0 of the period generator                              */
  int32_t sched_mode;     /* LSAM_SCHED_FIXED or LSAM_SCHED_REDRAW                    */
  int32_t algorithm;      /* LSAM_ALG_LSAM or LSAM_ALG_DATA_PARALLEL                  */
  float noise_scale;      /* sigma >= 0 of the Langevin sampler (Section "Langevin Dynamics
                             for Sampling"): x <- x - lr (G + mu v) + sigma sqrt(2 lr) xi with
                             xi ~ N(0, I) per replica, step and coordinate, drawn from
                             Philox4x32-10 counters (see csrc/langevin.h); 0 = noise-free,
                             as the paper's experiments run                            */
  uint64_t noise_seed;    /* key of that generator                                    */
  int32_t n_conv;         /* 0: dense model.  > 0: the first n_conv layers are 3x3 convolutions
                             (stride 1, zero rim 1, bias, ReLU), the rest dense; see below   */
  int32_t img_h, img_w;   /* input image sides (n_conv > 0)                           */
  float bn_eps;           /* epsilon of the normalisation, > 0 (or 0 with bn_mask = 0) */
  uint64_t pool_mask;     /* bit l set: a 2x2/stride-2 max-pool follows convolution l */
  uint64_t bn_mask;       /* bit l set: convolution l is batch-normalised before its ReLU */
  uint64_t stride_mask;   /* bit l set: convolution l has stride 2 (its output is [H/2, W/2]) */
  uint64_t skip_mask;     /* bit l set (l >= 2): convolutions l-1 and l form a residual block; the
                             block's input -- the image convolution l-1 read -- is added to the
                             normalised output of convolution l before its ReLU; see below   */
  uint64_t proj_mask;     /* bit l set (with bit l of skip_mask): that shortcut is a projection, a
                             1x1 convolution with batch normalisation; see below            */
  int32_t global_avg_pool; /* 1: the dense layers read the mean of the last image over its
                             positions (one value per channel) instead of the flattened image */
  int32_t preact;         /* 1: residual blocks are pre-activation blocks (wide residual
                             networks); see below                                      */
} lsam_config;

/* Which per-replica buffer `lsam_get_buffer` copies out. */
#define LSAM_BUF_PARAMS     0  /* x_i (replica -1: center y)                          */
#define LSAM_BUF_VELOCITY   1  /* v_i                                                  */
#define LSAM_BUF_ITER_SUM   2  /* S_i = sum of x_i's iterates since its last sync (zero
                                  right after the sync that served replica i)         */
#define LSAM_BUF_GRAD       3  /* gradient buffer (g2 after a step, but see
                                  lsam_set_fused_step; MLP mode only)                 */
#define LSAM_BUF_PERTURBED  4  /* fp32 mode: x~_i of the last step.  bf16 mode: the bf16
                                  operand copy of the weight matrices widened to fp32
                                  (it holds bf16(x_i) once a step has finished), with the
                                  biases, which have no bf16 copy, taken from x_i      */
#define LSAM_BUF_CENTER_DIR 5  /* g'_prev (replica ignored)                            */

/* Bytes of device workspace the configuration needs; 0 if the configuration is invalid
 * (then `lsam_last_error` says why).  Host-only, touches no GPU. */
size_t lsam_workspace_bytes(const lsam_config* cfg);

/* Creates a context (Algorithm 2, "Initialization").  `init_params` [host] holds either d
 * values, copied to all K replicas and to y, or (K+1)*d values: replicas 0..K-1, then y.
 * `n_init` is that count.  v, S, g'_prev and all counters start at zero.
 * `workspace` [device], `workspace_bytes` >= lsam_workspace_bytes(cfg).
 * `stream`: hipStream_t as void*.  The configuration (including dims/tau) is copied. */
int lsam_init(const lsam_config* cfg, const float* init_params, int64_t n_init,
              void* workspace, size_t workspace_bytes, void* stream, lsam_ctx** out);

/* One local iteration of every replica (Algorithm 2, asynchronous sampling step, with the
 * score of q(x|y) built from the SAM gradient of Theorem "Convergence of G_t with Constant
 * Perturbation"): forward/backward at x_i on (X_i, labels_i) -> g1; n = ||g1||_2 over the
 * whole replica; x~ = x + rho g1/(n + gamma); forward/backward at x~ on the same batch
 * -> g2; G = g2 + lambda_i (x_i - y); momentum update of x_i; S_i += x_i; c_i += 1.
 *   X      [device] [K, B, in_0] row-major; float in fp32 mode, bfloat16 in bf16 mode;
 *          convolutional model: [K, B, img_h, img_w, C_0] floats
 *   labels [device] [K, B] int32 class indices in [0, out_L)
 *   loss   [device] [K] floats receiving the first-pass mean cross-entropy, or NULL
 * MLP mode only (LSAM_ESTATE otherwise).  Labels are not range-checked on the host. */
int lsam_step(lsam_ctx* ctx, const void* X, const int32_t* labels, float* loss);

/* Raw-vector mode: same iteration with both gradients handed in.
 *   g1, g2 [device] [K, d_raw] floats, row stride d_raw.  Read only. */
int lsam_step_grads(lsam_ctx* ctx, const float* g1, const float* g2);

/* Center update (Algorithm 2, synchronous optimization step) for the due set
 * D = {i : c_i >= tau_i}: g' = sum_{i in D} S_i / sum_{i in D} c_i - y;
 * g = g' + beta (g' - g'_prev) (g = g' at the first sync); y += eta' g; g'_prev = g';
 * S_i = 0, c_i = 0 for i in D (and tau_i redrawn in redraw mode).
 * Returns |D| (0: nothing was due, nothing launched) or a negative error. */
int lsam_sync(lsam_ctx* ctx);

/* Copies replica `replica`'s parameters (or y for replica == -1) to `dst` [host] in the
 * flat layout; `n` must equal d.  Synchronises the stream. */
int lsam_get_params(lsam_ctx* ctx, int32_t replica, float* dst, int64_t n);

/* Same for the other per-replica buffers (LSAM_BUF_*). */
int lsam_get_buffer(lsam_ctx* ctx, int32_t which, int32_t replica, float* dst, int64_t n);

/* Overwrites one buffer from `src` [host] in the flat layout (restoring a snapshot taken
 * with lsam_get_buffer).  Checkpoint/resume of a run is: lsam_init with the same configuration,
 * this call for x_i, v_i, S_i, y and g'_prev, lsam_set_counters for the integer state, and
 * lsam_set_scalars if eta or rho had been changed.
 * Valid for LSAM_BUF_PARAMS (replica -1: y), LSAM_BUF_VELOCITY, LSAM_BUF_ITER_SUM and
 * LSAM_BUF_CENTER_DIR.  In bf16 mode setting a replica's parameters also refreshes its bf16
 * operand copy.  Synchronises the stream before and after the copy. */
int lsam_set_buffer(lsam_ctx* ctx, int32_t which, int32_t replica, const float* src, int64_t n);

/* Per-replica gradient norms ||g1_i|| of the last step: `dst` [host] [K]. Synchronises. */
int lsam_get_norms(lsam_ctx* ctx, float* dst);

/* Schedule state: any of the outputs may be NULL.  tau_out, count_out [host] [K]. */
int lsam_get_schedule(lsam_ctx* ctx, int32_t* tau_out, int32_t* count_out, int64_t* t_y_out);

/* In the bf16 dense model running Algorithm 2 without Langevin noise (and rho > 0), neither
 * gradient of a weight matrix is stored: both are used element by element only.  The
 * weight-gradient kernels of the first pass leave just the sums of squares the norm needs; once
 * the norm is known the same products are formed again and their epilogue writes the bf16
 * operand copy of x~ = x + rho g1/(||g1|| + gamma); the weight-gradient kernels of the pass at
 * the perturbed point take the sampler step on x, v, S and the operand copy where g2 is
 * produced.  Biases take the ordinary kernels.  Results are those of the separate kernels, bit
 * for bit.  With the fusion active the weight-matrix part of LSAM_BUF_GRAD is not written
 * (the bias parts hold g2); switch it off (on = 0) to have g1 / g2 stored as in the other
 * modes.  Returns 1 if steps of this context will use the fusion, 0 if not (other modes never
 * do), or a negative error. */
int lsam_set_fused_step(lsam_ctx* ctx, int32_t on);

/* Which kernels serve layer `layer` (0-based) of this context, for reports that attribute time
 * and work to kernel classes without restating the library's choices.  `info` [host] gets
 * LSAM_LAYER_INFO_FIELDS (8) values, `n` its capacity:
 *   [0] LSAM_LAYER_DENSE (GEMM kernels), LSAM_LAYER_HEAD (the two fused kernels of a narrow fp32
 *       classifier head), LSAM_LAYER_CONV_FIRST (first-layer convolution kernels),
 *       LSAM_LAYER_CONV_DIRECT (GEMM that unfolds the image on the fly), LSAM_LAYER_CONV_STORED
 *       (stored unfolded image + GEMM)
 *   [1] 1 if its input gradient goes through a stored unfolded gradient (convolutions)
 *   [2] 0: both weight gradients are stored; 1: fused path, norm from a weight-gradient product
 *       whose result is only summed; 2: fused path, norm from the Gram matrices of its factors
 *   [3] rows of its matrix products (B, or B H W of the layer's output for a convolution)
 *   [4], [5] columns of its weight matrix (fan-in) and its outputs
 *   [6] channels its projection shortcut reads (0: the layer closes no block with a projection;
 *       then three more products of [3] rows, [6] columns and [5] outputs belong to the layer)
 *   [7] pixel step of that projection (2: it reads every second pixel, through a gather) */
#define LSAM_LAYER_INFO_FIELDS 8
#define LSAM_LAYER_DENSE 0
#define LSAM_LAYER_HEAD 1
#define LSAM_LAYER_CONV_FIRST 2
#define LSAM_LAYER_CONV_DIRECT 3
#define LSAM_LAYER_CONV_STORED 4
int lsam_layer_info(lsam_ctx* ctx, int32_t layer, int32_t* info, int32_t n);

/* Tells the context that a HIP graph holding one captured lsam_step (or lsam_step_grads) has
 * been replayed once: the local counts c_i and the step number advance as they do in an eager
 * step, with no GPU work, so that an eager lsam_sync after the replay finds the replicas that
 * are due.  (Capturing a step advances them once as well.)  A captured step keeps the kernel
 * arguments it was captured with -- eta, rho, lambda_i = lambda0/(eta tau_i), the noise
 * counter -- so replay is only meaningful while those stay what they were: the call returns
 * LSAM_ESTATE with Langevin noise switched on, and in redraw mode when lambda_i depends on the
 * redrawn periods.  Call lsam_sync eagerly between replays: a captured lsam_sync would repeat the
 * center update for the due set it was captured with. */
int lsam_note_replay(lsam_ctx* ctx);

/* The integer state of Algorithm 2 that no buffer holds, `state` [host] [2K+3] int64:
 * the local iteration counts c_0..c_{K-1} since each replica's last sync (its t_x), the periods
 * tau_0..tau_{K-1} in force, the state of the period generator (as a bit pattern), the number
 * of center updates so far (t_y; 0 means g'_prev is not used by the next one) and the number of
 * sampler steps taken (the step word of the Langevin noise counters).  `n` must be 2K+3.
 * lsam_set_counters overwrites all of them (counts >= 0, periods >= 1, else LSAM_EINVAL and
 * nothing is changed).  Host-only, no GPU work. */
int lsam_get_counters(lsam_ctx* ctx, int64_t* state, int64_t n);
int lsam_set_counters(lsam_ctx* ctx, const int64_t* state, int64_t n);

/* Hidden activations A_layer = ReLU(Z_layer) [B, out_layer] of replica `replica` as the last
 * forward pass left them (after lsam_step: the pass at the perturbed point; the only pass when
 * rho = 0), for diagnosis: `dst` [host] row-major floats (bf16 mode: the stored bf16 values
 * widened), `n` = B * out_layer, layer in 1..L-1.  Dense models only (LSAM_ESTATE otherwise).
 * Synchronises the stream. */
int lsam_get_activation(lsam_ctx* ctx, int32_t layer, int32_t replica, float* dst, int64_t n);

/* Changes eta and rho from the next step on (decaying schedules eta_t, rho_t of the
 * convergence theorems are driven from the host through this call). */
int lsam_set_scalars(lsam_ctx* ctx, float lr, float rho);

/* Parameters per replica (d) of a configuration; -1 if invalid.  Host-only. */
int64_t lsam_num_params(const lsam_config* cfg);

/* Host-only replay of the schedule for `n_ticks` ticks (one step then one sync attempt
 * per tick): due_out [host] [n_ticks*K] gets 1 where replica i was served at that tick,
 * tau_out [host] [n_ticks*K] the period in force during that tick.  Touches no GPU. */
int lsam_schedule_replay(const lsam_config* cfg, int32_t n_ticks, int32_t* due_out,
                         int32_t* tau_out);

/* Per-kernel launch statistics gathered with HIP events when enabled: for profiling
 * only (it serialises nothing but adds two event records per launch).
 * `lsam_timing_read` synchronises the stream and fills, for up to `cap` kernel classes,
 * name pointers (static strings), launch counts and total milliseconds; returns the number
 * of classes.  `lsam_timing_enable(ctx, 0)` switches it off and clears the totals. */
int lsam_timing_enable(lsam_ctx* ctx, int32_t on);
int lsam_timing_read(lsam_ctx* ctx, int32_t cap, const char** names, int64_t* counts,
                     double* total_ms);

/* Ceilings of the device this process runs on, measured with the simplest kernels there are,
 * for reading kernel throughputs against (needs no context): a plain copy between the two
 * halves of `scratch` [device, 16-byte aligned, `scratch_bytes` >= 32 KiB; contents are
 * overwritten] in GB/s counting bytes read plus bytes written, and loops of independent MFMA
 * instructions on register operands in TFLOP/s, bf16 (32x32x16) and fp32 (32x32x2).
 * Runs on `stream` and blocks until done.  Returns LSAM_OK or LSAM_EINVAL / LSAM_EHIP. */
int lsam_probe_peaks(void* scratch, size_t scratch_bytes, void* stream, double* copy_gbytes_per_s,
                     double* mfma_bf16_tflops, double* mfma_fp32_tflops);

/* For callers that cannot allocate device memory or hold a context -- code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc: the raw-vector iteration of
 * lsam_step_grads as one stateless call.  Every array is the caller's; the scratch memory of
 * the gradient-norm reduction (K x 1024 partial sums, norms, scales: 512.5 KiB) is a fixed
 * device array inside the library, one copy per GPU, kept until the process ends.  The call
 * allocates and frees no device memory, calls no allocating library routine and does not
 * synchronise.
 *   x, v, S [device] [K, stride] floats, updated in place (x_i, v_i, S_i += new x_i)
 *   y       [device] [d] center, read only
 *   g1, g2  [device] [K, g_stride] gradients at x_i and at the perturbed point, read only
 *   xt      [device] [K, stride] receives x~_i = x_i + rho g1_i / (||g1_i|| + gamma); may be NULL
 *           when rho = 0 (then nothing is written)
 *   norms   [device] [K] receives ||g1_i||, or NULL
 *   lambda  [host] K coupling coefficients (the context-based call uses lambda0/(lr tau_i))
 * x, v, S, y, xt must be 16-byte aligned and `stride` a multiple of 4.  Limits: K <=
 * LSAM_MAX_REPLICAS, d <= LSAM_STATIC_MAX_D; beyond them the call returns LSAM_EINVAL and
 * launches nothing.  Results equal those of lsam_step_grads on the same values (same kernels).
 * All calls on one GPU share that GPU's scratch array: calls that may overlap in time on one
 * GPU (different streams, or different threads) race on it and must be serialised by the
 * caller; calls on one stream are ordered and safe.  Nothing in the array has to survive
 * between calls and every slot is written before it is read, so no clearing is needed. */
#define LSAM_STATIC_MAX_D (1LL << 34)
typedef struct {
  int32_t K;            /* replicas                                                  */
  int64_t d;            /* parameters per replica                                    */
  int64_t stride;       /* row stride of x, v, S, xt in floats, >= d                 */
  int64_t g_stride;     /* row stride of g1, g2 in floats, >= d                      */
  float rho, gamma;     /* perturbation radius and stabiliser                        */
  float lr, momentum;   /* eta and mu of the sampler step                            */
  int32_t nesterov;     /* 1: x -= lr (G + mu v);  0: x -= lr v                      */
  const float* lambda;  /* [host] K values                                           */
} lsam_update_desc;
int lsam_step_grads_static(const lsam_update_desc* u, float* x, float* v, float* S, const float* y,
                           const float* g1, const float* g2, float* xt, float* norms, void* stream);

void lsam_destroy(lsam_ctx* ctx);

const char* lsam_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LSAM_H */
