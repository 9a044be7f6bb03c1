/*
 * ols.h -- C boundary of the Overlap Local-SGD hot path on one MI355X (gfx950).
 *
 * The library holds m simulated workers as m model replicas resident in HBM and
 * runs the iteration of arXiv 2002.09539, Section 2 ("Proposed Algorithm"):
 *
 *   local step   x_{k+1/2}^{(i)} = x_k^{(i)} - gamma g_i(x_k^{(i)}; xi_k^{(i)})
 *   pull-back    x_{k+1}^{(i)}   = x_{k+1/2}^{(i)} - alpha (x_{k+1/2}^{(i)} - z_k)    when (k+1) mod tau == 0
 *   anchor       z_{k+1}         = (1/m) sum_i x_{k+1}^{(i)}                          when (k+1) mod tau == 0
 *
 * with the anchor refresh running on a side stream while the next round's local
 * steps run on the main stream (the overlap the paper describes around its
 * timeline figure), and the optional momentum variant of the same section.
 *
 * General conventions
 *   - Every pointer named *_dev is DEVICE memory owned by the caller and must stay
 *     valid until ols_destroy or until it is re-bound.  The library allocates no
 *     device memory; it owns only HIP events.  Streams are hipStream_t handles
 *     passed as void* and are owned by the caller (default priority).
 *   - All state tensors are fp32.  Replica-major layout: row i of x/buf/g is worker
 *     i's flat parameter / momentum / gradient vector; rows are `ld` elements apart,
 *     ld = ols_row_stride(d) (d rounded up to a multiple of 64 so rows are 256-byte
 *     aligned).  Elements [d, ld) of every row are padding: the caller zero-fills
 *     them once and never reads them.
 *   - Every call returns OLS_OK (0) or a negative error code; ols_last_error()
 *     returns a thread-local message for the last failure.  Calls are asynchronous
 *     with respect to the host unless stated otherwise.  A handle is not thread-safe.
 *   - There is no CPU fallback: every step runs in HIP kernels, and a missing
 *     device makes the first launching call fail with OLS_EHIP.
 */
#ifndef OLS_H
#define OLS_H

#include <stddef.h>
#include <stdint.h>

#if defined(__GNUC__)
#define OLS_API __attribute__((visibility("default")))
#else
#define OLS_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ols_ctx* ols_handle;

enum {
    OLS_OK = 0,
    OLS_EINVAL = -1, /* bad argument                                  */
    OLS_ESTATE = -2, /* call out of order for the algorithm's schedule */
    OLS_EHIP = -3,   /* HIP runtime failure                            */
    OLS_ENOMEM = -4  /* caller-provided workspace too small            */
};

/* keys of ols_set_option */
enum {
    OLS_OPT_NESTEROV = 1,      /* 1 (default): local step direction g + mu buf; 0: heavy ball (direction buf) */
    OLS_OPT_FUSE_PULL = 2,     /* 1 (default): the tau-th local step of a round defers its parameter write and
                                  ols_sync_pull applies step + pull-back in ONE pass over HBM; 0: two passes.
                                  Both orders execute the same fp32 operation sequence per element.           */
    OLS_OPT_SERIALIZE = 3,     /* 0: the anchor refresh runs on the side stream, overlapped with the next round
                                  (the paper's schedule); 1: on the main stream (blocking); 2 (default): overlapped
                                  unless the refresh moves at most 1 MiB ((4 m + 4) ld bytes), where the two
                                  cross-stream synchronisations of a round cost more than the refresh they would
                                  hide.  Results are identical bit for bit in all three.                        */
    OLS_OPT_DRY_RUN = 4,       /* 1: advance the schedule and record the launch trace but launch nothing
                                  (host-logic tests on machines without a GPU); default 0                     */
    OLS_OPT_KERNEL_TIMING = 5, /* 1: bracket every kernel with HIP events on its own stream and accumulate
                                  per-kernel durations (see ols_kernel_stats); default 0                      */
    OLS_OPT_TRACE = 6,         /* 1: keep a host-side log of launches (see ols_trace_get); default 0          */
    OLS_OPT_MEAN_SPLIT = 7,    /* anchor-mean kernel: 0 = choose from (m, d); 1, 2, 4, 8 or 16 = number of
                                  lane groups / wavefronts of a workgroup sharing the replica axis (combined by
                                  wavefront shuffles, then an LDS tree)                                       */
    OLS_OPT_FUSE_MEAN = 8,     /* 1: ols_sync_pull also produces the new anchor in the same pass (each thread
                                  owns a parameter column across all m replicas); ols_anchor_update_async then
                                  only publishes it.  Removes the separate reduction instead of hiding it.
                                  default 0                                                                   */
    OLS_OPT_TUNING = 9,            /* TUNING, UNSTABLE -- not part of the interface a caller should rely on.  Selects a
                                      tile-shape variant of one GEMM kernel for re-measurement: value = 256 * which +
                                      variant, which = 0 forward, 1 weight gradient, 2 delta GEMM; variant 0 (default)
                                      lets the library choose from the shape.  The default build carries only the
                                      variants that choice can pick (bit-identical among themselves where tests say
                                      so); building with -DOLS_TUNING_VARIANTS adds the others.  A variant the build
                                      does not carry makes the next local step fail with OLS_EHIP.  (Keys 10 and 11
                                      are unused.)                                                                 */
    OLS_OPT_GEMM_SPLITK = 12,      /* fp32 forward GEMM: K ranges per output tile where the shape calls for
                                      splitting (0 = from the shape, 1 = never, up to 8)                       */
    OLS_OPT_FUSE_GEMM_UPDATE = 13, /* 1 (default): with an attached MLP (or a least-squares model of at most 64 samples
                                      per batch and 4096 parameters) the kernels that form the gradients apply
                                      the local step (and on the tau-th step the pull-back) where each gradient
                                      element is produced, so g is never written nor re-read and ols_sync_pull only
                                      publishes the result; 0: gradients go to g and the streaming kernels update.
                                      With an MLP both routes execute the same fp32 operation sequence per element
                                      (identical bits); the one-launch least-squares kernel sums in another order. */
    OLS_OPT_GEMM_FORCE_GENERAL = 14, /* 1: the GEMMs always take their bounds-checked kernel, also on
                                      shapes the full-tile kernel covers (both give identical bits); default 0     */
    OLS_OPT_ANCHOR_DELAY_US = 15,  /* emulated communication latency, 0 (default) .. 1000000 microseconds: a kernel
                                      that only waits that long runs ahead of every anchor refresh on the refresh's
                                      stream, standing in for the all-reduce time of a real cluster (Section 2: the
                                      latency is hidden while it is shorter than tau local steps; Section 4's
                                      comparison with blocking synchronisation is OLS_OPT_SERIALIZE = 1 with the same
                                      delay).  Results do not depend on it.  Ignored where the anchor is produced by
                                      the pull pass itself (OLS_OPT_FUSE_MEAN, ols_set_mixing).                    */
    OLS_OPT_HEAD_DW_GUEST = 16     /* 1 (default): with an attached MLP that has a hidden layer, the output layer's
                                      weight / bias gradients (and their fused update) are computed by extra
                                      workgroups at the front of the launch of the last hidden layer's
                                      weight-gradient GEMM instead of a kernel of their own (OLS_K_HEAD_BWD then
                                      does not appear); same arithmetic, identical bits                          */
};

/* kernel kinds for ols_kernel_stats / the launch trace */
enum {
    OLS_K_INIT = 0,
    OLS_K_STEP = 1,       /* momentum / plain local step                */
    OLS_K_STEP_PULL = 2,  /* fused local step + pull-back               */
    OLS_K_PULL = 3,       /* stand-alone pull-back                      */
    OLS_K_MEAN = 4,       /* replica-axis mean (anchor refresh)         */
    OLS_K_STEP_PULL_MEAN = 5,
    OLS_K_LSQ_RESID = 6,
    OLS_K_LSQ_GRAD = 7,
    OLS_K_GEMM_FWD = 8,   /* hidden layer forward, bias + ReLU epilogue */
    OLS_K_GEMM_DW = 9,    /* weight gradient A^T dZ                     */
    OLS_K_GEMM_DA = 10,   /* back-propagated delta dZ W^T, ReLU mask    */
    OLS_K_HEAD_FWD = 11,  /* output layer + softmax cross-entropy       */
    OLS_K_HEAD_BWD = 12,  /* output layer gradients and delta           */
    OLS_K_MIX = 13,       /* general mixing X <- X W (ols_set_mixing)    */
    OLS_K_CAST = 14,      /* fp32 -> bf16 operand conversion            */
    OLS_K_DELAY = 15,     /* emulated communication latency (OLS_OPT_ANCHOR_DELAY_US) */
    OLS_K_LSQ_STEP = 16,  /* least squares, small problems: gradient and local step in one launch */
    OLS_K_STALE_SYNC = 17, /* stale-average synchronisation (ols_set_stale_average) */
    OLS_K_CONV_FWD = 18,  /* 3 x 3 convolution forward (bias, shortcut, ReLU in the epilogue) */
    OLS_K_CONV_DX = 19,   /* delta back-propagated through a 3 x 3 convolution, ReLU mask    */
    OLS_K_CONV_DW = 20,   /* kernel and bias gradient of a 3 x 3 convolution                 */
    OLS_K_POOL = 21,      /* global average pooling in front of the classifier               */
    OLS_K_POOL_BWD = 22,  /* its backward                                                    */
    OLS_K_BN_FWD = 23,    /* batch normalisation: statistics (two launches) + normalise, shortcut, ReLU */
    OLS_K_BN_BWD = 24,    /* its backward: scale / shift gradients (two launches) + gradient at the input */
    OLS_K_COUNT = 25
};

typedef struct ols_trace_entry {
    int32_t kind;      /* OLS_K_*                                         */
    int32_t stream;    /* 0 = main, 1 = side                              */
    int32_t src_buf;   /* which replica buffer was read: 0 = x, 1 = x_alt */
    int32_t dst_buf;   /* which replica buffer was written (-1: none)     */
    int32_t waited;    /* 1 if the launch was preceded by a cross-stream event wait */
    int32_t k;         /* local iterations completed when it was enqueued */
} ols_trace_entry;

/* ---- life cycle ------------------------------------------------------------------------------ */

/* Creates the schedule state for m workers with d parameters each (Section 2 notation: tau local
 * steps per round, pull-back strength alpha, learning rate gamma).  beta is the LOCAL momentum
 * factor mu of the "Momentum Variant" paragraph (0 disables the momentum buffer); the paper's own
 * beta (anchor momentum) is set with ols_set_anchor_momentum.
 * Requires m >= 1, d >= 1, tau >= 1, 0 <= alpha <= 1, gamma > 0, 0 <= beta < 1.
 * Touches no device.  Returns NULL on error (see ols_last_error). */
OLS_API ols_handle ols_create(int m, int64_t d, int tau, float alpha, float gamma, float beta);

/* Destroys the handle and its events.  Drains both streams first if anything was launched. */
OLS_API int ols_destroy(ols_handle h);

/* Row stride (elements) the state tensors must use for d parameters: d rounded up to 64. */
OLS_API int64_t ols_row_stride(int64_t d);

/* Binds caller-owned device state.
 *   x_dev      [m][ld]  replica parameters (current buffer)
 *   x_alt_dev  [m][ld]  second replica buffer for the overlap, or NULL.  With it, the first update
 *                       after an anchor refresh is written out-of-place so the side stream can
 *                       still read the round-boundary models; without it that update first waits
 *                       for the refresh (gradient computation still overlaps).
 *   buf_dev    [m][ld]  local momentum buffers; may be NULL iff beta == 0
 *   g_dev      [m][ld]  stochastic gradients (written by the attached model, or by the caller)
 *   z_dev      [ld]     anchor model
 *   ld         must equal ols_row_stride(d)
 *   main_stream, side_stream  hipStream_t; side_stream may equal main_stream (forces serial order)
 * All pointers must be 256-byte aligned.  Errors: OLS_EINVAL. */
OLS_API int ols_bind(ols_handle h, float* x_dev, float* x_alt_dev, float* buf_dev, float* g_dev, float* z_dev,
             int64_t ld, void* main_stream, void* side_stream);

/* Sets x^{(i)} = z = x0 for every worker (Theorem 1's common starting point), zeroes the momentum
 * buffers and resets k to 0.  x0_dev: [d] fp32 on the device.  Asynchronous on the main stream. */
OLS_API int ols_init_params(ols_handle h, const float* x0_dev);

/* Anchor momentum of the "Momentum Variant" paragraph: v <- beta_z v + (mean_i x^{(i)} - z),
 * z <- z + v.  v_dev: [ld] device buffer (zero-filled by the caller), or NULL with beta_z == 0 to
 * return to the plain average.  Must be called before the first local step. */
OLS_API int ols_set_anchor_momentum(ols_handle h, float beta_z, float* v_dev);

/* General mixing (Section 2, "Matrix-Form Update Rule": X_{k+1} = (X_k - gamma G_k) W_k with
 * X = [x^(1), ..., x^(m), z]; the section notes that other column-stochastic W can take the place of
 * the one printed there).  w_dev: (m + 1) x (m + 1) fp32, row-major, on the DEVICE, caller-owned and
 * valid until replaced; entry [i][j] is the weight of row i of X in output row j.  While a matrix is
 * set, every synchronisation point applies X <- X W in one pass on the main stream in place of the
 * pull-back and the anchor average: the tau-th local step is a plain local step, ols_sync_pull
 * launches the mixing kernel (each output row is the fma chain over i = 0..m in fp32) and
 * ols_anchor_update_async only completes the call sequence (the anchor is row m of the product, so
 * there is nothing left to overlap).  NULL returns to the paper's pull-back + anchor average.
 * m <= 128.  Not combinable with anchor momentum.  OLS_ESTATE in the middle of a synchronisation.
 * The matrix is not checked for column-stochasticity: that is the caller's modelling choice. */
OLS_API int ols_set_mixing(ols_handle h, const float* w_dev);

/* Stale-average synchronisation, the alternative way of decoupling communication from computation that
 * "Related Works" describes: a round's local updates are applied to the average of the models as they
 * stood tau iterations before.  snap_dev: [m][ld] fp32 device buffer, 256-byte aligned, caller-owned and
 * valid until replaced; the call fills it with the current models (on the main stream).  While it is set,
 * every tau-th local step is a plain local step, ols_sync_pull computes
 *     x^(i) <- z + (x^(i) - snap^(i)),   snap^(i) <- the new x^(i)        (fp32, z + (x - snap) as written)
 * in one pass on the main stream (z: the average of the snapshots, produced by the previous round's
 * refresh), and ols_anchor_update_async averages the new models on the side stream, overlapped with the
 * next round.  alpha is not used.  Legal only after ols_init_params and before the first local step (a
 * later ols_init_params refills the buffer); NULL returns to the paper's rule.  Not combinable with general mixing or anchor momentum. */
OLS_API int ols_set_stale_average(ols_handle h, float* snap_dev);

/* Changes the learning rate gamma for subsequent local steps (Section 4 uses a schedule). */
OLS_API int ols_set_lr(ols_handle h, float gamma);

/* ---- models that produce the stochastic gradients g_i --------------------------------------- */

/* Linear least squares: loss_i = (1/B) sum_s 0.5 (a_s . x^{(i)} - y_s)^2 over the worker's batch of
 * B rows; g_i = (1/B) A^T (A x^{(i)} - y).  Inputs per ols_set_batch: A [B][d] fp32, y [B] fp32. */
OLS_API int ols_attach_lsq(ols_handle h, int batch);

/* ReLU multi-layer perceptron with softmax cross-entropy (mean over the batch).
 *   dims[0..n_layers]: layer widths, input first; the last is the class count (<= 32).
 *   Flat parameter layout per layer l: W_l row-major [dims[l]][dims[l+1]] then b_l [dims[l+1]];
 *   d must equal the sum.  dims[0..n_layers-1] and batch must be multiples of 4.
 *   gemm_dtype 0: fp32 MFMA; 1: bf16 operands (round-to-nearest-even), fp32 accumulate, fp32 master
 *   weights and gradients.
 * Inputs per ols_set_batch: X [B][dims[0]] fp32, labels [B] int32 in [0, classes). */
OLS_API int ols_attach_mlp(ols_handle h, int n_layers, const int* dims, int batch, int gemm_dtype);

/* Residual convolutional block with a pooled linear classifier: the first residual stage of the network of Section 4
 * ("Experimental setting": ResNet-18 on 32 x 32 inputs, mini-batch 128 per node), biases in place of batch
 * normalisation:
 *     a1 = relu(conv3x3(X; Wa) + ba);  a2 = relu(conv3x3(a1; Wb) + bb + X);  logits = mean_positions(a2) Wh + bh,
 * softmax cross-entropy, mean over the batch.  3 x 3 kernels, stride 1, zero padding 1, cross-correlation
 * (out[y][x] = sum_{kh,kw} in[y + kh - 1][x + kw - 1] W[kh][kw]).
 *   channels: a multiple of 16, at most 256; classes <= 32; batch * height * width * channels < 2^31 - 2^16 channels.
 *   Flat parameter layout: Wa [3][3][channels][channels] (kh, kw, input channel, output channel), ba [channels],
 *   Wb, bb likewise, Wh [channels][classes], bh [classes]; d must equal the sum.
 * Inputs per ols_set_batch: X [B][height][width][channels] fp32 (channel contiguous), labels [B] int32.
 * Gradients go to g and the streaming kernels apply the update (the parameters are few: 74 k at 64 channels). */
OLS_API int ols_attach_convblock(ols_handle h, int channels, int height, int width, int classes, int batch);

/* The same block as the residual network of Section 4 has it, with batch normalisation: the convolutions carry no
 * bias and each is followed by a normalisation per channel over all samples and positions of the worker's own
 * mini-batch (training mode; every worker normalises alone, as every node of the paper's cluster does):
 *     z1 = conv3x3(X; Wa);   a1 = relu(bn(z1; ga, ba));
 *     z2 = conv3x3(a1; Wb);  a2 = relu(bn(z2; gb, bb) + X);   logits = mean_positions(a2) Wh + bh
 *     bn(z; g, b)[c] = g[c] (z - mean_c) / sqrt(var_c + eps) + b[c],  var_c the biased variance.
 * No running averages are kept (they play no part in training).  eps in (0, 1]; 1e-5 is the usual value.
 *   Flat parameter layout: Wa, ga [channels], ba [channels], Wb, gb, bb, Wh, bh (scale before shift);
 *   d = 2 (9 channels^2 + 2 channels) + channels classes + classes.  Other limits, inputs and errors as for
 *   ols_attach_convblock.  The workspace keeps z1 and z2 for the backward pass beside the activations. */
OLS_API int ols_attach_convblock_bn(ols_handle h, int channels, int height, int width, int classes, int batch, float eps);

/* The block of ols_attach_convblock with bf16 operands on the matrix cores (fp32 accumulation), by the rule of the
 * bf16 MLP: a tensor is rounded to bf16, to nearest even, where it becomes an operand of a convolution's products --
 * the input batch, both kernels (through a bf16 copy of the parameters that the update kernels keep in the workspace),
 * a1, and the deltas at both convolution outputs; biases, the shortcut, a2, pooling, classifier, gradients and the
 * master parameters stay fp32.  Same parameter layout, inputs and errors as ols_attach_convblock, and in addition:
 * channels a multiple of 64, width at most 128; attach (and bind the workspace) before ols_init_params, as for the
 * bf16 MLP.  Internally the operand tensors are stored with their zero border, (height + 2) x (width + 2) per sample;
 * the limit on batch * height * width * channels applies to those sizes. */
OLS_API int ols_attach_convblock_bf16(ols_handle h, int channels, int height, int width, int classes, int batch);

/* The batch-normalised block of ols_attach_convblock_bn with bf16 operands, by the same rule: the input batch, both
 * kernels, a1, and the gradients at the two convolution outputs are rounded to bf16 where they become operands of a
 * convolution; the convolution outputs, the normalisations with their statistics, scales and shifts, the shortcut, a2,
 * pooling, classifier, gradients and master parameters stay fp32 (the network of Section 4, "Experimental setting", has
 * the normalisation).  Parameter layout, eps and errors as for ols_attach_convblock_bn; shape limits and call order as
 * for ols_attach_convblock_bf16. */
OLS_API int ols_attach_convblock_bn_bf16(ols_handle h, int channels, int height, int width, int classes, int batch, float eps);

/* Bytes of caller-provided device workspace the attached model needs (activations, deltas, per-sample
 * losses, bf16 operand copies).  0 when no model is attached. */
OLS_API int64_t ols_workspace_bytes(ols_handle h);
OLS_API int ols_bind_workspace(ols_handle h, void* ws_dev, int64_t bytes); /* 256-byte aligned; OLS_ENOMEM if short */

/* Mini-batches for the NEXT local step: worker i reads X_dev + i * x_worker_stride (elements) and
 * y_dev + i * y_worker_stride (elements of int32 labels or fp32 targets).  Pointers only; no copy. */
OLS_API int ols_set_batch(ols_handle h, const float* X_dev, int64_t x_worker_stride, const void* y_dev,
                  int64_t y_worker_stride);

/* Without an attached model the caller supplies gradients itself: rebinds g ([m][ld] device) for the
 * next local step. */
OLS_API int ols_set_gradient(ols_handle h, float* g_dev);

/* ---- the iteration --------------------------------------------------------------------------- */

/* Iteration k for every worker -- the FIRST update rule of Section 2 ("Proposed Algorithm"),
 *     x_{k+1/2}^{(i)} = x_k^{(i)} - gamma g_i(x_k^{(i)}; xi_k^{(i)}),
 * with the local momentum of the "Momentum Variant" paragraph when beta > 0 (buffer fed by the local gradient
 * only): the stochastic gradients of the attached model at x_k^{(i)} on the current mini-batch (or the caller's
 * gradient tensor), then the step; k <- k + 1.  When the new k is a multiple of tau a pull-back is due.  On the
 * default route (OLS_OPT_FUSE_GEMM_UPDATE with an attached model) the kernels that form the gradients apply the
 * step, and on that tau-th step also the pull-back toward z_k, where each gradient element is produced; the main
 * stream waits for the previous round's anchor refresh only in front of the first such launch.  Otherwise, with
 * OLS_OPT_FUSE_PULL, the tau-th step's parameter write is left pending for ols_sync_pull.
 * OLS_ESTATE if unbound / uninitialised, if a pull or an anchor refresh is due, or if a model is
 * attached but no batch or workspace is set. */
OLS_API int ols_local_step(ols_handle h);

/* The SECOND update rule of Section 2, applied when (k+1) mod tau == 0 in the paper's indexing:
 *     x_{k+1}^{(i)} = x_{k+1/2}^{(i)} - alpha (x_{k+1/2}^{(i)} - z_k)        for every replica,
 * z_k being the anchor produced by the PREVIOUS round's refresh (the sentence after the anchor update rule: the
 * average started at iteration a tau is needed only for the models of iteration (a+1) tau).  The main stream first
 * waits for that refresh if it is still in flight, so the result does not depend on timing.  Where the tau-th
 * local step already applied the pull-back (default route) the call only marks the models as pulled for the
 * refresh.  Leaves the momentum buffers untouched.  Legal only when k > 0, k mod tau == 0 and not yet pulled. */
OLS_API int ols_sync_pull(ols_handle h);

/* The THIRD update rule of Section 2, the anchor refresh
 *     z_{k+1} = (1/m) sum_i x_{k+1}^{(i)}        over the POST-pull models
 * (with ols_set_anchor_momentum: v <- beta_z v + (mean - z), z <- z + v), enqueued on the side stream behind the
 * pull and overlapped with the following tau local steps -- the non-blocking synchronisation of the paper's
 * timeline figure, here a reduction over the replica axis in HBM.  Legal only right after a pull. */
OLS_API int ols_anchor_update_async(ols_handle h);

/* `steps` iterations in the order of the three calls above (ols_local_step; after every tau-th one
 * ols_sync_pull and ols_anchor_update_async) driven from inside the library, for workloads whose steps
 * are so short that the caller's loop would be the bottleneck.  The attached model's mini-batches come
 * from a resident data set visited cyclically and unshuffled (Section 4: the data is partitioned and not
 * shuffled): iteration k reads batch k mod nb of X_dev [m][nb][B][row] fp32 and y_dev [m][nb][B]
 * (int32 labels or fp32 targets), k being the handle's iteration count.  Same launches as the
 * separate calls; stops at the first error and returns it.  OLS_ESTATE without an attached model or
 * when a pull or an anchor refresh is due. */
OLS_API int ols_run_steps(ols_handle h, int64_t steps, const float* X_dev, const void* y_dev, int nb);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): ols_run_steps with the attached model's workspace (activations, deltas, split-K partial
 * sums, output-layer deltas, per-sample losses) taken from a static device array inside the library instead of a
 * caller-provided buffer.  The call allocates nothing (no hipMalloc / hipFree, no events); the handle must have
 * been bound and initialised beforehand, and state, data and streams remain the caller's.
 *   - The array holds ols_static_workspace_bytes() = 64 MiB, one copy per GPU, kept until the process ends;
 *     OLS_ENOMEM if ols_workspace_bytes(h) is larger.
 *   - fp32 models only (least squares, fp32 MLP): the bf16 MLP keeps weights in its workspace (OLS_EINVAL).
 *   - OLS_ESTATE while OLS_OPT_KERNEL_TIMING is on (timing creates events).
 *   - The handle's workspace becomes the static array (it replaces one bound with ols_bind_workspace); ols_get_loss
 *     afterwards reads the per-sample losses from it.  Nothing in it needs clearing between calls: every kernel
 *     writes what it later reads.
 *   - Every handle on one GPU shares the one array: calls (and the work they enqueue) that overlap on a GPU race;
 *     drain the streams (ols_sync) before another handle uses it.
 * Same launches, same results as ols_run_steps. */
OLS_API int ols_run_steps_static(ols_handle h, int64_t steps, const float* X_dev, const void* y_dev, int nb);
OLS_API int64_t ols_static_workspace_bytes(void);

/* ---- results --------------------------------------------------------------------------------- */

/* Reads the iterates of Section 2: which = 0..m-1 the local model x_k^{(i)} of worker which + 1, -1 the anchor
 * z_k (the paper does not say which of them "the model" is; both are exposed).  Copies d floats.  which = -2 computes the replica mean
 * (1/m) sum_i x^{(i)} into dst, which must then be a 256-byte aligned DEVICE buffer of
 * ols_row_stride(d) floats.  Drains both streams first (synchronous).  OLS_ESTATE while a fused pull
 * is pending.  dst_is_device selects the kind of dst. */
OLS_API int ols_get_params(ols_handle h, int which, float* dst, int dst_is_device);

/* Mean mini-batch loss of each worker at the most recent local step, per_worker_host [m].
 * Synchronous. */
OLS_API int ols_get_loss(ols_handle h, float* per_worker_host);

/* Blocks until both streams have drained. */
OLS_API int ols_sync(ols_handle h);

OLS_API int ols_set_option(ols_handle h, int key, int64_t value);

/* Local iterations completed so far (k). */
OLS_API int64_t ols_iteration(ols_handle h);

/* ---- instrumentation ------------------------------------------------------------------------- */

/* Accumulated HIP-event timing of one kernel kind since OLS_OPT_KERNEL_TIMING was enabled.
 * Synchronous (drains the streams). */
OLS_API int ols_kernel_stats(ols_handle h, int kind, int64_t* launches, double* total_ms);
OLS_API const char* ols_kernel_name(int kind);

/* Launch trace (OLS_OPT_TRACE): number of entries, and entry idx.  The trace keeps the first 65536
 * launches after it is enabled. */
OLS_API int64_t ols_trace_count(ols_handle h);
OLS_API int ols_trace_get(ols_handle h, int64_t idx, ols_trace_entry* out);

OLS_API const char* ols_last_error(void);
OLS_API const char* ols_version(void);

#ifdef __cplusplus
}
#endif
#endif /* OLS_H */
