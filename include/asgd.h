/*
 * asgd.h — C ABI of the MI355X (gfx950) hot path of GPU A-SGD (arXiv 1312.6186).
 *
 * The paper's protocol (Section 2.3, "Our contribution: GPU A-SGD"): each model
 * replica computes minibatch gradients on a GPU, pushes gradients to a central
 * parameter server and fetches updated parameters from it.  The three calls of
 * that protocol are
 *     asgd_snapshot      (a replica fetches the server's parameters)
 *     asgd_fwd_bwd       (one replica's minibatch gradient, Section 2)
 *     asgd_apply_update  (the server applies a pushed gradient)
 *     asgd_apply_update_snapshot (push and the same replica's next fetch, fused)
 *     asgd_train_step    (gradient, push and fetch of one replica, pipelined by layer)
 * plus the calls that describe the network and the on-one-GPU A-SGD replay.
 *
 * Conventions
 *   - "device" pointers are HIP device memory owned by the caller unless stated;
 *     "host" pointers are ordinary process memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work and return without synchronising the host
 *     (asgd_profile_end and asgd_net_destroy are the exceptions and say so).
 *   - Every call returns 0 on success or a negative asgd_status_t; the text of
 *     the last error of the calling thread is at asgd_last_error().  Nothing
 *     aborts or throws across this boundary.
 *   - Canonical layouts: images [B,C,H,W]; the flat parameter vector holds, for
 *     every conv / fc layer in descriptor order, the weights then the bias;
 *     conv weights [cout][cin][k][k], fc weights [out][in] with
 *     in = c*H*W + h*W + w.  Gradients and momentum use the same order.
 */
#ifndef ASGD_H
#define ASGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ASGD_OK = 0,
    ASGD_EINVAL = -1,  /* null pointer, bad enum, bad scalar argument        */
    ASGD_ESHAPE = -2,  /* layer list or sizes that do not form a valid net   */
    ASGD_ENOMEM = -3,  /* host or device allocation failed                   */
    ASGD_EHIP = -4,    /* a HIP runtime call failed (no device, launch error) */
    ASGD_EALIGN = -5   /* a buffer is not aligned as the call requires       */
} asgd_status_t;

typedef enum { ASGD_F32 = 0, ASGD_BF16 = 1 } asgd_dtype_t;

typedef enum {
    ASGD_LAYER_CONV = 1,       /* out, k, stride, pad                          */
    ASGD_LAYER_RELU = 2,       /* must follow a CONV or an FC                  */
    ASGD_LAYER_MAXPOOL = 3,    /* k, stride (unpadded, floor rule)             */
    ASGD_LAYER_FC = 4,         /* out                                          */
    ASGD_LAYER_DROPOUT = 5,    /* p, scale; must directly follow FC + RELU      */
    ASGD_LAYER_SOFTMAX_CE = 6, /* last layer; follows an FC                    */
    ASGD_LAYER_LRN = 7         /* k (window, odd, <= 9), p (alpha), scale (beta), bias; must directly follow CONV + RELU */
} asgd_layer_kind_t;

/* One entry of the network description.  Unused fields are ignored.
 * Dropout (Section 1 cites Hinton et al. 2012): a unit is dropped with
 * probability p; kept units are multiplied by `scale` (0 is read as 1, the
 * cited unscaled form).
 * LRN is the cross-channel response normalisation of the architecture the paper
 * trains (Section 3 cites it):  b[c] = a[c] * (bias + alpha * sum a[c']^2)^(-beta),
 * the sum over the `k` channels centred on c, clipped at the ends. */
typedef struct {
    int32_t kind;   /* asgd_layer_kind_t */
    int32_t out;    /* CONV: output channels; FC: output features */
    int32_t k;      /* CONV / MAXPOOL: square window size */
    int32_t stride; /* CONV / MAXPOOL */
    int32_t pad;    /* CONV: zero padding on each side */
    float p;        /* DROPOUT: drop probability, 0 <= p < 1; LRN: alpha */
    float scale;    /* DROPOUT: factor on kept units; LRN: beta */
    float bias;     /* LRN: the additive constant k of the formula */
    int32_t groups; /* CONV: number of channel groups ("columns"); 0 or 1 = ungrouped.  Group g maps input
                       channels [g*cin/groups, ...) to output channels [g*out/groups, ...); both per-group
                       counts must be multiples of 8; filters are [out][cin/groups][k][k] */
} asgd_layer_desc_t;

/* Where one parameterised layer lives in the flat parameter vector. */
typedef struct {
    int32_t layer;       /* index into the descriptor list */
    int32_t kind;        /* ASGD_LAYER_CONV or ASGD_LAYER_FC */
    uint64_t w_offset;   /* elements from the start of the flat vector */
    uint64_t w_count;
    uint64_t b_offset;
    uint64_t b_count;
    int32_t w_shape[4];  /* conv: cout,cin,k,k; fc: out,in,1,1 */
} asgd_tensor_info_t;

typedef struct asgd_net asgd_net_t;

/* Build the execution plan of a network (the Krizhevsky-style convnet of
 * Section 3: conv, ReLU, max-pool, fully connected, dropout, softmax
 * cross-entropy) for a fixed batch size and compute type.
 *   layers, n_layers : host array; copied.
 *   batch, in_c/h/w  : minibatch size and image shape.
 *   compute_dtype    : ASGD_F32 (fp32 MFMA) or ASGD_BF16 (bf16 MFMA, fp32
 *                      accumulation); it is also the type of the worker's
 *                      parameter copy and of the images given to asgd_fwd_bwd.
 *   out              : receives the plan; release with asgd_net_destroy.
 * Touches no GPU: shapes, parameter layout and workspace size can be queried
 * on a machine without one.  Device workspace (activations, pooling indices,
 * split-K partial sums; owned by the plan) is allocated by the first
 * asgd_fwd_bwd or by asgd_net_prepare.
 * Errors: ASGD_EINVAL (null, bad dtype), ASGD_ESHAPE (invalid sequence, a
 * window larger than its input, an FC fan-in that is not a multiple of 8,
 * sizes beyond 2^31 elements), ASGD_ENOMEM. */
int asgd_net_create(const asgd_layer_desc_t *layers, int n_layers, int batch, int in_c, int in_h,
                    int in_w, int compute_dtype, asgd_net_t **out);

/* Allocate the plan's device workspace on the current device now (optional). */
int asgd_net_prepare(asgd_net_t *net);

/* Free the plan, its workspace and its internal streams and events (the host
 * waits for the internal streams first).  The caller must have synchronised
 * every stream the plan was used on. */
int asgd_net_destroy(asgd_net_t *net);

/* on != 0: every kernel of asgd_fwd_bwd / asgd_train_step on this plan is
 * enqueued on the caller's stream, none on the plan's internal stream (for
 * profilers, which then see each kernel running alone).  New plans start with
 * on = 0, or with on = 1 if ASGD_SERIAL=1 is in the environment.  The results
 * are the same bit for bit either way.  Errors: ASGD_EINVAL (null plan). */
int asgd_net_set_serial(asgd_net_t *net, int on);

/* Number of elements of the flat parameter vector (0 if net is NULL). */
size_t asgd_param_count(const asgd_net_t *net);

/* Fill `info[0..cap)` with the parameterised layers in flat-vector order.
 * Returns the number of such layers (which may exceed cap), or a negative
 * status. */
int asgd_param_layout(const asgd_net_t *net, asgd_tensor_info_t *info, int cap);

/* Output shape of descriptor layer `layer` as (c,h,w); FC-side layers report
 * (features,1,1). */
int asgd_layer_shape(const asgd_net_t *net, int layer, int32_t chw[3]);

/* Bytes of device workspace the plan owns once prepared. */
size_t asgd_workspace_bytes(const asgd_net_t *net);

/* One replica's minibatch gradient (Section 2: the gradient of the objective
 * over a minibatch): forward, softmax cross-entropy averaged over the batch,
 * backward.
 *   params  : device, the worker's copy of the flat parameter vector in the
 *             plan's compute dtype (fp32, or bf16 as written by asgd_snapshot),
 *             16-byte aligned; read only.
 *   images  : device, [B,C,H,W] in the compute dtype; read only.
 *   labels  : device, int32 [B], each in [0, classes).  A label outside that
 *             range is never used as an address: the loss comes back NaN and
 *             that row's logit gradient is softmax / B (no class subtracted);
 *             every kernel still runs to its end.
 *   dropout_seed, step, worker : key of the stateless dropout mask generator
 *             (SplitMix64 finaliser over seed, step, worker, layer index and
 *             element index), so that a run can be replayed exactly.
 *   loss    : device, 1 float; overwritten.
 *   grads   : device, fp32 [param_count], 16-byte aligned; overwritten (not
 *             accumulated into).
 * No host synchronisation.  The call is ordered on `stream`: it starts after
 * the work already enqueued there and later work on `stream` sees its results.
 * Kernels that do not feed the next layer (parameter gradients, filter packing)
 * may run on an internal stream of default priority, forked from and joined back
 * into `stream` with events (never inside asgd_replay_run, never between
 * asgd_profile_begin / end, and not at all on a plan switched to serial, see
 * asgd_net_set_serial).  A plan must not be used on two streams at once (its workspace
 * is shared).
 * Errors: ASGD_EINVAL, ASGD_EALIGN, ASGD_ENOMEM, ASGD_EHIP. */
int asgd_fwd_bwd(asgd_net_t *net, const void *params, const void *images, const int32_t *labels,
                 uint64_t dropout_seed, uint64_t step, uint32_t worker, float *loss, float *grads,
                 void *stream);

/* asgd_fwd_bwd for callers that cannot allocate device memory or create streams
 * and events (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): same arguments, same results bit for bit, but the plan's
 * workspace is taken from an array that the library holds in the device image
 * of every GPU it runs on (asgd_static_workspace_bytes() bytes, 64 MiB, kept
 * until the process ends), every kernel is enqueued on `stream`, and the call
 * calls no hipMalloc / hipFree, creates no stream or event and needs no
 * asgd_net_prepare.  The array is cleared by a kernel at the start of the call.
 *   - A plan whose asgd_workspace_bytes() exceeds the array is refused with
 *     ASGD_ENOMEM and nothing is enqueued.
 *   - All calls on one GPU share the one array: two calls that overlap on a GPU
 *     (different streams, different plans) race; order them.
 *   - asgd_debug_get does not see the tensors of this call.
 * Errors: ASGD_EINVAL, ASGD_EALIGN, ASGD_ENOMEM (plan too large), ASGD_EHIP. */
int asgd_fwd_bwd_static(asgd_net_t *net, const void *params, const void *images, const int32_t *labels,
                        uint64_t dropout_seed, uint64_t step, uint32_t worker, float *loss, float *grads,
                        void *stream);
size_t asgd_static_workspace_bytes(void);

/* The parameter server's update for one pushed gradient (Section 3.1: the
 * single-GPU settings, i.e. momentum SGD with weight decay), one pass over the
 * buffers:   t = g + wd*w;  v = mu*v - lr*t;  w = w + v.
 *   params, momentum : device fp32 [n], updated in place.
 *   grads            : device fp32 [n], read only.
 * Errors: ASGD_EINVAL (null with n > 0), ASGD_EHIP. */
int asgd_apply_update(float *params, float *momentum, const float *grads, size_t n, float lr,
                      float mu, float wd, void *stream);

/* The two server updates the paper names as future work (Section 4), as the
 * same kind of single pass over the flat buffers, with t = g + wd*w:
 *   Adagrad :  h += t*t;  w -= lr * t / (sqrt(h) + eps)
 *   Adadelta:  a = rho*a + (1-rho)*t*t;  d = -sqrt(b + eps) / sqrt(a + eps) * t;
 *              b = rho*b + (1-rho)*d*d;  w += d
 *   params and the state buffers (hist; avg_sq_grad, avg_sq_step): device fp32
 *   [n], updated in place, state zero before the first update; grads read only.
 *   The square roots and quotients of the step are the hardware's approximate
 *   ones (about one ulp each); the state recurrences are exact fp32 FMAs.
 * Errors: ASGD_EINVAL (null with n > 0), ASGD_EALIGN, ASGD_EHIP. */
int asgd_apply_update_adagrad(float *params, float *hist, const float *grads, size_t n, float lr,
                              float eps, float wd, void *stream);
int asgd_apply_update_adadelta(float *params, float *avg_sq_grad, float *avg_sq_step,
                               const float *grads, size_t n, float rho, float eps, float wd,
                               void *stream);

/* A replica's fetch (Section 2.3): copy the server's fp32 parameters into the
 * worker's buffer, as fp32 (dst_dtype ASGD_F32) or rounded to bf16, ties to
 * even (ASGD_BF16; NaN stays a quiet NaN).
 *   params : device fp32 [n];  worker_copy : device, n elements of dst_dtype.
 * Errors: ASGD_EINVAL, ASGD_EHIP. */
int asgd_snapshot(const float *params, void *worker_copy, size_t n, int dst_dtype, void *stream);

/* The push and the next fetch of Section 2.3 in one pass over the parameters:
 * exactly asgd_apply_update followed by asgd_snapshot of the updated parameters
 * into `worker_copy` (the same values, bit for bit), without reading the
 * parameters a second time.  For the replica that fetches right after its own
 * push; other replicas' copies are untouched.
 * Errors: ASGD_EINVAL (null with n > 0, unknown dtype), ASGD_EALIGN, ASGD_EHIP. */
int asgd_apply_update_snapshot(float *params, float *momentum, const float *grads, size_t n,
                               float lr, float mu, float wd, void *worker_copy, int dst_dtype,
                               void *stream);

/* One whole cycle of a replica that shares the GPU with the server (the
 * single-replica loop of Section 2.3): asgd_fwd_bwd on `worker_copy`, then
 * asgd_apply_update_snapshot on every layer's slice of the parameters.  Results
 * are those of the two calls, bit for bit; the difference is the schedule: a
 * layer's slice is pushed as soon as its gradient is complete and its data
 * gradient (the last reader of the old values) has been queued, so the update
 * can run beside the rest of the backward pass wherever the GPU has room for it.
 *   master, momentum : device fp32 [P], updated in place.
 *   worker_copy : device [P] in the plan's compute dtype, 16-byte aligned; the
 *             parameters the gradient is computed on; holds the updated
 *             parameters (the next fetch) when the call completes.
 *   grads       : device fp32 [P]; holds this step's gradient afterwards.
 *   other arguments as for asgd_fwd_bwd / asgd_apply_update.
 * Errors: as asgd_fwd_bwd. */
int asgd_train_step(asgd_net_t *net, float *master, float *momentum, void *worker_copy,
                    const void *images, const int32_t *labels, uint64_t dropout_seed, uint64_t step,
                    uint32_t worker, float *loss, float *grads, float lr, float mu, float wd,
                    void *stream);

/* asgd_train_step with the push of the fully-connected weights done inside the
 * kernel that computes their gradient (Section 2.3: replica and server on one
 * GPU, n_push = n_fetch = 1): the gradient of such a weight matrix never goes
 * to memory; the kernel reads the parameters and momenta of its block, applies
 * the update of asgd_apply_update to them and writes the replica's copy, which
 * takes 8 bytes per parameter off the step's traffic.  master, momentum and
 * worker_copy end up as after asgd_train_step, bit for bit.
 *   grads : device fp32 [P]; afterwards holds this step's gradient EXCEPT in
 *           the weight slices of the fully-connected layers that were fused
 *           (no split-K in their gradient GEMM, in_features a multiple of 8,
 *           slice offset a multiple of 8 elements), which are left as they
 *           were; biases and convolution filters are written as usual.
 *   other arguments and errors as for asgd_train_step. */
int asgd_train_step_fused(asgd_net_t *net, float *master, float *momentum, void *worker_copy,
                          const void *images, const int32_t *labels, uint64_t dropout_seed,
                          uint64_t step, uint32_t worker, float *loss, float *grads, float lr,
                          float mu, float wd, void *stream);

/* Test hook: what the last asgd_fwd_bwd on this plan left behind, converted to
 * canonical layout into a caller-owned device buffer.
 *   what = ASGD_DEBUG_OUTPUT : fp32 [B,C,H,W] (or [B,F]) output of `layer`,
 *          which must be the last layer of a fused group (the RELU after a
 *          CONV, a MAXPOOL, the RELU/DROPOUT ending an FC group, the last FC).
 *   what = ASGD_DEBUG_ARGMAX : uint8 [B,C,Ho,Wo], window position ky*k+kx of
 *          the first maximum (row-major scan) of MAXPOOL `layer`.
 *   what = ASGD_DEBUG_MASK   : uint8 [B,F], 1 = kept, of DROPOUT `layer`.
 * `cap_bytes` is the size of dst; too small gives ASGD_EINVAL. */
typedef enum { ASGD_DEBUG_OUTPUT = 0, ASGD_DEBUG_ARGMAX = 1, ASGD_DEBUG_MASK = 2 } asgd_debug_what_t;
int asgd_debug_get(asgd_net_t *net, int what, int layer, void *dst, size_t cap_bytes, void *stream);

/* Per-kernel-class timing of asgd_fwd_bwd (and asgd_train_step), for roofline
 * reports.  Between asgd_profile_begin and asgd_profile_end every operation
 * enqueued by these calls on this plan is bracketed by a pair of HIP events on the stream it
 * runs on (an operation is one layer's GEMM including its split-K reduction, or
 * one streaming kernel).  asgd_profile_end synchronises those events (host
 * blocks) and fills out[0..ASGD_K_COUNT) with, per class: the number of
 * operations, their summed duration, and the algorithmic work they stand for
 * (2 * multiply-adds of the layer definition; bytes of the tensors an operation
 * must read and write once, at their true, unpadded sizes).
 * Errors: ASGD_EINVAL (null, end without begin), ASGD_EHIP. */
typedef enum {
    ASGD_K_CONV_FWD = 0, ASGD_K_CONV_DGRAD = 1, ASGD_K_CONV_WGRAD = 2,
    ASGD_K_FC_FWD = 3, ASGD_K_FC_DGRAD = 4, ASGD_K_FC_WGRAD = 5,
    ASGD_K_POOL_FWD = 6, ASGD_K_POOL_BWD = 7, ASGD_K_BIAS_GRAD = 8,
    ASGD_K_SOFTMAX_CE = 9, ASGD_K_LAYOUT = 10, ASGD_K_UPDATE = 11, ASGD_K_LRN = 12, ASGD_K_COUNT = 13
} asgd_kernel_class_t;
typedef struct {
    int32_t kclass;
    int32_t launches;
    double ms;
    double flops;
    double bytes;
} asgd_profile_entry_t;
int asgd_profile_begin(asgd_net_t *net);
int asgd_profile_end(asgd_net_t *net, asgd_profile_entry_t *out);

/* Staleness schedule of the A-SGD replay (Section 3.3 attributes artefacts of
 * the learning curves to stale updates).  Update a (0-based) is pushed by
 * worker a mod n_workers and was computed on parameter version
 * read_version[a] = a - min(a, h(seed, a) mod (max_stale + 1)).  Host arrays of
 * length T.  Requires 0 <= max_stale < n_workers so that every read is
 * causally possible.  Errors: ASGD_EINVAL. */
int asgd_schedule_generate(int32_t *worker, int32_t *read_version, int T, uint64_t seed,
                           int n_workers, int max_stale);

/* A-SGD on one GPU (Sections 2.2-2.3): n_workers replicas as concurrent HIP
 * streams, one server stream applying pushed gradients to the shared fp32
 * parameters in schedule order.  Update a: its worker snapshots the parameters
 * when exactly read_version[a] updates have been applied, computes the
 * gradient of minibatch a on that copy, and the server applies it as update a.
 *   nets          : host array of n_workers plans (same network), one each.
 *   params, momentum : device fp32 [param_count], shared, updated in place.
 *   worker_copy, worker_grads : host arrays of n_workers device buffers
 *                   (param_count elements of the compute dtype / of fp32).
 *   images, labels : device, T minibatches back to back ([T][B,C,H,W], [T][B]).
 *   worker, read_version : host, length T (asgd_schedule_generate).
 *   losses        : device fp32 [T], loss of each pushed gradient.
 *   log           : device int32 [T][3] = (update, worker, version counter read
 *                   on the device when the snapshot was taken).
 *   stream        : the caller's stream; the replay starts after the work
 *                   already on it and the stream waits for the replay's end.
 * The call only enqueues: it does not wait for the GPU.  The worker and server
 * streams and the events between them are created by the first replay on
 * nets[0] (more events when a later replay is longer), kept by that plan and
 * released by asgd_net_destroy(nets[0]).  The plans must not be used for
 * anything else until `stream` has passed the replay.
 * Errors: ASGD_EINVAL (a read_version outside [a - max over schedule, a], a
 * worker index out of range, a worker whose next read precedes its previous
 * push), ASGD_EHIP. */
int asgd_replay_run(asgd_net_t *const *nets, int n_workers, float *params, float *momentum,
                    void *const *worker_copy, float *const *worker_grads, const void *images,
                    const int32_t *labels, const int32_t *worker, const int32_t *read_version, int T,
                    float lr, float mu, float wd, uint64_t dropout_seed, float *losses, int32_t *log,
                    void *stream);

/* The regime the paper runs, n_fetch = n_push = n_sync (Section 2.3: the
 * parameters are updated on the GPU for n_sync steps between two exchanges with
 * the server).  The paper gives one sentence; the reading implemented here:
 * cycle a belongs to replica worker[a].  The replica fetches the server's
 * parameters when exactly read_version[a] updates have been applied, into its
 * own fp32 parameters (and its compute copy), runs n_sync momentum-SGD steps on
 * them with its own momentum buffer (same rule and hyper-parameters as the
 * server; the momentum persists across fetches), and pushes the SUM of the
 * n_sync minibatch gradients, which the server applies as one gradient
 * (update a).  Local step i of cycle a uses minibatch a*n_sync + i, which is
 * also its dropout step.  n_sync = 1 gives asgd_replay_run's results.
 *   worker_params, worker_momentum, worker_accum : host arrays of n_workers
 *             device fp32 [param_count] buffers: each replica's parameters
 *             (overwritten by every fetch), momentum (read and updated; zero it
 *             before the first call) and gradient accumulator (scratch).
 *   images, labels : device, T*n_sync minibatches back to back.
 *   losses  : device fp32 [T*n_sync].
 *   everything else as for asgd_replay_run.
 * Errors: as asgd_replay_run; ASGD_EINVAL for n_sync < 1. */
int asgd_replay_nsync_run(asgd_net_t *const *nets, int n_workers, int n_sync, float *params,
                          float *momentum, float *const *worker_params,
                          float *const *worker_momentum, float *const *worker_accum,
                          void *const *worker_copy, float *const *worker_grads, const void *images,
                          const int32_t *labels, const int32_t *worker,
                          const int32_t *read_version, int T, float lr, float mu, float wd,
                          uint64_t dropout_seed, float *losses, int32_t *log, void *stream);

/* The replica's gradient accumulator of that regime: accum = grads (first != 0)
 * or accum + grads, device fp32 [n].
 * Errors: ASGD_EINVAL (null with n > 0), ASGD_EALIGN, ASGD_EHIP. */
int asgd_accumulate(float *accum, const float *grads, size_t n, int first, void *stream);

/* Text of the last error on the calling thread ("" if none). */
const char *asgd_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ASGD_H */
