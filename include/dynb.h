/*
 * dynb -- data-parallel hot path of dynamic mini-batching on one MI355X (gfx950).
 *
 * K simulated workers each compute the gradient of the mean loss over their own
 * variable-sized mini-batch b_k (paper, Section "Key Idea: Variable Mini-Batch
 * Sizes"); the gradients are combined with weights lambda_k = b_k / sum_i b_i
 * (Eq. 2), applied by SGD (Eq. 3), and a host-side proportional controller
 * resizes the b_k so that iteration times equalise (Section
 * "Proportional-Control Based Dynamic Policy", Eq. 4 and Eq. 5, and the
 * four-step summary at the end of "Control stability").
 *
 * Conventions for every call
 *   - plain C ABI; every function returns DYNB_OK (0) or a negative error code and
 *     never throws; dynb_last_error() returns a thread-local message for the last
 *     failure on the calling thread.
 *   - "device" pointers are HIP device memory owned by the caller; the library
 *     allocates no device memory.  "host" pointers are ordinary host memory, read
 *     or written before the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Device
 *     work is enqueued on it and the call returns without synchronising.
 *   - b[K] is a HOST array of non-negative batch sizes; worker k owns the rows
 *     [off_k, off_k + b_k) of the global batch, off_k = sum_{j<k} b_j.  b_k = 0 is
 *     legal: that worker's gradient is all zeros and its weight lambda_k is 0.
 *   - Flat parameter layout (params, grads, aggregated gradient, velocity): for each
 *     layer that has parameters, in model order, its weight in C order (dense:
 *     [n_in][n_out]; conv3x3: [3][3][c_in][c_out]) followed by its bias [n_out].
 *     P = number of parameters; P_pad = P rounded up to a multiple of 256 floats.
 *     Vectors have P_pad elements; the tail beyond P is ignored on input and written
 *     as zero.
 */
#ifndef DYNB_H
#define DYNB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DYNB_MAX_WORKERS 64
#define DYNB_MAX_LAYERS 64

enum {
  DYNB_OK = 0,
  DYNB_ERR_BADARG = -1,      /* null pointer, K out of range, sum(b) mismatch, bad value */
  DYNB_ERR_UNSUPPORTED = -2, /* a model or size this build has no kernel for */
  DYNB_ERR_HIP = -3,         /* a HIP runtime call failed */
  DYNB_ERR_STATE = -4        /* call order violated (e.g. model not bound) */
};

enum { DYNB_F32 = 0, DYNB_BF16 = 1 };
enum {
  DYNB_LAYER_DENSE = 0,
  DYNB_LAYER_CONV3X3 = 1,
  DYNB_LAYER_GAP = 2,
  DYNB_LAYER_BN = 3,
  DYNB_LAYER_ADD = 4
};

/* One layer.  DENSE: n_in -> n_out.  CONV3X3: c_in = n_in, c_out = n_out, 3x3 kernel,
 * zero padding 1, `stride` 1 or 2, NHWC.  GAP: global average pool over H x W (n_in,
 * n_out, stride ignored).  BN: batch normalisation of n_in = n_out channels over the rows
 * (samples x pixels) of each worker's OWN mini-batch (biased variance, `eps` under the root),
 * learnable scale and shift: parameters [scale n_out][shift n_out] in the flat vector.
 * ADD: adds the stored output of layer `skip_from` (an earlier layer of the same shape; at
 * most one ADD per source layer).  relu != 0 applies max(., 0) to the layer output.
 * The ResNet-style blocks these two serve are the shape of the paper's first workload
 * (Section "Experimental Evaluation"). */
typedef struct {
  int32_t kind;
  int32_t n_in;
  int32_t n_out;
  int32_t stride;
  int32_t relu;
  int32_t skip_from; /* ADD */
  float eps;         /* BN */
} dynb_layer_desc;

/* dtype DYNB_F32: fp32 storage and arithmetic.  DYNB_BF16: weights (not biases),
 * the input, stored activations and stored activation-gradients are rounded to
 * bfloat16 (nearest-even); products accumulate in fp32; biases, logits, softmax,
 * gradients and master parameters are fp32.  The input is [n][in_h][in_w][in_c]
 * (a dense-only model uses in_h = in_w = 1, in_c = features).  The last layer must
 * produce n_classes logits. */
typedef struct {
  int32_t dtype;
  int32_t in_h, in_w, in_c;
  int32_t n_classes;
  int32_t n_layers;
  const dynb_layer_desc* layers; /* host, copied by dynb_model_create */
} dynb_model_desc;

/* Controller constants.  kp = 1 is the paper's rule (gain = measured throughput);
 * deadband is the paper's Delta_min(b) (0.05 in its evaluation); b_min/b_max are the
 * per-worker size bounds; ewma_alpha is the smoothing constant of dynb_ewma_update. */
typedef struct {
  double kp;
  double deadband;
  double ewma_alpha;
  int32_t b_min;
  int32_t b_max;
} dynb_gains;

typedef struct dynb_model dynb_model;

const char* dynb_last_error(void);

/* ---- model handle (host bookkeeping only) ------------------------------------- */

/* Validates the description and builds the layer plan.  *m is owned by the caller
 * and released with dynb_model_destroy. */
int dynb_model_create(const dynb_model_desc* desc, dynb_model** m);
void dynb_model_destroy(dynb_model* m);
int64_t dynb_model_num_params(const dynb_model* m);    /* P     */
int64_t dynb_model_padded_params(const dynb_model* m); /* P_pad */

/* Bytes of device workspace needed for global batches up to max_global_batch split
 * over up to max_workers workers (activations, activation-gradients, 16-bit weight
 * copies, logits, losses).  Returns 0 on bad arguments. */
size_t dynb_model_workspace_bytes(const dynb_model* m, int32_t max_global_batch,
                                  int32_t max_workers);

/* Attaches caller-owned device memory: params = fp32 master parameters [P_pad];
 * workspace of at least dynb_model_workspace_bytes(...) bytes, 256-byte aligned.  The
 * workspace is cleared and the weight copies are derived from params on `stream`. */
int dynb_model_bind(dynb_model* m, float* params, void* workspace, size_t workspace_bytes,
                    int32_t max_global_batch, int32_t max_workers, void* stream);

/* Re-derives the weight copies used by the kernels from the bound master parameters.
 * Call after writing params by any means other than the dynb_model_*update calls. */
int dynb_model_sync_weights(dynb_model* m, void* stream);

/* Device pointer to float[max_workers]: mean loss of each worker's mini-batch from the
 * most recent dynb_forward_backward (0 for an idle worker). */
const float* dynb_model_worker_loss(const dynb_model* m);

/* Copies those K losses to host_loss[K] (host): enqueues the copy behind the work already
 * on `stream` and waits for it.  The only call of this library that blocks on the device. */
int dynb_model_read_worker_loss(const dynb_model* m, float* host_loss, int32_t K, void* stream);

/* ---- the hot path -------------------------------------------------------------- */

/* Per-worker gradient grad f(x_{b_k,t}): for every worker k, forward pass, mean
 * softmax-cross-entropy loss over its own b_k samples, and backward pass; writes
 * grads[k][0..P_pad) (device, fp32, row stride P_pad).
 *   x : device fp32 [sum(b)][in_h][in_w][in_c];  y : device int32 [sum(b)], labels in
 *   [0, n_classes);  b : host int32 [K], 1 <= K <= max_workers, sum(b) <= max_global_batch. */
int dynb_forward_backward(dynb_model* m, const float* x, const int32_t* y, const int32_t* b,
                          int32_t K, float* grads, void* stream);

/* dynb_forward_backward that also returns the weighted average of Eq. 2,
 * out[p] = sum_k (b_k / sum_i b_i) * grads[k][p] (fp32; device fp32 [P_pad], 16-byte aligned):
 * what dynb_weighted_aggregate(grads, b, K, P_pad, out) would give, but for large dense layers
 * the sum is formed in the weight-gradient kernel while each worker's tile is still in
 * registers, so the K*P_pad floats are written once and not read again.  There the K terms of
 * an element are added in a fixed order that depends on the element's tile (a rotation of
 * 0..K-1, so that the compute units do not all write a worker's tile at the same moment):
 * reproducible from run to run, equal to the ascending-k sum up to fp32 rounding.  grads is
 * written in full as before.  sum(b) must be > 0. */
int dynb_forward_backward_aggregate(dynb_model* m, const float* x, const int32_t* y,
                                    const int32_t* b, int32_t K, float* grads, float* out,
                                    void* stream);

/* dynb_forward_backward for callers that cannot allocate device memory or hand over a
 * workspace (code under HIP graph capture, serving loops, harnesses that forbid hipMalloc): the
 * same kernels, but everything the bound workspace would hold lives in a static device array of
 * DYNB_STATIC_SCRATCH_BYTES inside the library (each GPU the library runs on holds its own copy
 * until the process ends).  The call allocates and frees nothing, records no memset, and needs
 * no dynb_model_bind: `m` is only read (a handle from dynb_model_create, bound or not), `params`
 * is the device fp32 parameter vector [P_pad] (16-byte aligned) the gradients are taken at; the
 * 16-bit weight copies are derived from it inside the call.  x, y, b, K, grads, stream as for
 * dynb_forward_backward; the per-worker losses are not returned.
 * DYNB_ERR_UNSUPPORTED when dynb_model_workspace_bytes(m, sum(b), K) exceeds
 * DYNB_STATIC_SCRATCH_BYTES (nothing is launched then).  All calls on one GPU share that GPU's
 * array, which keeps the previous call's contents (the call clears what it needs): calls that
 * overlap in time on one GPU -- different streams or threads -- race; serialise them. */
#define DYNB_STATIC_SCRATCH_BYTES (32u << 20)
size_t dynb_static_scratch_bytes(void);
int dynb_forward_backward_static(const dynb_model* m, const float* params, const float* x,
                                 const int32_t* y, const int32_t* b, int32_t K, float* grads,
                                 void* stream);

/* Weighted average of Eq. 2: out[p] = sum_k (b_k / sum_i b_i) * grads[k*n + p], summed in
 * worker order.  grads device fp32 [K][n]; out device fp32 [n]; n % 4 == 0; both 16-byte
 * aligned.  sum(b) must be > 0. */
int dynb_weighted_aggregate(const float* grads, const int32_t* b, int32_t K, int64_t n, float* out,
                            void* stream);

/* Eq. 3 (read without its stray 1/K): params[p] -= lr * g[p] for p < n. */
int dynb_sgd_update(float* params, const float* g, int64_t n, float lr, void* stream);

/* Heavy-ball momentum: v = mu * v + g ; params -= lr * v. */
int dynb_sgd_momentum_update(float* params, float* velocity, const float* g, int64_t n, float lr,
                             float mu, void* stream);

/* The update on the model's bound parameters followed by a refresh of the weight copies
 * the next dynb_forward_backward reads.  velocity == NULL selects plain SGD (mu ignored). */
int dynb_model_sgd_update(dynb_model* m, const float* g, float lr, float mu, float* velocity,
                          void* stream);

/* Adam (Kingma & Ba, Algorithm 1; the optimizer of the paper's MNIST workload, Section
 * "Experimental Evaluation"), step number `step` >= 1:
 *   m = beta1 m + (1-beta1) g;  v = beta2 v + (1-beta2) g^2;
 *   params -= lr * (m / (1-beta1^step)) / (sqrt(v / (1-beta2^step)) + eps).
 * params, m, v, g: device fp32 [n], 16-byte aligned, n % 4 == 0.  fp32 arithmetic on the
 * device; the betas are doubles so that 1 - beta and the bias corrections are formed in
 * double on the host before they are rounded to fp32 (0.999 is not a float: 1 - 0.999f is
 * off by 1.3e-5 relative). */
int dynb_adam_update(float* params, float* m, float* v, const float* g, int64_t n, float lr,
                     double beta1, double beta2, float eps, int64_t step, void* stream);

/* Choice of optimizer for the model-level updates.  momentum is read by
 * DYNB_OPT_MOMENTUM; beta1, beta2, eps and step (1-based) by DYNB_OPT_ADAM. */
enum { DYNB_OPT_SGD = 0, DYNB_OPT_MOMENTUM = 1, DYNB_OPT_ADAM = 2 };
typedef struct {
  int32_t kind;
  float lr;
  float momentum;
  float eps;
  double beta1, beta2;
  int64_t step;
} dynb_optimizer;

/* One optimizer step on the model's bound parameters from the finished gradient g (device
 * fp32 [P_pad], 16-byte aligned), followed by the refresh of the weight copies the next
 * dynb_forward_backward reads.  state1: velocity (momentum) or first moment (Adam); state2:
 * second moment (Adam); device fp32 [P_pad], 16-byte aligned, caller-owned, zero before the
 * first step; ignored (may be NULL) when the optimizer has no such state.
 * DYNB_ERR_BADARG: null/misaligned pointers, unknown kind, missing state, Adam step < 1 or
 * betas outside [0,1).  DYNB_ERR_STATE: model not bound. */
int dynb_model_update(dynb_model* m, const float* g, const dynb_optimizer* opt, float* state1,
                      float* state2, void* stream);

/* Eq. 2 and Eq. 3 in one pass: the same result as dynb_weighted_aggregate(grads, b, K,
 * P_pad, tmp) followed by dynb_model_update(m, tmp, ...), but every parameter's K per-worker
 * gradients are read and summed (ascending k, fp32) where the step is applied, so the
 * aggregate is never written to or re-read from device memory.  grads: device fp32
 * [K][P_pad] as written by dynb_forward_backward; b: host int32 [K], sum(b) > 0. */
int dynb_model_aggregate_update(dynb_model* m, const float* grads, const int32_t* b, int32_t K,
                                const dynb_optimizer* opt, float* state1, float* state2,
                                void* stream);

/* Piecewise-constant learning rate (the paper gives the values 0.1, 0.01, 0.001, 0.0002 for
 * its ResNet workload, Section "Experimental Evaluation"): *lr = values[i] for
 * boundaries[i-1] <= step < boundaries[i].  values: host [n_values], boundaries: host
 * [n_values - 1], non-decreasing (may be NULL when n_values == 1). */
int dynb_lr_schedule(int64_t step, const int64_t* boundaries, const double* values,
                     int32_t n_values, double* lr);

/* ---- controller (host only) ---------------------------------------------------- */

/* One controller invocation (four-step summary of "Control stability"): from the
 * (smoothed) iteration times t[K] > 0 and the current sizes b[K] (sum = global_batch)
 * compute b_next[K]:
 *   tbar = mean_k t_k;  X_k = b_k / t_k;  r_k = b_k - kp * X_k * (t_k - tbar)   (Eq. 4, 5)
 *   clamp r_k to [b_min, b_max]; rescale to sum global_batch; largest-remainder rounding
 *   (ties to the lowest k); move entries back inside the bounds one sample at a time;
 *   if max_k |b_next_k - b_k| / b_k > deadband take the new sizes, else keep b.
 * IEEE double arithmetic in a fixed order: results are reproducible bit for bit.
 * Errors (DYNB_ERR_BADARG): null pointer, K outside [1, DYNB_MAX_WORKERS], b_k < 0,
 * sum(b) != global_batch, t_k not finite or <= 0, K*b_min > global_batch,
 * K*b_max < global_batch, non-finite gains, deadband < 0. */
int dynb_controller_step(const double* iter_times, const int32_t* b, int32_t K,
                         int32_t global_batch, const dynb_gains* gains, int32_t* b_next);

/* ---- the controller with its state between iterations ---------------------------
 * Subsection "Control stability": the smoothed iteration times are an EWMA over the
 * iterations since the last readjustment, and a worker whose throughput fell after its
 * batch size was raised keeps the size it had before as its upper bound.  The object
 * holds the sizes b[K], the smoothed times mu[K], the learnt upper bounds and the sizes
 * and throughputs replaced by the last readjustment.  Host memory only; not thread-safe.
 *   adaptive_b_max   != 0: learn upper bounds from throughput drops
 *   drop_tolerance   relative drop of the smoothed throughput b_k/mu_k that counts as a
 *                    drop (0: any); should exceed the noise of the iteration times
 *   min_observations iterations that must have been smoothed since the last readjustment
 *                    before the next one is considered (>= 1; 1 = check every iteration) */
typedef struct {
  dynb_gains gains;
  double drop_tolerance;
  int32_t min_observations;
  int32_t adaptive_b_max;
} dynb_controller_config;

typedef struct dynb_controller dynb_controller;

/* b0[K] (host) are the starting sizes, sum = global_batch.  Errors as for
 * dynb_controller_step, plus ewma_alpha outside [0,1], drop_tolerance < 0 or not finite,
 * min_observations < 1.  *out is owned by the caller (dynb_controller_destroy). */
int dynb_controller_create(const dynb_controller_config* cfg, const int32_t* b0, int32_t K,
                           int32_t global_batch, dynb_controller** out);
void dynb_controller_destroy(dynb_controller* c);

/* Feed the iteration times t[K] > 0 (host) of the iteration that just ran with the current
 * sizes; b_next[K] (host) receives the sizes for the next iteration, *resized (may be null)
 * whether they changed.  In order: (1) mu_k = t_k on the first iteration after a
 * readjustment, else mu_k = alpha t_k + (1 - alpha) mu_k; (2) for a worker whose size was
 * raised at the last readjustment from b_old and whose throughput b_k/mu_k is now below
 * (1 - drop_tolerance) times the throughput it had then: upper bound = b_old, unless the
 * bounds could then no longer hold the global batch (bounds only shrink); (3) once
 * min_observations iterations are smoothed, or at once if a size exceeds its bound: the step
 * of dynb_controller_step on mu with the per-worker bounds (a size above its bound overrides
 * the dead-band); (4) after a change the smoothing restarts.  Bit-reproducible like
 * dynb_controller_step.  DYNB_ERR_BADARG: null pointer, t_k not finite or <= 0 (state
 * unchanged). */
int dynb_controller_observe(dynb_controller* c, const double* iter_times, int32_t* b_next,
                            int32_t* resized);

/* Copy out the state; every output pointer may be null.  b, mu, b_hi: K entries (host). */
int dynb_controller_read(const dynb_controller* c, int32_t* b, double* mu, int32_t* b_hi,
                         int32_t* observations, int32_t* readjustments);

/* Exponentially weighted moving average of iteration times since the last
 * readjustment ("Exponential Smoothing"): reset != 0 sets mu = t, otherwise
 * mu_k = alpha * t_k + (1 - alpha) * mu_k.  mu is caller-owned state. */
int dynb_ewma_update(double* mu, const double* t, int32_t K, double alpha, int32_t reset);

/* Open-loop sizes proportional to throughput estimates X[K] > 0 with the global batch
 * K * b0 kept ("Static Mini-batch Allocation Policy"), largest-remainder rounding. */
int dynb_static_allocate(const double* X, int32_t K, int32_t b0, int32_t* b_out);

/* Throughput estimates for dynb_static_allocate from the servers' resources (same section,
 * paragraph "Estimating throughput"): X_k = number of CPU cores when the workers use only CPUs
 * (no worker states a FLOPs figure: half_precision_flops == 0 for all), X_k = the server's
 * half-precision FLOPs when CPU and GPU servers are mixed (stated, > 0, for all).  r: host [K];
 * X_out: host [K].  DYNB_ERR_BADARG: null pointer, K out of range, FLOPs stated for some
 * workers only, a negative or non-finite figure, no cores where cores are the estimate. */
typedef struct {
  int32_t cpu_cores;
  double half_precision_flops;
} dynb_worker_resources;
int dynb_estimate_throughput(const dynb_worker_resources* r, int32_t K, double* X_out);

/* ---- per-kernel timing (measurement aid) ---------------------------------------- */

/* When enabled, every kernel launch is bracketed by HIP events on its stream and
 * accumulated per kernel class.  dynb_profile_collect synchronises and folds pending
 * events into the totals.  Classes: see dynb_profile_name. */
int dynb_profile_enable(int32_t on);
int dynb_profile_reset(void);
int dynb_profile_collect(void);
int32_t dynb_profile_num_classes(void);
const char* dynb_profile_name(int32_t cls);
int dynb_profile_get(int32_t cls, double* total_ms, int64_t* launches, double* flops,
                     double* bytes);

#ifdef __cplusplus
}
#endif
#endif /* DYNB_H */
