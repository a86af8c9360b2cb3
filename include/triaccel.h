/*
 * triaccel.h -- C ABI of the MI355X (gfx950) Tri-Accel optimizer-step library.
 *
 * The library runs, for a list of parameter tensors ("layers"), the per-layer
 * fused optimizer step of Tri-Accel (arXiv 2508.16905):
 *
 *   gradient statistics        Var[grad_l(t)] and the EMA v_l(t)         Sec. 3.1, first equation
 *   precision rule             p_l(t) in {FP16, BF16, FP32}              Sec. 3.1, second equation
 *   sparse curvature signal    diagonal Hutchinson EMA, top-k magnitude  Sec. 3.2 (and Sec. 1:
 *                              mask, lambda_l = largest kept magnitude   "top-k Hessian or Fisher entries")
 *   step-size scaling          eta_l = eta_0 / (1 + alpha lambda_l)      Sec. 3.2, "Step size scaling"
 *   precision promotion        lambda_l > tau_curv -> one level up       Sec. 3.2, "Precision promotion"
 *   memory-elastic batch rule  B(t+1) from MemUsage / MemMax             Sec. 3.3
 *   control loop               the order of the stages                   Sec. 3.4
 *   overflow skip, loss scale  dynamic loss scaling (prior art, Sec. 2)
 *
 * All pointers inside triaccel_tensor are DEVICE pointers owned by the caller
 * (allocated e.g. by PyTorch-ROCm).  All other pointers are HOST pointers.  The
 * library owns only its internal workspace, released by triaccel_destroy().
 *
 * Every device operation is enqueued on the HIP stream given to triaccel_init();
 * triaccel_step() never synchronises; steps may be enqueued back to back, and
 * triaccel_result() reports the last one.
 * A handle belongs to the device that was current when it was created; calls that
 * enqueue work must be made with that device current (TRIACCEL_E_HIP otherwise).
 * Calls on one handle must not overlap in time; different handles are independent.
 *
 * Precision codes / dtypes:  0 = FP16 (IEEE binary16), 1 = BF16, 2 = FP32 --
 * the order of the cases in the precision rule, so "promotion" is +1.
 *
 * Return values: 0 on success, a negative TRIACCEL_E_* code otherwise.  Arguments
 * are validated before anything is enqueued: a call that returns an argument error
 * (any code but TRIACCEL_E_HIP) has changed no optimizer state and does not count as
 * a step.  TRIACCEL_E_HIP from a call that enqueues work means the HIP runtime failed
 * part-way through the enqueue: the call does not count as a step and its result cannot
 * be read, but kernels already enqueued may have changed the tensors, so the handle
 * should be destroyed.  A skipped step (non-finite gradient) is not an error.
 * Steps are counted in 64 bits (the flags of a skipped step carry the count as their epoch).
 */
#ifndef TRIACCEL_H
#define TRIACCEL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TRIACCEL_FP16 0
#define TRIACCEL_BF16 1
#define TRIACCEL_FP32 2

#define TRIACCEL_OK 0
#define TRIACCEL_E_INVALID_ARG (-1)     /* value out of range, wrong struct_size, n <= 0 ...        */
#define TRIACCEL_E_BAD_DTYPE (-2)       /* dtype code not in {0, 1, 2}                               */
#define TRIACCEL_E_SHAPE_MISMATCH (-3)  /* tensor list differs from the one given to triaccel_init   */
#define TRIACCEL_E_NULL_PTR (-4)        /* a required pointer is NULL                                */
#define TRIACCEL_E_ALIGNMENT (-5)       /* a device pointer is not 16-byte aligned                   */
#define TRIACCEL_E_HIP (-6)             /* a HIP runtime call failed; see triaccel_last_error()      */
#define TRIACCEL_E_NOT_INITIALISED (-7) /* NULL / destroyed handle, or result before any step        */
#define TRIACCEL_E_NO_MEMORY (-8)       /* host or device allocation failed                          */

typedef struct triaccel_ctx *triaccel_handle;

/* Hyper-parameters, fixed at init.  Symbols are the paper's where it has one. */
typedef struct {
  uint32_t struct_size;    /* sizeof(triaccel_config) */
  float beta_var;          /* beta of the variance EMA (Sec. 3.1), in [0, 1)                       */
  float beta_curv;         /* smoothing factor of the curvature EMA, in [0, 1)                     */
  float tau_low, tau_high; /* precision thresholds (Sec. 3.1), tau_low <= tau_high                  */
  float tau_curv;          /* promotion threshold on lambda_l (Sec. 3.2)                            */
  float alpha;             /* step-size coefficient (Sec. 3.2), >= 0                                */
  uint32_t sparsity_ppm;   /* curvature sparsity s in parts per million: the mask keeps the
                              k_l = clamp(n_l - floor(n_l * s / 1e6), 1, n_l) largest |h_i|         */
  float momentum;          /* mu of the base SGD update (Sec. 4.1 uses 0.9); 0 = no buffer          */
  float weight_decay;      /* coupled L2 coefficient                                                */
  int32_t ctrl_interval;   /* T_ctrl (Sec. 3.4): codes and the curvature used for eta_l are
                              re-evaluated on applied steps t with t % T_ctrl == 0; >= 1            */
  float scale_backoff;     /* loss-scale factor after a skipped step (e.g. 0.5)                     */
  float scale_growth;      /* loss-scale factor after growth_interval good steps (e.g. 2)           */
  int32_t growth_interval; /* >= 1                                                                  */
  double rho_low, rho_high;     /* memory utilisation thresholds (Sec. 3.3)                         */
  int32_t delta_up, delta_down; /* batch-size steps (Sec. 3.3)                                      */
  int32_t b_min, b_max;         /* clamp of the batch size                                          */
  int32_t power_k;         /* vectors per layer that triaccel_power_iter may be called with (top-k
                              eigenvalues, Sec. 3.2 / 4.1: k = 5); 0 = no workspace for it; <= 8      */
  int32_t lambda_source;   /* lambda_l of the step-size and promotion rules (Sec. 3.2):
                              0 = largest kept |h_i| of the diagonal curvature EMA,
                              1 = max_j |Rayleigh quotient| latched by triaccel_power_iter            */
  int32_t curvature_source; /* sample behind the diagonal curvature EMA ("Hessian or Fisher", Sec. 1 / 3.2):
                              0 = Hutchinson pair, u_i = z_i (Hz)_i / S (the caller supplies z and hz),
                              1 = empirical Fisher, u_i = (g_i / S)^2 (no probe; z and hz must be NULL)  */
  int32_t elementwise_scale; /* 0 = one step size per layer, eta_l = eta_0 / (1 + alpha lambda_l) (Sec. 3.2);
                              1 = the same rule applied per entry of the sparsified curvature,
                              eta_i = eta_0 / (1 + alpha a_i), a_i = |h_i| for entries in the mask, else 0
                              (lambda_l still drives the promotion rule); reads h once more in the update */
  uint32_t topk_abs;       /* > 0: the mask keeps this many entries per layer (the paper's fixed top-k,
                              Sec. 4.1: k = 5), clamped to [1, n_l]; 0: the fraction given by sparsity_ppm */
} triaccel_config;

/* One parameter tensor.  Contiguous, flat; numel elements. */
typedef struct {
  void *param;       /* device; capacity 4*numel bytes.  Holds numel elements of the tensor's CURRENT
                        precision code at the start of the buffer (the library tracks the code;
                        param_dtype below is only read by triaccel_init)                            */
  const void *grad;  /* device; numel elements of grad_dtype; the true gradient times loss_scale   */
  const float *z;    /* device; Rademacher probe (+-1.0f); NULL = no curvature probe this step      */
  const float *hz;   /* device; Hessian-vector product H z times loss_scale; NULL iff z is NULL     */
  float *curv;       /* device; fp32[numel]; diagonal curvature EMA h (library-updated state)       */
  float *mom;        /* device; fp32[numel]; momentum buffer m; may be NULL iff momentum == 0       */
  uint32_t *mask;    /* device; ceil(numel/32) words; bit (i % 32) of word (i / 32) = element i kept */
  int64_t numel;     /* 0 < numel < 2^31                                                            */
  int32_t grad_dtype;  /* precision code of the gradient buffer                                     */
  int32_t param_dtype; /* precision code of the parameters at init; ignored by triaccel_step        */
} triaccel_tensor;

/* Per-step scalars. */
typedef struct {
  uint32_t struct_size;     /* sizeof(triaccel_step_args) */
  float lr;                 /* eta_0 of this step (the caller applies its own schedule)             */
  float loss_scale;         /* S > 0: gradients and hz arrive multiplied by S                       */
  int32_t batch_size;       /* B(t), input of the batch rule                                        */
  uint64_t mem_used_bytes;  /* MemUsage(t); with mem_total_bytes == 0 the library asks the HIP      */
  uint64_t mem_total_bytes; /* MemMax       runtime (hipMemGetInfo) for both: a driver round trip,
                               so it samples them on the first call and on every 16th call after it
                               and uses the last sample in between                                  */
  int32_t update_curvature; /* only read with curvature_source == 1: non-zero = this step refreshes the
                               curvature EMA, threshold and mask from its gradient (the "every T
                               iterations" of Sec. 3.2 is the caller's schedule); with curvature_source
                               == 0 the presence of z decides, per tensor                              */
  int32_t reserved_;        /* set to 0 */
} triaccel_step_args;

typedef struct {
  uint32_t struct_size;    /* sizeof(triaccel_step_result), set by the caller */
  int32_t skipped;         /* 1: a gradient held inf/NaN; no optimizer state was changed            */
  uint64_t step_index;     /* number of triaccel_step calls so far                                  */
  float next_loss_scale;   /* loss scale to use for the next step                                   */
  int32_t next_batch_size; /* B(t+1), Sec. 3.3                                                      */
} triaccel_step_result;

/* Per-layer record; same layout on the device and in the host copy. */
typedef struct {
  int64_t numel;
  float mean, var;      /* of the unscaled gradient at the last applied step (population variance)  */
  float v;              /* variance EMA v_l (Sec. 3.1)                                              */
  float theta;          /* magnitude threshold of the mask                                          */
  uint32_t nnz;         /* popcount of the mask                                                     */
  float lambda;         /* lambda_l: largest kept |h_i|, or with lambda_source == 1 the latched
                           power-iteration value                                                    */
  float lambda_ctrl;    /* lambda latched at the last control step (used by eta and promotion)      */
  float eta;            /* per-layer step size (Sec. 3.2)                                           */
  int32_t code;         /* precision the parameters are stored in now                               */
  int32_t prev_code;    /* precision before the last applied step                                   */
  uint32_t found_inf;   /* this tensor's gradient held inf/NaN at the last step                     */
  uint32_t curv_nonfinite; /* a probe sample was non-finite at the last probed step (element frozen) */
  uint32_t sel_passes;  /* diagnostic: passes over h, beyond the one that updates it, that the threshold
                           selection of the last probed step needed (0 when the prediction held)        */
  uint32_t sel_listed;  /* diagnostic: keys listed by the curvature kernel at the last probed step          */
  uint32_t sel_outcome; /* diagnostic: 0 small tensor (all keys listed), 1 predicted band held, 2 no band
                           this step, 3 threshold above the band, 4 below it, 5 too many keys listed,
                           6 fewer non-zero magnitudes than k                                              */
} triaccel_layer_info;

/* Stage timings of one step (only recorded while profiling is on). */
#define TRIACCEL_N_STAGES 7
#define TRIACCEL_PROFILE_RING 64
typedef struct {
  float ms[TRIACCEL_N_STAGES]; /* 0 gradient statistics, 1 curvature EMA + provisional mask + band list,
                                  2 per-layer kernel (band check, assign), 3 fallback radix select
                                  (histogram passes), 4 update + cast of tensors whose storage size is
                                  unchanged (+ fallback mask pass), 5 in-place update of tensors whose
                                  size changes, 6 threshold resolution among listed keys + mask patch   */
} triaccel_stage_times;

/*
 * Create a handle for n tensors.  `tensors` gives shapes, dtypes and the initial pointers;
 * curv / mom / mask contents are taken as the initial state (normally zero).  `hip_stream` is a
 * hipStream_t (NULL = the default stream).  Allocates the workspace (chunk table, partials,
 * histograms, candidate lists, per-layer state, eight device copies of the tensor table; a few MB plus
 * 40 bytes per 4096 parameters, plus up to 4 MB of candidate lists per tensor of 262,144 elements or more).
 */
int triaccel_init(triaccel_handle *out, const triaccel_config *config, const triaccel_tensor *tensors,
                  int32_t n, void *hip_stream);

/*
 * Enqueue one optimizer step (Sec. 3.4 control loop, stages 1-3; stage 4 runs on the host).
 * `tensors` must have the n, numel and grad_dtype given at init; pointers may differ from call
 * to call.  Asynchronous: returns once the kernels are enqueued.
 */
int triaccel_step(triaccel_handle h, const triaccel_tensor *tensors, int32_t n, const triaccel_step_args *args);

/* Wait for the last enqueued step and return its record. */
int triaccel_result(triaccel_handle h, triaccel_step_result *out);

/* Wait for the stream and copy the n per-layer records to `out` (host). */
int triaccel_layer_state(triaccel_handle h, triaccel_layer_info *out, int32_t n);

/* Batch rule of Sec. 3.3 as a pure host function; returns B(t+1), or B unchanged if config is NULL. */
int32_t triaccel_batch_next(const triaccel_config *config, int32_t batch_size, uint64_t mem_used_bytes,
                            uint64_t mem_total_bytes);

/* Release the workspace.  Waits for the stream first.  NULL is allowed. */
void triaccel_destroy(triaccel_handle h);

/* Static text for an error code. */
const char *triaccel_strerror(int code);

/* Text of the last HIP failure on this thread ("" if none). */
const char *triaccel_last_error(void);

/*
 * on != 0: the following triaccel_step calls replay the step as a HIP graph instead of launching its
 * kernels one by one; results are identical.  A graph is captured the first time it is needed: one for
 * steps that refresh the curvature and one for steps that do not, for each of the (up to eight) device
 * copies of the tensor table in use.  Meant for small parameter sets, where the
 * step is bound by launch overhead.  While profiling is on the kernels are launched one by one.
 * The handle must have been created on a stream of its own (the default stream cannot be captured).
 */
int triaccel_set_graph(triaccel_handle h, int32_t on);

/*
 * Record HIP events in every following step: on = 1 at every stage boundary, on = 2 only around the
 * update kernel (stage 4; the other stage times then read 0), on = 0 stop.  Every recorded event
 * costs a few microseconds of the stream's time.
 */
int triaccel_set_profiling(triaccel_handle h, int32_t on);

/*
 * Wait for the stream and return the stage timings of the step enqueued `steps_back` calls ago
 * (0 = the last one; at most TRIACCEL_PROFILE_RING - 1).  That step must have run with profiling on.
 */
int triaccel_stage_times_get(triaccel_handle h, int32_t steps_back, triaccel_stage_times *out);

/*
 * Checkpointing (for callers that cannot re-run a job from step 0).  The tensors are the caller's; what the
 * library holds is small: the per-layer records (variance EMA, codes, latched curvature, threshold
 * predictor, power-iteration lambda), the loss-scale counter and the step count.
 * triaccel_state_size returns the number of bytes of the blob (negative error code on failure);
 * triaccel_get_state waits for the stream and writes the blob to `buf` (host, `size` bytes as returned);
 * triaccel_set_state replaces the state of a handle created with the same tensor list (same n, numel and
 * gradient dtypes) and the same hyper-parameters; a blob that does not match is refused and nothing changes.
 * After set_state, with the caller's tensors restored to their saved contents, the following steps are
 * bit-identical to those of the run that saved the state.
 */
int64_t triaccel_state_size(triaccel_handle h);
int triaccel_get_state(triaccel_handle h, void *buf, int64_t size);
int triaccel_set_state(triaccel_handle h, const void *buf, int64_t size);

/*
 * Power iteration for the top-k eigenvalues of each layer's Hessian (Sec. 3.2, third equation:
 * u <- H u / ||H u||, lambda ~ u^T H u / u^T u).  The caller owns the Hessian-vector products; one
 * call performs one iteration on k vectors per layer.  On entry u holds the current vectors u_j and
 * hu the products H_l u_j; on return (stream order) u_j holds the normalised H_l u_j with the
 * directions j' < j projected out first (ordered Gram-Schmidt: for k = 1 exactly the printed
 * iteration; for k > 1 vector j converges to the j-th eigenvector), and the per-layer record holds
 *   rayleigh_j = u_j . H u_j / u_j . u_j,   hnorm_j = ||H u_j||,
 *   resid_j = ||H u_j - rayleigh_j u_j|| / ||u_j||   (convergence measure).
 * A vector with no direction left (remainder <= 1e-6 of ||H u_j||) is set to zero and flagged.
 */
typedef struct {
  float *u;         /* device; fp32; vector j occupies elements [j*stride, j*stride + numel); in/out   */
  const float *hu;  /* device; fp32; same layout; read only                                            */
  int64_t stride;   /* elements between consecutive vectors: >= numel and a multiple of 4              */
} triaccel_power_tensor;

typedef struct {
  float rayleigh[8]; /* entries j >= k of the last call are 0                                           */
  float resid[8];
  float hnorm[8];
  uint32_t deficient; /* bit j: vector j had no direction left and was zeroed                           */
  float lambda_max;   /* max_j |rayleigh_j| of the last call                                            */
  float lambda_latched; /* the value triaccel_step uses when lambda_source == 1 (0 before any latch)    */
} triaccel_power_info;

/*
 * Enqueue one iteration.  n must equal the n of triaccel_init (numel per tensor as given there);
 * 1 <= k <= config.power_k.  latch != 0: lambda_l <- max_j |rayleigh_j| of this call, used by the
 * following triaccel_step calls when config.lambda_source == 1.  Asynchronous.
 */
int triaccel_power_iter(triaccel_handle h, const triaccel_power_tensor *vectors, int32_t n, int32_t k,
                        int32_t latch);

/* Wait for the stream and copy the n per-layer records of the last triaccel_power_iter call. */
int triaccel_power_state(triaccel_handle h, triaccel_power_info *out, int32_t n);

/*
 * Wait for the stream and return the durations (ms) of the three kernels of the last
 * triaccel_power_iter call -- Gram pass, per-layer factorisation, apply pass -- into ms[0..2] (host).
 * That call must have been made with profiling on (triaccel_set_profiling).
 */
int triaccel_power_times_get(triaccel_handle h, float *ms);

/*
 * For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): one power iteration exactly as triaccel_power_iter performs it, but
 * without a handle and without any allocation, host or device.  The tables and partial sums its kernels
 * need live in a fixed array inside the library's device code (about 4.3 MiB per GPU, held from the
 * first call on that GPU until the process ends), which bounds the size of one call:
 *   n <= TRIACCEL_STATIC_MAX_TENSORS, 1 <= k <= 8, and sum_i ceil(numel[i] / 4096) <=
 *   TRIACCEL_STATIC_MAX_CHUNKS (268,435,456 elements); larger calls return TRIACCEL_E_INVALID_ARG
 *   (text in triaccel_last_error) and do nothing.
 * vectors (host): n entries, u / hu device pointers as for triaccel_power_iter, 16-byte aligned.
 * numel (host): n element counts, each in (0, 2^31), stride >= numel[i] and a multiple of 4.
 * info (DEVICE, caller-owned): n records, written in stream order; lambda_latched is set to 0 (nothing is
 * latched: there is no optimizer handle).  u is overwritten as by triaccel_power_iter, bit for bit.
 * Asynchronous on `hip_stream` (NULL = the default stream), on the current device.  All calls on one GPU
 * share that GPU's array: calls that overlap in time on one GPU (different streams or threads) race.
 * The first call on a GPU looks up the array's address; n = 0 does only that (for use before a capture).
 */
#define TRIACCEL_STATIC_MAX_TENSORS 256
#define TRIACCEL_STATIC_MAX_CHUNKS 65536
int triaccel_power_iter_static(const triaccel_power_tensor *vectors, const int64_t *numel, int32_t n, int32_t k,
                               triaccel_power_info *info, void *hip_stream);

/*
 * Utility: convert n fp32 values (device) to `dtype` (device) with the same round-to-nearest-even
 * store the update kernel uses; dtype FP32 copies.  Enqueued on `hip_stream`.  Both pointers
 * 16-byte aligned.
 */
int triaccel_cast_f32(const float *src, void *dst, int64_t n, int32_t dtype, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* TRIACCEL_H */
