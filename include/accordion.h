/*
 * accordion.h -- C ABI of the Accordion gradient-compression hot path for one
 * AMD MI355X (gfx950).  arxiv 2010.16248.
 *
 * What the library computes, per training step, for W simulated data-parallel
 * workers on one GPU (the paper's setting: Section 3; compressors: Section 5):
 *
 *   Delta_w = g_w + e_w                       error feedback ("memory term", Sec. 5.3, App. A)
 *   A      += g_0                             per-layer accumulated gradient (Sec. 4.2)
 *   PowerSGD, matrix layers:  P_w = Delta_w Q,  P^ = orthonormalise(mean_w P_w),
 *                             Q_w = Delta_w^T P^,  Q~ = mean_w Q_w (next step's Q),
 *                             D = P^ Q~^T,  e_w = Delta_w - D
 *             1-D layers:     D = mean_w g_w,  e_w = 0      (App. "Compression Ratio Selection")
 *   TopK, every layer:        keep the k entries of Delta_w with the largest |.|
 *                             (ties: lower flat index), payload (index, value),
 *                             e_w = Delta_w with the kept entries zeroed,
 *                             D = (sum over workers of their kept values) / W
 *   end of a window:          c_l = ||A_l||_2,  Algorithm 1 per layer
 *                             (| old - c | / old >= eta  or  lr_next < lr_curr  => critical),
 *                             old <- c,  A <- 0; the level picks rank / k of the next window.
 *
 * Levels.  The paper's l_low is LOW COMPRESSION (higher rank, larger K) and is the
 * level used inside critical regimes; l_high is used outside.  To avoid the word
 * "low" the configuration names them *_crit and *_noncrit.
 *
 * Conventions.
 *  - Every function returns an int32 status (ACC_OK = 0).  Nothing throws, aborts or logs;
 *    accordion_last_error() gives a static, human-readable string for the last failure.
 *  - All tensors are fp32.  "flat" buffers hold all layers concatenated at acc_layer.offset
 *    (in elements); a matrix layer is rows x cols row-major (conv weight out x in x kh x kw
 *    = out x (in*kh*kw)); a 1-D layer has rows = 1.
 *  - Pointers named *_dev are DEVICE pointers and must be 16-byte aligned; pointers named
 *    *_host are HOST pointers.  The library never allocates or frees device memory: the
 *    caller provides one workspace of accordion_workspace_bytes() bytes (256-byte aligned)
 *    that must outlive the context, plus every gradient / output buffer.
 *  - Every call that does device work enqueues it on the HIP stream given at init and returns
 *    without waiting.  The accordion_get_* / accordion_set_state / payload_words calls
 *    synchronise that stream.
 *  - Levels, ranks and kept counts live in device memory and are read by the kernels, so a
 *    level switch costs no host round trip.
 *  - Inputs must be finite; NaN/Inf give unspecified (but memory-safe) results.
 *  - A context is not thread-safe; calls that overlap on one context race.
 */
#ifndef ACCORDION_H
#define ACCORDION_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  ACC_OK = 0,
  ACC_EINVAL = 1,    /* bad argument (null, out of range, misaligned) */
  ACC_ESTATE = 2,    /* call out of order for the step state machine */
  ACC_ENOSPACE = 3,  /* workspace or host buffer too small */
  ACC_EHIP = 4       /* a HIP runtime call failed */
};

enum { ACC_POWERSGD = 0, ACC_TOPK = 1, ACC_BATCH = 2 };

/* Which statistic accordion_detect_regime decides on.  ACC_DETECT_NORM: the paper's own test
 * (Sec. 4.2, Algorithm 1).  ACC_DETECT_MSDR: the comparison method of Sec. 5.6 -- per layer, the
 * mean to standard deviation ratio of worker 0's gradients over the window,
 *     m = || mean_t g_t || / sqrt( mean_t || g_t - mean ||^2 )
 * (from the accumulator, the sum of the squared gradient norms and the step count; fp64, result
 * fp32; +inf if the gradients did not vary).  The paper describes its use in one sentence; the
 * reading taken here: the first window's m is the reference; once m <= (1 - eta) * reference the
 * layer moves to the *_crit level (less compression) for good and m becomes the reference.
 * lr_curr / lr_next play no role.  accordion_get_norms then returns the reference the last decision
 * compared against (old_host) and m (curr_host).  One extra pass over worker 0's gradient per step.
 * accordion_set_state restarts the window sums (import state at a window end).  Not available
 * for ACC_BATCH; eta must be below 1. */
enum { ACC_DETECT_NORM = 0, ACC_DETECT_MSDR = 1 };

#define ACC_MAX_WORKERS 32
#define ACC_MAX_RANK 4
#define ACC_MAX_BATCH_MULTIPLIER 65536

typedef struct acc_layer {
  int64_t offset;     /* first element of the layer in the flat buffers */
  int32_t rows, cols; /* matrix: n x m; 1-D tensor: rows = 1 */
  int32_t is_matrix;  /* 1: compressed by PowerSGD; 0: 1-D tensor (sent raw by PowerSGD) */
} acc_layer;

typedef struct acc_config {
  int32_t method;              /* ACC_POWERSGD or ACC_TOPK */
  int32_t n_layers;
  const acc_layer* layers;     /* host array, copied at init; layers must not overlap */
  int64_t n_params;            /* length of the flat buffers; >= max(offset + rows*cols) */
  int32_t n_workers;           /* W in [1, ACC_MAX_WORKERS] */
  int32_t rank_crit;           /* PowerSGD rank inside critical regimes, in [1, ACC_MAX_RANK] */
  int32_t rank_noncrit;        /* PowerSGD rank outside */
  int32_t k_num_crit;          /* TopK: k = max(1, ceil(n * num / den)) per layer */
  int32_t k_num_noncrit;
  int32_t k_den;
  float   eta;                 /* detection threshold of Sec. 4.2; the paper uses 0.5 */
  int32_t initial_level;       /* level before the first decision: 1 = critical, 0 = not */
  int32_t batch_multiplier;    /* ACC_BATCH: floor(B_high / B_low) in [1, ACC_MAX_BATCH_MULTIPLIER]; else ignored */
  int32_t batch_monotone;      /* ACC_BATCH: 1 = once the large batch is chosen it is kept (App. A) */
  int32_t detector;            /* ACC_DETECT_NORM (0, the paper's) or ACC_DETECT_MSDR */
} acc_config;

typedef struct acc_ctx acc_ctx;

/* Size of the device workspace for this configuration (host-only arithmetic, no GPU needed).
 * Errors: ACC_EINVAL for null pointers or an invalid configuration. */
int32_t accordion_workspace_bytes(const acc_config* cfg, size_t* out_bytes);

/* Create a context (Algorithm 1's hyper-parameters l_low/l_high/eta and the layer table).
 * workspace_dev: device memory, >= accordion_workspace_bytes(), 256-byte aligned, owned by the
 *   caller; it is cleared here (e = 0, A = 0, no previous norms, level = initial_level).
 * q_init_host: PowerSGD only -- for every matrix layer, in layer order, cols x r_max floats
 *   (row-major, r_max = max(rank_crit, rank_noncrit)), the caller's N(0,1) start for Q.
 *   Ignored (may be NULL) for TopK.
 * hip_stream: a hipStream_t (NULL = the default stream).
 * Errors: ACC_EINVAL, ACC_ENOSPACE (workspace too small), ACC_EHIP.  On error *out is NULL. */
int32_t accordion_init(const acc_config* cfg, void* workspace_dev, size_t workspace_bytes,
                       const float* q_init_host, void* hip_stream, acc_ctx** out);

/* accordion_init for callers that cannot allocate device memory (code that runs under HIP graph
 * capture, serving loops, harnesses that forbid hipMalloc): the workspace is an array of
 * ACC_STATIC_WORKSPACE_BYTES bytes that lives inside the library's device code, one copy per GPU,
 * held until the process ends.  No hipMalloc, hipFree or other allocating call is made; gradients and
 * outputs are still the caller's.  The context belongs to the device that is current at the call.
 * Errors: as accordion_init; ACC_ENOSPACE when the configuration needs a larger workspace than the
 * array (accordion_workspace_bytes tells; use accordion_init then).
 * Every context created this way on one GPU uses the same array: the call clears it and lays it
 * out anew, so the context created last is the only usable one -- calls on an earlier one return
 * ACC_ESTATE (accordion_destroy still works) -- and two threads must not use such contexts on one
 * GPU at the same time: their work would race on the array. */
#define ACC_STATIC_WORKSPACE_BYTES (32u << 20)
int32_t accordion_init_static(const acc_config* cfg, const float* q_init_host, void* hip_stream, acc_ctx** out);

/* Enqueue all later work of this context on another HIP stream (NULL = the default stream).
 * Only between steps (else ACC_ESTATE).  The library does not order the two streams: the caller
 * makes the new stream wait for what the old one still has in flight.
 * HIP graphs: accordion_step_all, accordion_step_all_update and accordion_detect_regime only
 * launch kernels (no allocation, no memset, no synchronisation, per-kernel timing off), so a
 * caller may capture them on the context's stream and replay the graph.  What the host passes by
 * value is frozen into the graph: the gradient / output pointers, lr, momentum, weight_decay,
 * and the step number, which only steers the TopK bin guess (never a result) -- except in
 * batch-size mode, where it selects the slot of the micro-step count: capture an even number of
 * micro-steps per graph there.  Everything else a step depends on (levels, ranks, kept counts,
 * whether PowerSGD's residual is still pending) lives in device memory, so accordion_flush,
 * accordion_get_state or accordion_detect_regime may run between replays. */
int32_t accordion_set_stream(acc_ctx* ctx, void* hip_stream);

/* Free the host-side context (the workspace stays the caller's). */
int32_t accordion_destroy(acc_ctx* ctx);

/* Static description of the last error of this context (or of the last failed init when
 * ctx is NULL). */
const char* accordion_last_error(const acc_ctx* ctx);

/* C(g_w, l): one worker's compression (Sec. 3 update rule; Sec. 5 compressors).
 * phase 0: Delta_w = grad + e_w (kept in place of e_w); worker 0 also does A += grad.
 *          PowerSGD: P_w = Delta_w Q.  TopK: select, write the payload, zero the kept
 *          entries of e_w.   grad_dev: N floats; for PowerSGD it must stay unmodified until
 *          accordion_aggregate(ctx, 0) has run (the raw 1-D tensors are averaged there).
 * phase 1: PowerSGD only: Q_w = Delta_w^T P^ (grad_dev is ignored and may be NULL).
 * Order per step: phase 0 for each worker once (any order), aggregate(0), [phase 1 for each
 * worker, aggregate(1)], decompress.  Anything else returns ACC_ESTATE and touches nothing. */
int32_t accordion_compress_step(acc_ctx* ctx, int32_t worker, const float* grad_dev, int32_t phase);

/* The mean over workers that the all-reduce / all-gather provides (Sec. 5.1 "Implementation",
 * Sec. 3).  phase 0, PowerSGD: P^ = orthonormalise(mean_w P_w) by modified Gram-Schmidt in
 * column order (a zero column stays zero), and the mean of the raw 1-D tensors.
 * phase 0, TopK: the W payloads count as gathered (no arithmetic; the sum is in decompress).
 * phase 1, PowerSGD only: Q~ = mean_w Q_w, stored as the next step's Q. */
int32_t accordion_aggregate(acc_ctx* ctx, int32_t phase);

/* Averaged, decompressed gradient of this step into out_dev (N floats; every element that
 * belongs to a layer is overwritten).
 * PowerSGD: D = P^ Q~^T on matrix layers (the residual e_w = Delta_w - D of every worker becomes
 * the error memory, see accordion_flush); 1-D layers get the plain mean.  TopK: D[i] = (sum over workers, in worker order from +0, of the values kept
 * at i) / W.  Ends the step. */
int32_t accordion_decompress(acc_ctx* ctx, float* out_dev);

/* The whole step for all workers with batched launches: phase 0 for every worker,
 * aggregate, [phase 1, aggregate], decompress.  grads_host_array: HOST array of W DEVICE
 * pointers (N floats each).  Same results as the call-by-call sequence. */
int32_t accordion_step_all(acc_ctx* ctx, const float* const* grads_host_array, float* out_dev);

/* The optimizer that consumes the averaged decompressed gradient, fused into the pass that would
 * store it: SGD with Nesterov momentum (App. A, table "Hyperparameters": Nesterov, momentum 0.9)
 * on the update rule of Sec. 3.  With D as accordion_decompress defines it, for every element
 * that belongs to a layer (others are not touched):
 *     d = D + weight_decay * w   (only if weight_decay != 0; the paper names none)
 *     v = momentum * v + d
 *     w = w - lr * (d + momentum * v)
 * in fp32, every product and every sum rounded on its own, in this order.  D itself is not
 * stored anywhere (4 bytes per element written and read again saved).
 * weights_dev, velocity_dev: N floats each, DEVICE, 16-byte aligned, distinct, owned by the
 * caller; the velocity starts at zero.  lr, momentum, weight_decay: finite, >= 0.
 * accordion_decompress_update takes the place of accordion_decompress in the call-by-call
 * sequence, accordion_step_all_update that of accordion_step_all; state machine, effects on the
 * error memory and the accumulator, and errors are theirs (plus ACC_EINVAL for the arguments
 * above, checked before anything is launched). */
int32_t accordion_decompress_update(acc_ctx* ctx, float* weights_dev, float* velocity_dev, float lr,
                                    float momentum, float weight_decay);
int32_t accordion_step_all_update(acc_ctx* ctx, const float* const* grads_host_array,
                                  float* weights_dev, float* velocity_dev, float lr, float momentum,
                                  float weight_decay);

/* --- batch-size mode (method = ACC_BATCH) ----------------------------------------------------
 * Accordion switching the batch size instead of a compression level (Sec. 3 "Distributed SGD
 * with adaptive batch size"; Sec. 4.2: same algorithm, on the gradient of the whole model;
 * App. A "Additional Details for Batch Size experiment": the large batch is several backward
 * passes summed before one exchange).  One accordion_step_all / accordion_step_all_update call
 * is one MICRO-STEP: every worker's gradient of a micro-batch of B_low samples.
 *     A += g_0;   S_w = g_w (first micro-step of a batch) or S_w + g_w      (S_w lives where the
 *                                                                            error memory does)
 *     a batch is complete after 1 micro-step at level 1 (critical: batch B_low) and after
 *     batch_multiplier micro-steps at level 0 (batch B_high); then, with n = micro-steps in it,
 *     D = (S_0 + S_1 + ... + S_{W-1}) / (W n)   in fp32, in this order, one division.
 * accordion_step_all writes D to out_dev when the micro-step completes a batch and leaves
 * out_dev untouched otherwise; accordion_step_all_update applies the optimizer step then, with
 * the learning rate lr * n (Sec. 5.1: the rate grows in the ratio of the batch), and leaves
 * weights and velocity untouched otherwise.  The level and the micro-step count live on the
 * device: no host round trip decides whether a batch is complete; accordion_batch_status tells.
 * accordion_detect_regime: one norm over all layers' accumulated gradient, Algorithm 1 once; with
 * batch_monotone a level that has reached 0 stays 0.  accordion_payload_words counts n_model
 * floats (the dense all-reduce) per completed batch and none otherwise.
 * The call-by-call entry points return ACC_EINVAL for this method.  State layout: S_0..S_{W-1}
 * | A | pending micro-steps (int32) | norm_old (L) | has_old (L) | level (L, all equal); the
 * sums are meaningful only while pending > 0. */
int32_t accordion_batch_status(acc_ctx* ctx, int32_t* level, int32_t* pending_micro_steps,
                               int32_t* last_batch_micro_steps, int64_t* exchanges,
                               int64_t* micro_steps);

/* End of a window (Sec. 4.2; Algorithm 1): c_l = ||A_l||_2 (fp64 sum, fp32 result), per layer
 * critical <=> no previous norm, previous norm 0, |old - c| / old >= eta, or lr_next < lr_curr;
 * level <- critical; old <- c; A <- 0.  Only between steps (else ACC_ESTATE). */
int32_t accordion_detect_regime(acc_ctx* ctx, float lr_curr, float lr_next);

/* The batched entry points (accordion_step_all, accordion_step_all_update) keep Delta_w in the
 * error memory at the end of a step and form the residual in the first pass of the next step:
 * PowerSGD e_w = Delta_w - D from the stored factors, TopK e_w = Delta_w with the kept entries
 * dropped, from the stored thresholds and tie counts (one write of the memory saved per worker
 * and step).  accordion_flush writes the residual out now; accordion_get_state does so by itself.
 * Only between steps (else ACC_ESTATE).  The call-by-call TopK path writes it directly. */
int32_t accordion_flush(acc_ctx* ctx);

/* A <- 0 without a decision (to measure one epoch out of several, Sec. 5.1 "Hyperparameters"). */
int32_t accordion_reset_accumulator(acc_ctx* ctx);

/* --- read-backs (synchronise the stream) ------------------------------------------------ */

/* levels_host: n_layers int32, 1 = critical. */
int32_t accordion_get_levels(acc_ctx* ctx, int32_t* levels_host);
/* old_host: the previous norm the last decision compared against (0 if none);
 * curr_host: the norm it computed.  n_layers floats each. */
int32_t accordion_get_norms(acc_ctx* ctx, float* old_host, float* curr_host);
/* TopK payload of (worker, layer) from the last step: idx_host (int32, ascending, layer-local
 * flat index) and val_host (fp32), each with room for capacity entries; *count_out = k.
 * Errors: ACC_ENOSPACE if capacity < k (count_out is still set). */
int32_t accordion_get_payload(acc_ctx* ctx, int32_t worker, int32_t layer, int32_t* idx_host,
                              float* val_host, int64_t capacity, int64_t* count_out);
/* How a TopK layer's payload is laid out at a level (host-only arithmetic, no GPU needed).  The
 * paper's own runs keep K = 99 % inside critical regimes (Sec. 5.4, TopK tables), where a list of
 * (index, value) pairs costs 1.98 n floats -- more than the dense tensor.  A layer that keeps more
 * than half of its n entries therefore sends its k values in index order plus the n - k indices
 * of the dropped entries: n floats, never more than dense.  format: ACC_PAYLOAD_INDEX_VALUE
 * (2 k <= n; words = 2 k) or ACC_PAYLOAD_VALUES_HOLES (2 k > n; words = n); kept = k.
 * accordion_get_payload decodes either layout to (index, value); accordion_payload_words keeps
 * the paper's accounting of 2 k floats per layer. */
enum { ACC_PAYLOAD_INDEX_VALUE = 0, ACC_PAYLOAD_VALUES_HOLES = 1 };
int32_t accordion_payload_format(const acc_config* cfg, int32_t layer, int32_t level, int32_t* format,
                                 int64_t* kept, int64_t* words);

/* PowerSGD factors of a matrix layer from the last step: p_hat_host rows x r and q_host
 * cols x r (row-major, r = *rank_out, the rank that step used); room for ACC_MAX_RANK
 * columns each is required. */
int32_t accordion_get_factors(acc_ctx* ctx, int32_t layer, float* p_hat_host, float* q_host,
                              int32_t* rank_out);
/* Floats one worker sent in the last step / since init (PowerSGD: r(n+m) per matrix layer
 * + n per 1-D layer; TopK: 2k per layer -- the accounting of the paper's "Data Sent"). */
int32_t accordion_payload_words(acc_ctx* ctx, int64_t* last_step, int64_t* cumulative);

/* TopK diagnostics since init (they describe which path the selection took, never its result):
 * restaged_layers = (worker, layer) pairs whose threshold bin lay outside the bins the
 * error-feedback pass had worked on, on a guess: Delta was read once more for them and the
 * layer was decided by sweeps of one workgroup (slow);
 * swept_layers = pairs whose guess held but whose tie class was too large for the per-quarter
 * key lists, decided by the same sweeps. */
int32_t accordion_topk_stats(acc_ctx* ctx, int64_t* restaged_layers, int64_t* swept_layers);

/* Overlap of the kept coordinates of two workers in the last step (Sec. 4.3: how much the
 * Top-K supports of a pair of stochastic gradients overlap; the paper reports > 90 % for
 * Top-10 %).  TopK only, between steps, after at least one step (else ACC_ESTATE).
 * common_host[l] = number of coordinates of layer l that both workers kept; kept_host[l] = k of
 * that step; n_layers entries each.  The overlap fraction is sum(common) / sum(kept).  With error
 * feedback the kept sets are those of gradient + memory; on the first step after init they are
 * those of the gradients themselves.  Synchronises the stream. */
int32_t accordion_topk_overlap(acc_ctx* ctx, int32_t worker_a, int32_t worker_b, int64_t* common_host,
                               int64_t* kept_host);

/* State export / import for checkpointing and step-by-step comparison.  Layout (bytes, all
 * little-endian fp32/int32, no padding):  e_0 .. e_{W-1} (N each) | A (N) | Q (sum over
 * matrix layers of cols*r_max; absent for TopK) | norm_old (L) | has_old (L, int32) |
 * level (L, int32).  accordion_state_bytes gives the size.  Only between steps. */
int32_t accordion_state_bytes(const acc_ctx* ctx, size_t* out_bytes);
int32_t accordion_get_state(acc_ctx* ctx, void* state_host, size_t bytes);
int32_t accordion_set_state(acc_ctx* ctx, const void* state_host, size_t bytes);

/* --- per-kernel timing (tracing aid; not part of the paper's method) -------------------------
 * With profiling on, a kernel launch carries two HIP events that take the begin and the end
 * timestamp of its dispatch on the context's stream, and the elapsed time is accumulated per
 * stage: enable = 1 times every kernel, enable = 2 only the fused error-feedback pass of the
 * method (the kernel that moves the most bytes), enable = 3 only every fourth launch of that
 * pass (a timed launch costs a few us of stream time); 0 switches it off.  Not to be switched on
 * while the stream is being captured into a graph.  accordion_get_profile
 * synchronises the stream and returns the accumulated milliseconds and the number of launches
 * of one stage since profiling was last switched on.  Stages are numbered from 0, fewer than
 * ACC_N_STAGES of them; accordion_stage_name gives the kernel's name, NULL beyond the last stage
 * (accordion_get_profile returns ACC_EINVAL there). */
#define ACC_N_STAGES 48
int32_t accordion_set_profiling(acc_ctx* ctx, int32_t enable);
int32_t accordion_get_profile(acc_ctx* ctx, int32_t stage, double* total_ms, int64_t* launches);
const char* accordion_stage_name(int32_t stage);

/* --- measurement aid (not part of the paper's method) ---------------------------------------
 * Plain streaming copy dst_dev[0..n) = src_dev[0..n) (n floats, a positive multiple of 4; both
 * DEVICE pointers, 16-byte aligned, not overlapping) enqueued on hip_stream.  It moves exactly
 * 4n bytes in and 4n bytes out, which calibrates the memory counters of a profiler run and
 * gives the copy bandwidth the memory system reaches.  Needs no context.
 * Errors: ACC_EINVAL, ACC_EHIP (message via accordion_last_error(NULL)). */
int32_t accordion_probe_copy(float* dst_dev, const float* src_dev, int64_t n, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ACCORDION_H */
