/*
 * ga3c.h -- C ABI of the MI355X (gfx950) library for the GPU side of hybrid
 * CPU/GPU A3C (arXiv 1611.06256, "GA3C").
 *
 * The paper keeps ONE copy of the policy/value network on the GPU
 * (Sec. 4.1).  Predictor threads send it batches of states and get back the
 * policy and the value; trainer threads send it batches of experiences and
 * the network is updated in place.  This library is that network: two calls
 * that do all of their work in hand-written HIP kernels, plus parameter
 * access.
 *
 * Conventions that hold for every entry point
 *   - Pointers named *_dev are DEVICE memory owned by the caller; pointers
 *     without the suffix are HOST memory.  The library never frees or keeps a
 *     caller's pointer beyond the kernels it enqueues in that call.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Calls only enqueue work on it and never synchronise the host; outputs
 *     are valid once the caller has synchronised the stream.  ga3c_predict
 *     calls must be stream-ordered among themselves, and so must
 *     ga3c_train_step calls (each kind owns one set of workspaces), but the
 *     two kinds may run on two different streams: the context keeps two
 *     copies of the parameters, an update writes the copy that is not being
 *     read and publishes it, and HIP events order that against the
 *     predictions (a prediction sees the parameters of the last update that
 *     was ENQUEUED before it, never a half-written set).
 *   - One HOST thread at a time drives a context: the calls keep host-side
 *     state without locks (which parameter copy is published, where each event
 *     was last recorded, the profiler's lists).  The paper's predictor and
 *     trainer THREADS exist because its GPU calls block their caller; here a
 *     call only enqueues, so one thread can feed both streams (ga3c_sched_*
 *     does exactly that).  Callers that do use several threads must serialise
 *     their calls on one context themselves; the concurrency that matters, the
 *     overlap of prediction and training on the GPU, comes from the two streams.
 *     Different contexts are independent, except that ga3c_predict_static calls
 *     on one GPU share one scratch array.
 *   - Return value: GA3C_OK or a negative GA3C_E* code.  Nothing is printed,
 *     no C++ exception crosses the boundary.  ga3c_last_error() returns a
 *     thread-local description of the last failure on the calling thread.
 *   - Float tensors are IEEE fp32, row-major, the last index fastest.
 *
 * Flat parameter vector (what ga3c_params_get / _set speak), in this order:
 *   for each conv layer l: W[oc][ic][kh][kw], b[oc];
 *   fc W[fc_units][flat] with flat index = c*H*W + h*W + w of the last conv
 *   output, fc b[fc_units]; policy W[n_actions][fc_units], policy b[n_actions];
 *   value W[fc_units], value b[1].
 */
#ifndef GA3C_H
#define GA3C_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GA3C_OK        0
#define GA3C_EINVAL   -1   /* null pointer, bad shape, batch above the capacity given at create */
#define GA3C_ENOMEM   -2   /* device or host allocation failed */
#define GA3C_EHIP     -3   /* a HIP runtime call failed; see ga3c_last_error() */

#define GA3C_MAX_CONV  4
#define GA3C_MAX_ACTIONS 63

typedef struct ga3c_ctx ga3c_ctx;   /* opaque: parameters, RMSProp state, gradient, workspaces */

/* Network shape.  Sec. 3.2 describes the small network: conv 16 filters 8x8
 * stride 4, conv 32 filters 4x4 stride 2, fully connected 256, a rectifier
 * after each hidden layer, a softmax policy output and a linear value
 * output.  Convolutions are VALID cross-correlations.  Limits: n_conv in
 * [1,4]; n_actions in [1,63]; (n_actions + 5) * (fc_units + 16) <= 40960 (the
 * heads keep their weights in LDS); every spatial size must stay >= 1. */
typedef struct {
    int in_c, in_h, in_w;                 /* input planes / height / width (4, 84, 84) */
    int n_conv;
    struct { int oc, k, stride; } conv[GA3C_MAX_CONV];
    int fc_units;
    int n_actions;
    int math;                             /* 0 = fp32 accuracy; 1 = both operands of every contraction rounded to bfloat16 */
} ga3c_net_desc;

/* Hyper-parameters of one update, read on the host at call time.
 *   gamma      discount of the n-step return (text after Eq. 1)
 *   beta       weight of the entropy term (Eq. 1)
 *   value_coef weight of the value cost (Eq. 2 has none: 1.0)
 *   log_eps    epsilon added inside the logarithms (Eq. 5); 0 = plain Eq. 1
 *   lr, rms_decay, rms_eps   eta, alpha, epsilon of RMSProp (Eq. 3; epsilon
 *              is inside the square root)
 *   clip_norm  threshold of the global L2-norm rescale of the summed
 *              gradient; <= 0 disables it */
typedef struct {
    float gamma, beta, value_coef, log_eps;
    float lr, rms_decay, rms_eps, clip_norm;
} ga3c_hparams;

/* Written by ga3c_train_step to device memory when asked for.  Losses are
 * SUMS over the frames of the call (Sec. 5.3 sums gradients over the batch).
 * nonfinite is 1 when the gradient norm is NaN or infinite. */
typedef struct {
    float policy_loss, value_loss, entropy, grad_norm, clip_scale;
    int32_t nonfinite;
} ga3c_train_stats;

/* Create a context on the current HIP device.  Allocates (with hipMalloc)
 * the parameters theta, the RMSProp accumulator g, the gradient and all
 * workspaces for up to max_predict_batch frames per ga3c_predict and
 * max_train_frames frames (= N*T) per ga3c_train_step.  theta and g start at
 * zero.  On failure *out is NULL. */
int ga3c_create(const ga3c_net_desc *desc, int max_predict_batch, int max_train_frames,
                ga3c_ctx **out);

/* Waits for the device, then frees everything the context owns. */
int ga3c_destroy(ga3c_ctx *ctx);

/* Number of floats in the flat parameter vector (0 for a NULL context). */
size_t ga3c_params_count(const ga3c_ctx *ctx);

/* Offsets of the tensors in the flat vector, in the order listed at the top,
 * followed by the total: 2*n_conv + 7 entries.  `off` is host memory with
 * room for `cap` entries; returns the number written or GA3C_EINVAL. */
int ga3c_params_offsets(const ga3c_ctx *ctx, int64_t *off, int cap);

/* theta: weights ~ N(0, 2/fan_in) ("He normal"), biases 0; g = 0.  The
 * normal deviates come from a counter-based generator keyed by (seed, flat
 * index), so the result depends on nothing else.  (The paper does not state
 * its initialisation.) */
int ga3c_params_init(ga3c_ctx *ctx, uint64_t seed, void *stream);

/* Copy n = ga3c_params_count() floats out of / into the context.
 * which: 0 = theta, 1 = RMSProp accumulator g, 2 = gradient of the last
 * ga3c_train_step (unclipped sum over its frames; get only). */
int ga3c_params_get(ga3c_ctx *ctx, int which, float *dst_dev, size_t n, void *stream);
int ga3c_params_set(ga3c_ctx *ctx, int which, const float *src_dev, size_t n, void *stream);

/* Prediction (Sec. 4.1, the predictor's inference query): states in, policy
 * and value out.
 *   frames_dev   u8 [B][in_c][in_h][in_w], raw pixels; scaled by 1/255 inside
 *   uniforms_dev f32 [B] in [0,1), or NULL.  Needed iff actions_dev != NULL.
 *   logits_dev   f32 [B][n_actions]  pre-softmax policy output (may be NULL)
 *   values_dev   f32 [B]             V(s) (may be NULL)
 *   probs_dev    f32 [B][n_actions]  softmax policy pi(.|s) (may be NULL)
 *   actions_dev  i32 [B] (may be NULL): a = the first j whose running fp32 sum
 *                p_0 + ... + p_j (added left to right) exceeds u, else
 *                n_actions - 1.
 * 0 <= B <= max_predict_batch; B = 0 is a no-op.  Calls on one context share
 * its workspace: issue them on one stream, or order them with events. */
int ga3c_predict(ga3c_ctx *ctx, const uint8_t *frames_dev, int B,
                 const float *uniforms_dev,
                 float *logits_dev, float *values_dev, float *probs_dev, int32_t *actions_dev,
                 void *stream);

/* One A3C update on N agents x T steps (Sec. 3.2; Sec. 4.1, the trainer's
 * model update; gradients summed over all N*T frames, Sec. 5.3):
 *   R[n][T] = bootstrap[n]; R[n][t] = r[n][t] + gamma (1 - done[n][t]) R[n][t+1]
 *   minimise  sum_i  -log(pi_i[a_i] + log_eps) (R_i - V_i)        (R_i - V_i constant here)
 *                    - beta H(pi_i) + value_coef (R_i - V_i)^2    (Eq. 1, 2, 5)
 *   d = min(1, clip_norm / ||grad||) * grad;  g = alpha g + (1 - alpha) d^2;
 *   theta -= lr d / sqrt(g + rms_eps)                             (Eq. 3)
 *   frames_dev    u8  [N][T][in_c][in_h][in_w]
 *   actions_dev   i32 [N][T], each in [0, n_actions)
 *   rewards_dev   f32 [N][T]
 *   dones_dev     u8  [N][T], non-zero = the episode ended with this step
 *   bootstrap_dev f32 [N] value of the state after the last step, or NULL = 0
 *   hp            host pointer
 *   stats_dev     device pointer or NULL
 * N*T <= max_train_frames; N*T = 0 is a no-op. */
int ga3c_train_step(ga3c_ctx *ctx, const uint8_t *frames_dev, const int32_t *actions_dev,
                    const float *rewards_dev, const uint8_t *dones_dev,
                    const float *bootstrap_dev, int N, int T,
                    const ga3c_hparams *hp, ga3c_train_stats *stats_dev, void *stream);

/* The same update on N segments of unequal length laid end to end (Sec. 4.1:
 * an agent hands in its experiences after t_max actions or when its episode
 * ends, so a training batch also holds shorter segments):
 *   frames_dev    u8  [n_frames][in_c][in_h][in_w]
 *   actions_dev   i32 [n_frames];  rewards_dev f32 [n_frames];  dones_dev u8 [n_frames]
 *   seg_start_dev i32 [N+1], device memory: segment n is the frames
 *                 seg_start[n] .. seg_start[n+1]-1; seg_start[0] = 0,
 *                 seg_start[N] = n_frames, never decreasing (an empty segment
 *                 is allowed and contributes nothing).  The table is read on
 *                 the device only, so it is not checked: with a table that
 *                 breaks these rules the returns are meaningless, but no
 *                 access leaves the arrays.
 *   bootstrap_dev f32 [N] value of the state after each segment's last step
 *                 (0 where the episode ended), or NULL = 0
 * The return of frame i in segment n is r[i] + gamma (1 - done[i]) R[i+1],
 * with R[seg_start[n+1]] = bootstrap[n]; everything else is as above.
 * n_frames <= max_train_frames; n_frames = 0 is a no-op; N >= 1 otherwise. */
int ga3c_train_step_ragged(ga3c_ctx *ctx, const uint8_t *frames_dev, const int32_t *actions_dev,
                           const float *rewards_dev, const uint8_t *dones_dev, const int32_t *seg_start_dev,
                           const float *bootstrap_dev, int N, int n_frames,
                           const ga3c_hparams *hp, ga3c_train_stats *stats_dev, void *stream);

/* Intermediates of the last ga3c_train_step, for checking it step by step.
 * which: 0 = returns R [N*T]; 1 = logits [N*T][A]; 2 = values [N*T];
 * 3 = dL/d(logits, value) [N*T][A+1];
 * 4 + l = output of conv layer l after its rectifier [N*T][oc][oh][ow];
 * 8 = output of the fully connected layer after its rectifier [N*T][fc_units];
 * 9 = dL/d(pre-activation of the fully connected layer) [N*T][fc_units];
 * 10 + l = dL/d(pre-activation of conv layer l), shaped like 4 + l.
 * Copies n floats (n must not exceed the tensor's size for the last call's
 * N*T).  With these a test can hand each layer of a reference the inputs the
 * library itself used. */
int ga3c_train_debug_get(ga3c_ctx *ctx, int which, float *dst_dev, size_t n, void *stream);

/* RMSProp alone (Eq. 3) on caller-owned flat buffers of any length, with the
 * same kernel ga3c_train_step uses; scale multiplies the gradient first.
 * Exists so that the kernel can be measured on a buffer far larger than the
 * last-level cache. */
int ga3c_rmsprop_flat(float *theta_dev, float *g_dev, const float *grad_dev, size_t n,
                      float scale, float lr, float rms_decay, float rms_eps, void *stream);

/* Layers whose shape matches one of the paper's networks run on kernels
 * compiled for that shape; every other shape runs on the general gather
 * kernels.  on != 0 forces the general kernels for all layers (used to test
 * them at the paper's shapes too); on == 0 restores the default. */
int ga3c_use_generic_kernels(ga3c_ctx *ctx, int on);

/* Per-stage timing for measurement, off by default.  While it is on, every
 * kernel that ga3c_predict and ga3c_train_step launch carries a pair of HIP
 * events which the runtime stamps with the start and the end of that very
 * dispatch: a stage's time is the sum of the execution times of its kernels
 * (what a kernel trace shows), without queueing or dispatch latency.
 * ga3c_profile_read waits for the recorded events, adds up the elapsed times
 * and writes one text line per stage into the HOST buffer buf:
 *   "<stage> <calls> <total_ms> <algorithmic_flop> <algorithmic_bytes>\n"
 * then forgets what it has reported.  Returns GA3C_EINVAL if cap is too small.
 * The flop and byte figures are those of the method (2 per multiply-add of
 * the layer's definition; 20 bytes per parameter for RMSProp), not counters. */
int ga3c_profile_enable(ga3c_ctx *ctx, int on);
int ga3c_profile_read(ga3c_ctx *ctx, char *buf, size_t cap);

/* ---- queue-driven batching on one GPU (Sec. 4.1 and 4.3) -------------------
 *
 * The paper's predictors drain "as many prediction requests as are
 * immediately available" into one inference call, its trainers merge the
 * agents' experience batches into one update (at least a minimum number of
 * frames, Sec. 5.3), and every period one of the system's knobs is changed at
 * random by one step and the change kept if trainings per second did not drop
 * (Sec. 4.3).  Here the knobs are the two batch caps; the two kinds of call
 * run on two HIP streams of default priority that the scheduler owns.  A
 * request or segment leaves its queue only after the GPU work that serves it
 * has been enqueued without error.
 *
 * One host thread drives a scheduler: submit, tick and poll are not
 * thread-safe against each other.  Frames are DEVICE memory owned by the
 * caller, 16-byte aligned, and must stay unchanged until the tick that
 * consumed them has finished on the GPU (ga3c_sched_drain, or the
 * prediction's result has been polled).  A segment has 1 .. t_max steps (fewer
 * than t_max when the agent's episode ended, Sec. 4.1); actions / rewards /
 * dones are HOST arrays of that many entries, copied at submit time.
 *
 * Policy lag (Sec. 4.2: the policy that acted may be several updates older
 * than the parameters its experiences update): every prediction carries the
 * number of updates that had been issued before the parameters it read; an
 * agent hands that number back with the segment, and the scheduler adds up,
 * per segment, how many updates were issued between the two. */
typedef struct ga3c_sched ga3c_sched;
typedef struct ga3c_tuner ga3c_tuner;

typedef struct {
    int t_max;                              /* steps per trajectory (the paper's t_max = 5) */
    int predict_cap;                        /* frames per prediction batch, 1 .. max_predict_batch */
    int train_min;                          /* an update waits until this many frames are queued */
    int train_cap;                          /* frames per update, t_max .. max_train_frames */
    int adjust_period;                      /* ticks per adjustment window; 0 = caps stay fixed.  With the adjustment
                                               on, its training knob is the batch size itself: an update waits for
                                               train_cap frames (never fewer than train_min) and takes at most as many */
    int predict_cap_lo, predict_cap_hi;     /* bounds for the adjustment (cap moves by factors of 2) */
    int train_cap_lo, train_cap_hi, train_cap_step;   /* bounds and step (frames) for the adjustment */
    uint64_t seed;                          /* of the adjustment's random choices */
    ga3c_hparams hp;                        /* used for every update */
    float adjust_margin;                    /* a trial is kept iff throughput >= (1 - margin) * reference; 0 = 0.03 */
} ga3c_sched_config;

typedef struct {
    int32_t agent; int32_t action; float value;
    int32_t policy_version;                 /* updates issued before the parameters this prediction read */
} ga3c_prediction;

typedef struct {
    int64_t ticks, predictions, predict_batches, trained_frames, train_batches;
    int64_t sum_predict_queue, sum_train_queue;   /* queue lengths (requests / trajectories) summed over ticks */
    int64_t predict_queue, train_queue;           /* now */
    int64_t trials_accepted, trials_rejected;
    int32_t predict_cap, train_cap;               /* now */
    double last_window_frames_per_s;
    int64_t short_segments;                       /* trained segments with fewer than t_max steps */
    int64_t lag_sum, lag_count, lag_max;          /* policy lag in updates over the trained segments that gave a version */
    int64_t windows, last_change_window;          /* adjustment windows so far; the one in which the kept caps last changed */
} ga3c_sched_stats;

int ga3c_sched_create(ga3c_ctx *ctx, const ga3c_sched_config *cfg, ga3c_sched **out);
/* Waits for the scheduler's streams, frees its buffers; the context stays. */
int ga3c_sched_destroy(ga3c_sched *s);
/* Agent `agent` asks for an action for the state in frame_dev (u8 [C][H][W]);
 * uniform in [0,1) drives the draw. */
int ga3c_sched_submit_predict(ga3c_sched *s, int agent, const uint8_t *frame_dev, float uniform);
/* Agent `agent` hands in len experiences, 1 <= len <= t_max: frames_dev u8
 * [len][C][H][W] (device), actions / rewards / dones (host, len entries), the
 * value of the state after the last step (ignored when that step is terminal),
 * and the policy_version of the prediction that chose the first action, or a
 * negative number to leave the segment out of the lag statistics. */
int ga3c_sched_submit_segment(ga3c_sched *s, int agent, const uint8_t *frames_dev, int len, const int32_t *actions,
                              const float *rewards, const uint8_t *dones, float bootstrap, int64_t policy_version);
/* The same with len = t_max and no version. */
int ga3c_sched_submit_trajectory(ga3c_sched *s, int agent, const uint8_t *frames_dev, const int32_t *actions,
                                 const float *rewards, const uint8_t *dones, float bootstrap);
/* The same for n agents at once (host arrays of n entries; actions, rewards
 * and dones are [n][t_max]).  Entries are queued in index order; on an error
 * the entries before the offending one stay queued (trajectories) or nothing
 * is queued (predictions). */
int ga3c_sched_submit_predict_many(ga3c_sched *s, int n, const int32_t *agents, const uint8_t *const *frames_dev,
                                   const float *uniforms);
int ga3c_sched_submit_trajectory_many(ga3c_sched *s, int n, const int32_t *agents, const uint8_t *const *frames_dev,
                                      const int32_t *actions, const float *rewards, const uint8_t *dones,
                                      const float *bootstrap);
/* Segments of n agents at once: lens [n]; actions, rewards and dones are
 * [n][t_max] with the first lens[i] entries of row i used; policy_versions [n]
 * or NULL (no versions).  Queued in index order; on an error the entries
 * before the offending one stay queued. */
int ga3c_sched_submit_segment_many(ga3c_sched *s, int n, const int32_t *agents, const uint8_t *const *frames_dev,
                                   const int32_t *lens, const int32_t *actions, const float *rewards,
                                   const uint8_t *dones, const float *bootstrap, const int64_t *policy_versions);
/* One pass of predictor and trainer: at most one prediction batch (all queued
 * requests up to the cap; fewer requests than the cap go out only when no
 * earlier prediction batch is still in flight, otherwise they wait for it and
 * are joined by what arrives meanwhile, as with a single predictor that is
 * busy with its batch; full batches are issued back to back, up to four in
 * flight) and at most one update (queued trajectories up to
 * the cap, if at least train_min frames wait; whole segments, oldest first;
 * ga3c_train_step when all have t_max steps, ga3c_train_step_ragged
 * otherwise) are enqueued on the GPU.
 * *predicted / *trained (may be NULL) receive the frames issued.  At the end of
 * an adjustment window the call waits for the window's GPU work to read the
 * clock. */
int ga3c_sched_tick(ga3c_sched *s, int *predicted, int *trained);
/* Copies up to cap finished predictions to out (host), oldest first; returns
 * how many, or a negative error code.  Never blocks. */
int ga3c_sched_poll(ga3c_sched *s, ga3c_prediction *out, int cap);
/* Waits until everything issued so far has finished. */
int ga3c_sched_drain(ga3c_sched *s);
int ga3c_sched_get_stats(const ga3c_sched *s, ga3c_sched_stats *out);
const char *ga3c_sched_last_error(void);

/* The adjustment rule alone (host only, no GPU): caps within [lo, hi]; the
 * prediction cap moves by a factor 2 per step, the training cap by a factor
 * 1 + 2^-k up or down: k = 0 at first (a factor 2 as well), one finer after
 * every rejected step of that knob (down to 1 + 1/64), one coarser after a
 * step that brought a clear gain; training caps are multiples of t_step, a
 * step is at least t_step, the last step to a bound may be shorter.
 * ga3c_tuner_report closes a window that ran the current caps at the given
 * throughput.  The first two windows measure the starting caps (the
 * reference; the first window also pays for the start of the run).  A trial
 * is kept iff its throughput >= (1 - margin) * reference (margin 0.03 unless
 * set): then the caps are kept and the reference becomes the larger of the two
 * readings; if the gain exceeded half the margin ("clear gain") the same knob
 * is stepped in the same direction again.  A trial that is not kept is undone
 * and the kept caps run again before the next trial: for 1, 2, 4, then 8
 * windows after the first, second, ... rejected trial since the last clear
 * gain (the search cools down once it has settled and picks its pace up again
 * with the next clear gain); each such window's reading replaces the reference
 * if higher and is averaged into it if lower.  Otherwise one knob is stepped
 * in a random direction (not the same knob three times in a row; not a
 * direction that was rejected from the knob's present value, unless the other
 * one has been rejected since).  The new caps are returned.  Deterministic for
 * a given seed and sequence of readings. */
int ga3c_tuner_create(int p_lo, int p_hi, int p0, int t_lo, int t_hi, int t_step, int t0, uint64_t seed,
                      ga3c_tuner **out);
int ga3c_tuner_report(ga3c_tuner *t, double throughput, int *predict_cap, int *train_cap);
int ga3c_tuner_state(const ga3c_tuner *t, int *kept_predict_cap, int *kept_train_cap, int64_t *accepted,
                     int64_t *rejected);
int ga3c_tuner_set_margin(ga3c_tuner *t, double margin);
/* Windows reported so far, and the window in which the kept caps last changed (0 = never). */
int ga3c_tuner_progress(const ga3c_tuner *t, int64_t *windows, int64_t *last_change_window);
int ga3c_tuner_destroy(ga3c_tuner *t);

/* Prediction without allocation, for callers that cannot call hipMalloc: code
 * under HIP graph capture, tight serving loops, harnesses that forbid device
 * allocation.  The same kernels as ga3c_predict, for the network of Sec. 3.2
 * only (4x84x84 input, 16 filters 8x8 stride 4, 32 filters 4x4 stride 2, 256
 * fully connected units) with n_actions outputs, and no context: theta_dev is
 * the caller's flat parameter vector in the order given at the top of this file
 * (what ga3c_params_get writes), 16-byte aligned, as are the frames.  All
 * intermediate results (filter fragments, activations, partial sums, tickets)
 * live in one array of GA3C_STATIC_SCRATCH_BYTES that is part of the library's
 * device image: every GPU the library runs on holds it until the process ends.
 * The call allocates and frees nothing, on the device or through any library.
 * 0 <= B <= GA3C_STATIC_MAX_FRAMES; a larger B is rejected with GA3C_EINVAL.
 * The other arguments are those of ga3c_predict.
 * All calls on one GPU share that GPU's array: calls that may overlap (two
 * streams, two threads) race; order them on one stream or with events.  The
 * array keeps the last call's contents; the only part that must start at zero
 * (the tickets) is returned to zero by the kernel that uses it. */
#define GA3C_STATIC_MAX_FRAMES 256
#define GA3C_STATIC_SCRATCH_BYTES (14u << 20)
int ga3c_predict_static(int n_actions, int math, const float *theta_dev, const uint8_t *frames_dev, int B,
                        const float *uniforms_dev, float *logits_dev, float *values_dev, float *probs_dev,
                        int32_t *actions_dev, void *stream);

/* Shape and capacities the context was created with (any pointer may be NULL). */
int ga3c_get_desc(const ga3c_ctx *ctx, ga3c_net_desc *desc, int *max_predict_batch, int *max_train_frames);

/* Thread-local text of the last error on this thread ("" if none). */
const char *ga3c_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* GA3C_H */
