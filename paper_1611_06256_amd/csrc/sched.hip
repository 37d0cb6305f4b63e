// Queue-driven batching on one GPU (paper Sec. 4.1: prediction queue +
// predictors, training queue + trainers) and the dynamic adjustment of the
// batching knobs (Sec. 4.3), on top of ga3c_predict / ga3c_train_step.
//
// The paper runs predictor and trainer THREADS because each GPU call blocks
// its Python caller.  Here every GPU call only enqueues, so one host thread
// (the caller of ga3c_sched_tick) drains both queues: prediction requests that
// are "immediately available" (Sec. 4.1) go out as one batch on the predict
// stream, trajectories are merged until a minimum batch is reached (Sec. 5.3)
// and go out as one update on the train stream.  The two streams overlap on
// the GPU; the context's parameter snapshots keep a prediction from reading
// half-updated weights.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <deque>
#include <new>
#include <vector>

#include "../../include/ga3c.h"
#include "sched_error.hpp"

using ga3c::sfail;

namespace {

#define SHIP(expr)                                                                                   \
    do {                                                                                             \
        hipError_t e_ = (expr);                                                                      \
        if (e_ != hipSuccess)                                                                        \
            return sfail(e_ == hipErrorOutOfMemory ? GA3C_ENOMEM : GA3C_EHIP, "%s: %s", #expr,       \
                         hipGetErrorString(e_));                                                     \
    } while (0)

// Copies whole frames by pointer: dst[i] = *src[i], frame_vecs 16-byte vectors each.
__global__ __launch_bounds__(256) void gather_frames_kernel(const uint4 *const *__restrict__ src, uint4 *__restrict__ dst,
                                                            int frame_vecs) {
    const uint4 *s = src[blockIdx.y];
    uint4 *d = dst + (size_t)blockIdx.y * frame_vecs;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < frame_vecs; i += gridDim.x * 256) d[i] = s[i];
}

}  // namespace

// ------------------------------------------------------------- scheduler ----

namespace {

constexpr int RING = 4;    // batches in flight per stream

struct PredReq { int agent; const uint8_t *frame; float uniform; };
struct Traj {
    int agent;
    int len;                 // experiences in the segment, 1 .. t_max
    int64_t version;         // updates issued before the policy that chose its first action was read; -1 = not given
    const uint8_t *frames;
    std::vector<int32_t> actions;
    std::vector<float> rewards;
    std::vector<uint8_t> dones;
    float bootstrap;
};

struct PredSlot {
    hipEvent_t done = nullptr;
    bool busy = false;
    int n = 0;
    const uint4 **ptrs_h = nullptr, **ptrs_d = nullptr;   // pinned host / device pointer lists
    float *unif_h = nullptr, *unif_d = nullptr;
    uint8_t *frames_d = nullptr;
    int32_t *act_d = nullptr, *act_h = nullptr;
    float *val_d = nullptr, *val_h = nullptr;
    std::vector<int> agents;
    int64_t version = 0;     // updates issued before this batch
};

struct TrainSlot {
    hipEvent_t done = nullptr;
    bool busy = false;
    int n_agents = 0;
    const uint4 **ptrs_h = nullptr, **ptrs_d = nullptr;
    uint8_t *frames_d = nullptr;
    int32_t *act_h = nullptr, *act_d = nullptr;
    float *rew_h = nullptr, *rew_d = nullptr;
    uint8_t *done_h = nullptr, *done_d = nullptr;
    float *boot_h = nullptr, *boot_d = nullptr;
    int32_t *seg_h = nullptr, *seg_d = nullptr;          // first frame of every segment, and the frame count
};

}  // namespace

struct ga3c_sched {
    ga3c_ctx *ctx;
    ga3c_sched_config cfg;
    ga3c_net_desc desc;
    int max_pred, max_train;
    size_t frame_bytes;
    int predict_cap, train_cap;
    hipStream_t sp, st;
    std::deque<PredReq> pq;
    std::deque<Traj> tq;
    int64_t tq_frames;       // experiences waiting in tq
    PredSlot ps[RING];
    TrainSlot ts[RING];
    int ps_next, ts_next;
    std::deque<ga3c_prediction> ready;
    ga3c_tuner *tuner;
    ga3c_sched_stats stats;
    int64_t window_ticks, window_frames;
    std::chrono::steady_clock::time_point window_start;
};

namespace {

template <class T>
int pinned(T **p, size_t n) {
    SHIP(hipHostMalloc((void **)p, sizeof(T) * std::max<size_t>(n, 1), hipHostMallocDefault));
    return GA3C_OK;
}
template <class T>
int device(T **p, size_t n) {
    SHIP(hipMalloc((void **)p, sizeof(T) * std::max<size_t>(n, 1)));
    return GA3C_OK;
}
#define STRY(expr) do { int rc_ = (expr); if (rc_ != GA3C_OK) return rc_; } while (0)

int alloc_slots(ga3c_sched *s) {
    const int maxN = s->max_train;      // a segment has at least one frame
    for (int i = 0; i < RING; ++i) {
        PredSlot &p = s->ps[i];
        SHIP(hipEventCreateWithFlags(&p.done, hipEventDisableTiming));
        STRY(pinned(&p.ptrs_h, s->max_pred)); STRY(device(&p.ptrs_d, s->max_pred));
        STRY(pinned(&p.unif_h, s->max_pred)); STRY(device(&p.unif_d, s->max_pred));
        STRY(device(&p.frames_d, (size_t)s->max_pred * s->frame_bytes));
        STRY(device(&p.act_d, s->max_pred)); STRY(pinned(&p.act_h, s->max_pred));
        STRY(device(&p.val_d, s->max_pred)); STRY(pinned(&p.val_h, s->max_pred));
        TrainSlot &t = s->ts[i];
        SHIP(hipEventCreateWithFlags(&t.done, hipEventDisableTiming));
        STRY(pinned(&t.ptrs_h, maxN)); STRY(device(&t.ptrs_d, maxN));
        STRY(device(&t.frames_d, (size_t)s->max_train * s->frame_bytes));
        STRY(pinned(&t.act_h, s->max_train)); STRY(device(&t.act_d, s->max_train));
        STRY(pinned(&t.rew_h, s->max_train)); STRY(device(&t.rew_d, s->max_train));
        STRY(pinned(&t.done_h, s->max_train)); STRY(device(&t.done_d, s->max_train));
        STRY(pinned(&t.boot_h, maxN)); STRY(device(&t.boot_d, maxN));
        STRY(pinned(&t.seg_h, maxN + 1)); STRY(device(&t.seg_d, maxN + 1));
    }
    return GA3C_OK;
}

// Moves the results of finished prediction batches to the ready list.
int harvest(ga3c_sched *s, bool wait) {
    for (int k = 0; k < RING; ++k) {
        PredSlot &p = s->ps[(s->ps_next + k) % RING];        // oldest first
        if (!p.busy) continue;
        if (wait) SHIP(hipEventSynchronize(p.done));
        else {
            const hipError_t q = hipEventQuery(p.done);
            if (q == hipErrorNotReady) continue;
            if (q != hipSuccess) return sfail(GA3C_EHIP, "hipEventQuery: %s", hipGetErrorString(q));
        }
        for (int i = 0; i < p.n; ++i)
            s->ready.push_back(ga3c_prediction{p.agents[i], p.act_h[i], p.val_h[i], (int32_t)p.version});
        p.busy = false;
    }
    for (int k = 0; k < RING; ++k) {
        TrainSlot &t = s->ts[k];
        if (!t.busy) continue;
        if (wait) SHIP(hipEventSynchronize(t.done));
        else if (hipEventQuery(t.done) != hipSuccess) continue;
        t.busy = false;
    }
    return GA3C_OK;
}

int issue_predict(ga3c_sched *s, int *count) {
    *count = 0;
    if (s->pq.empty()) return GA3C_OK;
    if ((int)s->pq.size() < s->predict_cap) {
        // Fewer requests than a full batch: they go out at once only if no earlier batch is still in flight;
        // otherwise they wait for it, and what arrives meanwhile joins them.  (A single predictor of Sec. 4.1 behaves
        // like this: it is busy with its batch.  Full batches are issued back to back, up to RING of them, like
        // several predictors.)  Under light load this makes batches as large as the GPU's own pace allows.
        STRY(harvest(s, false));
        for (int k = 0; k < RING; ++k)
            if (s->ps[k].busy) return GA3C_OK;
    }
    PredSlot &p = s->ps[s->ps_next];
    if (p.busy) {                                   // ring full: wait for the oldest batch
        SHIP(hipEventSynchronize(p.done));
        STRY(harvest(s, false));
    }
    // the requests leave the queue only when the whole batch has been enqueued: a failing GPU call loses none
    const int n = (int)std::min<size_t>(s->pq.size(), (size_t)s->predict_cap);
    p.agents.resize(n);
    for (int i = 0; i < n; ++i) {
        const PredReq &r = s->pq[i];
        p.agents[i] = r.agent; p.ptrs_h[i] = (const uint4 *)r.frame; p.unif_h[i] = r.uniform;
    }
    SHIP(hipMemcpyAsync(p.ptrs_d, p.ptrs_h, sizeof(void *) * n, hipMemcpyHostToDevice, s->sp));
    SHIP(hipMemcpyAsync(p.unif_d, p.unif_h, sizeof(float) * n, hipMemcpyHostToDevice, s->sp));
    const int vecs = (int)(s->frame_bytes / 16);
    hipLaunchKernelGGL(gather_frames_kernel, dim3(std::min(8, (vecs + 255) / 256), n), dim3(256), 0, s->sp, p.ptrs_d,
                       (uint4 *)p.frames_d, vecs);
    SHIP(hipGetLastError());
    if (ga3c_predict(s->ctx, p.frames_d, n, p.unif_d, nullptr, p.val_d, nullptr, p.act_d, s->sp) != GA3C_OK)
        return sfail(GA3C_EHIP, "ga3c_predict: %s", ga3c_last_error());
    SHIP(hipMemcpyAsync(p.act_h, p.act_d, sizeof(int32_t) * n, hipMemcpyDeviceToHost, s->sp));
    SHIP(hipMemcpyAsync(p.val_h, p.val_d, sizeof(float) * n, hipMemcpyDeviceToHost, s->sp));
    SHIP(hipEventRecord(p.done, s->sp));
    s->pq.erase(s->pq.begin(), s->pq.begin() + n);
    p.busy = true; p.n = n;
    p.version = s->stats.train_batches;      // the call above reads the parameters that this many updates produced
    s->ps_next = (s->ps_next + 1) % RING;
    s->stats.predictions += n; s->stats.predict_batches += 1;
    *count = n;
    return GA3C_OK;
}

int issue_train(ga3c_sched *s, int *count) {
    *count = 0;
    const int T = s->cfg.t_max;
    // merge until the minimum batch is there (Sec. 5.3).  With the adjustment on, its training knob is the batch size
    // itself: an update waits for train_cap frames and takes at most as many, so the knob decides how large the
    // updates are whatever the pace at which segments arrive
    const int need = s->tuner ? std::max(s->cfg.train_min, s->train_cap) : s->cfg.train_min;
    if (s->tq.empty() || s->tq_frames < need) return GA3C_OK;
    TrainSlot &t = s->ts[s->ts_next];
    if (t.busy) {
        SHIP(hipEventSynchronize(t.done));
        t.busy = false;
    }
    // whole segments, oldest first, while they fit the cap (the first one always goes); they leave the queue, and
    // enter the statistics, only when the update has been enqueued: a failing GPU call loses none
    int n = 0, B = 0;
    bool equal = true;
    while ((size_t)n < s->tq.size() && (n == 0 || B + s->tq[n].len <= s->train_cap)) {
        const Traj &tr = s->tq[n];
        const int L = tr.len;
        for (int k = 0; k < L; ++k) t.ptrs_h[B + k] = (const uint4 *)(tr.frames + (size_t)k * s->frame_bytes);
        memcpy(t.act_h + B, tr.actions.data(), sizeof(int32_t) * L);
        memcpy(t.rew_h + B, tr.rewards.data(), sizeof(float) * L);
        memcpy(t.done_h + B, tr.dones.data(), L);
        t.boot_h[n] = tr.bootstrap;
        t.seg_h[n] = B;
        if (L != T) equal = false;
        B += L; n += 1;
    }
    t.seg_h[n] = B;
    SHIP(hipMemcpyAsync(t.ptrs_d, t.ptrs_h, sizeof(void *) * B, hipMemcpyHostToDevice, s->st));
    SHIP(hipMemcpyAsync(t.act_d, t.act_h, sizeof(int32_t) * B, hipMemcpyHostToDevice, s->st));
    SHIP(hipMemcpyAsync(t.rew_d, t.rew_h, sizeof(float) * B, hipMemcpyHostToDevice, s->st));
    SHIP(hipMemcpyAsync(t.done_d, t.done_h, B, hipMemcpyHostToDevice, s->st));
    SHIP(hipMemcpyAsync(t.boot_d, t.boot_h, sizeof(float) * n, hipMemcpyHostToDevice, s->st));
    if (!equal) SHIP(hipMemcpyAsync(t.seg_d, t.seg_h, sizeof(int32_t) * (n + 1), hipMemcpyHostToDevice, s->st));
    const int vecs = (int)(s->frame_bytes / 16);
    hipLaunchKernelGGL(gather_frames_kernel, dim3(std::min(8, (vecs + 255) / 256), B), dim3(256), 0, s->st, t.ptrs_d,
                       (uint4 *)t.frames_d, vecs);
    SHIP(hipGetLastError());
    const int rc = equal ? ga3c_train_step(s->ctx, t.frames_d, t.act_d, t.rew_d, t.done_d, t.boot_d, n, T, &s->cfg.hp,
                                           nullptr, s->st)
                         : ga3c_train_step_ragged(s->ctx, t.frames_d, t.act_d, t.rew_d, t.done_d, t.seg_d, t.boot_d, n, B,
                                                  &s->cfg.hp, nullptr, s->st);
    if (rc != GA3C_OK) return sfail(GA3C_EHIP, "ga3c_train_step: %s", ga3c_last_error());
    SHIP(hipEventRecord(t.done, s->st));
    const int64_t now = s->stats.train_batches;       // updates issued before this one = the version it starts from
    for (int i = 0; i < n; ++i) {
        const Traj &tr = s->tq[i];
        if (tr.len != T) s->stats.short_segments += 1;
        if (tr.version >= 0) {
            const int64_t lag = now - tr.version;
            s->stats.lag_sum += lag; s->stats.lag_count += 1;
            s->stats.lag_max = std::max(s->stats.lag_max, lag);
        }
        s->tq_frames -= tr.len;
    }
    s->tq.erase(s->tq.begin(), s->tq.begin() + n);
    t.busy = true; t.n_agents = n;
    s->ts_next = (s->ts_next + 1) % RING;
    s->stats.trained_frames += (int64_t)B; s->stats.train_batches += 1;
    *count = B;
    return GA3C_OK;
}

}  // namespace

extern "C" int ga3c_sched_create(ga3c_ctx *ctx, const ga3c_sched_config *cfg, ga3c_sched **out) {
    if (out) *out = nullptr;
    if (!ctx || !cfg || !out) return sfail(GA3C_EINVAL, "ga3c_sched_create: null argument");
    ga3c_net_desc d;
    int mp, mt;
    if (ga3c_get_desc(ctx, &d, &mp, &mt) != GA3C_OK) return sfail(GA3C_EINVAL, "ga3c_sched_create: bad context");
    const size_t fb = (size_t)d.in_c * d.in_h * d.in_w;
    if (fb % 16 != 0) return sfail(GA3C_EINVAL, "ga3c_sched_create: frame size must be a multiple of 16 bytes");
    if (cfg->t_max < 1 || cfg->predict_cap < 1 || cfg->predict_cap > mp || cfg->train_min < 1 ||
        cfg->train_cap < cfg->t_max || cfg->train_cap > mt || cfg->train_min > cfg->train_cap)
        return sfail(GA3C_EINVAL, "ga3c_sched_create: caps outside the context's capacity (predict %d, train %d)", mp, mt);
    if (cfg->adjust_period > 0 &&
        (cfg->predict_cap_lo < 1 || cfg->predict_cap_hi > mp || cfg->predict_cap_lo > cfg->predict_cap ||
         cfg->predict_cap_hi < cfg->predict_cap || cfg->train_cap_lo < cfg->train_min || cfg->train_cap_hi > mt ||
         cfg->train_cap_lo > cfg->train_cap || cfg->train_cap_hi < cfg->train_cap || cfg->train_cap_step < 1))
        return sfail(GA3C_EINVAL, "ga3c_sched_create: adjustment bounds must contain the initial caps and fit the context");
    ga3c_sched *s = new (std::nothrow) ga3c_sched();
    if (!s) return sfail(GA3C_ENOMEM, "ga3c_sched_create: out of memory");
    s->ctx = ctx; s->cfg = *cfg; s->desc = d; s->max_pred = mp; s->max_train = mt; s->frame_bytes = fb;
    s->predict_cap = cfg->predict_cap; s->train_cap = cfg->train_cap;
    s->sp = s->st = nullptr; s->ps_next = s->ts_next = 0; s->tuner = nullptr; s->tq_frames = 0;
    memset(&s->stats, 0, sizeof(s->stats));
    s->stats.predict_cap = s->predict_cap; s->stats.train_cap = s->train_cap;
    s->window_ticks = s->window_frames = 0;
    int rc = GA3C_OK;
    // default priority for both streams
    if (hipStreamCreateWithFlags(&s->sp, hipStreamNonBlocking) != hipSuccess ||
        hipStreamCreateWithFlags(&s->st, hipStreamNonBlocking) != hipSuccess)
        rc = sfail(GA3C_EHIP, "ga3c_sched_create: hipStreamCreate failed");
    if (rc == GA3C_OK) rc = alloc_slots(s);
    if (rc == GA3C_OK && cfg->adjust_period > 0)
        rc = ga3c_tuner_create(cfg->predict_cap_lo, cfg->predict_cap_hi, cfg->predict_cap, cfg->train_cap_lo,
                               cfg->train_cap_hi, cfg->train_cap_step, cfg->train_cap, cfg->seed, &s->tuner);
    if (rc == GA3C_OK && s->tuner && cfg->adjust_margin > 0.f) rc = ga3c_tuner_set_margin(s->tuner, cfg->adjust_margin);
    if (rc != GA3C_OK) {
        char keep[512];
        snprintf(keep, sizeof(keep), "%s", ga3c::sched_error_text());
        ga3c_sched_destroy(s);
        sfail(rc, "%s", keep);
        return rc;
    }
    s->window_start = std::chrono::steady_clock::now();
    *out = s;
    return GA3C_OK;
}

extern "C" int ga3c_sched_destroy(ga3c_sched *s) {
    if (!s) return GA3C_OK;
    if (s->sp) (void)hipStreamSynchronize(s->sp);
    if (s->st) (void)hipStreamSynchronize(s->st);
    for (int i = 0; i < RING; ++i) {
        PredSlot &p = s->ps[i];
        if (p.done) (void)hipEventDestroy(p.done);
        (void)hipHostFree(p.ptrs_h); (void)hipFree(p.ptrs_d); (void)hipHostFree(p.unif_h); (void)hipFree(p.unif_d);
        (void)hipFree(p.frames_d); (void)hipFree(p.act_d); (void)hipHostFree(p.act_h); (void)hipFree(p.val_d);
        (void)hipHostFree(p.val_h);
        TrainSlot &t = s->ts[i];
        if (t.done) (void)hipEventDestroy(t.done);
        (void)hipHostFree(t.ptrs_h); (void)hipFree(t.ptrs_d); (void)hipFree(t.frames_d);
        (void)hipHostFree(t.act_h); (void)hipFree(t.act_d); (void)hipHostFree(t.rew_h); (void)hipFree(t.rew_d);
        (void)hipHostFree(t.done_h); (void)hipFree(t.done_d); (void)hipHostFree(t.boot_h); (void)hipFree(t.boot_d);
        (void)hipHostFree(t.seg_h); (void)hipFree(t.seg_d);
    }
    if (s->sp) (void)hipStreamDestroy(s->sp);
    if (s->st) (void)hipStreamDestroy(s->st);
    ga3c_tuner_destroy(s->tuner);
    delete s;
    return GA3C_OK;
}

extern "C" int ga3c_sched_submit_predict(ga3c_sched *s, int agent, const uint8_t *frame_dev, float uniform) {
    if (!s || !frame_dev) return sfail(GA3C_EINVAL, "ga3c_sched_submit_predict: null argument");
    if (((uintptr_t)frame_dev) & 15) return sfail(GA3C_EINVAL, "ga3c_sched_submit_predict: frame must be 16-byte aligned");
    s->pq.push_back(PredReq{agent, frame_dev, uniform});
    return GA3C_OK;
}

extern "C" int ga3c_sched_submit_segment(ga3c_sched *s, int agent, const uint8_t *frames_dev, int len,
                                         const int32_t *actions, const float *rewards, const uint8_t *dones,
                                         float bootstrap, int64_t policy_version) {
    if (!s || !frames_dev || !actions || !rewards || !dones)
        return sfail(GA3C_EINVAL, "ga3c_sched_submit_segment: null argument");
    if (((uintptr_t)frames_dev) & 15)
        return sfail(GA3C_EINVAL, "ga3c_sched_submit_segment: frames must be 16-byte aligned");
    if (len < 1 || len > s->cfg.t_max)
        return sfail(GA3C_EINVAL, "ga3c_sched_submit_segment: length %d outside 1..t_max = %d", len, s->cfg.t_max);
    for (int i = 0; i < len; ++i)
        if (actions[i] < 0 || actions[i] >= s->desc.n_actions)
            return sfail(GA3C_EINVAL, "ga3c_sched_submit_segment: action %d out of range", (int)actions[i]);
    Traj tr;
    tr.agent = agent; tr.len = len; tr.version = policy_version < 0 ? -1 : policy_version;
    tr.frames = frames_dev; tr.bootstrap = bootstrap;
    tr.actions.assign(actions, actions + len);
    tr.rewards.assign(rewards, rewards + len);
    tr.dones.assign(dones, dones + len);
    s->tq.push_back(std::move(tr));
    s->tq_frames += len;
    return GA3C_OK;
}

extern "C" int ga3c_sched_submit_trajectory(ga3c_sched *s, int agent, const uint8_t *frames_dev, const int32_t *actions,
                                            const float *rewards, const uint8_t *dones, float bootstrap) {
    if (!s) return sfail(GA3C_EINVAL, "ga3c_sched_submit_trajectory: null scheduler");
    return ga3c_sched_submit_segment(s, agent, frames_dev, s->cfg.t_max, actions, rewards, dones, bootstrap, -1);
}

extern "C" int ga3c_sched_submit_predict_many(ga3c_sched *s, int n, const int32_t *agents,
                                              const uint8_t *const *frames_dev, const float *uniforms) {
    if (!s || n < 0 || (n > 0 && (!agents || !frames_dev || !uniforms)))
        return sfail(GA3C_EINVAL, "ga3c_sched_submit_predict_many: bad argument");
    for (int i = 0; i < n; ++i)
        if (!frames_dev[i] || (((uintptr_t)frames_dev[i]) & 15))
            return sfail(GA3C_EINVAL, "ga3c_sched_submit_predict_many: frame %d is null or not 16-byte aligned", i);
    for (int i = 0; i < n; ++i) s->pq.push_back(PredReq{agents[i], frames_dev[i], uniforms[i]});
    return GA3C_OK;
}

extern "C" int ga3c_sched_submit_trajectory_many(ga3c_sched *s, int n, const int32_t *agents,
                                                 const uint8_t *const *frames_dev, const int32_t *actions,
                                                 const float *rewards, const uint8_t *dones, const float *bootstrap) {
    if (!s || n < 0 || (n > 0 && (!agents || !frames_dev || !actions || !rewards || !dones || !bootstrap)))
        return sfail(GA3C_EINVAL, "ga3c_sched_submit_trajectory_many: bad argument");
    const int T = s->cfg.t_max;
    for (int i = 0; i < n; ++i) {
        const int rc = ga3c_sched_submit_trajectory(s, agents[i], frames_dev[i], actions + (size_t)i * T,
                                                    rewards + (size_t)i * T, dones + (size_t)i * T, bootstrap[i]);
        if (rc != GA3C_OK) return rc;
    }
    return GA3C_OK;
}

extern "C" int ga3c_sched_submit_segment_many(ga3c_sched *s, int n, const int32_t *agents,
                                              const uint8_t *const *frames_dev, const int32_t *lens,
                                              const int32_t *actions, const float *rewards, const uint8_t *dones,
                                              const float *bootstrap, const int64_t *policy_versions) {
    if (!s || n < 0 || (n > 0 && (!agents || !frames_dev || !lens || !actions || !rewards || !dones || !bootstrap)))
        return sfail(GA3C_EINVAL, "ga3c_sched_submit_segment_many: bad argument");
    const int T = s->cfg.t_max;
    for (int i = 0; i < n; ++i) {
        const int rc = ga3c_sched_submit_segment(s, agents[i], frames_dev[i], lens[i], actions + (size_t)i * T,
                                                 rewards + (size_t)i * T, dones + (size_t)i * T, bootstrap[i],
                                                 policy_versions ? policy_versions[i] : -1);
        if (rc != GA3C_OK) return rc;
    }
    return GA3C_OK;
}

extern "C" int ga3c_sched_tick(ga3c_sched *s, int *predicted, int *trained) {
    if (!s) return sfail(GA3C_EINVAL, "ga3c_sched_tick: null scheduler");
    int np = 0, nt = 0;
    s->stats.ticks += 1;
    s->stats.sum_predict_queue += (int64_t)s->pq.size();
    s->stats.sum_train_queue += (int64_t)s->tq.size();
    STRY(issue_predict(s, &np));
    STRY(issue_train(s, &nt));
    STRY(harvest(s, false));
    if (predicted) *predicted = np;
    if (trained) *trained = nt;
    if (s->tuner) {
        s->window_ticks += 1; s->window_frames += nt;
        if (s->window_ticks >= s->cfg.adjust_period) {
            // throughput of the window that just ended: finish its GPU work, then read the clock
            SHIP(hipStreamSynchronize(s->st));
            SHIP(hipStreamSynchronize(s->sp));
            const auto now = std::chrono::steady_clock::now();
            const double sec = std::chrono::duration<double>(now - s->window_start).count();
            const double thr = sec > 0 ? (double)s->window_frames / sec : 0.0;
            ga3c_tuner_report(s->tuner, thr, &s->predict_cap, &s->train_cap);
            s->stats.last_window_frames_per_s = thr;
            s->stats.predict_cap = s->predict_cap; s->stats.train_cap = s->train_cap;
            ga3c_tuner_state(s->tuner, nullptr, nullptr, &s->stats.trials_accepted, &s->stats.trials_rejected);
            ga3c_tuner_progress(s->tuner, &s->stats.windows, &s->stats.last_change_window);
            s->window_ticks = s->window_frames = 0;
            s->window_start = std::chrono::steady_clock::now();
        }
    }
    return GA3C_OK;
}

extern "C" int ga3c_sched_poll(ga3c_sched *s, ga3c_prediction *out, int cap) {
    if (!s || (!out && cap > 0) || cap < 0) return sfail(GA3C_EINVAL, "ga3c_sched_poll: bad argument");
    STRY(harvest(s, false));
    int n = 0;
    while (n < cap && !s->ready.empty()) {
        out[n++] = s->ready.front();
        s->ready.pop_front();
    }
    return n;
}

extern "C" int ga3c_sched_drain(ga3c_sched *s) {
    if (!s) return sfail(GA3C_EINVAL, "ga3c_sched_drain: null scheduler");
    SHIP(hipStreamSynchronize(s->sp));
    SHIP(hipStreamSynchronize(s->st));
    return harvest(s, true);
}

extern "C" int ga3c_sched_get_stats(const ga3c_sched *s, ga3c_sched_stats *out) {
    if (!s || !out) return sfail(GA3C_EINVAL, "ga3c_sched_get_stats: null argument");
    *out = s->stats;
    out->predict_queue = (int64_t)s->pq.size();
    out->train_queue = (int64_t)s->tq.size();
    return GA3C_OK;
}

