// Drives the scheduler (csrc/sched.hip) and, through it, the two GPU calls, with the HOST side of the whole library
// built with -fsanitize=address,undefined (device code is not instrumented).  Built by
// paper_1611_06256_amd/build.py (build_sched_sanitized) into paper_1611_06256_amd/sched_sanitized and run on a GPU by
// tests/test_gpu_sched.py: any out-of-bounds access, use after free, signed overflow or misaligned access in the
// scheduler's queues, slot rings and staging buffers turns into a non-zero exit status.
//
// Synthetic closed loop: N agents ask for actions and hand in segments (some shorter than t_max, Sec. 4.1) with the
// policy version they were given (Sec. 4.2); the batch caps are adjusted every few ticks (Sec. 4.3); a second phase
// uses fixed caps and the many-at-once submit calls; error paths are exercised too.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "../include/ga3c.h"

#define HIPCK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("hip error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)

static uint64_t lcg(uint64_t &s) { s = s * 6364136223846793005ull + 1442695040888963407ull; return s >> 11; }
static float unif(uint64_t &s) { return (float)(lcg(s) & 0xFFFFFF) / 16777216.0f; }

int main() {
    int ndev = 0;
    HIPCK(hipGetDeviceCount(&ndev));
    if (ndev < 1) { printf("no GPU\n"); return 2; }
    HIPCK(hipSetDevice(0));
    int bad = 0;
    const int N = 24, T = 5, A = 6;
    const size_t fb = 4 * 84 * 84;
    ga3c_net_desc d;
    memset(&d, 0, sizeof(d));
    d.in_c = 4; d.in_h = 84; d.in_w = 84; d.n_conv = 2;
    d.conv[0].oc = 16; d.conv[0].k = 8; d.conv[0].stride = 4;
    d.conv[1].oc = 32; d.conv[1].k = 4; d.conv[1].stride = 2;
    d.fc_units = 256; d.n_actions = A; d.math = 0;
    ga3c_ctx *ctx = nullptr;
    if (ga3c_create(&d, 64, 160, &ctx) != GA3C_OK || !ctx) { printf("create: %s\n", ga3c_last_error()); return 1; }
    if (ga3c_params_init(ctx, 7, nullptr) != GA3C_OK) ++bad;

    // frames of all agents: N x T frames of pseudo-random bytes, in device memory
    std::vector<uint8_t> host((size_t)N * T * fb);
    uint64_t rs = 2024;
    for (size_t i = 0; i < host.size(); i += 8) {
        const uint64_t v = lcg(rs) * 0x9E3779B97F4A7C15ull;
        memcpy(&host[i], &v, 8);
    }
    uint8_t *frames = nullptr;
    HIPCK(hipMalloc(&frames, host.size()));
    HIPCK(hipMemcpy(frames, host.data(), host.size(), hipMemcpyHostToDevice));

    ga3c_sched_config cfg;
    memset(&cfg, 0, sizeof(cfg));
    cfg.t_max = T; cfg.predict_cap = 8; cfg.train_min = 10; cfg.train_cap = 40;
    cfg.adjust_period = 5; cfg.predict_cap_lo = 2; cfg.predict_cap_hi = 64;
    cfg.train_cap_lo = 10; cfg.train_cap_hi = 160; cfg.train_cap_step = 10; cfg.seed = 3;
    cfg.hp.gamma = 0.99f; cfg.hp.beta = 0.01f; cfg.hp.value_coef = 1.f; cfg.hp.log_eps = 0.f;
    cfg.hp.lr = 1e-4f; cfg.hp.rms_decay = 0.99f; cfg.hp.rms_eps = 0.1f; cfg.hp.clip_norm = 40.f;
    cfg.adjust_margin = 0.05f;

    // bad configurations are refused and leave nothing behind
    {
        ga3c_sched *s = nullptr;
        ga3c_sched_config b = cfg;
        b.predict_cap = 65;
        if (ga3c_sched_create(ctx, &b, &s) == GA3C_OK || s) ++bad;
        b = cfg; b.train_cap_hi = 161;
        if (ga3c_sched_create(ctx, &b, &s) == GA3C_OK || s) ++bad;
        if (ga3c_sched_create(nullptr, &cfg, &s) == GA3C_OK || s) ++bad;
        if (!ga3c_sched_last_error()[0]) ++bad;
    }

    for (int phase = 0; phase < 2; ++phase) {
        ga3c_sched *s = nullptr;
        ga3c_sched_config c = cfg;
        if (phase == 1) { c.adjust_period = 0; c.predict_cap = 16; c.train_min = 20; c.train_cap = 60; }
        if (ga3c_sched_create(ctx, &c, &s) != GA3C_OK || !s) { printf("sched_create: %s\n", ga3c_sched_last_error()); return 1; }
        std::vector<int> step(N, 0), seglen(N, 0);
        std::vector<int64_t> segver(N, -1);
        std::vector<char> waiting(N, 0);
        std::vector<int32_t> acts((size_t)N * T, 0);
        std::vector<ga3c_prediction> out(64);
        int64_t asked = 0, answered = 0, handed = 0;
        for (int it = 0; it < 400; ++it) {
            if (phase == 0) {
                for (int a = 0; a < N; ++a)
                    if (!waiting[a] && (lcg(rs) & 3) != 0) {        // three in four ready agents ask now
                        if (ga3c_sched_submit_predict(s, a, frames + ((size_t)a * T + step[a] % T) * fb, unif(rs)) != GA3C_OK) ++bad;
                        waiting[a] = 1; ++asked;
                    }
            } else {
                std::vector<int32_t> ag; std::vector<const uint8_t *> fp; std::vector<float> un;
                for (int a = 0; a < N; ++a)
                    if (!waiting[a]) { ag.push_back(a); fp.push_back(frames + ((size_t)a * T + step[a] % T) * fb); un.push_back(unif(rs)); waiting[a] = 1; }
                if (!ag.empty()) {
                    if (ga3c_sched_submit_predict_many(s, (int)ag.size(), ag.data(), fp.data(), un.data()) != GA3C_OK) ++bad;
                    asked += (int64_t)ag.size();
                }
            }
            int np = 0, nt = 0;
            if (ga3c_sched_tick(s, &np, &nt) != GA3C_OK) { printf("tick: %s\n", ga3c_sched_last_error()); ++bad; break; }
            if (np < 0 || np > 64 || nt < 0 || nt > 160) ++bad;
            if (phase == 1 && ga3c_sched_drain(s) != GA3C_OK) ++bad;      // lockstep rounds: every tick's work finishes before the poll
            const int got = ga3c_sched_poll(s, out.data(), (int)out.size());
            if (got < 0) { ++bad; break; }
            for (int i = 0; i < got; ++i) {
                const int a = out[i].agent;
                if (a < 0 || a >= N || !waiting[a] || out[i].action < 0 || out[i].action >= A) { ++bad; continue; }
                if (seglen[a] == 0) segver[a] = out[i].policy_version;
                acts[(size_t)a * T + seglen[a]] = out[i].action;
                ++seglen[a]; ++step[a]; waiting[a] = 0; ++answered;
                const bool ended = (lcg(rs) % 10) == 0;              // the episode ends: a short segment goes in at once
                if (seglen[a] == T || ended) {
                    float rew[5]; uint8_t done[5];
                    for (int k = 0; k < T; ++k) { rew[k] = (float)((int)(lcg(rs) % 3) - 1); done[k] = 0; }
                    if (ended) done[seglen[a] - 1] = 1;
                    const int rc = (seglen[a] == T && phase == 1 && !ended)
                                       ? ga3c_sched_submit_trajectory(s, a, frames + (size_t)a * T * fb, &acts[(size_t)a * T], rew, done, out[i].value)
                                       : ga3c_sched_submit_segment(s, a, frames + (size_t)a * T * fb, seglen[a], &acts[(size_t)a * T], rew, done,
                                                                   out[i].value, segver[a]);
                    if (rc != GA3C_OK) ++bad;
                    handed += seglen[a];
                    seglen[a] = 0;
                }
            }
        }
        // what is still queued goes out, then everything finishes
        for (int k = 0; k < 64; ++k) {
            ga3c_sched_stats st;
            if (ga3c_sched_get_stats(s, &st) != GA3C_OK) { ++bad; break; }
            if (st.predict_queue == 0) break;
            int np = 0, nt = 0;
            if (ga3c_sched_tick(s, &np, &nt) != GA3C_OK) { ++bad; break; }
            if (ga3c_sched_drain(s) != GA3C_OK) { ++bad; break; }
        }
        if (ga3c_sched_drain(s) != GA3C_OK) ++bad;
        int got;
        while ((got = ga3c_sched_poll(s, out.data(), (int)out.size())) > 0) answered += got;
        if (got < 0) ++bad;
        ga3c_sched_stats st;
        if (ga3c_sched_get_stats(s, &st) != GA3C_OK) ++bad;
        if (st.predictions != asked || answered != asked || st.predict_queue != 0) { printf("phase %d: asked %lld answered %lld issued %lld\n", phase, (long long)asked, (long long)answered, (long long)st.predictions); ++bad; }
        if (st.trained_frames > handed || st.trained_frames <= 0 || st.train_batches <= 0) ++bad;
        if (phase == 0 && (st.windows < 50 || st.predict_cap < 2 || st.predict_cap > 64 || st.train_cap < 10 || st.train_cap > 160)) ++bad;
        if (st.lag_count <= 0 || st.lag_max < 0 || st.short_segments <= 0) ++bad;
        // errors after creation: a segment longer than t_max, an action out of range
        {
            float rew[6] = {0}; uint8_t done[6] = {0}; int32_t ac[6] = {0, 0, 0, 0, 0, 0};
            if (ga3c_sched_submit_segment(s, 0, frames, 6, ac, rew, done, 0.f, -1) == GA3C_OK) ++bad;
            ac[0] = A;
            if (ga3c_sched_submit_segment(s, 0, frames, 5, ac, rew, done, 0.f, -1) == GA3C_OK) ++bad;
        }
        if (ga3c_sched_destroy(s) != GA3C_OK) ++bad;
        printf("phase %d: %lld predictions, %lld trained frames in %lld updates, %lld windows, caps %d / %d\n", phase,
               (long long)st.predictions, (long long)st.trained_frames, (long long)st.train_batches, (long long)st.windows,
               st.predict_cap, st.train_cap);
    }
    HIPCK(hipFree(frames));
    if (ga3c_destroy(ctx) != GA3C_OK) ++bad;
    printf("%d problems\n", bad);
    return bad ? 1 : 0;
}
