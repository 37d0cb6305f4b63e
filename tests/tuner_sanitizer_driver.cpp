// Drives the adjustment rule (csrc/tuner.cpp, host code only) through its whole interface on synthetic throughput
// models; built by tests/test_tuner_cpu.py with -fsanitize=address,undefined, which turn any out-of-bounds access,
// use after free, leak, signed overflow or misaligned access into a non-zero exit status.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>

#include "../include/ga3c.h"

static uint64_t lcg(uint64_t &s) { s = s * 6364136223846793005ull + 1442695040888963407ull; return s >> 11; }
static double gauss(uint64_t &s) {     // sum of 12 uniforms - 6
    double a = 0.0;
    for (int i = 0; i < 12; ++i) a += (double)(lcg(s) & 0xFFFFFF) / 16777216.0;
    return a - 6.0;
}
static double model(int p, int t, int ps, int ts) {
    const double lp = std::log2((double)p) - std::log2((double)ps);
    return 1e6 - 4e4 * lp * lp - 0.5 * (double)(t - ts) * (double)(t - ts);
}

int main() {
    int bad = 0;
    for (uint64_t seed = 0; seed < 16; ++seed) {
        ga3c_tuner *t = nullptr;
        const int p0 = 1 << (seed % 9), t0 = 40 + 40 * (int)(seed * 7 % 32);
        if (ga3c_tuner_create(1, 256, p0, 40, 1280, 40, t0, seed, &t) != GA3C_OK || !t) { ++bad; continue; }
        if (ga3c_tuner_set_margin(t, 0.03) != GA3C_OK) ++bad;
        if (ga3c_tuner_set_margin(t, 2.0) == GA3C_OK) ++bad;
        uint64_t rs = 99 + seed;
        int p = p0, c = t0;
        for (int w = 0; w < 500; ++w) {
            const double thr = model(p, c, 64, 640) * (1.0 + 0.01 * gauss(rs));
            if (ga3c_tuner_report(t, thr, &p, &c) != GA3C_OK) ++bad;
            if (p < 1 || p > 256 || (p & (p - 1)) || c < 40 || c > 1280 || c % 40) { ++bad; break; }
        }
        int kp = 0, kt = 0;
        int64_t acc = 0, rej = 0, win = 0, last = 0;
        if (ga3c_tuner_state(t, &kp, &kt, &acc, &rej) != GA3C_OK) ++bad;
        if (ga3c_tuner_progress(t, &win, &last) != GA3C_OK || win != 500 || last < 0 || last > win) ++bad;
        if (model(kp, kt, 64, 640) < 0.9e6) ++bad;
        if (ga3c_tuner_report(t, 1.0, nullptr, nullptr) != GA3C_OK) ++bad;      // optional outputs
        ga3c_tuner_destroy(t);
    }
    // degenerate ranges: a single value per knob, and refusals
    ga3c_tuner *t = nullptr;
    if (ga3c_tuner_create(8, 8, 8, 80, 80, 40, 80, 1, &t) != GA3C_OK) ++bad;
    for (int w = 0; w < 20; ++w) {
        int p = 0, c = 0;
        if (ga3c_tuner_report(t, 5.0 + w, &p, &c) != GA3C_OK || p != 8 || c != 80) ++bad;
    }
    ga3c_tuner_destroy(t);
    if (ga3c_tuner_create(4, 2, 3, 40, 80, 40, 40, 0, &t) == GA3C_OK) ++bad;
    if (ga3c_tuner_create(1, 2, 1, 40, 80, 40, 40, 0, nullptr) == GA3C_OK) ++bad;
    if (ga3c_tuner_report(nullptr, 1.0, nullptr, nullptr) == GA3C_OK) ++bad;
    if (std::strlen(ga3c_sched_last_error()) == 0) ++bad;
    ga3c_tuner_destroy(nullptr);
    std::printf("tuner sanitizer driver: %d problems\n", bad);
    return bad ? 1 : 0;
}
