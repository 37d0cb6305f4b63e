// The dynamic adjustment of the batching knobs (paper Sec. 4.3) as a pure host object: no HIP in this file, so it
// also builds for the CPU alone (the tests build it with the address and undefined-behaviour sanitizers).
#include <algorithm>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <new>

#include "../../include/ga3c.h"
#include "sched_error.hpp"

namespace ga3c {
static thread_local char s_err[512] = "";
int sfail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(s_err, sizeof(s_err), fmt, ap);
    va_end(ap);
    return code;
}
const char *sched_error_text() { return s_err; }
}  // namespace ga3c
using ga3c::sfail;

extern "C" const char *ga3c_sched_last_error(void) { return ga3c::sched_error_text(); }

namespace {
uint64_t splitmix(uint64_t &x) {
    x += 0x9E3779B97F4A7C15ull;
    uint64_t z = x;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
}  // namespace

// Sec. 4.3: every period one knob is changed by one step; the change is kept if the throughput did not drop,
// otherwise undone.  Knobs here are the two batch caps: the prediction cap moves on the ladder lo, 2 lo, 4 lo, ...
// (one step = a factor 2), the training cap by a factor 1 + 2^-k up or down (k = 0 at first, i.e. a factor 2 as
// well; one finer after a rejected step of that knob, down to 1/64; one coarser again after a step that brought a
// clear gain; values
// are multiples of t_step and a step is at least t_step), so that both knobs cross their range in a handful of steps
// and still settle finely.
// What the paper leaves open, and what this does:
//  * "did not drop" is judged against a relative margin (window-to-window noise of a few per cent would otherwise
//    reject every neutral step): a trial is kept iff its throughput >= (1 - margin) * reference;
//  * the reference is the throughput of the kept configuration: measured when it was accepted, never lowered by a
//    neutral step, and measured again in the window after every rejected trial (a higher reading replaces it, a
//    lower one is averaged in), so that one lucky reading cannot lock the tuner in; the starting configuration is
//    measured twice, because the first window also pays for the start of the run;
//  * the search cools down ("annealing"): after the k-th rejected trial in a row without a clear gain in between the
//    kept configuration runs for 1, 2, 4, then 8 windows before the next trial, so that a settled system spends one
//    window in nine on a trial that is likely to cost throughput; the first clear gain brings the pace back;
//  * after a step that raised the throughput by more than half the margin the same knob is stepped in the same
//    direction again; otherwise knob and direction are drawn at random (seeded), except that a knob is not drawn a
//    third time in a row and the step that was rejected last is not repeated at once.
struct ga3c_tuner {
    int p_lo, p_hi, t_lo, t_hi, t_step;
    int p, t;              // configuration now running
    int kept_p, kept_t;    // last accepted configuration
    double kept_thr;       // its throughput (the reference)
    double margin;
    bool have_ref, trial, persist;
    int rest;              // windows the kept configuration still runs before the next trial
    int rej_run;           // rejected trials since the last clear gain
    bool last_knob_p, last_up;
    bool have_rej[2], rej_up[2];           // per knob (0 training, 1 prediction): the direction rejected last from the
                                           // kept value (not tried again until that knob's kept value has moved)
    int knob_run;          // trials in a row on the knob of the last trial
    int t_shift;           // the training cap moves by the factor 1 + 2^-t_shift: 0 at first, finer after a rejected step
                           // of that knob (up to 6), coarser again after a clear gain
    uint64_t rng;
    int64_t accepted, rejected, windows, last_change;
};

extern "C" int ga3c_tuner_create(int p_lo, int p_hi, int p0, int t_lo, int t_hi, int t_step, int t0, uint64_t seed,
                                 ga3c_tuner **out) {
    if (out) *out = nullptr;
    if (!out || p_lo < 1 || p_hi < p_lo || p0 < p_lo || p0 > p_hi || t_lo < 1 || t_hi < t_lo || t0 < t_lo || t0 > t_hi ||
        t_step < 1)
        return sfail(GA3C_EINVAL, "ga3c_tuner_create: bad bounds");
    ga3c_tuner *t = new (std::nothrow) ga3c_tuner();
    if (!t) return sfail(GA3C_ENOMEM, "ga3c_tuner_create: out of memory");
    t->p_lo = p_lo; t->p_hi = p_hi; t->t_lo = t_lo; t->t_hi = t_hi; t->t_step = t_step;
    t->p = t->kept_p = p0; t->t = t->kept_t = t0;
    t->kept_thr = 0.0; t->margin = 0.03;
    t->have_ref = false; t->trial = false; t->persist = false; t->rest = 0; t->rej_run = 0;
    t->last_knob_p = false; t->last_up = false; t->t_shift = 0;
    t->have_rej[0] = t->have_rej[1] = false; t->rej_up[0] = t->rej_up[1] = false; t->knob_run = 0;
    t->rng = seed; t->accepted = t->rejected = 0; t->windows = 0; t->last_change = 0;
    *out = t;
    return GA3C_OK;
}

extern "C" int ga3c_tuner_destroy(ga3c_tuner *t) {
    delete t;
    return GA3C_OK;
}

extern "C" int ga3c_tuner_set_margin(ga3c_tuner *t, double margin) {
    if (!t || !(margin >= 0.0) || margin >= 1.0) return sfail(GA3C_EINVAL, "ga3c_tuner_set_margin: margin must be in [0, 1)");
    t->margin = margin;
    return GA3C_OK;
}

namespace {
// One step of a knob from the kept configuration; false if it would leave the bounds or change nothing.
bool tuner_move(const ga3c_tuner *t, bool knob_p, bool up, int &np, int &nt) {
    np = t->kept_p; nt = t->kept_t;
    if (knob_p) {
        const int c = up ? t->kept_p * 2 : t->kept_p / 2;
        if (c < t->p_lo || c > t->p_hi || c == t->kept_p) return false;
        np = c;
    } else {
        // a factor 1 + 2^-t_shift up or down, rounded to the ladder of t_step, at least one rung
        const double f = 1.0 + 1.0 / (double)(1 << t->t_shift);
        const double want = up ? t->kept_t * f : t->kept_t / f;
        int c = (int)(want / t->t_step + 0.5) * t->t_step;
        if (up) c = std::max(c, t->kept_t + t->t_step); else c = std::min(c, t->kept_t - t->t_step);
        c = std::min(std::max(c, t->t_lo), t->t_hi);      // the last step to a bound may be shorter
        if (c == t->kept_t) return false;
        nt = c;
    }
    return true;
}
}  // namespace

// End of a measurement window that ran the current configuration with the
// given throughput.  Decides about the trial (if one was running), then
// proposes the next configuration and returns it.
extern "C" int ga3c_tuner_report(ga3c_tuner *t, double throughput, int *predict_cap, int *train_cap) {
    if (!t) return sfail(GA3C_EINVAL, "ga3c_tuner_report: null tuner");
    t->windows += 1;
    if (!t->have_ref) {
        // the first window also pays for whatever starts up with the run: it gives a provisional reference, and the
        // starting configuration runs once more before the first trial
        t->kept_thr = throughput; t->have_ref = true;
        t->rest = 1;
    } else if (t->trial) {
        if (throughput >= (1.0 - t->margin) * t->kept_thr) {
            t->accepted += 1;
            t->kept_p = t->p; t->kept_t = t->t;
            // a clear gain: step the same knob the same way again; a neutral step is kept but earns no repeat
            t->persist = throughput > (1.0 + 0.5 * t->margin) * t->kept_thr;
            t->kept_thr = std::max(t->kept_thr, throughput);
            t->last_change = t->windows;
            t->have_rej[t->last_knob_p ? 1 : 0] = false;
            if (!t->last_knob_p && t->persist) t->t_shift = std::max(0, t->t_shift - 1);
            if (t->persist) t->rej_run = 0;
        } else {
            t->rejected += 1;                    // undo, and look at the kept configuration again before the next trial
            t->persist = false;
            t->rest = 1 << std::min(t->rej_run, 3);           // 1, 2, 4, 8, 8, ... windows
            t->rej_run += 1;
            // both directions rejected: start over (conditions may have changed since the first of the two)
            const int kn = t->last_knob_p ? 1 : 0;
            if (t->have_rej[kn] && t->rej_up[kn] != t->last_up) t->have_rej[kn] = false;
            else { t->have_rej[kn] = true; t->rej_up[kn] = t->last_up; }
            if (!t->last_knob_p) t->t_shift = std::min(6, t->t_shift + 1);
        }
    } else {
        // the kept configuration again: a higher reading replaces the reference, a lower one is averaged in (readings
        // err on the low side: stalls, start-up; and a reference that was a lucky high decays this way)
        t->kept_thr = throughput >= t->kept_thr ? throughput : 0.5 * (t->kept_thr + throughput);
    }
    int np = t->kept_p, nt = t->kept_t;
    bool moved = false;
    if (t->rest > 0) {
        t->rest -= 1;
    } else {
        if (t->persist) moved = tuner_move(t, t->last_knob_p, t->last_up, np, nt);
        t->persist = false;
        if (!moved) {
            // one knob, one step, random direction, except: the same knob is not drawn a third time in a row, the step
            // that was rejected last is not repeated at once, and a step that would leave the bounds goes the other way
            const uint64_t r = splitmix(t->rng);
            bool knob_p = (r & 1) == 0, up = (r & 2) != 0;
            if (t->knob_run >= 2 && knob_p == t->last_knob_p) knob_p = !knob_p;
            for (int k = 0; k < 2 && !moved; ++k, knob_p = !knob_p) {
                bool u = k == 0 ? up : (r & 4) != 0;
                if (t->have_rej[knob_p ? 1 : 0] && u == t->rej_up[knob_p ? 1 : 0]) u = !u;
                moved = tuner_move(t, knob_p, u, np, nt);
                if (!moved) { u = !u; moved = tuner_move(t, knob_p, u, np, nt); }
                if (moved) {
                    t->knob_run = knob_p == t->last_knob_p ? t->knob_run + 1 : 1;
                    t->last_knob_p = knob_p; t->last_up = u;
                    break;
                }
            }
        }
    }
    t->p = np; t->t = nt;
    t->trial = moved;
    if (predict_cap) *predict_cap = t->p;
    if (train_cap) *train_cap = t->t;
    return GA3C_OK;
}

// Windows reported so far, and the window in which the kept configuration last changed (0: never).
extern "C" int ga3c_tuner_progress(const ga3c_tuner *t, int64_t *windows, int64_t *last_change_window) {
    if (!t) return sfail(GA3C_EINVAL, "ga3c_tuner_progress: null tuner");
    if (windows) *windows = t->windows;
    if (last_change_window) *last_change_window = t->last_change;
    return GA3C_OK;
}

extern "C" int ga3c_tuner_state(const ga3c_tuner *t, int *kept_predict_cap, int *kept_train_cap, int64_t *accepted,
                                int64_t *rejected) {
    if (!t) return sfail(GA3C_EINVAL, "ga3c_tuner_state: null tuner");
    if (kept_predict_cap) *kept_predict_cap = t->kept_p;
    if (kept_train_cap) *kept_train_cap = t->kept_t;
    if (accepted) *accepted = t->accepted;
    if (rejected) *rejected = t->rejected;
    return GA3C_OK;
}

