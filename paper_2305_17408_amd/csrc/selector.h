// The adaptive selector's state machine (paper Sec. 3.3, "Adaptive Selector"): host logic only,
// no HIP calls, so that it can be driven with made-up timings in a CPU test.
//
// Feedback-driven kernel selection for one direction: during the first calls every candidate runs
// one warm-up and `trials` timed repetitions, with events around each subgraph kernel; afterwards
// the candidate with the smallest median per subgraph class is kept (ties: lowest id).  A second
// round compares the ways of composing the pieces by their total time.  A candidate whose FIRST
// TIMED repetition (never the cold warm-up run) is more than four times the best median so far
// is abandoned: that warm sample stays its only one and its remaining repetitions are skipped.
#pragma once
#include <algorithm>

#include "adaptgear.h"

namespace ag {

constexpr int kMaxTrials = 15;      // timed repetitions per candidate (upper limit of the option)

struct Selector {
    int forced[AG_NUM_CLS];
    int choice[AG_NUM_CLS];
    int ncand[AG_NUM_CLS];
    int phase = 0;          // 0: per-class trials, 1: composition trials, 2: frozen
    int cand = 0, rep = 0, calls = 0;
    float samples[AG_NUM_CLS][4][kMaxTrials];
    int nsamples[AG_NUM_CLS][4];
    float median_ms[AG_NUM_CLS][4];
    float best_ms[AG_NUM_CLS];      // smallest median among the finished candidates of a class
    float total_trial_ms = 0.f;

    void reset(bool keep_forced)
    {
        for (int c = 0; c < AG_NUM_CLS; ++c) {
            if (!keep_forced) forced[c] = -1;
            choice[c] = 0;
            best_ms[c] = -1.f;
            for (int k = 0; k < 4; ++k) { nsamples[c][k] = 0; median_ms[c][k] = -1.f; }
        }
        phase = 0; cand = 0; rep = 0; total_trial_ms = 0.f;
    }
};

inline float selector_median(const Selector &s, int c, int k)
{
    const int n = s.nsamples[c][k];
    if (n == 0) return -1.f;                            // not measured
    float v[kMaxTrials];
    std::copy(s.samples[c][k], s.samples[c][k] + n, v);
    std::sort(v, v + n);
    return v[n / 2];
}

inline int selector_fastest(Selector &s, int c)
{
    int best = -1;
    for (int k = 0; k < s.ncand[c]; ++k) {
        s.median_ms[c][k] = selector_median(s, c, k);
        if (s.median_ms[c][k] >= 0 && (best < 0 || s.median_ms[c][k] < s.median_ms[c][best])) best = k;
    }
    return best < 0 ? 0 : best;                         // ties and "nothing measured" -> lowest id
}

// Decide what this call runs (k[class] = kernel id); returns true when the call is a trial, whose
// four intervals must then be reported with selector_record.
inline bool selector_next(Selector &s, int *k)
{
    for (;;) {
        if (s.phase == 0) {
            int maxc = 1;
            bool any_free = false;
            for (int c = 0; c < AG_CLS_COMPOSE; ++c)
                if (s.forced[c] < 0 && s.ncand[c] > 1) { maxc = std::max(maxc, s.ncand[c]); any_free = true; }
            if (!any_free || s.cand >= maxc) {
                for (int c = 0; c < AG_CLS_COMPOSE; ++c)
                    s.choice[c] = s.forced[c] >= 0 ? s.forced[c] : selector_fastest(s, c);
                s.phase = 1; s.cand = 0; s.rep = 0;
                continue;
            }
            for (int c = 0; c < AG_CLS_COMPOSE; ++c)
                k[c] = s.forced[c] >= 0 ? s.forced[c] : std::min(s.cand, s.ncand[c] - 1);
            k[AG_CLS_COMPOSE] = AG_COMPOSE_SPLIT;        // without blocks this is the remainder kernel alone
            return true;
        }
        if (s.phase == 1) {
            const int c = AG_CLS_COMPOSE;
            if (s.forced[c] >= 0 || s.cand >= s.ncand[c]) {
                s.choice[c] = s.forced[c] >= 0 ? s.forced[c] : selector_fastest(s, c);
                s.phase = 2;
                continue;
            }
            for (int q = 0; q < AG_CLS_COMPOSE; ++q) k[q] = s.choice[q];
            k[c] = s.cand;
            return true;
        }
        for (int q = 0; q < AG_NUM_CLS; ++q) k[q] = s.choice[q];
        return false;
    }
}

// Report a trial call: ms[0..2] = the three subgraph-kernel intervals, ms[3] = the whole call.
// `trials` = timed repetitions per candidate (1..kMaxTrials); repetition 0 is the warm-up.
inline void selector_record(Selector &s, int trials, const int *k, const float *ms)
{
    trials = std::max(1, std::min(trials, kMaxTrials));
    s.total_trial_ms += ms[3];
    const bool timed = s.rep > 0;
    if (timed) {
        auto push = [&](int c, int id, float v) {
            if (s.nsamples[c][id] < kMaxTrials) s.samples[c][id][s.nsamples[c][id]++] = v;
        };
        if (s.phase == 0) {
            for (int c = 0; c < AG_CLS_COMPOSE; ++c)
                if (s.forced[c] < 0 && s.cand < s.ncand[c]) push(c, k[c], ms[c]);
        } else {
            push(AG_CLS_COMPOSE, k[AG_CLS_COMPOSE], ms[3]);
        }
    }
    // hopeless after its first timed repetition: more than 4x the best finished candidate
    // (in the class trials: in every class this candidate is still being measured for)
    bool hopeless = false;
    if (s.rep == 1) {
        if (s.phase == 0) {
            bool any = false, all_slow = true;
            for (int c = 0; c < AG_CLS_COMPOSE; ++c)
                if (s.forced[c] < 0 && s.cand < s.ncand[c] && s.ncand[c] > 1) {
                    any = true;
                    if (!(s.best_ms[c] > 0 && ms[c] > 4.f * s.best_ms[c])) all_slow = false;
                }
            hopeless = any && all_slow;
        } else {
            const float b = s.best_ms[AG_CLS_COMPOSE];
            hopeless = b > 0 && ms[3] > 4.f * b;
        }
    }
    if (++s.rep > trials || hopeless) {
        // candidate finished: remember the smallest median per class
        for (int c = 0; c < AG_NUM_CLS; ++c) {
            if ((s.phase == 0) == (c == AG_CLS_COMPOSE)) continue;
            if (s.forced[c] >= 0 || s.cand >= s.ncand[c]) continue;
            const float m = selector_median(s, c, k[c]);
            if (m > 0 && (s.best_ms[c] < 0 || m < s.best_ms[c])) s.best_ms[c] = m;
        }
        s.rep = 0;
        ++s.cand;
    }
}

}  // namespace ag
