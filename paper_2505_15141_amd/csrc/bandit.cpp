// Host-side arm selection: UCBSpec (Alg. 4 and its full version) and EXP3Spec (full version of Alg. 5).
// O(K) double arithmetic per round on per-arm sufficient statistics; the history H_t of Alg. 3 is only
// ever used through the pull counts and the accepted lengths.
#include <cmath>
#include <limits>
#include <new>
#include <vector>
#include "common.h"

struct bs_bandit {
    int kind, K;
    double L, delta;
    uint64_t seed;
    int64_t t;                    // completed rounds
    std::vector<double> n, sum;   // pulls; sum of y (UCB) or cumulative estimated loss (EXP3)
    std::vector<double> p;        // EXP3: probabilities used for the pending selection
    int pending;                  // arm handed out by select and not yet updated, or -1
};

static double ucb_radius(const bs_bandit* b, int i) {
    const double n = b->n[i], t = (double)b->t;
    const double inner = 1.0 + 2.0 * std::log((double)b->K * t * t * std::sqrt(1.0 + n) / b->delta);
    return 0.5 * b->L * std::sqrt((1.0 + n) / (n * n) * inner);
}

static void exp3_probs(const bs_bandit* b, double* p) {
    const double t = (double)(b->t + 1);
    const double eta = std::sqrt(std::log((double)b->K) / (t * (double)b->K));
    double lo = b->sum[0];
    for (int i = 1; i < b->K; ++i) lo = std::fmin(lo, b->sum[i]);
    double z = 0.0;
    for (int i = 0; i < b->K; ++i) {
        p[i] = std::exp(-eta * (b->sum[i] - lo));   // the common factor exp(eta*lo) cancels
        z += p[i];
    }
    for (int i = 0; i < b->K; ++i) p[i] /= z;
}

extern "C" __attribute__((visibility("default"))) int bs_bandit_create(int kind, int K, int L, double delta, uint64_t seed, bs_bandit** out) {
    BS_REQUIRE(out, BS_EINVAL, "bs_bandit_create: out is NULL");
    BS_REQUIRE(kind == BS_UCBSPEC || kind == BS_EXP3SPEC, BS_EINVAL, "bs_bandit_create: unknown kind %d", kind);
    BS_REQUIRE(K >= 1 && K <= 4096, BS_EINVAL, "bs_bandit_create: K=%d out of range", K);
    BS_REQUIRE(L >= 1, BS_EINVAL, "bs_bandit_create: L=%d must be >= 1", L);
    BS_REQUIRE(kind != BS_UCBSPEC || (delta > 0.0 && delta <= 1.0), BS_EINVAL,
               "bs_bandit_create: delta=%g must be in (0,1]", delta);
    bs_bandit* b = new (std::nothrow) bs_bandit();
    BS_REQUIRE(b, BS_EINVAL, "bs_bandit_create: out of host memory");
    b->kind = kind; b->K = K; b->L = (double)L; b->delta = delta; b->seed = seed; b->t = 0; b->pending = -1;
    b->n.assign(K, 0.0); b->sum.assign(K, 0.0); b->p.assign(K, 1.0 / K);
    *out = b;
    return BS_OK;
}

extern "C" __attribute__((visibility("default"))) int bs_bandit_destroy(bs_bandit* b) {
    delete b;
    return BS_OK;
}

extern "C" __attribute__((visibility("default"))) int bs_bandit_probs(bs_bandit* b, double* out) {
    BS_REQUIRE(b && out, BS_EINVAL, "bs_bandit_probs: NULL argument");
    if (b->kind == BS_EXP3SPEC) {
        exp3_probs(b, out);
    } else {
        for (int i = 0; i < b->K; ++i)
            out[i] = (b->n[i] > 0 && b->t >= b->K) ? b->sum[i] / b->n[i] + ucb_radius(b, i)
                                                   : std::numeric_limits<double>::infinity();
    }
    return BS_OK;
}

extern "C" __attribute__((visibility("default"))) int bs_bandit_select(bs_bandit* b, int* arm_out) {
    BS_REQUIRE(b && arm_out, BS_EINVAL, "bs_bandit_select: NULL argument");
    int arm = 0;
    if (b->kind == BS_UCBSPEC) {
        if (b->t < b->K) {
            arm = (int)b->t;                              // round-robin start
        } else {
            double best = -std::numeric_limits<double>::infinity();
            for (int i = 0; i < b->K; ++i) {
                const double u = b->sum[i] / b->n[i] + ucb_radius(b, i);
                if (u > best) { best = u; arm = i; }     // strict: ties keep the lowest index
            }
        }
    } else {
        exp3_probs(b, b->p.data());
        const double u = (double)bs::u_closed_open(bs::philox_word(b->seed, 0u, (uint32_t)b->t, 0u, bs::PURPOSE_BANDIT));
        double total = 0.0;
        for (int i = 0; i < b->K; ++i) total += b->p[i];
        const double x = u * total;
        double c = 0.0;
        arm = b->K - 1;
        for (int i = 0; i < b->K; ++i) {
            c += b->p[i];
            if (c > x) { arm = i; break; }
        }
    }
    b->pending = arm;
    *arm_out = arm;
    return BS_OK;
}

extern "C" __attribute__((visibility("default"))) int bs_bandit_update(bs_bandit* b, int arm, double y) {
    BS_REQUIRE(b, BS_EINVAL, "bs_bandit_update: NULL handle");
    BS_REQUIRE(arm >= 0 && arm < b->K, BS_EINVAL, "bs_bandit_update: arm %d not in [0,%d)", arm, b->K);
    BS_REQUIRE(y >= 1.0 && y <= b->L + 1.0, BS_EINVAL, "bs_bandit_update: y=%g outside [1, L+1=%g]", y, b->L + 1.0);
    if (b->kind == BS_EXP3SPEC) {
        BS_REQUIRE(b->pending == arm, BS_ESTATE, "bs_bandit_update: arm %d was not the selected arm (%d)", arm, b->pending);
        b->sum[arm] += (b->L + 1.0 - y) / (b->L * b->p[arm]);
    } else {
        b->sum[arm] += y;
    }
    b->n[arm] += 1.0;
    b->t += 1;
    b->pending = -1;
    return BS_OK;
}

extern "C" __attribute__((visibility("default"))) int bs_bandit_stats(bs_bandit* b, double* n, double* sum, int64_t* rounds) {
    BS_REQUIRE(b, BS_EINVAL, "bs_bandit_stats: NULL handle");
    for (int i = 0; i < b->K; ++i) {
        if (n) n[i] = b->n[i];
        if (sum) sum[i] = b->sum[i];
    }
    if (rounds) *rounds = b->t;
    return BS_OK;
}

extern "C" __attribute__((visibility("default"))) int bs_throughput_reward(double tokens, double seconds, double canonical_seconds, int L, double* y_out) {
    BS_REQUIRE(y_out, BS_EINVAL, "bs_throughput_reward: NULL output");
    BS_REQUIRE(L >= 1 && tokens >= 0.0 && seconds > 0.0 && canonical_seconds > 0.0, BS_EINVAL,
               "bs_throughput_reward: tokens=%g seconds=%g canonical_seconds=%g L=%d", tokens, seconds, canonical_seconds, L);
    const double rate = tokens / seconds, ref = (double)(L + 1) / canonical_seconds;
    const double frac = rate / ref < 1.0 ? rate / ref : 1.0;
    *y_out = 1.0 + (double)L * frac;
    return BS_OK;
}

// One bandit per batch: the reward of a round is the mean accepted length over the sequences that took part in it.
extern "C" __attribute__((visibility("default"))) int bs_batch_reward(const int32_t* host_n_emitted, int B, double* y_out, int* n_active_out) {
    BS_REQUIRE(host_n_emitted && y_out, BS_EINVAL, "bs_batch_reward: NULL argument");
    BS_REQUIRE(B >= 1, BS_EINVAL, "bs_batch_reward: B=%d", B);
    long long sum = 0;
    int active = 0;
    for (int b = 0; b < B; ++b) {
        BS_REQUIRE(host_n_emitted[b] >= 0, BS_EINVAL, "bs_batch_reward: n_emitted[%d]=%d is negative", b, host_n_emitted[b]);
        if (host_n_emitted[b] > 0) { sum += host_n_emitted[b]; ++active; }
    }
    if (n_active_out) *n_active_out = active;
    BS_REQUIRE(active > 0, BS_ESTATE, "bs_batch_reward: no sequence took part in the round (all at their goal, or skipped)");
    *y_out = (double)sum / (double)active;
    return BS_OK;
}
