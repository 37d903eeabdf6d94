// Device code of the bandit (Section 3.2 rewards, Section 3.3 policies), shared by the bandit kernels and by the
// final-token locate kernel, which in tapout_round applies a sequence's reward and picks its next arm at its end.
// Every translation unit that includes this is compiled without floating-point contraction: every product, quotient
// and sum below is a separately rounded IEEE double operation.
#pragma once

#include "common.h"

namespace tapout {

constexpr int kAttempts = 8;

__device__ inline double unit_open(float u)
{
    double x = (double)u;
    return x > 0.0 ? x : 0x1p-25;
}

// Gamma(shape >= 1) by Marsaglia-Tsang squeeze-free rejection from caller uniforms.
__device__ inline double gamma_draw(double shape, const float *u, bool *exhausted)
{
    const double d = shape - 1.0 / 3.0;
    const double c = 1.0 / sqrt(9.0 * d);
    for (int i = 0; i < kAttempts; ++i) {
        double u1 = unit_open(u[3 * i]), u2 = (double)u[3 * i + 1], u3 = unit_open(u[3 * i + 2]);
        double z = sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2);
        double t = 1.0 + c * z;
        double v = t * t * t;
        if (v > 0.0 && log(u3) < 0.5 * z * z + d - d * v + d * log(v))
            return d * v;
    }
    *exhausted = true;
    return shape;
}

__device__ inline int ucb1_arm(const double *S, const int64_t *N, int A)
{
    int64_t t = 1;
    for (int a = 0; a < A; ++a) t += N[a];
    int best = 0;
    double best_v = -INFINITY;
    for (int a = 0; a < A; ++a) {
        if (N[a] == 0) return a;                       // every arm is played once first, in index order
        double n = (double)N[a];
        double v = S[a] / n + sqrt((2.0 * log((double)t)) / n);
        if (a == 0 || v > best_v) { best = a; best_v = v; }
    }
    return best;
}

// UCB-Tuned: bonus sqrt((ln t / N) min(1/4, V)), V = var + sqrt(2 ln t / N), var = Q/N - mean^2.
__device__ inline int ucb_tuned_arm(const double *S, const double *Q, const int64_t *N, int A)
{
    int64_t t = 1;
    for (int a = 0; a < A; ++a) t += N[a];
    const double lt = log((double)t);
    int best = 0;
    double best_v = -INFINITY;
    for (int a = 0; a < A; ++a) {
        if (N[a] == 0) return a;
        const double n = (double)N[a];
        const double mean = S[a] / n;
        const double var = Q[a] / n - mean * mean;
        const double V = var + sqrt((2.0 * lt) / n);
        const double cap = V < 0.25 ? V : 0.25;
        const double v = mean + sqrt((lt / n) * cap);
        if (a == 0 || v > best_v) { best = a; best_v = v; }
    }
    return best;
}

// Gaussian posterior N(S/(N+1), 1/(N+1)); one Box-Muller normal from the arm's first two uniforms.
__device__ inline int ts_gauss_arm(const double *S, const int64_t *N, int A, const float *u)
{
    int best = 0;
    double best_v = -INFINITY;
    for (int a = 0; a < A; ++a) {
        const float *ua = u + (size_t)a * TAPOUT_TS_UNIFORMS_PER_ARM;
        const double n1 = (double)N[a] + 1.0;
        const double z = sqrt(-2.0 * log(unit_open(ua[0]))) * cos(6.283185307179586476925 * (double)ua[1]);
        const double th = S[a] / n1 + z / sqrt(n1);
        if (a == 0 || th > best_v) { best = a; best_v = th; }
    }
    return best;
}

__device__ inline int ts_arm(const double *S, const int64_t *N, int A, const float *u, bool *exhausted)
{
    int best = 0;
    double best_v = -INFINITY;
    for (int a = 0; a < A; ++a) {
        double alpha = 1.0 + S[a];
        double beta = 1.0 + ((double)N[a] - S[a]);
        const float *ua = u + (size_t)a * TAPOUT_TS_UNIFORMS_PER_ARM;
        double g1 = gamma_draw(alpha, ua, exhausted);
        double g2 = gamma_draw(beta, ua + kAttempts * 3, exhausted);
        double th = g1 / (g1 + g2);
        if (a == 0 || th > best_v) { best = a; best_v = th; }
    }
    return best;
}

__device__ inline int select_arm(const BanditArgs &a, size_t nb, const float *u_ts, bool *ex)
{
    const double *S = a.sum_r + nb;
    const int64_t *N = a.count + nb;
    const float *u = u_ts ? u_ts + nb * TAPOUT_TS_UNIFORMS_PER_ARM : nullptr;
    if (a.policy == TAPOUT_UCB1) return ucb1_arm(S, N, a.n_arms);
    if (a.policy == TAPOUT_UCB_TUNED) return ucb_tuned_arm(S, a.sum_r2 + nb, N, a.n_arms);
    if (a.policy == TAPOUT_TS_GAUSS) return ts_gauss_arm(S, N, a.n_arms, u);
    return ts_arm(S, N, a.n_arms, u, ex);
}

__device__ inline void apply_reward(const BanditArgs &a, int nb, int arm, int m, int n, int g)
{
    const double r = a.reward == TAPOUT_REWARD_SIMPLE
                         ? (double)m / (double)g
                         : (a.alpha * (double)m) / (double)g + ((1.0 - a.alpha) * (double)m) / (double)n;
    a.count[(size_t)nb * a.n_arms + arm] += 1;
    a.sum_r[(size_t)nb * a.n_arms + arm] += r;
    a.sum_r2[(size_t)nb * a.n_arms + arm] += r * r;
}

// Token-level bandits (Section 3.1 / 3.2): position k < m is an accepted play (reward 1) of the arm chosen
// there, position m < n the rejected one (reward 0); later positions were never evaluated.
__device__ inline void apply_token_rewards(const BanditArgs &a, int nb, const int32_t *arm_b, int m, int n)
{
    if (n > a.positions) n = a.positions;
    for (int k = 0; k < n && k <= m; ++k) {
        const int arm = arm_b[k];
        if (arm < 0 || arm >= a.n_arms) continue;
        const size_t i = ((size_t)nb * a.positions + k) * a.n_arms + arm;
        const double r = k < m ? 1.0 : 0.0;
        a.count[i] += 1;
        a.sum_r[i] += r;
        a.sum_r2[i] += r;
    }
}

// Carried state of the stateful stop rules after one draft of sequence b (Appendix A.1).
__device__ inline void advance_rule_state(const BanditArgs &a, int b, int m, int n)
{
    if (a.round_K > 0) a.prev_entropy[b] = a.round_entropy[(int64_t)b * a.round_K + (n - 1)];
    const double r = (double)m / (double)n;
    const double rate = a.ad_beta1 * a.accept_rate[b] + (1.0 - a.ad_beta1) * r;
    a.accept_rate[b] = rate;
    const double s = a.ad_steer ? r : rate;       // what steers the threshold: the smoothed rate, or r as printed
    const double sg = a.ad_alpha > s ? 1.0 : (a.ad_alpha < s ? -1.0 : 0.0);
    for (int j = 0; j < a.n_arms; ++j) {
        if (a.rule[j] != TAPOUT_RULE_ADAEDL) continue;
        const double lam = a.lambda[(int64_t)b * a.n_arms + j];
        a.lambda[(int64_t)b * a.n_arms + j] = a.ad_beta2 * lam + (1.0 - a.ad_beta2) * (lam + a.ad_eps * sg);
    }
}

__device__ inline bool playable(const BanditArgs &a, int b, const int32_t *arm, const int32_t *n_draft,
                                const int32_t *gamma, const uint8_t *active)
{
    if (active && !active[b]) return false;
    if (n_draft[b] < 1 || gamma[b] < 1) return false;
    return a.positions > 1 || (arm[b] >= 0 && arm[b] < a.n_arms);           // token-level arms are checked per position
}

__device__ inline void play(const BanditArgs &a, int nb, int b, const int32_t *arm, const int32_t *accept_len,
                            const int32_t *n_draft, const int32_t *gamma)
{
    if (a.positions > 1) apply_token_rewards(a, nb, arm + (size_t)b * a.positions, accept_len[b], n_draft[b]);
    else apply_reward(a, nb, arm[b], accept_len[b], n_draft[b], gamma[b]);
}

// Update of sequence b's own sequence-level bandit followed by its next selection, by one thread: the selection
// reads the state the thread has just written (program order).
__device__ inline void update_select_one(const BanditArgs &a, int b, const int32_t *arm, const int32_t *accept_len,
                                         const int32_t *n_draft, const int32_t *gamma, const uint8_t *active,
                                         const float *u_ts, int32_t *arm_out, uint32_t *flags)
{
    if (playable(a, b, arm, n_draft, gamma, active)) play(a, b, b, arm, accept_len, n_draft, gamma);
    if (a.accept_rate && !(active && !active[b])) {
        const int n = n_draft[b];
        if (n >= 1 && (a.round_K == 0 || n <= a.round_K)) advance_rule_state(a, b, accept_len[b], n);
    }
    bool ex = false;
    arm_out[b] = select_arm(a, (size_t)b * a.n_arms, u_ts, &ex);
    if (flags) flags[b] = ex ? TAPOUT_FLAG_SAMPLER_EXHAUSTED : 0u;
}

// The same restricted to the UCB policies (no caller uniforms, no Gamma / Gaussian draws in the code).
__device__ inline void update_select_ucb(const BanditArgs &a, int b, const int32_t *arm, const int32_t *accept_len,
                                         const int32_t *n_draft, const int32_t *gamma, const uint8_t *active,
                                         int32_t *arm_out, uint32_t *flags)
{
    if (playable(a, b, arm, n_draft, gamma, active)) play(a, b, b, arm, accept_len, n_draft, gamma);
    if (a.accept_rate && !(active && !active[b])) {
        const int n = n_draft[b];
        if (n >= 1 && (a.round_K == 0 || n <= a.round_K)) advance_rule_state(a, b, accept_len[b], n);
    }
    const size_t nb = (size_t)b * a.n_arms;
    arm_out[b] = a.policy == TAPOUT_UCB1 ? ucb1_arm(a.sum_r + nb, a.count + nb, a.n_arms)
                                         : ucb_tuned_arm(a.sum_r + nb, a.sum_r2 + nb, a.count + nb, a.n_arms);
    if (flags) flags[b] = 0u;
}

// The same on the first TAPOUT_MAX_ARMS lanes of a wavefront, one arm per lane, in two steps for a kernel that has
// other work in between.  ucb_lane_prefetch requests what the update and the selection read (the lane's arm of the
// sequence's bandit state; the sequence's arm, lengths and cap) in one memory round trip.  ucb_lane_finish works on the
// register copies: the lane of the played arm applies the reward and writes its state back, every lane forms the index
// of its arm (the logarithm, quotient and square root of the arms side by side instead of one after the other), and
// the argmax runs over the lanes, lowest arm on ties, an unplayed arm first.  Per arm the same double operations as
// ucb1_arm / ucb_tuned_arm, hence the same bits.  All TAPOUT_MAX_ARMS lanes must be active in both calls.
struct UcbLane {
    double S, Q;
    int64_t N;
    int32_t arm, n_draft, gamma;
    bool active;
};

__device__ inline UcbLane ucb_lane_prefetch(const BanditArgs &a, int b, int lane, const int32_t *arm, const int32_t *n_draft,
                                            const int32_t *gamma, const uint8_t *active)
{
    UcbLane r;
    const size_t nb = (size_t)b * a.n_arms;
    const bool on = lane < a.n_arms;
    r.S = on ? a.sum_r[nb + lane] : 0.0;
    r.Q = on ? a.sum_r2[nb + lane] : 0.0;
    r.N = on ? a.count[nb + lane] : 0;
    r.arm = arm[b]; r.n_draft = n_draft[b]; r.gamma = gamma[b];
    r.active = !(active && !active[b]);
    return r;
}

__device__ inline void ucb_lane_finish(const BanditArgs &a, int b, int lane, UcbLane r, int32_t accept_len, int32_t *arm_out, uint32_t *flags)
{
    const size_t nb = (size_t)b * a.n_arms;
    const bool on = lane < a.n_arms;
    if (r.active && r.n_draft >= 1 && r.gamma >= 1 && r.arm >= 0 && r.arm < a.n_arms && lane == r.arm) {
        const double m = (double)accept_len;
        const double rew = a.reward == TAPOUT_REWARD_SIMPLE
                               ? m / (double)r.gamma
                               : (a.alpha * m) / (double)r.gamma + ((1.0 - a.alpha) * m) / (double)r.n_draft;
        r.N += 1; r.S += rew; r.Q += rew * rew;
        a.count[nb + lane] = r.N; a.sum_r[nb + lane] = r.S; a.sum_r2[nb + lane] = r.Q;
    }
    if (lane == 0 && a.accept_rate && r.active && r.n_draft >= 1 && (a.round_K == 0 || r.n_draft <= a.round_K))
        advance_rule_state(a, b, accept_len, r.n_draft);
    // t = 1 + all plays (an integer: any order)
    int64_t t = on ? r.N : 0;
#pragma unroll
    for (int d = 1; d < TAPOUT_MAX_ARMS; d <<= 1) {
        const int lo = __shfl_xor((int)(uint32_t)t, d), hi = __shfl_xor((int)(t >> 32), d);
        t += (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
    }
    t += 1;
    const double n = (double)r.N;
    double v;
    if (a.policy == TAPOUT_UCB1) {
        v = r.S / n + sqrt((2.0 * log((double)t)) / n);
    } else {
        const double lt = log((double)t);
        const double mean = r.S / n;
        const double var = r.Q / n - mean * mean;
        const double V = var + sqrt((2.0 * lt) / n);
        const double cap = V < 0.25 ? V : 0.25;
        v = mean + sqrt((lt / n) * cap);
    }
    // an arm never played goes first (lowest index); else the first maximum in index order
    const uint64_t unplayed = __ballot(on && r.N == 0) & 0xffull;
    int best = on ? lane : 0x7fffffff;
    if (!on) v = -INFINITY;
#pragma unroll
    for (int d = 1; d < TAPOUT_MAX_ARMS; d <<= 1) {
        const double ov = __shfl_xor(v, d);
        const int ob = __shfl_xor(best, d);
        if (ov > v || (ov == v && ob < best)) { v = ov; best = ob; }
    }
    if (lane == 0) {
        arm_out[b] = unplayed ? __builtin_ctzll(unplayed) : (best == 0x7fffffff ? 0 : best);
        if (flags) flags[b] = 0u;
    }
}

// The same for Thompson Sampling with Beta posteriors on 16 consecutive lanes of a wavefront (lane16 = 0..15 = 2 * arm +
// variate; b >= a.B: idle group): every lane holds the count and the reward sum of its arm in registers and applies
// the reward to its own copy if its arm was the one played; one lane writes the state back.  No lane reads what
// another lane wrote.  All 16 lanes of the group must be active.
__device__ inline void update_select_ts_lanes(const BanditArgs &a, const int b, const int lane16, const int32_t *arm_in, const int32_t *accept_len,
                                              const int32_t *n_draft, const int32_t *gamma, const uint8_t *active,
                                              const float *u_ts, int32_t *arm_out, uint32_t *flags)
{
    const int arm = lane16 >> 1, which = lane16 & 1;
    const bool live = b < a.B && arm < a.n_arms;
    double g = 1.0;
    bool ex = false;
    if (live) {
        const size_t nb = (size_t)b * a.n_arms;
        double S = a.sum_r[nb + arm];
        int64_t Ni = a.count[nb + arm];
        if (playable(a, b, arm_in, n_draft, gamma, active) && arm_in[b] == arm) {
            const int m = accept_len[b], n = n_draft[b], gm = gamma[b];
            const double r = a.reward == TAPOUT_REWARD_SIMPLE
                                 ? (double)m / (double)gm
                                 : (a.alpha * (double)m) / (double)gm + ((1.0 - a.alpha) * (double)m) / (double)n;
            Ni += 1;
            S += r;
            if (which == 0) {
                a.count[nb + arm] = Ni;
                a.sum_r[nb + arm] = S;
                a.sum_r2[nb + arm] += r * r;
            }
        }
        const double N = (double)Ni;
        const double shape = which == 0 ? 1.0 + S : 1.0 + (N - S);
        const float *ua = u_ts + (nb + arm) * TAPOUT_TS_UNIFORMS_PER_ARM + which * kAttempts * 3;
        g = gamma_draw(shape, ua, &ex);
    }
    if (b < a.B && lane16 == 0 && a.accept_rate && !(active && !active[b])) {
        const int n = n_draft[b];
        if (n >= 1 && (a.round_K == 0 || n <= a.round_K)) advance_rule_state(a, b, accept_len[b], n);
    }
    const double other = __shfl_xor(g, 1);
    double th = (live && which == 0) ? g / (g + other) : -INFINITY;
    int best = (live && which == 0) ? arm : 0x7fffffff;
    uint32_t exm = ex ? 1u : 0u;
#pragma unroll
    for (int d = 2; d < 16; d <<= 1) {
        const double oth = __shfl_xor(th, d);
        const int ob = __shfl_xor(best, d);
        if (oth > th || (oth == th && ob < best)) { th = oth; best = ob; }
    }
#pragma unroll
    for (int d = 1; d < 16; d <<= 1) exm |= __shfl_xor(exm, d);
    if (b < a.B && lane16 == 0) {
        arm_out[b] = best == 0x7fffffff ? 0 : best;
        if (flags) flags[b] = exm ? TAPOUT_FLAG_SAMPLER_EXHAUSTED : 0u;
    }
}

}  // namespace tapout
