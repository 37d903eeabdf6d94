// Sequence-level bandit over the stop rules (Section 3.3) and the blended
// reward (Section 3.2).  State: per bandit and arm the number of plays N and
// the summed reward S, in double / int64.  One thread per sequence; the work
// is O(B * arms) and never touches the vocabulary.
//
// This file is compiled without floating-point contraction: every product,
// quotient and sum below is a separately rounded IEEE double operation.
#include "common.h"

namespace tapout {

namespace {

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

__global__ void bandit_select_kernel(BanditArgs a, const float *u_ts, int32_t *arm_out, uint32_t *flags)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= a.B) return;
    const int nb = a.n_bandits == 1 ? 0 : b;
    const double *S = a.sum_r + (size_t)nb * a.n_arms;
    const int64_t *N = a.count + (size_t)nb * a.n_arms;
    bool ex = false;
    int arm;
    if (a.policy == TAPOUT_UCB1) arm = ucb1_arm(S, N, a.n_arms);
    else arm = ts_arm(S, N, a.n_arms, u_ts + (size_t)nb * a.n_arms * TAPOUT_TS_UNIFORMS_PER_ARM, &ex);
    arm_out[b] = arm;
    if (flags) flags[b] = ex ? TAPOUT_FLAG_SAMPLER_EXHAUSTED : 0u;
}

__device__ inline void apply_reward(const BanditArgs &a, int nb, int arm, int m, int n, int g)
{
    double r = (a.alpha * (double)m) / (double)g + ((1.0 - a.alpha) * (double)m) / (double)n;
    a.count[(size_t)nb * a.n_arms + arm] += 1;
    a.sum_r[(size_t)nb * a.n_arms + arm] += r;
}

__device__ inline bool playable(const BanditArgs &a, int b, const int32_t *arm, const int32_t *n_draft,
                                const int32_t *gamma, const uint8_t *active)
{
    if (active && !active[b]) return false;
    return arm[b] >= 0 && arm[b] < a.n_arms && n_draft[b] >= 1 && gamma[b] >= 1;
}

__global__ void bandit_update_kernel(BanditArgs a, const int32_t *arm, const int32_t *accept_len,
                                     const int32_t *n_draft, const int32_t *gamma, const uint8_t *active)
{
    if (a.n_bandits == 1) {
        // shared bandit: the B plays are applied in index order by one thread
        if (blockIdx.x == 0 && threadIdx.x == 0)
            for (int b = 0; b < a.B; ++b)
                if (playable(a, b, arm, n_draft, gamma, active))
                    apply_reward(a, 0, arm[b], accept_len[b], n_draft[b], gamma[b]);
        return;
    }
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= a.B) return;
    if (playable(a, b, arm, n_draft, gamma, active))
        apply_reward(a, b, arm[b], accept_len[b], n_draft[b], gamma[b]);
}

}  // namespace

hipError_t launch_bandit_select(const BanditArgs &a, const float *u_ts, int32_t *arm_out, uint32_t *flags, hipStream_t st, Timing tm)
{
    const int block = 64;
    launch_kernel(bandit_select_kernel, dim3((a.B + block - 1) / block), dim3(block), st, tm, a, u_ts, arm_out, flags);
    return hipGetLastError();
}

hipError_t launch_bandit_update(const BanditArgs &a, const int32_t *arm, const int32_t *accept_len,
                                const int32_t *n_draft, const int32_t *gamma, const uint8_t *active, hipStream_t st, Timing tm)
{
    const int block = 64;
    int grid = a.n_bandits == 1 ? 1 : (a.B + block - 1) / block;
    launch_kernel(bandit_update_kernel, dim3(grid), dim3(block), st, tm, a, arm, accept_len, n_draft, gamma, active);
    return hipGetLastError();
}

}  // namespace tapout
