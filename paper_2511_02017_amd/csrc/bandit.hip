// Sequence-level bandit over the stop rules (Section 3.3: UCB1, UCB-Tuned,
// Thompson Sampling with Beta or Gaussian posteriors) and the rewards of
// Section 3.2.  State: per bandit and arm the number of plays N, the summed
// reward S and the summed squared reward Q, in int64 / double.  The update also
// advances the carried state of the stateful stop rules of Appendix A.1
// (SVIP-Difference's previous entropy, AdaEDL's acceptance rate and thresholds).
// One thread per sequence; the work is O(B * arms) and never touches the
// vocabulary.
//
// This file is compiled without floating-point contraction: every product,
// quotient and sum below is a separately rounded IEEE double operation.
#include "common.h"
#include "bandit_device.h"

namespace tapout {

namespace {

// Sequence-level bandit: one thread per sequence.
__global__ void bandit_select_kernel(BanditArgs a, const float *u_ts, int32_t *arm_out, uint32_t *flags)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= a.B) return;
    bool ex = false;
    arm_out[b] = select_arm(a, (size_t)(a.n_bandits == 1 ? 0 : b) * a.n_arms, u_ts, &ex);
    if (flags) flags[b] = ex ? TAPOUT_FLAG_SAMPLER_EXHAUSTED : 0u;
}

// Sequence-level Thompson Sampling with Beta posteriors, lane-parallel: the Marsaglia-Tsang loops of the 2 * arms
// Gamma variates of a sequence are long serial chains of double-precision log / sqrt / cos, so each gets a lane
// of its own (16 lanes per sequence: lane = 2 * arm + variate), the pair is combined with one lane exchange and
// the argmax runs over the sequence's 16 lanes.  Same operations per variate as the one-thread version, hence
// the same bits.
__global__ __launch_bounds__(64) void bandit_select_ts_kernel(BanditArgs a, const float *u_ts, int32_t *arm_out, uint32_t *flags)
{
    static_assert(TAPOUT_MAX_ARMS * 2 == 16, "16 lanes per sequence");
    const int lane16 = threadIdx.x & 15;
    const int b = blockIdx.x * 4 + (threadIdx.x >> 4);
    const int arm = lane16 >> 1, which = lane16 & 1;
    const bool live = b < a.B && arm < a.n_arms;
    double g = 1.0;
    bool ex = false;
    if (live) {
        const size_t nb = (size_t)(a.n_bandits == 1 ? 0 : b) * a.n_arms;
        const double S = a.sum_r[nb + arm], N = (double)a.count[nb + arm];
        const double shape = which == 0 ? 1.0 + S : 1.0 + (N - S);
        const float *ua = u_ts + (nb + arm) * TAPOUT_TS_UNIFORMS_PER_ARM + which * kAttempts * 3;
        g = gamma_draw(shape, ua, &ex);
    }
    // theta = g1 / (g1 + g2) on the even lane of each pair
    const double other = __shfl_xor(g, 1);
    double th = (live && which == 0) ? g / (g + other) : -INFINITY;
    int best = (live && which == 0) ? arm : 0x7fffffff;
    uint32_t exm = ex ? 1u : 0u;
    // argmax over the 16 lanes of the sequence; ties go to the lowest arm (the one-thread loop keeps the first maximum)
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

// Token-level bandits: one workgroup per sequence, its threads take the positions; the sequence's flag word
// is the OR over its positions.
__global__ void bandit_select_token_kernel(BanditArgs a, const float *u_ts, int32_t *arm_out, uint32_t *flags)
{
    __shared__ uint32_t sh_flag;
    const int b = blockIdx.x;
    if (threadIdx.x == 0) sh_flag = 0;
    __syncthreads();
    bool any = false;
    for (int k = threadIdx.x; k < a.positions; k += blockDim.x) {
        bool ex = false;
        const size_t nb = ((size_t)(a.n_bandits == 1 ? 0 : b) * a.positions + k) * a.n_arms;
        arm_out[(size_t)b * a.positions + k] = select_arm(a, nb, u_ts, &ex);
        any |= ex;
    }
    if (any) atomicOr(&sh_flag, TAPOUT_FLAG_SAMPLER_EXHAUSTED);
    __syncthreads();
    if (threadIdx.x == 0 && flags) flags[b] = sh_flag;
}

__global__ void bandit_update_kernel(BanditArgs a, const int32_t *arm, const int32_t *accept_len,
                                     const int32_t *n_draft, const int32_t *gamma, const uint8_t *active)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (a.n_bandits == 1) {
        // shared bandit: the B plays are applied in index order by one thread
        if (b == 0)
            for (int i = 0; i < a.B; ++i)
                if (playable(a, i, arm, n_draft, gamma, active)) play(a, 0, i, arm, accept_len, n_draft, gamma);
    } else if (b < a.B && playable(a, b, arm, n_draft, gamma, active)) {
        play(a, b, b, arm, accept_len, n_draft, gamma);
    }
    if (a.accept_rate && b < a.B && !(active && !active[b])) {
        const int n = n_draft[b];
        if (n >= 1 && (a.round_K == 0 || n <= a.round_K)) advance_rule_state(a, b, accept_len[b], n);
    }
}

// ---- update and next selection in one launch ---------------------------------------------------------
// Sequence-level bandits, one per sequence: the thread that applies sequence b's reward is the one that picks its
// next arm, so the selection reads the state it has just written (program order within a thread) and the round
// saves a launch.  Same operations as the two kernels: same bits.
__global__ void bandit_update_select_kernel(BanditArgs a, const int32_t *arm, const int32_t *accept_len,
                                            const int32_t *n_draft, const int32_t *gamma, const uint8_t *active,
                                            const float *u_ts, int32_t *arm_out, uint32_t *flags)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= a.B) return;
    update_select_one(a, b, arm, accept_len, n_draft, gamma, active, u_ts, arm_out, flags);
}

// The same for Thompson Sampling with Beta posteriors, lane-parallel (update_select_ts_lanes): four sequences per wavefront.
__global__ __launch_bounds__(64) void bandit_update_select_ts_kernel(BanditArgs a, const int32_t *arm_in, const int32_t *accept_len,
                                                                      const int32_t *n_draft, const int32_t *gamma, const uint8_t *active,
                                                                      const float *u_ts, int32_t *arm_out, uint32_t *flags)
{
    update_select_ts_lanes(a, blockIdx.x * 4 + (threadIdx.x >> 4), threadIdx.x & 15, arm_in, accept_len, n_draft, gamma, active, u_ts, arm_out, flags);
}

}  // namespace

// Update followed by the next selection.  One launch where every sequence has a sequence-level bandit of its own;
// otherwise (shared bandit, token-level bandits) the two kernels one after the other.
hipError_t launch_bandit_update_select(const BanditArgs &a, const int32_t *arm, const int32_t *accept_len,
                                       const int32_t *n_draft, const int32_t *gamma, const uint8_t *active,
                                       const float *u_ts, int32_t *arm_out, uint32_t *flags, hipStream_t st, Timing tm)
{
    if (a.positions > 1 || a.n_bandits == 1) {
        hipError_t e = launch_bandit_update(a, arm, accept_len, n_draft, gamma, active, st, tm);
        if (e != hipSuccess) return e;
        return launch_bandit_select(a, u_ts, arm_out, flags, st, Timing{});
    }
    if (a.policy == TAPOUT_TS_BETA)
        launch_kernel(bandit_update_select_ts_kernel, dim3((a.B + 3) / 4), dim3(64), st, tm, a, arm, accept_len, n_draft, gamma, active, u_ts, arm_out, flags);
    else
        launch_kernel(bandit_update_select_kernel, dim3((a.B + 63) / 64), dim3(64), st, tm, a, arm, accept_len, n_draft, gamma, active, u_ts, arm_out, flags);
    return hipGetLastError();
}

hipError_t launch_bandit_select(const BanditArgs &a, const float *u_ts, int32_t *arm_out, uint32_t *flags, hipStream_t st, Timing tm)
{
    const int block = 64;
    if (a.positions > 1) launch_kernel(bandit_select_token_kernel, dim3(a.B), dim3(block), st, tm, a, u_ts, arm_out, flags);
    else if (a.policy == TAPOUT_TS_BETA) launch_kernel(bandit_select_ts_kernel, dim3((a.B + 3) / 4), dim3(64), st, tm, a, u_ts, arm_out, flags);
    else launch_kernel(bandit_select_kernel, dim3((a.B + block - 1) / block), dim3(block), st, tm, a, u_ts, arm_out, flags);
    return hipGetLastError();
}

hipError_t launch_bandit_update(const BanditArgs &a, const int32_t *arm, const int32_t *accept_len,
                                const int32_t *n_draft, const int32_t *gamma, const uint8_t *active, hipStream_t st, Timing tm)
{
    const int block = 64;
    int grid = (a.n_bandits == 1 && !a.accept_rate) ? 1 : (a.B + block - 1) / block;
    launch_kernel(bandit_update_kernel, dim3(grid), dim3(block), st, tm, a, arm, accept_len, n_draft, gamma, active);
    return hipGetLastError();
}

}  // namespace tapout
