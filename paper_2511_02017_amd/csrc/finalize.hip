// Per-sequence epilogues of the two streaming passes.
//
// draft_finalize : merges the slice partials of every draft row into the
//   signals of Table 1 / Appendix A.1 and runs the stop scan of Algorithm 1's
//   draft loop (the token drafted at the firing step is kept).
// verify_finalize: merges the partials of the target rows, forms
//   log p(tok), takes the accept decisions  u < p(tok)/q(tok)  of speculative
//   sampling, finds the first rejection, handles greedy sequences completely
//   and leaves a SampleJob for the sequences whose final token must be drawn.
//
// Both run one workgroup per sequence; the work is O(K * nsplit) per sequence.
#include "common.h"

namespace tapout {

namespace {

constexpr int kFinalBlock = 64;

__device__ inline bool rule_fires(int rule, float h, float H, float p1, float margin)
{
    // decisions on the returned binary32 signals, widened to double (strict inequalities of Table 1)
    switch (rule) {
    case TAPOUT_RULE_SVIP:    return sqrt((double)H) > (double)h;
    case TAPOUT_RULE_MAXCONF: return (double)p1 < (double)h;
    default:                  return (double)margin < (double)h;
    }
}

__global__ __launch_bounds__(kFinalBlock) void draft_finalize_kernel(DraftFinalArgs a)
{
    extern __shared__ float sh[];             // [3][K] entropy, p_top1, margin
    __shared__ uint32_t sh_flags;
    const int b = blockIdx.x;
    const int K = a.K;
    int kb = a.k_len ? a.k_len[b] : K;
    kb = kb > K ? K : kb;
    if (threadIdx.x == 0) sh_flags = 0;
    __syncthreads();
    for (int k = threadIdx.x; k < kb; k += blockDim.x) {
        const int64_t i = (int64_t)b * K + k;
        const void *row = row_address(a.base, a.dtype, a.stride_b, a.stride_k, b, k);
        RowTotal r = merge_partials(a.part + i * a.nsplit, a.nsplit);
        uint32_t f = 0;
        float lse, H, p1, p2, mg;
        double lse_d = NAN;
        if (r.bad) {
            f |= TAPOUT_FLAG_BAD_ROW;
            lse = H = p1 = p2 = mg = NAN;
        } else {
            double l2S = log2(r.S);
            lse_d = (r.R + l2S) * kLn2;
            double Hd = (l2S - r.T / r.S) * kLn2;
            double p1d = exp2((double)r.M * (double)kLog2e - r.R) / r.S;
            double p2d = (a.V > 1) ? exp2((double)r.v2 * (double)kLog2e - r.R) / r.S : 0.0;
            lse = (float)lse_d; H = (float)(Hd > 0.0 ? Hd : 0.0);
            p1 = (float)p1d; p2 = (float)p2d; mg = (float)(p1d - p2d);
        }
        if (a.lse) a.lse[i] = lse;
        if (a.entropy) a.entropy[i] = H;
        if (a.p_top1) a.p_top1[i] = p1;
        if (a.p_top2) a.p_top2[i] = p2;
        if (a.margin) a.margin[i] = mg;
        if (a.top1_id) a.top1_id[i] = resolve_argmax(row, a.dtype, a.V, r.cand, r.M);
        if (a.draft_tok && a.logq_tok) {
            int32_t t = a.draft_tok[i];
            if (t < 0 || t >= a.V) { f |= TAPOUT_FLAG_BAD_TOKEN; a.logq_tok[i] = NAN; }
            else a.logq_tok[i] = (float)((double)load_elem_rt(row, a.dtype, t) - lse_d);
        }
        sh[k] = H; sh[K + k] = p1; sh[2 * K + k] = mg;
        if (f) atomicOr(&sh_flags, f);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (a.flags) a.flags[b] = sh_flags;
        if (a.arm) {
            int arm = a.arm[b];
            int ns = kb;
            bool stopped = false;
            for (int k = 0; k < kb; ++k) {
                bool fire = false;
                if (arm >= 0 && arm < a.n_arms)
                    fire = rule_fires(a.rule[arm], a.threshold[arm], sh[k], sh[K + k], sh[2 * K + k]);
                if (a.stop_fired) a.stop_fired[(int64_t)b * K + k] = fire ? 1 : 0;
                if (fire && !stopped) { ns = k + 1; stopped = true; }
            }
            if (a.n_stop) a.n_stop[b] = ns;
        }
    }
}

__global__ __launch_bounds__(kFinalBlock) void verify_finalize_kernel(VerifyFinalArgs a)
{
    extern __shared__ unsigned char sh_raw[];
    // per row k: accept decision (u8), argmax (i32), max (f32)
    int32_t *sh_top1 = (int32_t *)sh_raw;                  // [K+1]
    float *sh_max = (float *)(sh_top1 + (a.K + 1));        // [K+1]
    unsigned char *sh_acc = (unsigned char *)(sh_max + (a.K + 1));   // [K]
    __shared__ uint32_t sh_flags;
    const int b = blockIdx.x;
    const int K = a.K;
    int n = a.n_draft[b];
    uint32_t f0 = 0;
    if (n < 1 || n > K) { f0 |= TAPOUT_FLAG_BAD_NDRAFT; n = n < 1 ? 1 : K; }
    const bool greedy = a.greedy ? a.greedy[b] != 0 : false;
    if (threadIdx.x == 0) sh_flags = f0;
    __syncthreads();
    for (int k = threadIdx.x; k <= n; k += blockDim.x) {
        const int64_t it = (int64_t)b * (K + 1) + k;
        const void *row = row_address(a.tbase, a.t_dtype, a.t_stride_b, a.t_stride_k, b, k);
        RowTotal r = merge_partials(a.part + it * a.nsplit, a.nsplit);
        uint32_t f = 0;
        double lse_d = NAN;
        if (r.bad) f |= TAPOUT_FLAG_BAD_ROW;
        else lse_d = (r.R + log2(r.S)) * kLn2;
        int32_t top1 = resolve_argmax(row, a.t_dtype, a.V, r.cand, r.M);
        if (a.target_lse) a.target_lse[it] = (float)lse_d;
        if (a.target_top1) a.target_top1[it] = top1;
        sh_top1[k] = top1;
        sh_max[k] = r.M;
        if (k < n) {
            const int64_t i = (int64_t)b * K + k;
            int32_t t = a.draft_tok[i];
            bool acc = false;
            float lp = NAN;
            if (t < 0 || t >= a.V) f |= TAPOUT_FLAG_BAD_TOKEN;
            else if (!r.bad) {
                lp = (float)((double)load_elem_rt(row, a.t_dtype, t) - lse_d);
                if (greedy) acc = (t == top1);
                else acc = (double)a.u_accept[i] < exp((double)lp - (double)a.logq_tok[i]);
            }
            if (a.logp_tok) a.logp_tok[i] = lp;
            sh_acc[k] = acc ? 1 : 0;
        }
        if (f) atomicOr(&sh_flags, f);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t f = sh_flags;
        int m = 0;
        SampleJob job;
        job.kind = 0; job.row = 0; job.ref_p = 0.0f; job.ref_q = 0.0f;
        int32_t final_tok = -1;
        if (f & (TAPOUT_FLAG_BAD_NDRAFT | TAPOUT_FLAG_BAD_TOKEN | TAPOUT_FLAG_BAD_ROW)) {
            m = 0;
            final_tok = sh_top1[0];
            if (a.logp_tok)
                for (int k = 0; k < n; ++k) a.logp_tok[(int64_t)b * K + k] = NAN;
        } else {
            while (m < n && sh_acc[m]) ++m;
            if (greedy) final_tok = sh_top1[m];
            else {
                job.kind = m < n ? 1 : 2;
                job.row = m;
                job.ref_p = sh_max[m];
                job.ref_q = m < n ? a.draft_lse[(int64_t)b * K + m] : 0.0f;
            }
        }
        a.accept_len[b] = m;
        a.n_out[b] = m + 1;
        int32_t *o = a.out_tok + (int64_t)b * (K + 1);
        for (int k = 0; k <= K; ++k)
            o[k] = k < m ? a.draft_tok[(int64_t)b * K + k] : (k == m ? final_tok : -1);
        a.jobs[b] = job;
        a.flags_ws[b] = f;
        if (a.flags) a.flags[b] = f;
    }
}

}  // namespace

hipError_t launch_draft_finalize(const DraftFinalArgs &a, hipStream_t st)
{
    size_t shmem = (size_t)3 * a.K * sizeof(float);
    hipLaunchKernelGGL(draft_finalize_kernel, dim3(a.B), dim3(kFinalBlock), shmem, st, a);
    return hipGetLastError();
}

hipError_t launch_verify_finalize(const VerifyFinalArgs &a, hipStream_t st)
{
    size_t shmem = (size_t)(a.K + 1) * 8 + (size_t)a.K + 8;
    hipLaunchKernelGGL(verify_finalize_kernel, dim3(a.B), dim3(kFinalBlock), shmem, st, a);
    return hipGetLastError();
}

}  // namespace tapout
