// Device code of the draft epilogue (see finalize.hip), in a header because two kernels run it: the epilogue kernel
// of its own, and the final-token locate kernel of a whole-round call, whose launch carries the epilogue's
// workgroups beside its own.
#pragma once
#include <type_traits>

#include "common.h"

namespace tapout {

constexpr int kFinalBlock = 256;
static_assert(kFinalBlock == kBlock, "stage_partials strides by kBlock");

__device__ inline bool rule_fires(int rule, float h, float H, float p1, float margin)
{
    // decisions on the returned binary32 signals, widened to double (strict inequalities of Table 1)
    switch (rule) {
    case TAPOUT_RULE_SVIP:    return sqrt((double)H) > (double)h;
    case TAPOUT_RULE_MAXCONF: return (double)p1 < (double)h;
    default:                  return (double)margin < (double)h;
    }
}

// SVIP-Difference (Table 1): sqrt(H_t) - sqrt(H_{t-1}) > h; no previous entropy (NaN) or a bad row: no stop.
__device__ inline bool svip_diff_fires(float h, float H, float H_prev)
{
    if (H != H || H_prev != H_prev) return false;
    return sqrt((double)H) - sqrt((double)H_prev) > (double)h;
}

// AdaEDL (Table 1): 1 - sqrt(g H) < lambda.
__device__ inline bool adaedl_fires(double g, double lambda, float H)
{
    if (H != H) return false;
    return 1.0 - sqrt(g * (double)H) < lambda;
}

// The epilogue of sequence b; called by all kFinalBlock threads of a workgroup.
template <bool SHARDED>
__device__ inline void draft_finalize_body(const DraftFinalArgs &a, const int b)
{
    __shared__ Partial sh_part[kStageCap];
    __shared__ uint8_t sh_dec[kScanCap];
    __shared__ float sh_H[kScanCap];                           // entropies of the sequence (stateful rules only)
    __shared__ uint32_t sh_flags;
    const int K = a.K;
    // few rows and slices: one partial per thread, merged across lanes (see lane_merge_commit); else staged in LDS
    const int msh = SHARDED ? -1 : lane_merge_shift(K, a.nsplit);
    // The lane-parallel merge leaves the totals of all K <= 64 rows in LDS at once and row k with thread k: it is one
    // stage whatever the slice count.  The staged merge takes kStageCap partials at a time (nsplit <= kStageCap is
    // guaranteed by the host).
    const int rows_per_stage = msh >= 0 ? kWave : kStageCap / a.nsplit;
    const bool want_tok = a.draft_tok && a.logq_tok;
    static_assert(kFinalBlock == 256, "stage_issue / stage_commit assume 256 threads");
    // First memory round trip: k_len, the arm, the carried entropy, the drafted tokens and the partials, all
    // requested before anything is waited for.  (Rows beyond k_len hold stale partials and unused tokens:
    // read, never used.)  The empty asm keeps the compiler from sinking the small loads below the barrier.
    const bool tok_mode = a.arm_stride > 0;
    int kb = a.k_len ? a.k_len[b] : K;
    const int arm = (a.arm && !tok_mode) ? a.arm[b] : -1;     // sequence-level bandit: one arm for all steps
    float H_carry = a.prev_entropy ? a.prev_entropy[b] : NAN;
    int32_t tok0 = -1;
    if (want_tok && (int)threadIdx.x < K) tok0 = a.draft_tok[(int64_t)b * K + threadIdx.x];
    const int count0 = min(K, rows_per_stage) * a.nsplit;
    RowSlot *sh_rows = (RowSlot *)sh_part;
    static_assert(sizeof(RowSlot) * 64 <= sizeof(Partial) * kStageCap, "the row totals reuse the staging buffer");
    StageRegs st0;
    LaneRegs ln0;
    st0.w0 = st0.w1 = ln0.p[0].w0 = ln0.p[0].w1 = ln0.p[1].w0 = ln0.p[1].w1 = u32x4{0u, 0u, 0u, 0u};
    if constexpr (SHARDED) st0 = stage_issue_shards(a.part, (int64_t)a.B * K, (int64_t)b * K, a.nsplit, count0);
    else if (__builtin_expect(msh >= 0, 1)) ln0 = lane_merge_issue(a.part + (int64_t)b * K * a.nsplit, K, a.nsplit, msh);
    else st0 = stage_issue(a.part + (int64_t)b * K * a.nsplit, count0);
    asm volatile("" :: "v"(kb), "v"(arm), "v"(H_carry), "v"(tok0), "v"(st0.w0), "v"(st0.w1), "v"(ln0.p[0].w0), "v"(ln0.p[0].w1), "v"(ln0.p[1].w0), "v"(ln0.p[1].w1));
    kb = kb > K ? K : (kb < 0 ? 0 : kb);
    // Second round trip: the logit of the drafted token (its address needs the token, not k_len: rows up to K
    // exist) and, on the lane path, the left-out batch of this thread's (row, slice) pieces.
    float xtok_first = 0.0f;
    if constexpr (!SHARDED)
        if (want_tok && (int)threadIdx.x < K && tok0 >= 0 && tok0 < a.V)
            xtok_first = load_elem_rt(row_address(a.base, a.dtype, a.stride_b, a.stride_k, b, threadIdx.x), a.dtype, tok0);
    if (threadIdx.x == 0) sh_flags = 0;                       // ahead of the barrier in the commit: rows of other wavefronts OR into it
    if (__builtin_expect(msh >= 0, 1)) {
        Piece e[2];
        BatchRegs bt[2];
        const int sl = threadIdx.x & ((1 << msh) - 1);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int row = (threadIdx.x >> msh) + q * (256 >> msh);
            e[q] = lane_piece(ln0, q, kb, a.nsplit, msh);     // rows beyond k_len hold stale partials: empty pieces
            bt[q].valid = 0;
            if (q == 0 || (256 >> msh) < kb)                      // uniform; a thread without a piece asks for nothing (candidate -1)
                bt[q] = batch_issue(row_address(a.base, a.dtype, a.stride_b, a.stride_k, b, row), a.dtype, a.V,
                                    (row < kb && sl < a.nsplit) ? e[q].idx : -1, sl, a.per, a.part);
        }
        // While the batches travel, the pieces are merged as they are.  Then every lane adds what its own batch holds
        // besides the first maximum: rescaled to the row's reference, summed over the row's lanes (binary32: small
        // terms, a fixed butterfly), together with the exact index of the row's first maximum from the lane that won.
        const bool two = (256 >> msh) < kb;                     // uniform
        Piece m[2];
        m[0] = lane_group_merge<true>(e[0], msh);
        if (two) m[1] = lane_group_merge<true>(e[1], msh);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            if (q == 1 && !two) break;
            const BatchExtra x = batch_extra(e[q], bt[q], a.dtype);
            const float d = ref_of_max(m[q].M) - ref_of_max(e[q].M);              // >= 0 for a piece that holds anything
            const int di = (int)fminf(fmaxf(d, -1.0e9f), 1.0e9f);
            float sa = ldexpf(x.sa, -di), ta = ldexpf(x.ta - d * x.sa, -di);
            if (x.sa == 0.0f) { sa = 0.0f; ta = 0.0f; }                           // empty piece or empty batch (0 * inf)
            int32_t idx = (e[q].M == m[q].M && e[q].idx == m[q].idx) ? x.idx : 0x7fffffff;
            auto step = [&](auto ctrl) {
                constexpr int C = decltype(ctrl)::value;
                sa += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(sa), C, 0xf, 0xf, true));
                ta += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(ta), C, 0xf, 0xf, true));
                idx = min(idx, __builtin_amdgcn_update_dpp(0, idx, C, 0xf, 0xf, true));
            };
            if (msh >= 1) step(std::integral_constant<int, 0xB1>{});
            if (msh >= 2) step(std::integral_constant<int, 0x4E>{});
            if (msh >= 3) step(std::integral_constant<int, 0x141>{});
            if (msh >= 4) step(std::integral_constant<int, 0x140>{});
            const int row = (threadIdx.x >> msh) + q * (256 >> msh);
            if (row < kb && sl == 0) {
                Piece f = m[q];
                f.S += (double)sa; f.T += (double)ta; f.idx = idx;
                RowSlot o;
                o.r = row_total<true>(f);
                o.xt = f.xt;
                sh_rows[row] = o;
            }
        }
        __syncthreads();
    } else {
        stage_commit(sh_part, st0, count0);
    }
    // Staged path: the `count` partials of rows k0.. lie in LDS; every thread completes some of them (left-out batch
    // back in, exact index of the first maximum into the cand slot) before the rows are merged one by one.
    auto complete_stage = [&](int k0, int count) {
        if constexpr (!SHARDED) {
            for (int i = threadIdx.x; i < count; i += kFinalBlock) {
                const int k = k0 + i / a.nsplit, sl = i % a.nsplit;
                if (k >= kb) continue;                          // stale partial of a row that was not drafted
                Piece e = piece_from_partial(sh_part[i]);
                const BatchRegs bt = batch_issue(row_address(a.base, a.dtype, a.stride_b, a.stride_k, b, k), a.dtype, a.V, e.idx, sl, a.per, a.part);
                batch_fix(e, bt, a.dtype);
                sh_part[i].S = (float)e.S; sh_part[i].T = (float)e.T; sh_part[i].cand = e.idx;
            }
            __syncthreads();
        }
    };
    if (__builtin_expect(msh < 0, 0)) complete_stage(0, count0);
    const bool arm_ok = arm >= 0 && arm < a.n_arms;
    const int rule_b = arm_ok ? pick8(a.rule, arm) : -1;
    // rows whose rule looks beyond their own signals are decided in a second sweep (uniform over the workgroup);
    // token-level bandits: the arm of step k is arm[b, k]
    const bool sweep = tok_mode ? (a.round_entropy != nullptr)
                                : (rule_b == TAPOUT_RULE_SVIP_DIFF || rule_b == TAPOUT_RULE_ADAEDL);
    bool fire_mine = false; uint32_t f_mine = 0;      // this thread's row: rule fired, flags (used on the lane-merge path)
    for (int k0 = 0; k0 < kb; k0 += rows_per_stage) {
        const int k1 = min(kb, k0 + rows_per_stage);
        const int kmine = k0 + threadIdx.x;                   // first (usually only) row of this thread in the stage
        float xtok0 = xtok_first;
        if (__builtin_expect(k0 > 0, 0)) {                                         // further stages (K > rows_per_stage): load late
            tok0 = (want_tok && kmine < k1) ? a.draft_tok[(int64_t)b * K + kmine] : -1;
            __syncthreads();
            if constexpr (SHARDED) {
                stage_commit(sh_part, stage_issue_shards(a.part, (int64_t)a.B * K, (int64_t)b * K + k0, a.nsplit, (k1 - k0) * a.nsplit),
                             (k1 - k0) * a.nsplit);
            } else {
                stage_partials(sh_part, a.part + ((int64_t)b * K + k0) * a.nsplit, (k1 - k0) * a.nsplit);
                complete_stage(k0, (k1 - k0) * a.nsplit);
            }
            xtok0 = 0.0f;
            if constexpr (!SHARDED)
                if (want_tok && kmine < k1 && tok0 >= 0 && tok0 < a.V)
                    xtok0 = load_elem_rt(row_address(a.base, a.dtype, a.stride_b, a.stride_k, b, kmine), a.dtype, tok0);
        }
        for (int k = kmine; k < k1; k += kFinalBlock) {
            const int64_t i = (int64_t)b * K + k;
            const void *row = SHARDED ? nullptr : row_address(a.base, a.dtype, a.stride_b, a.stride_k, b, k);
            const RowTotal r = msh >= 0 ? sh_rows[k].r : merge_partials<true>(sh_part + (k - k0) * a.nsplit, a.nsplit);
            const int32_t top1 = (r.cand >= 0 && r.cand < a.V) ? r.cand : 0;                      // exact: the pieces carry the index of their first maximum
            uint32_t f = 0;
            float lse, H, p1, p2, mg;
            double lse_d = NAN;
            if (__builtin_expect(r.bad, 0)) {
                f |= TAPOUT_FLAG_BAD_ROW;
                lse = H = p1 = p2 = mg = NAN;
            } else {
                const RowSignals g = row_signals(r, a.V > 1);
                lse_d = g.lse;
                lse = (float)g.lse; H = (float)g.H;
                p1 = (float)g.p1; p2 = (float)g.p2; mg = (float)g.margin;
            }
            if (a.lse) a.lse[i] = lse;
            if (a.entropy) a.entropy[i] = H;
            if (a.p_top1) a.p_top1[i] = p1;
            if (a.p_top2) a.p_top2[i] = p2;
            if (a.margin) a.margin[i] = mg;
            if (a.top1_id) a.top1_id[i] = top1;
            if (a.draft_tok && a.logq_tok) {
                int32_t t = tok0;
                float xt = xtok0;
                if (k != kmine) t = a.draft_tok[i];            // more rows than threads: load late
                if constexpr (SHARDED) {
                    // the shard that owns the token sent its logit; the others sent NaN
                    xt = NAN;
                    for (int g = 0; g < a.nsplit; ++g) {
                        const float v = __int_as_float(sh_part[(k - k0) * a.nsplit + g].pad[0]);
                        if (v == v) xt = v;
                    }
                } else if (k != kmine) {
                    if (t >= 0 && t < a.V) xt = load_elem_rt(row, a.dtype, t);
                }
                if (t < 0 || t >= a.V) { f |= TAPOUT_FLAG_BAD_TOKEN; a.logq_tok[i] = NAN; }
                else a.logq_tok[i] = (float)((double)xt - lse_d);
            }
            if (a.round_entropy) a.round_entropy[i] = H;
            if (a.arm) {
                const int arm_k = tok_mode ? a.arm[(int64_t)b * a.arm_stride + k] : arm;
                const bool ok_k = arm_k >= 0 && arm_k < a.n_arms;
                const int rule_k = ok_k ? pick8(a.rule, arm_k) : -1;
                if (sweep) sh_H[k] = H;
                if (rule_k == TAPOUT_RULE_SVIP_DIFF || rule_k == TAPOUT_RULE_ADAEDL) {
                    sh_dec[k] = 2;                             // decided below, once every row's entropy is known
                } else {
                    const bool fire = ok_k && rule_fires(rule_k, pick8(a.threshold, arm_k), H, p1, mg);
                    if (a.stop_fired) a.stop_fired[i] = fire ? 1 : 0;
                    sh_dec[k] = fire ? 1 : 0;                  // k < K <= kScanCap
                    fire_mine = fire;
                }
            }
            f_mine = f;
            if (f) atomicOr(&sh_flags, f);
        }
    }
    if (__builtin_expect(msh >= 0 && !sweep, 1)) {
        // Lane-merge path without a second sweep: row k was thread k's, so the rows are lanes of the first wavefront
        // and ballots give the stop position and the flags; no barrier, no scan through LDS.
        if (threadIdx.x < kWave) {
            const uint64_t fired = __builtin_amdgcn_ballot_w64((int)threadIdx.x < kb && fire_mine);
            uint32_t fa = 0;
            if (__builtin_amdgcn_ballot_w64((f_mine & TAPOUT_FLAG_BAD_ROW) != 0)) fa |= TAPOUT_FLAG_BAD_ROW;
            if (__builtin_amdgcn_ballot_w64((f_mine & TAPOUT_FLAG_BAD_TOKEN) != 0)) fa |= TAPOUT_FLAG_BAD_TOKEN;
            if (threadIdx.x == 0) {
                if (a.flags) a.flags[b] = fa;
                if (a.arm && a.n_stop) a.n_stop[b] = fired ? __builtin_ctzll(fired) + 1 : kb;
            }
        }
        return;
    }
    __syncthreads();                       // orders the LDS / scratch writes above before the scan
    if (__builtin_expect(sweep, 0)) {
        for (int k = threadIdx.x; k < kb; k += kFinalBlock) {
            if (sh_dec[k] != 2) continue;
            const int arm_k = tok_mode ? a.arm[(int64_t)b * a.arm_stride + k] : arm;      // in range: checked when it was marked
            const float H = sh_H[k];
            bool fire;
            if (pick8(a.rule, arm_k) == TAPOUT_RULE_SVIP_DIFF) {
                fire = svip_diff_fires(pick8(a.threshold, arm_k), H, k > 0 ? sh_H[k - 1] : H_carry);
            } else {
                const double lam = a.lambda ? a.lambda[(int64_t)b * a.n_arms + arm_k] : (double)pick8(a.threshold, arm_k);
                fire = adaedl_fires(a.adaedl_gamma, lam, H);
            }
            if (a.stop_fired) a.stop_fired[(int64_t)b * K + k] = fire ? 1 : 0;
            sh_dec[k] = fire ? 1 : 0;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        if (a.flags) a.flags[b] = sh_flags;
        if (a.arm && a.n_stop) {
            int ns = kb;
            for (int k = 0; k < kb; ++k) {
                if (sh_dec[k] != 0) { ns = k + 1; break; }
            }
            a.n_stop[b] = ns;
        }
    }
}

}  // namespace tapout
