// Verification of the drafted tokens and the final token (Algorithm 1, lines
// 10-11; "verify" = speculative sampling as in the works the paper cites).
//
// After the streaming pass over the target rows (row_reduce.hip) three small
// launches finish the job:
//
//   pass 1  head: every workgroup of a sequence merges the target partials,
//           forms log p(tok), takes the accept decisions u < p(tok)/q(tok) and
//           finds the first rejection m (slice 0 writes the outputs); then it
//           sums its slice of e_p = exp(t - ref_p), e_q = exp(d - ref_q) of
//           the row pair (m, m) the final token is drawn from
//   pass 2  slice sums of w = max(0, e_p/S_p - e_q/S_q)   (or e_p/S_p: bonus token)
//   pass 3  one workgroup per sequence: scan the slice sums, then a block scan
//           inside the slice that contains u * Z: token = smallest j whose
//           inclusive prefix sum exceeds u * Z
//
// Passes 1-3 are double precision.  With ~1e5 CDF cell edges in [0,1) a binary32
// evaluation would move an edge across u for about one draw in a hundred; in
// double the chance is ~1e-11, so the token agrees with a sequential fp64
// evaluation.  Only one row pair per sequence is touched (2/(2K+1) of the
// round's logits).  exp() is evaluated as 2^(n/256) * (1 + r + r^2/2 + r^3/6),
// |r| <= ln2/512, with a 256-entry table in LDS: relative error < 2e-13, far
// inside what the 1e-9 decision margin needs, at a third of the instructions of
// a correctly rounded exp.
#include "common.h"

namespace tapout {

namespace {

constexpr int kVBlock = 256;
constexpr int kPer = 8;                       // consecutive elements per thread: kSampleSlice = kVBlock * kPer
static_assert(kVBlock * kPer == kSampleSlice, "slice = one 8-element run per thread");

// ---- double-precision helpers ---------------------------------------------------
__device__ inline double exp_tab(double y, const double *T)
{
    // y <= ~0 in all uses; anything below -745 is 0 in double anyway
    y = fmax(y, -800.0);
    const double t = y * 369.3299304675746;                 // 256 / ln 2
    const double n = rint(t);
    const double r = fma(n, -0.0027076061740622863, y);      // y - n * ln2/256
    const int ni = (int)n;
    const double tk = T[ni & 255];
    const double q = r * fma(r, fma(r, 1.0 / 6.0, 0.5), 1.0);
    return ldexp(fma(tk, q, tk), ni >> 8);
}

__device__ inline double wave_sum_d(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// Sum over the workgroup in a fixed order (same result in every workgroup that sums the same values).
__device__ inline double block_sum_d(double v, double *sh4)
{
    v = wave_sum_d(v);
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) sh4[threadIdx.x / kWave] = v;
    __syncthreads();
    return (sh4[0] + sh4[1]) + (sh4[2] + sh4[3]);
}

// Inclusive scan over the workgroup of one double per thread; returns the exclusive prefix of this
// thread, the workgroup total through *total.
__device__ inline double block_excl_scan_d(double v, double *sh4, double *total)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    double inc = v;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        double up = __shfl_up(inc, o, kWave);
        if (lane >= o) inc += up;
    }
    __syncthreads();
    if (lane == kWave - 1) sh4[wave] = inc;
    __syncthreads();
    double base = 0.0;
    for (int w2 = 0; w2 < wave; ++w2) base += sh4[w2];
    *total = ((sh4[0] + sh4[1]) + sh4[2]) + sh4[3];
    return base + (inc - v);
}

// Eight consecutive elements j .. j+7 of a row, exact in binary32; -inf beyond V.
template <int DT>
__device__ inline void load8(const char *rowp, bool aligned, int j, int V, float (&x)[kPer])
{
    if (aligned && j + kPer <= V) {
        if constexpr (DT == TAPOUT_BF16) {
            u32x4 w = *(const u32x4 *)(rowp + (int64_t)j * 2);
            unpack<TAPOUT_BF16>(w, x);
        } else {
            u32x4 w0 = *(const u32x4 *)(rowp + (int64_t)j * 4), w1 = *(const u32x4 *)(rowp + (int64_t)j * 4 + 16);
            float lo[4], hi[4];
            unpack<TAPOUT_F32>(w0, lo); unpack<TAPOUT_F32>(w1, hi);
#pragma unroll
            for (int i = 0; i < 4; ++i) { x[i] = lo[i]; x[4 + i] = hi[i]; }
        }
    } else {
#pragma unroll
        for (int i = 0; i < kPer; ++i) x[i] = (j + i < V) ? load_elem<DT>(rowp, j + i) : -INFINITY;
    }
}

struct Weights {
    int kind;          // 1 residual max(0, p - q), 2 target row only
    double ref_p, ref_q, inv_Sp, inv_Sq;
};

// The eight weights of this thread in slice `s` (elements s*kSampleSlice + tid*8 ..).
template <int TD, int DD>
__device__ inline void thread_weights(const Weights &w, const char *trow, bool t_al, const char *drow, bool d_al,
                                      int s, int V, const double *T, double (&wv)[kPer])
{
    const int j = s * kSampleSlice + threadIdx.x * kPer;
    float xt[kPer], xd[kPer];
    load8<TD>(trow, t_al, j, V, xt);
    if (w.kind == 1) load8<DD>(drow, d_al, j, V, xd);
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        double p = exp_tab((double)xt[i] - w.ref_p, T) * w.inv_Sp;
        if (w.kind == 1) {
            double q = exp_tab((double)xd[i] - w.ref_q, T) * w.inv_Sq;
            p = p - q;
            p = p > 0.0 ? p : 0.0;
        }
        wv[i] = p;
    }
}

__device__ inline void load_table(double *shT, const double *T)
{
    for (int i = threadIdx.x; i < 256; i += blockDim.x) shT[i] = T[i];
    __syncthreads();
}

// ---- head: accept decisions of one sequence -----------------------------------------
// Called by all threads of a workgroup.  Returns the sequence's job (identical in every
// workgroup of the sequence); with `writer` also writes the sequence's outputs.
// Accept decisions exist for rows k < n <= K <= kScanCap, so the LDS byte buffer always holds them.
__device__ inline SampleJob verify_head(const VerifyArgs &a, int b, bool writer,
                                        Partial *sh_part, uint8_t *sh_dec, uint32_t *sh_flags, int32_t *sh_bcast)
{
    const int K = a.K;
    int n = a.n_draft[b];
    uint32_t f0 = 0;
    if (n < 1 || n > K) { f0 |= TAPOUT_FLAG_BAD_NDRAFT; n = n < 1 ? 1 : K; }
    const bool greedy = a.greedy ? a.greedy[b] != 0 : false;
    SampleJob job;
    job.kind = 0; job.row = 0; job.ref_p = 0.0f; job.ref_q = 0.0f;
    if (greedy && !writer) return job;           // greedy sequences have nothing to sample
    if (threadIdx.x == 0) { *sh_flags = f0; sh_bcast[4] = 0; }
    const bool need_top1 = writer || greedy;
    int last_k = -1; float last_M = 0.0f; int32_t last_top1 = 0;     // the last row this thread merged
    const int rows_per_stage = kStageCap / a.nsplit;
    for (int k0 = 0; k0 <= n; k0 += rows_per_stage) {
        const int k1 = min(n + 1, k0 + rows_per_stage);
        // loads that do not depend on the partials go out first
        const int kmine = k0 + threadIdx.x;
        int32_t tok0 = -1;
        float xtok0 = 0.0f, u0 = 0.0f, lq0 = 0.0f;
        if (kmine < k1 && kmine < n) {
            const int64_t i = (int64_t)b * K + kmine;
            tok0 = a.draft_tok[i];
            u0 = a.u_accept[i];
            lq0 = a.logq_tok[i];
            if (tok0 >= 0 && tok0 < a.V)
                xtok0 = load_elem_rt(row_address(a.tbase, a.t_dtype, a.t_stride_b, a.t_stride_k, b, kmine), a.t_dtype, tok0);
        }
        __syncthreads();
        stage_partials(sh_part, a.part + ((int64_t)b * (K + 1) + k0) * a.nsplit, (k1 - k0) * a.nsplit);
        for (int k = kmine; k < k1; k += blockDim.x) {
            const int64_t it = (int64_t)b * (K + 1) + k;
            const void *row = row_address(a.tbase, a.t_dtype, a.t_stride_b, a.t_stride_k, b, k);
            RowTotal r = merge_partials(sh_part + (k - k0) * a.nsplit, a.nsplit);
            const int32_t top1 = need_top1 ? resolve_argmax(row, a.t_dtype, a.V, r.cand, r.M) : 0;   // loads overlap the math below
            uint32_t f = 0;
            double lse_d = NAN;
            if (r.bad) f |= TAPOUT_FLAG_BAD_ROW;
            else lse_d = (r.R + log2(r.S)) * kLn2;
            if (writer) {
                if (a.target_lse) a.target_lse[it] = (float)lse_d;
                if (a.target_top1) a.target_top1[it] = top1;
            }
            if (k < n) {
                const int64_t i = (int64_t)b * K + k;
                int32_t t = tok0;
                float xt = xtok0, u = u0, lq = lq0;
                if (k != kmine) {                              // more rows than threads: load late
                    t = a.draft_tok[i]; u = a.u_accept[i]; lq = a.logq_tok[i];
                    if (t >= 0 && t < a.V) xt = load_elem_rt(row, a.t_dtype, t);
                }
                bool acc = false;
                float lp = NAN;
                if (t < 0 || t >= a.V) f |= TAPOUT_FLAG_BAD_TOKEN;
                else if (!r.bad) {
                    lp = (float)((double)xt - lse_d);
                    if (greedy) acc = (t == top1);
                    else acc = (double)u < exp((double)lp - (double)lq);
                }
                if (writer && a.logp_tok) a.logp_tok[i] = lp;
                sh_dec[k] = acc ? 1 : 0;
            }
            last_k = k; last_M = r.M; last_top1 = top1;
            if (f) atomicOr(sh_flags, f);
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t f = *sh_flags;
        const bool flagged = f & (TAPOUT_FLAG_BAD_NDRAFT | TAPOUT_FLAG_BAD_TOKEN | TAPOUT_FLAG_BAD_ROW);
        int m = 0;
        if (!flagged)
            while (m < n && sh_dec[m] != 0) ++m;
        sh_bcast[0] = m;
        sh_bcast[1] = flagged ? 1 : 0;
        sh_bcast[2] = (int32_t)f;
    }
    __syncthreads();
    const int m = sh_bcast[0];                   // a flagged sequence has m = 0 and emits the argmax of row 0
    const bool flagged = sh_bcast[1] != 0;
    const uint32_t f = (uint32_t)sh_bcast[2];
    // maximum and argmax of row m: from the thread that merged it, if it still holds them
    if (last_k == m) { sh_bcast[4] = 1; sh_bcast[5] = __float_as_int(last_M); sh_bcast[6] = last_top1; }
    __syncthreads();
    float Mm; int32_t top1m;
    if (sh_bcast[4]) {
        Mm = __int_as_float(sh_bcast[5]); top1m = sh_bcast[6];
    } else {                                     // more rows than threads: merge row m once more
        __syncthreads();
        stage_partials(sh_part, a.part + ((int64_t)b * (K + 1) + m) * a.nsplit, a.nsplit);
        RowTotal r = merge_partials(sh_part, a.nsplit);
        Mm = r.M;
        top1m = need_top1 ? resolve_argmax(row_address(a.tbase, a.t_dtype, a.t_stride_b, a.t_stride_k, b, m), a.t_dtype, a.V, r.cand, r.M) : 0;
    }
    if (!flagged && !greedy) {
        job.kind = m < n ? 1 : 2;
        job.row = m;
        job.ref_p = Mm;                          // exponent references: the target row's maximum, the draft row's lse
        job.ref_q = m < n ? a.draft_lse[(int64_t)b * K + m] : 0.0f;
    }
    if (writer) {
        const int32_t final_tok = (flagged || greedy) ? top1m : -1;   // sampled sequences: written by pass 3
        if (threadIdx.x == 0) {
            a.accept_len[b] = m;
            a.n_out[b] = m + 1;
            a.jobs[b] = job;
            a.flags_ws[b] = f;
            if (a.flags) a.flags[b] = f;
        }
        int32_t *o = a.out_tok + (int64_t)b * (K + 1);
        for (int k = threadIdx.x; k <= K; k += blockDim.x) {
            o[k] = k < m ? a.draft_tok[(int64_t)b * K + k] : (k == m ? final_tok : -1);
            if (flagged && a.logp_tok && k < n) a.logp_tok[(int64_t)b * K + k] = NAN;
        }
    }
    return job;
}

struct Rows {
    const char *trow, *drow;
    bool t_al, d_al;
};

template <int TD, int DD>
__device__ inline Rows job_rows(const VerifyArgs &a, int b, const SampleJob &job)
{
    Rows r;
    r.trow = (const char *)row_address(a.tbase, TD, a.t_stride_b, a.t_stride_k, b, job.row);
    r.drow = (const char *)row_address(a.dbase, DD, a.d_stride_b, a.d_stride_k, b, job.kind == 1 ? job.row : 0);
    r.t_al = ((uintptr_t)r.trow & 15u) == 0;
    r.d_al = ((uintptr_t)r.drow & 15u) == 0;
    return r;
}

// ---- pass 1 ----------------------------------------------------------------------
template <int TD, int DD>
__global__ __launch_bounds__(kVBlock) void verify_pass1(VerifyArgs a)
{
    __shared__ Partial sh_part[kStageCap];
    __shared__ uint8_t sh_dec[kScanCap];
    __shared__ uint32_t sh_flags;
    __shared__ int32_t sh_bcast[8];
    __shared__ double shT[256];
    __shared__ double sh4[4];
    const int b = blockIdx.y, s = blockIdx.x;
    const SampleJob job = verify_head(a, b, s == 0, sh_part, sh_dec, &sh_flags, sh_bcast);
    if (job.kind == 0) return;
    load_table(shT, a.exp_table);
    const Rows r = job_rows<TD, DD>(a, b, job);
    const int j = s * kSampleSlice + threadIdx.x * kPer;
    const double ref_p = (double)job.ref_p, ref_q = (double)job.ref_q;
    float xt[kPer], xd[kPer];
    load8<TD>(r.trow, r.t_al, j, a.V, xt);
    if (job.kind == 1) load8<DD>(r.drow, r.d_al, j, a.V, xd);
    double sp = 0.0, sq = 0.0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        sp += exp_tab((double)xt[i] - ref_p, shT);
        if (job.kind == 1) sq += exp_tab((double)xd[i] - ref_q, shT);
    }
    sp = block_sum_d(sp, sh4);
    sq = block_sum_d(sq, sh4);
    if (threadIdx.x == 0) {
        a.part1[((int64_t)b * a.nsl + s) * 2 + 0] = sp;
        a.part1[((int64_t)b * a.nsl + s) * 2 + 1] = sq;
    }
}

// Normalisers of the sequence from the slice sums of pass 1: every workgroup adds the same numbers
// in the same order.  A draft row whose sum is not a positive finite number cannot be resampled
// from: the draw then comes from the target row alone.
__device__ inline Weights make_weights(const VerifyArgs &a, const SampleJob &job, int b, double *sh4, bool *draft_bad)
{
    double sp = 0.0, sq = 0.0;
    for (int s = threadIdx.x; s < a.nsl; s += blockDim.x) {
        sp += a.part1[((int64_t)b * a.nsl + s) * 2 + 0];
        sq += a.part1[((int64_t)b * a.nsl + s) * 2 + 1];
    }
    const double Sp = block_sum_d(sp, sh4);
    const double Sq = block_sum_d(sq, sh4);
    Weights w;
    w.kind = job.kind;
    w.ref_p = (double)job.ref_p; w.ref_q = (double)job.ref_q;
    w.inv_Sp = 1.0 / Sp;
    w.inv_Sq = 1.0 / Sq;
    *draft_bad = false;
    if (job.kind == 1 && (!(Sq > 0.0) || !(Sq < INFINITY))) {
        w.kind = 2;
        *draft_bad = true;
    }
    return w;
}

// ---- pass 2 ----------------------------------------------------------------------
template <int TD, int DD>
__global__ __launch_bounds__(kVBlock) void verify_pass2(VerifyArgs a)
{
    __shared__ double shT[256];
    __shared__ double sh4[4];
    const int b = blockIdx.y, s = blockIdx.x;
    const SampleJob job = a.jobs[b];
    if (job.kind == 0) return;
    load_table(shT, a.exp_table);
    bool draft_bad;
    const Weights w = make_weights(a, job, b, sh4, &draft_bad);
    const Rows r = job_rows<TD, DD>(a, b, job);
    double wv[kPer];
    thread_weights<TD, DD>(w, r.trow, r.t_al, r.drow, r.d_al, s, a.V, shT, wv);
    double z = 0.0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) z += wv[i];
    z = block_sum_d(z, sh4);
    if (threadIdx.x == 0) a.part2[(int64_t)b * a.nsl + s] = z;
}

// ---- pass 3 ----------------------------------------------------------------------
// Locate inside slice s: first element whose running sum (starting at `cum`) exceeds `target`.
// Returns the element index or -1; *last_pos collects the largest index with positive weight seen.
template <int TD, int DD>
__device__ inline int locate_in_slice(const Weights &w, const Rows &r, int s, int V, const double *shT,
                                      double cum, double target, double *sh4, int *sh_hit, int *last_pos, double *slice_total)
{
    double wv[kPer];
    thread_weights<TD, DD>(w, r.trow, r.t_al, r.drow, r.d_al, s, V, shT, wv);
    double sum = 0.0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) sum += wv[i];
    const double excl = block_excl_scan_d(sum, sh4, slice_total);
    if (threadIdx.x == 0) *sh_hit = 0x7fffffff;
    __syncthreads();
    const int j0 = s * kSampleSlice + threadIdx.x * kPer;
    double c = cum + excl;
    int hit = 0x7fffffff, lp = -1;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        c += wv[i];
        if (wv[i] > 0.0) lp = j0 + i;
        if (hit == 0x7fffffff && j0 + i < V && c > target) hit = j0 + i;
    }
    if (hit != 0x7fffffff) atomicMin(sh_hit, hit);
    if (lp >= 0) atomicMax(last_pos, lp);
    __syncthreads();
    const int h = *sh_hit;
    __syncthreads();
    return h == 0x7fffffff ? -1 : h;
}

template <int TD, int DD>
__global__ __launch_bounds__(kVBlock) void verify_pass3(VerifyArgs a)
{
    __shared__ double shT[256];
    __shared__ double sh4[4];
    __shared__ int sh_hit, sh_last, sh_slice;
    const int b = blockIdx.x;
    const SampleJob job = a.jobs[b];
    if (job.kind == 0) return;
    load_table(shT, a.exp_table);
    bool draft_bad;
    Weights w = make_weights(a, job, b, sh4, &draft_bad);
    const Rows r = job_rows<TD, DD>(a, b, job);
    if (threadIdx.x == 0) { sh_last = -1; sh_slice = 0x7fffffff; }
    __syncthreads();
    const double u = (double)a.u_sample[b];
    double *zs = a.part2 + (int64_t)b * a.nsl;

    // total weight (fixed order), then the slice that holds u * Z
    double zt = 0.0;
    for (int s = threadIdx.x; s < a.nsl; s += blockDim.x) zt += zs[s];
    double Z = block_sum_d(zt, sh4);
    if (!(Z > 0.0) && w.kind == 1) {
        // the residual vanished (p == q up to rounding): draw from the target row itself
        w.kind = 2;
        __syncthreads();
        for (int s = 0; s < a.nsl; ++s) {
            double wv[kPer];
            thread_weights<TD, DD>(w, r.trow, r.t_al, r.drow, r.d_al, s, a.V, shT, wv);
            double z = 0.0;
#pragma unroll
            for (int i = 0; i < kPer; ++i) z += wv[i];
            z = block_sum_d(z, sh4);
            if (threadIdx.x == 0) zs[s] = z;
        }
        __threadfence_block();
        __syncthreads();
        zt = 0.0;
        for (int s = threadIdx.x; s < a.nsl; s += blockDim.x) zt += zs[s];
        Z = block_sum_d(zt, sh4);
    }
    int token = -1;
    if (Z > 0.0) {
        const double target = u * Z;
        // prefix over the slice sums, 256 slices at a time
        double carry = 0.0, cum_at = 0.0;
        int s_found = -1;
        for (int s0 = 0; s0 < a.nsl && s_found < 0; s0 += kVBlock) {
            const int s = s0 + threadIdx.x;
            const double v = s < a.nsl ? zs[s] : 0.0;
            double tot;
            const double excl = block_excl_scan_d(v, sh4, &tot);
            if (s < a.nsl && carry + excl + v > target) atomicMin(&sh_slice, s);
            __syncthreads();
            const int sf = sh_slice;
            if (sf != 0x7fffffff) {
                s_found = sf;
                // every thread needs the prefix in front of slice sf: the owning thread publishes it
                if (s == sf) sh4[0] = carry + excl;
                __syncthreads();
                cum_at = sh4[0];
                __syncthreads();
            }
            carry += tot;
        }
        // slice sums and the in-slice scan round differently: if the crossing is not inside the chosen
        // slice, continue into the following ones
        if (s_found >= 0) {
            double cum = cum_at;
            for (int s = s_found; s < a.nsl && token < 0; ++s) {
                double slice_total;
                token = locate_in_slice<TD, DD>(w, r, s, a.V, shT, cum, target, sh4, &sh_hit, &sh_last, &slice_total);
                cum += slice_total;
            }
        }
        if (token < 0) {
            // rounding left no crossing: the largest index with positive weight
            __syncthreads();
            if (sh_last < 0) {
                for (int s = 0; s < a.nsl; ++s) {
                    double slice_total;
                    locate_in_slice<TD, DD>(w, r, s, a.V, shT, 0.0, INFINITY, sh4, &sh_hit, &sh_last, &slice_total);
                }
                __syncthreads();
            }
            token = sh_last;
        }
    }
    if (threadIdx.x == 0) {
        if (token < 0) token = 0;
        a.out_tok[(int64_t)b * (a.K + 1) + job.row] = token;
        if (draft_bad) {
            uint32_t f = a.flags_ws[b] | TAPOUT_FLAG_BAD_ROW;
            a.flags_ws[b] = f;
            if (a.flags) a.flags[b] = f;
        }
    }
}

template <int TD, int DD>
hipError_t launch_typed(const VerifyArgs &a, int pass, hipStream_t st)
{
    dim3 grid12(a.nsl, a.B), block(kVBlock);
    if (pass == 1) hipLaunchKernelGGL((verify_pass1<TD, DD>), grid12, block, 0, st, a);
    else if (pass == 2) hipLaunchKernelGGL((verify_pass2<TD, DD>), grid12, block, 0, st, a);
    else hipLaunchKernelGGL((verify_pass3<TD, DD>), dim3(a.B), block, 0, st, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_verify(const VerifyArgs &a, int pass, hipStream_t st)
{
    if (a.t_dtype == TAPOUT_F32)
        return a.d_dtype == TAPOUT_F32 ? launch_typed<TAPOUT_F32, TAPOUT_F32>(a, pass, st) : launch_typed<TAPOUT_F32, TAPOUT_BF16>(a, pass, st);
    return a.d_dtype == TAPOUT_F32 ? launch_typed<TAPOUT_BF16, TAPOUT_F32>(a, pass, st) : launch_typed<TAPOUT_BF16, TAPOUT_BF16>(a, pass, st);
}

}  // namespace tapout
