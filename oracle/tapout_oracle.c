/*
 * CPU oracle for the per-round logits path of TapOut (dynamic speculative
 * decoding with a bandit over training-free stop rules).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, fp64 statement of
 * what the GPU library must compute, written from the paper's definitions:
 *
 *   - draft-distribution signals and stop rules ....... Table 1, Appendix A.1
 *   - the draft / stop / verify / final-token round ... Algorithm 1
 *   - speculative-sampling verification ............... Algorithm 1 "Verify X
 *     with M_p" as defined by the speculative-sampling works the Introduction
 *     cites: accept x with probability min(1, p(x)/q(x)); at the first
 *     rejection draw from normalise(max(0, p - q)); if nothing is rejected
 *     draw the extra token from the next target distribution
 *   - blended reward ................................... Section 3.2
 *   - UCB1 and Thompson Sampling ....................... Section 3.3
 *
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may call
 * it.  It shares no code, table or constant with the HIP path.  Every sum is a
 * sequential index-order loop in double precision; there is no blocking or
 * fusion.  OpenMP is used only ACROSS independent rows / sequences (the
 * arithmetic inside one row is untouched by the thread count).
 *
 * Parity pins (tests/test_oracle_*.py): closed-form rows (uniform, two- and
 * three-point), library cross-checks of the row statistics, threshold edges,
 * exact enumeration of the speculative-sampling output law on tiny
 * vocabularies, UCB1 and reward hand cases, Gamma/Beta sampler moments,
 * closed-form rows for SVIPDifference / AdaEDL, the empirical variance of
 * UCB-Tuned against a two-pass library variance, Gaussian posterior moments.
 * Every function in this file is covered by at least one of those pins,
 * except the VALUES of AdaEDL's hyper-parameters and the exact form of its
 * threshold update, which the paper prints garbled: PARITY UNPINNED for
 * those (the arithmetic of the reading taken here is pinned by closed
 * forms; whether it is the authors' reading cannot be).
 *
 * Conventions shared with the boundary (they are the boundary's, restated
 * here, not imported from it):
 *   dtype 0 = IEEE binary32 logits, dtype 1 = bfloat16 logits (upper 16 bits
 *   of a binary32); both widen exactly to double.
 *   rule 0 = SVIP (sqrt(H) > h), 1 = Max-Confidence (p_top1 < h),
 *   rule 2 = LogitMargin (p_top1 - p_top2 < h), 3 = SVIPDifference
 *   (sqrt(H_t) - sqrt(H_{t-1}) > h), 4 = AdaEDL (1 - sqrt(g H) < lambda)
 *                                             -- Table 1, Appendix A.1
 *   policy 0 = UCB1, 1 = Thompson Sampling with Beta posteriors,
 *   2 = UCB-Tuned, 3 = Thompson Sampling with a Gaussian posterior.
 *   reward 0 = r_blend, 1 = r_simple                      -- Section 3.2
 *   flag bits: 1 = a processed row holds NaN or has no finite maximum,
 *              2 = drafted token id outside [0, V), 4 = n_draft outside [1, K].
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_API __attribute__((visibility("default")))

enum { FLAG_BAD_ROW = 1, FLAG_BAD_TOKEN = 2, FLAG_BAD_NDRAFT = 4, FLAG_SAMPLER_EXHAUSTED = 8 };

/* ---- exact widening of a stored logit ---------------------------------- */
static double logit_at(const void *row, int dtype, int64_t j)
{
    if (dtype == 0)
        return (double)((const float *)row)[j];
    uint32_t bits = (uint32_t)((const uint16_t *)row)[j] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static const void *row_ptr(const void *base, int dtype, int64_t stride_b, int64_t stride_k, int b, int k)
{
    int64_t off = (int64_t)b * stride_b + (int64_t)k * stride_k;
    return (const char *)base + off * (dtype == 0 ? 4 : 2);
}

/* ---- row statistics (Appendix A.1: p = softmax of the draft logits; H its
 *      Shannon entropy in nats; Table 1: top-1 probability, top-1/top-2
 *      margin) ----------------------------------------------------------- */
typedef struct {
    double M;      /* max_j x_j (NaN entries ignored)                         */
    double S;      /* sum_j exp(x_j - M)                                      */
    double lse;    /* M + ln S                                                */
    double H;      /* -sum_j p_j ln p_j, with 0 ln 0 = 0                      */
    double p1, p2; /* largest and second largest probability (duplicates count) */
    int32_t top1;  /* smallest j with x_j = M                                 */
    int bad;       /* row holds a NaN or has no finite maximum                */
} row_stats_t;

static void row_stats(const void *row, int dtype, int64_t V, row_stats_t *r)
{
    double M = -INFINITY;
    int32_t top1 = 0;
    int has_nan = 0, seen = 0;
    for (int64_t j = 0; j < V; ++j) {
        double x = logit_at(row, dtype, j);
        if (x != x) { has_nan = 1; continue; }
        if (!seen || x > M) { M = x; top1 = (int32_t)j; seen = 1; }
    }
    r->M = M; r->top1 = top1;
    r->bad = has_nan || !seen || isinf(M);
    if (r->bad) {
        r->S = r->lse = r->H = r->p1 = r->p2 = NAN;
        return;
    }
    double S = 0.0;
    for (int64_t j = 0; j < V; ++j)
        S += exp(logit_at(row, dtype, j) - M);
    double lnS = log(S);
    double H = 0.0, x2 = -INFINITY;
    for (int64_t j = 0; j < V; ++j) {
        double x = logit_at(row, dtype, j);
        double p = exp(x - M) / S;
        if (p > 0.0)
            H -= p * ((x - M) - lnS);          /* ln p_j = x_j - M - ln S */
        if (j != top1 && x > x2) x2 = x;
    }
    r->S = S; r->lse = M + lnS; r->H = H;
    r->p1 = 1.0 / S;                           /* exp(M - M) / S */
    r->p2 = (V > 1) ? exp(x2 - M) / S : 0.0;
}

/* One row, all statistics, for tests.  out = {lse, H, p1, p2, margin, M, S}. */
ORACLE_API int tapout_oracle_row_stats(const void *row, int dtype, int64_t V, double *out, int32_t *top1)
{
    row_stats_t r;
    row_stats(row, dtype, V, &r);
    out[0] = r.lse; out[1] = r.H; out[2] = r.p1; out[3] = r.p2;
    out[4] = r.p1 - r.p2; out[5] = r.M; out[6] = r.S;
    *top1 = r.top1;
    return r.bad;
}

/* ---- stop rules (Table 1; strict inequalities as printed) -------------- *
 * The decision is taken on the binary32 values the boundary returns (the
 * kernel's output precision), widened to double, so that it is a function of
 * the returned signals alone.  margin_out = |signal - h| / |h|.             */
static int rule_fires(int rule, float h, float H, float p1, float margin, double *margin_out)
{
    double sig, thr = (double)h;
    int fire;
    switch (rule) {
    case 0: sig = sqrt((double)H); fire = sig > thr; break;          /* SVIP            */
    case 1: sig = (double)p1;      fire = sig < thr; break;          /* Max-Confidence  */
    default: sig = (double)margin; fire = sig < thr; break;          /* LogitMargin     */
    }
    if (margin_out) *margin_out = fabs(sig - thr) / (fabs(thr) > 0 ? fabs(thr) : 1.0);
    return fire;
}

/* SVIPDifference (Table 1, Appendix A.1): sqrt(H_t) - sqrt(H_{t-1}) > h, the
 * entropies being those of the current and the previous token step.  At the
 * first step of a draft the previous step is the last drafted position of the
 * sequence's previous draft (carried by the caller); without one (has_prev =
 * 0, or a NaN) the rule cannot fire.                                          */
static int svip_diff_fires(float h, float H, int has_prev, float H_prev, double *margin_out)
{
    double thr = (double)h;
    if (!has_prev || H_prev != H_prev || H != H) { if (margin_out) *margin_out = INFINITY; return 0; }
    double sig = sqrt((double)H) - sqrt((double)H_prev);
    if (margin_out) *margin_out = fabs(sig - thr) / (fabs(thr) > 0 ? fabs(thr) : 1.0);
    return sig > thr;
}

/* AdaEDL (Table 1, Appendix A.1): 1 - sqrt(g * H) < lambda_t, g a fixed
 * hyper-parameter, lambda_t the sequence's adaptive threshold.               */
static int adaedl_fires(double g, double lambda, float H, double *margin_out)
{
    if (H != H) { if (margin_out) *margin_out = INFINITY; return 0; }
    double sig = 1.0 - sqrt(g * (double)H);
    if (margin_out) *margin_out = fabs(sig - lambda) / (fabs(lambda) > 0 ? fabs(lambda) : 1.0);
    return sig < lambda;
}

/*
 * Draft pass: signals of every draft row (b,k), k < k_len[b], and the stop
 * position of Algorithm 1's draft loop: the token of the step at which the
 * selected rule fires is kept, so n_stop = (first firing k) + 1, or k_len[b]
 * if it never fires.  Rows k >= k_len[b] are left untouched.  When arm is
 * given, entropy, p_top1 and margin must be given too (the scan reads them).
 * prev_entropy [B] (or NULL): entropy of the last drafted position of each
 * sequence's previous draft, NaN for none (SVIPDifference).  lambda [B,
 * n_arms] (or NULL): adaptive thresholds (AdaEDL arms read their column).
 * arm_stride = 0: sequence-level bandit, arm[b] decides at every step;
 * arm_stride > 0: token-level bandits (Section 3.1), the arm of step k is
 * arm[b * arm_stride + k].
 */
ORACLE_API int tapout_oracle_draft_stats(
    const void *draft, int dtype, int64_t stride_b, int64_t stride_k,
    int B, int K, int64_t V,
    const int32_t *draft_tok, const int32_t *k_len, const int32_t *arm,
    int n_arms, const int32_t *rule, const float *threshold,
    float *lse, float *entropy, float *p_top1, float *p_top2, float *margin,
    int32_t *top1_id, float *logq_tok,
    int32_t *n_stop, uint8_t *stop_fired, double *stop_margin, uint32_t *flags,
    const float *prev_entropy, const double *lambda, double adaedl_g,
    int arm_stride, int nthreads)
{
    if (nthreads < 1) nthreads = 1;
    if (flags) memset(flags, 0, (size_t)B * sizeof *flags);
#pragma omp parallel for collapse(2) schedule(dynamic, 1) num_threads(nthreads)
    for (int b = 0; b < B; ++b)
        for (int k = 0; k < K; ++k) {
            int kb = k_len ? k_len[b] : K;
            if (kb > K) kb = K;
            if (k >= kb) continue;
            const void *row = row_ptr(draft, dtype, stride_b, stride_k, b, k);
            row_stats_t r;
            row_stats(row, dtype, V, &r);
            int64_t i = (int64_t)b * K + k;
            if (lse) lse[i] = (float)r.lse;
            if (entropy) entropy[i] = (float)r.H;
            if (p_top1) p_top1[i] = (float)r.p1;
            if (p_top2) p_top2[i] = (float)r.p2;
            if (margin) margin[i] = (float)(r.p1 - r.p2);
            if (top1_id) top1_id[i] = r.top1;
            uint32_t f = r.bad ? FLAG_BAD_ROW : 0;
            if (draft_tok && logq_tok) {
                int32_t t = draft_tok[i];
                if (t < 0 || t >= V) { f |= FLAG_BAD_TOKEN; logq_tok[i] = NAN; }
                else logq_tok[i] = (float)(logit_at(row, dtype, t) - r.lse);
            }
            if (f && flags) {
#pragma omp atomic
                flags[b] |= f;
            }
        }
    if (!arm) return 0;
    for (int b = 0; b < B; ++b) {
        int kb = k_len ? k_len[b] : K;
        if (kb > K) kb = K;
        int ns = kb;
        int stopped = 0;
        for (int k = 0; k < kb; ++k) {
            int a = arm_stride > 0 ? arm[(size_t)b * arm_stride + k] : arm[b];
            int64_t i = (int64_t)b * K + k;
            double mg = INFINITY;
            int fire = 0;
            if (a >= 0 && a < n_arms) {
                if (rule[a] == 3) {
                    int has_prev = k > 0 ? 1 : (prev_entropy != NULL);
                    float Hp = k > 0 ? entropy[i - 1] : (prev_entropy ? prev_entropy[b] : NAN);
                    fire = svip_diff_fires(threshold[a], entropy[i], has_prev, Hp, &mg);
                } else if (rule[a] == 4) {
                    fire = adaedl_fires(adaedl_g, lambda ? lambda[(size_t)b * n_arms + a] : (double)threshold[a], entropy[i], &mg);
                } else {
                    fire = rule_fires(rule[a], threshold[a], entropy[i], p_top1[i], margin[i], &mg);
                }
            }
            if (stop_fired) stop_fired[i] = (uint8_t)fire;
            if (stop_margin) stop_margin[i] = mg;
            if (fire && !stopped) { ns = k + 1; stopped = 1; }
        }
        if (n_stop) n_stop[b] = ns;
    }
    return 0;
}

/* ---- final token: inverse CDF over non-negative weights ---------------- *
 * token = min{ j : C_j > target }, C_j the inclusive index-order prefix sums.
 * If rounding leaves no such j, the largest j with w_j > 0.  margin_out is
 * the distance of target to the nearer edge of the chosen cell, over Z.     */
typedef double (*weight_fn)(const void *ctx, int64_t j);

static int32_t inverse_cdf(weight_fn w, const void *ctx, int64_t V, double u, double *Z_out, double *margin_out)
{
    double Z = 0.0;
    for (int64_t j = 0; j < V; ++j) Z += w(ctx, j);
    *Z_out = Z;
    if (!(Z > 0.0)) return -1;
    double target = u * Z, C = 0.0;
    int64_t last_pos = -1;
    for (int64_t j = 0; j < V; ++j) {
        double wj = w(ctx, j);
        double Cn = C + wj;
        if (wj > 0.0) last_pos = j;
        if (Cn > target) {
            if (margin_out) {
                double lo = target - C, hi = Cn - target;
                *margin_out = (lo < hi ? lo : hi) / Z;
            }
            return (int32_t)j;
        }
        C = Cn;
    }
    if (margin_out) *margin_out = 0.0;
    return (int32_t)last_pos;
}

typedef struct {
    const void *t_row, *d_row;
    int t_dtype, d_dtype;
    double Mp, Sp, Mq, Sq;
} resid_ctx;

static double w_target(const void *c_, int64_t j)
{
    const resid_ctx *c = c_;
    return exp(logit_at(c->t_row, c->t_dtype, j) - c->Mp) / c->Sp;
}

static double w_residual(const void *c_, int64_t j)
{
    const resid_ctx *c = c_;
    double p = exp(logit_at(c->t_row, c->t_dtype, j) - c->Mp) / c->Sp;
    double q = exp(logit_at(c->d_row, c->d_dtype, j) - c->Mq) / c->Sq;
    double w = p - q;
    return w > 0.0 ? w : 0.0;
}

/* Exposed for the inverse-CDF special-case pins: explicit weights. */
typedef struct { const double *w; } plain_ctx;
static double w_plain(const void *c_, int64_t j) { return ((const plain_ctx *)c_)->w[j]; }

ORACLE_API int32_t tapout_oracle_inverse_cdf(const double *w, int64_t V, double u, double *Z, double *margin)
{
    plain_ctx c = { w };
    return inverse_cdf(w_plain, &c, V, u, Z, margin);
}

/*
 * Draft-token sampling (Algorithm 1: x_i ~ M_q(prefix + X)): the token of every
 * live draft row (b,k), k < k_len[b], is the inverse CDF of softmax(row) at the
 * caller's uniform u_draft[b,k], with the conventions of the final token
 * (smallest j whose inclusive prefix sum exceeds u * Z; index-order sums in
 * double).  A row holding NaN or without a finite maximum gives token -1 and
 * sets the bad-row flag of its sequence.  Rows k >= k_len[b] are untouched.
 */
ORACLE_API int tapout_oracle_draft_sample(
    const void *draft, int dtype, int64_t stride_b, int64_t stride_k,
    int B, int K, int64_t V, const int32_t *k_len, const float *u_draft,
    int32_t *tok_out, double *icdf_margin, uint32_t *flags, int nthreads)
{
    if (nthreads < 1) nthreads = 1;
    if (flags) memset(flags, 0, (size_t)B * sizeof *flags);
#pragma omp parallel for collapse(2) schedule(dynamic, 1) num_threads(nthreads)
    for (int b = 0; b < B; ++b)
        for (int k = 0; k < K; ++k) {
            int kb = k_len ? k_len[b] : K;
            if (kb > K) kb = K;
            if (k >= kb) continue;
            int64_t i = (int64_t)b * K + k;
            resid_ctx c;
            row_stats_t r;
            c.t_row = row_ptr(draft, dtype, stride_b, stride_k, b, k);
            c.t_dtype = dtype;
            row_stats(c.t_row, dtype, V, &r);
            double mg = INFINITY, Z = 0.0;
            if (r.bad) {
                tok_out[i] = -1;
                if (flags) {
#pragma omp atomic
                    flags[b] |= FLAG_BAD_ROW;
                }
            } else {
                c.Mp = r.M; c.Sp = r.S;
                tok_out[i] = inverse_cdf(w_target, &c, V, (double)u_draft[i], &Z, &mg);
            }
            if (icdf_margin) icdf_margin[i] = mg;
        }
    return 0;
}

/*
 * Verification of the n_draft[b] drafted tokens of each sequence and the
 * final token (Algorithm 1: verify, then sample the final token from the
 * target at prefix + Y).
 *
 * Sampled sequence: position k is accepted iff u_accept[b,k] < p_k(tok)/q_k(tok),
 * evaluated as exp(logp_tok - logq_tok) on the binary32 log-probabilities
 * the boundary carries (logq_tok is an input, logp_tok an output), widened
 * to double.  accept_len = number of leading accepts (the paper's m; the
 * final token is not counted).  Final token: at the first rejection m, from
 * normalise(max(0, p_m - q_m)); with none, from target row n_draft (bonus).
 * Greedy sequence: accept iff tok == argmax of the target row (lowest index
 * on ties); final token = argmax of target row accept_len.
 * A flagged sequence (bad row among 0..n_draft, bad token, bad n_draft)
 * yields accept_len 0 and the argmax of target row 0.
 */
ORACLE_API int tapout_oracle_verify(
    const void *target, int t_dtype, int64_t t_stride_b, int64_t t_stride_k,
    const void *draft, int d_dtype, int64_t d_stride_b, int64_t d_stride_k,
    int B, int K, int64_t V,
    const float *logq_tok, const int32_t *draft_tok, const int32_t *n_draft,
    const uint8_t *greedy, const float *u_accept, const float *u_sample,
    int32_t *accept_len, int32_t *out_tok, int32_t *n_out,
    float *target_lse, float *logp_tok, int32_t *target_top1,
    double *accept_margin, double *icdf_margin, uint32_t *flags, int nthreads)
{
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int b = 0; b < B; ++b) {
        uint32_t f = 0;
        int n = n_draft[b];
        int is_greedy = greedy ? greedy[b] != 0 : 0;
        if (n < 1 || n > K) { f |= FLAG_BAD_NDRAFT; n = n < 1 ? 1 : K; }
        row_stats_t *rs = malloc((size_t)(n + 1) * sizeof *rs);
        for (int k = 0; k <= n; ++k) {
            row_stats(row_ptr(target, t_dtype, t_stride_b, t_stride_k, b, k), t_dtype, V, &rs[k]);
            if (rs[k].bad) f |= FLAG_BAD_ROW;
            int64_t it = (int64_t)b * (K + 1) + k;
            if (target_lse) target_lse[it] = (float)rs[k].lse;
            if (target_top1) target_top1[it] = rs[k].top1;
        }
        for (int k = 0; k < n; ++k) {
            int32_t t = draft_tok[(int64_t)b * K + k];
            if (t < 0 || t >= V) f |= FLAG_BAD_TOKEN;
        }
        int m = 0;
        int32_t final_tok;
        double imargin = INFINITY;
        if (f & (FLAG_BAD_NDRAFT | FLAG_BAD_TOKEN | FLAG_BAD_ROW)) {
            m = 0;
            final_tok = rs[0].top1;
            for (int k = 0; k < n; ++k) {
                if (logp_tok) logp_tok[(int64_t)b * K + k] = NAN;
                if (accept_margin) accept_margin[(int64_t)b * K + k] = INFINITY;
            }
        } else {
            int rejected = 0;
            for (int k = 0; k < n; ++k) {
                int64_t i = (int64_t)b * K + k;
                int32_t t = draft_tok[i];
                const void *trow = row_ptr(target, t_dtype, t_stride_b, t_stride_k, b, k);
                float lp = (float)(logit_at(trow, t_dtype, t) - rs[k].lse);
                if (logp_tok) logp_tok[i] = lp;
                int acc;
                double mg = INFINITY;
                if (is_greedy) {
                    acc = (t == rs[k].top1);
                } else {
                    double rho = exp((double)lp - (double)logq_tok[i]);
                    double u = (double)u_accept[i];
                    acc = u < rho;
                    double r1 = rho < 1.0 ? rho : 1.0;
                    mg = fabs(u - r1) / (r1 > 1e-30 ? r1 : 1e-30);
                }
                if (accept_margin) accept_margin[i] = mg;
                if (!rejected) { if (acc) ++m; else rejected = 1; }
            }
            if (is_greedy) {
                final_tok = rs[m].top1;
            } else {
                resid_ctx c;
                c.t_row = row_ptr(target, t_dtype, t_stride_b, t_stride_k, b, m);
                c.t_dtype = t_dtype; c.Mp = rs[m].M; c.Sp = rs[m].S;
                double u = (double)u_sample[b], Z = 0.0;
                final_tok = -1;
                if (m < n) {
                    row_stats_t rq;
                    c.d_row = row_ptr(draft, d_dtype, d_stride_b, d_stride_k, b, m);
                    c.d_dtype = d_dtype;
                    row_stats(c.d_row, d_dtype, V, &rq);
                    if (rq.bad) f |= FLAG_BAD_ROW;
                    else {
                        c.Mq = rq.M; c.Sq = rq.S;
                        final_tok = inverse_cdf(w_residual, &c, V, u, &Z, &imargin);
                    }
                }
                /* bonus token, or an (only by rounding) empty residual: draw from p_m */
                if (final_tok < 0) final_tok = inverse_cdf(w_target, &c, V, u, &Z, &imargin);
                if (final_tok < 0) final_tok = rs[m].top1;
            }
        }
        accept_len[b] = m;
        for (int k = 0; k <= K; ++k)
            out_tok[(int64_t)b * (K + 1) + k] = k < m ? draft_tok[(int64_t)b * K + k] : (k == m ? final_tok : -1);
        n_out[b] = m + 1;
        if (icdf_margin) icdf_margin[b] = imargin;
        if (flags) flags[b] = f;
        free(rs);
    }
    return 0;
}

/* ---- carried state of the stateful stop rules (Appendix A.1) ------------- *
 * After each draft of an active sequence with 1 <= n_draft <= K:
 *   prev_entropy <- entropy of the last drafted position (row n_draft - 1);
 *   AdaEDL:  r = n_acc / n_drafted
 *            accept_rate <- beta1 * accept_rate + (1 - beta1) * r
 *            lambda <- beta2 * lambda + (1 - beta2) * (lambda + eps * sign(alpha - s))
 *   for the lambda of every AdaEDL arm of the sequence (each arm keeps its own,
 *   they start at different values).  The printed update is garbled (a doubled
 *   "+", an accept_rate that nothing reads).  Two readings of s:
 *     steer_raw = 0   s = the new smoothed accept_rate: the running average the
 *                     appendix defines is what steers the threshold;
 *     steer_raw = 1   s = r, this draft's own rate: the equation as printed
 *                     with the doubled "+" dropped (accept_rate is then kept
 *                     but read by nothing).
 *   sign(0) = 0.                                                              */
ORACLE_API int tapout_oracle_rule_state_update(
    int B, int K, int n_arms, const int32_t *rule,
    const float *entropy /* [B,K] or NULL */, const int32_t *n_draft, const int32_t *accept_len,
    const uint8_t *active,
    float *prev_entropy /* [B] */, double *accept_rate /* [B] */, double *lambda /* [B,n_arms] */,
    double ad_alpha, double beta1, double beta2, double eps, int steer_raw)
{
    for (int b = 0; b < B; ++b) {
        if (active && !active[b]) continue;
        int n = n_draft[b];
        if (n < 1 || n > K) continue;
        if (entropy) prev_entropy[b] = entropy[(size_t)b * K + (n - 1)];
        volatile double r = (double)accept_len[b] / (double)n;
        volatile double keep = beta1 * accept_rate[b];
        volatile double add = (1.0 - beta1) * r;
        double rate = keep + add;
        accept_rate[b] = rate;
        double s = steer_raw ? r : rate;
        double sg = ad_alpha > s ? 1.0 : (ad_alpha < s ? -1.0 : 0.0);
        for (int a = 0; a < n_arms; ++a) {
            if (rule[a] != 4) continue;
            double lam = lambda[(size_t)b * n_arms + a];
            volatile double step = eps * sg;
            volatile double moved = lam + step;
            volatile double t1 = beta2 * lam;
            volatile double t2 = (1.0 - beta2) * moved;
            lambda[(size_t)b * n_arms + a] = t1 + t2;
        }
    }
    return 0;
}

/* ---- reward (Section 3.2): r_blend = a*|Y|/gamma + (1-a)*|Y|/|X| -------- */
ORACLE_API double tapout_oracle_reward(int m, int n_drafted, int gamma, double alpha)
{
    volatile double t1 = (alpha * (double)m) / (double)gamma;
    volatile double t2 = ((1.0 - alpha) * (double)m) / (double)n_drafted;
    return t1 + t2;
}

/* r_simple = |Y| / gamma (Section 3.2), the normalised acceptance length. */
ORACLE_API double tapout_oracle_reward_simple(int m, int gamma)
{
    return (double)m / (double)gamma;
}

/* ---- UCB1 (Section 3.3): argmax_a mean_a + sqrt(2 ln t / N_a) ----------- *
 * N_a = plays of arm a so far, t = 1 + sum_a N_a (the index of the current
 * play).  Every arm is played once first, in index order; exact ties go to
 * the lowest index.  index_out[a] (optional) receives the UCB value, or
 * +inf for an unplayed arm.                                                */
ORACLE_API int tapout_oracle_ucb1_select(const double *sum_r, const int64_t *count, int A, double *index_out)
{
    int64_t t = 1;
    for (int a = 0; a < A; ++a) t += count[a];
    int best = -1;
    double best_v = -INFINITY;
    int unplayed = -1;
    for (int a = 0; a < A; ++a) {
        double v;
        if (count[a] == 0) { v = INFINITY; if (unplayed < 0) unplayed = a; }
        else {
            double n = (double)count[a];
            volatile double mean = sum_r[a] / n;
            volatile double bonus = sqrt((2.0 * log((double)t)) / n);
            v = mean + bonus;
        }
        if (index_out) index_out[a] = v;
        if (best < 0 || v > best_v) { best = a; best_v = v; }
    }
    return unplayed >= 0 ? unplayed : best;
}

/* ---- Thompson Sampling with Beta posteriors ----------------------------- *
 * Posterior of arm a after rewards in [0,1]: Beta(1 + sum_r, 1 + N - sum_r)
 * (uniform prior, fractional-count update).  A draw is G1/(G1+G2) with
 * G ~ Gamma(shape >= 1) from Marsaglia & Tsang's method driven by caller
 * uniforms: 8 attempts of 3 uniforms each (two for a Box-Muller normal, one
 * for the acceptance test), consumed in order; u = 0 is replaced by 2^-25.
 * If all attempts reject, the shape itself (the mean) is returned and the
 * exhausted flag raised.                                                    */
#define TS_ATTEMPTS 8
#define TS_UNIFORMS_PER_ARM (2 * TS_ATTEMPTS * 3)

static double unit_open(float u)
{
    double x = (double)u;
    return x > 0.0 ? x : 0x1p-25;
}

ORACLE_API double tapout_oracle_gamma(double shape, const float *u, int *exhausted)
{
    double d = shape - 1.0 / 3.0;
    double c = 1.0 / sqrt(9.0 * d);
    for (int i = 0; i < TS_ATTEMPTS; ++i) {
        double u1 = unit_open(u[3 * i]), u2 = (double)u[3 * i + 1], u3 = unit_open(u[3 * i + 2]);
        double z = sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2);
        double t = 1.0 + c * z;
        double v = t * t * t;
        if (v > 0.0 && log(u3) < 0.5 * z * z + d - d * v + d * log(v))
            return d * v;
    }
    if (exhausted) *exhausted = 1;
    return shape;
}

ORACLE_API double tapout_oracle_beta(double a, double b, const float *u, int *exhausted)
{
    double g1 = tapout_oracle_gamma(a, u, exhausted);
    double g2 = tapout_oracle_gamma(b, u + TS_ATTEMPTS * 3, exhausted);
    return g1 / (g1 + g2);
}

ORACLE_API int tapout_oracle_ts_select(const double *sum_r, const int64_t *count, int A, const float *u,
                                       double *theta_out, int *exhausted)
{
    int best = 0;
    double best_v = -INFINITY;
    for (int a = 0; a < A; ++a) {
        double alpha = 1.0 + sum_r[a];
        double beta = 1.0 + ((double)count[a] - sum_r[a]);
        double th = tapout_oracle_beta(alpha, beta, u + (size_t)a * TS_UNIFORMS_PER_ARM, exhausted);
        if (theta_out) theta_out[a] = th;
        if (a == 0 || th > best_v) { best = a; best_v = th; }
    }
    return best;
}

/* ---- UCB-Tuned (Section 3.3) -------------------------------------------- *
 * argmax_a mean_a + sqrt( (ln t / N_a) * min(1/4, V_a) ),
 * V_a = var_a + sqrt(2 ln t / N_a), var_a the empirical (population)
 * variance of the rewards of arm a, here from the running sums:
 * sum_r2/N - mean^2.  t, the initial plays and ties as for UCB1.            */
ORACLE_API int tapout_oracle_ucb_tuned_select(const double *sum_r, const double *sum_r2, const int64_t *count,
                                              int A, double *index_out)
{
    int64_t t = 1;
    for (int a = 0; a < A; ++a) t += count[a];
    int best = -1, unplayed = -1;
    double best_v = -INFINITY;
    for (int a = 0; a < A; ++a) {
        double v;
        if (count[a] == 0) { v = INFINITY; if (unplayed < 0) unplayed = a; }
        else {
            double n = (double)count[a];
            double lt = log((double)t);
            volatile double mean = sum_r[a] / n;
            volatile double m2 = sum_r2[a] / n;
            volatile double msq = mean * mean;
            volatile double var = m2 - msq;
            volatile double two_lt = 2.0 * lt;
            volatile double wide = sqrt(two_lt / n);
            volatile double V = var + wide;
            double cap = V < 0.25 ? V : 0.25;
            volatile double ratio = lt / n;
            volatile double prod = ratio * cap;
            volatile double bonus = sqrt(prod);
            v = mean + bonus;
        }
        if (index_out) index_out[a] = v;
        if (best < 0 || v > best_v) { best = a; best_v = v; }
    }
    return unplayed >= 0 ? unplayed : best;
}

/* ---- Thompson Sampling with a Gaussian posterior (Section 3.3) ----------- *
 * The paper names a Gaussian prior with known noise variance and gives no
 * values; taken here: prior N(0, 1), unit noise variance, so that after N_a
 * plays with summed reward S_a the posterior is N(S_a/(N_a+1), 1/(N_a+1)).
 * theta_a = mean + z / sqrt(N_a + 1), z = sqrt(-2 ln u1) cos(2 pi u2) from
 * the first two of the arm's caller uniforms (u1 = 0 read as 2^-25).         */
ORACLE_API int tapout_oracle_ts_gauss_select(const double *sum_r, const int64_t *count, int A, const float *u,
                                             double *theta_out)
{
    int best = 0;
    double best_v = -INFINITY;
    for (int a = 0; a < A; ++a) {
        const float *ua = u + (size_t)a * TS_UNIFORMS_PER_ARM;
        double n1 = (double)count[a] + 1.0;
        double z = sqrt(-2.0 * log(unit_open(ua[0]))) * cos(6.283185307179586476925 * (double)ua[1]);
        volatile double mean = sum_r[a] / n1;
        volatile double dev = z / sqrt(n1);
        double th = mean + dev;
        if (theta_out) theta_out[a] = th;
        if (a == 0 || th > best_v) { best = a; best_v = th; }
    }
    return best;
}

/*
 * Batched bandit calls.  n_bandits == B: one bandit per sequence slot.
 * n_bandits == 1: one shared bandit; select draws one arm for the round
 * (from the first sequence's uniforms) and update applies the B rewards in
 * index order, each as one play.
 *
 * positions = 1: sequence-level bandits.  positions = P > 1: token-level
 * bandits (Section 3.1: every position of the drafting sequence is itself a
 * bandit): state [n_bandits, P, A], arms [B, P], uniforms [B, P, A, 48].
 * The token-level reward (Section 3.2) is 1 for an accepted token and 0 for a
 * rejected one: position k < m = accept_len is an accepted play of its arm,
 * position m (if m < n_draft) a rejected one; later positions were never
 * evaluated by the target model and are not played.
 */
ORACLE_API int tapout_oracle_bandit_select(int policy, int n_bandits, int B, int A, int positions,
                                           const double *sum_r, const double *sum_r2, const int64_t *count,
                                           const float *u_ts, int32_t *arm_out, uint32_t *flags)
{
    for (int b = 0; b < B; ++b) {
        if (flags) flags[b] = 0;
        for (int k = 0; k < positions; ++k) {
            size_t nb = ((size_t)(n_bandits == 1 ? 0 : b) * positions + k) * A;
            int ex = 0, a;
            const double *S = sum_r + nb;
            const int64_t *N = count + nb;
            const float *u = u_ts ? u_ts + nb * TS_UNIFORMS_PER_ARM : NULL;
            if (policy == 0) a = tapout_oracle_ucb1_select(S, N, A, NULL);
            else if (policy == 2) a = tapout_oracle_ucb_tuned_select(S, sum_r2 + nb, N, A, NULL);
            else if (policy == 3) a = tapout_oracle_ts_gauss_select(S, N, A, u, NULL);
            else a = tapout_oracle_ts_select(S, N, A, u, NULL, &ex);
            arm_out[(size_t)b * positions + k] = a;
            if (flags && ex) flags[b] |= FLAG_SAMPLER_EXHAUSTED;
        }
    }
    return 0;
}

ORACLE_API int tapout_oracle_bandit_update(int n_bandits, int B, int A, int positions, int reward_kind, double alpha,
                                           double *sum_r, double *sum_r2, int64_t *count,
                                           const int32_t *arm, const int32_t *accept_len,
                                           const int32_t *n_draft, const int32_t *gamma,
                                           const uint8_t *active)
{
    for (int b = 0; b < B; ++b) {
        if (active && !active[b]) continue;
        if (n_draft[b] < 1 || gamma[b] < 1) continue;
        int nb = n_bandits == 1 ? 0 : b;
        if (positions == 1) {
            int a = arm[b];
            if (a < 0 || a >= A) continue;
            double r = reward_kind == 1 ? tapout_oracle_reward_simple(accept_len[b], gamma[b])
                                        : tapout_oracle_reward(accept_len[b], n_draft[b], gamma[b], alpha);
            count[(size_t)nb * A + a] += 1;
            sum_r[(size_t)nb * A + a] += r;
            if (sum_r2) { volatile double sq = r * r; sum_r2[(size_t)nb * A + a] += sq; }
            continue;
        }
        int m = accept_len[b], n = n_draft[b] < positions ? n_draft[b] : positions;
        for (int k = 0; k < n && k <= m; ++k) {
            int a = arm[(size_t)b * positions + k];
            if (a < 0 || a >= A) continue;
            size_t i = ((size_t)nb * positions + k) * A + a;
            double r = k < m ? 1.0 : 0.0;
            count[i] += 1;
            sum_r[i] += r;
            if (sum_r2) sum_r2[i] += r;
        }
    }
    return 0;
}
