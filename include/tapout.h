/*
 * libtapout -- per-round logits processing of TapOut (bandit-controlled dynamic
 * speculative decoding) on one AMD MI355X (gfx950).  C ABI, no C++ or torch
 * types.
 *
 * One decode round (Algorithm 1 of the paper) maps onto four calls:
 *
 *   tapout_bandit_select   arm of every sequence for this drafting session
 *   tapout_draft_stats     signals of the draft distributions + stop position
 *   tapout_verify          accept the drafted prefix, draw the final token
 *   tapout_bandit_update   blended reward -> bandit state
 *
 * General rules
 *   Pointers.  Unless a parameter says "host", every array pointer is a DEVICE
 *     pointer into memory owned by the caller; the library never keeps it
 *     after the call returns.  "or NULL" marks optional arrays.  The output
 *     arrays of a call must not overlap its input arrays or each other
 *     (several workgroups read a sequence's inputs while one writes its
 *     outputs).
 *   Asynchrony.  Calls enqueue kernels on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and return without waiting.  Calls on
 *     one context must be issued in stream order on one stream at a time: the
 *     context owns scratch memory that consecutive calls reuse.  The four
 *     calls of a round (and the sharded variants) only launch kernels — no
 *     allocation, no memset, no copy, no host synchronisation — so they can
 *     be captured into a HIP graph and replayed; launch shapes are fixed at
 *     capture time from the arguments and the context's options.
 *   Memory.  Device memory is allocated in tapout_create and released in
 *     tapout_destroy, never in between.
 *   Errors.  Every call returns a tapout_status.  Argument errors are found on
 *     the host before anything is launched and leave all outputs untouched;
 *     tapout_last_error() describes the last failure on that context.
 *     Data-dependent problems cannot be reported synchronously: they set bits
 *     in the per-sequence device array `flags` and produce the documented
 *     fallback result.
 *   Determinism.  No floating-point atomics; same inputs give bit-identical
 *     outputs from run to run.
 *   Logits layout.  A logits tensor is [B, K, V] (draft) or [B, K+1, V]
 *     (target) with the vocabulary axis contiguous; stride_b / stride_k are in
 *     elements.  Rows may start at any element-aligned address; rows that are
 *     16-byte aligned take the fast path.
 */
#ifndef TAPOUT_H
#define TAPOUT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define TAPOUT_API __attribute__((visibility("default")))
#else
#define TAPOUT_API
#endif

#define TAPOUT_MAX_ARMS 8
/* caller uniforms per arm for one Thompson draw: 2 Gamma variates x 8 attempts x 3 */
#define TAPOUT_TS_UNIFORMS_PER_ARM 48

typedef struct tapout_ctx tapout_ctx;

typedef enum {
    TAPOUT_OK = 0,
    TAPOUT_EINVAL = 1,       /* bad argument (see tapout_last_error)           */
    TAPOUT_EUNSUPPORTED = 2, /* valid request the build does not implement      */
    TAPOUT_ENOMEM = 3,       /* device allocation failed in tapout_create       */
    TAPOUT_EHIP = 4          /* a HIP runtime call or kernel launch failed      */
} tapout_status;

typedef enum { TAPOUT_F32 = 0, TAPOUT_BF16 = 1 } tapout_dtype;

/* Stop rules of Table 1 / Appendix A.1.  A rule fires, i.e. drafting stops
 * after the current token, when its strict inequality holds (H = entropy of
 * the draft distribution of the current step, in nats):
 *   SVIP       sqrt(H) > h                        h = 0.6
 *   MAXCONF    p(top-1) < h                       h = 0.8
 *   MARGIN     p(top-1) - p(top-2) < h            h = 0.2
 *   SVIP_DIFF  sqrt(H_t) - sqrt(H_{t-1}) > h      h = 0.2
 *              At the first step of a draft, H_{t-1} is the entropy of the last
 *              drafted position of the sequence's previous draft (carried in
 *              the context, see tapout_rule_state_get); a sequence without a
 *              previous draft cannot stop at its first step.
 *   ADAEDL     1 - sqrt(g * H) < lambda           g = tapout_config.adaedl_gamma
 *              lambda is kept per sequence and arm, starts at the arm's
 *              threshold[] entry and is moved by tapout_bandit_update.       */
typedef enum {
    TAPOUT_RULE_SVIP = 0, TAPOUT_RULE_MAXCONF = 1, TAPOUT_RULE_MARGIN = 2,
    TAPOUT_RULE_SVIP_DIFF = 3, TAPOUT_RULE_ADAEDL = 4
} tapout_rule;

/* Bandit policies of Section 3.3 (sequence-level). */
typedef enum { TAPOUT_UCB1 = 0, TAPOUT_TS_BETA = 1, TAPOUT_UCB_TUNED = 2, TAPOUT_TS_GAUSS = 3 } tapout_policy;

/* Rewards of Section 3.2: r_blend = alpha |Y|/gamma + (1 - alpha) |Y|/|X|,
 * r_simple = |Y|/gamma.                                                       */
typedef enum { TAPOUT_REWARD_BLEND = 0, TAPOUT_REWARD_SIMPLE = 1 } tapout_reward;

/* Action granularity of Section 3.1.  SEQUENCE: one bandit decides the stop
 * rule of a whole drafting session.  TOKEN: every draft position is a bandit of
 * its own (max_k of them per bandit slot); its reward (Section 3.2) is 1 if the
 * token drafted at that position is accepted and 0 if it is the first rejected
 * one; positions after the first rejection are not played.  In TOKEN mode the
 * arm arrays of all calls are [B, max_k] (row stride max_k whatever K is),
 * u_ts is [B, max_k, n_arms, 48], the bandit state is [n_bandits, max_k,
 * n_arms], and tapout_config.reward is ignored.                               */
typedef enum { TAPOUT_SEQUENCE_LEVEL = 0, TAPOUT_TOKEN_LEVEL = 1 } tapout_granularity;

/* per-sequence flag bits written by the kernels */
#define TAPOUT_FLAG_BAD_ROW 1u           /* a processed row holds NaN or has no finite maximum */
#define TAPOUT_FLAG_BAD_TOKEN 2u         /* drafted token id outside [0, V)                    */
#define TAPOUT_FLAG_BAD_NDRAFT 4u        /* n_draft outside [1, K]                             */
#define TAPOUT_FLAG_SAMPLER_EXHAUSTED 8u /* all Gamma attempts rejected (Thompson)             */

typedef struct {
    int32_t device;                       /* HIP device ordinal                                 */
    int32_t max_batch;                    /* largest B of any call                              */
    int32_t max_k;                        /* largest K (draft positions per sequence)           */
    int32_t vocab;                        /* largest V of any call                              */
    int32_t n_arms;                       /* 1 .. TAPOUT_MAX_ARMS                               */
    int32_t rule[TAPOUT_MAX_ARMS];        /* tapout_rule of each arm                            */
    float threshold[TAPOUT_MAX_ARMS];     /* h of each arm (Table 1 values are the defaults)    */
    int32_t policy;                       /* tapout_policy                                      */
    int32_t n_bandits;                    /* max_batch: one bandit per sequence slot; 1: shared */
    double alpha;                         /* weight of |Y|/gamma in the blended reward (0.5)    */
    int32_t reward;                       /* tapout_reward                                      */
    int32_t granularity;                  /* tapout_granularity                                 */
    /* AdaEDL (Appendix A.1).  The paper leaves all of these unvalued; the defaults are this
     * library's choice.  After every draft of a sequence, with r = accepted / drafted:
     *   rate   <- beta1 * rate + (1 - beta1) * r
     *   lambda <- beta2 * lambda + (1 - beta2) * (lambda + eps * sign(alpha_target - s))
     * with s = the new smoothed rate (adaedl_steer = 0, the default: the appendix defines the running
     * average, and this reading is the one in which something reads it) or s = r, this draft's own
     * rate (adaedl_steer = 1: the update as Appendix A.1 prints it, its doubled "+" dropped).          */
    double adaedl_gamma;                  /* g in the stop rule (0.5)                           */
    double adaedl_alpha;                  /* acceptance rate the threshold is steered to (0.9)  */
    double adaedl_beta1;                  /* smoothing of the acceptance rate (0.5)             */
    double adaedl_beta2;                  /* smoothing of lambda (0.9)                          */
    double adaedl_eps;                    /* step of lambda (0.01)                              */
    double adaedl_rate0;                  /* initial smoothed acceptance rate (= adaedl_alpha)  */
    int32_t draft_sampling;               /* 1: tapout_draft_stats may draw the draft tokens    */
                                          /* (u_draft); sizes the final-token scratch for one   */
                                          /* job per draft row instead of one per sequence      */
    int32_t adaedl_steer;                 /* 0: lambda follows the smoothed rate; 1: r itself   */
} tapout_config;

typedef struct {
    const void *ptr;                      /* device pointer to element [0,0,0]                  */
    int32_t dtype;                        /* tapout_dtype                                       */
    int64_t stride_b, stride_k;           /* elements; the vocabulary axis has stride 1         */
} tapout_logits;

/* Fill *cfg with the set-up of the paper's main experiments restricted to the
 * stateless rules: three arms SVIP / MAXCONF / MARGIN at the Table 1
 * thresholds, UCB1, r_blend with alpha = 0.5, one bandit per sequence.  host. */
TAPOUT_API void tapout_default_config(tapout_config *cfg, int32_t max_batch, int32_t max_k, int32_t vocab);

/* Create a context on cfg->device: validates cfg (host), allocates scratch
 * and bandit state (all plays zero).  *out is NULL on failure.               */
TAPOUT_API tapout_status tapout_create(tapout_ctx **out, const tapout_config *cfg);
TAPOUT_API tapout_status tapout_destroy(tapout_ctx *ctx);
/* Text of the last error on ctx (valid until the next call on ctx); with
 * ctx == NULL the text of the last failed tapout_create or context-free call
 * (tapout_draft_stats_static) on this thread.                                 */
TAPOUT_API const char *tapout_last_error(const tapout_ctx *ctx);

/*
 * Arm selection at the start of a drafting session (Section 3.1: sequence-
 * level bandit; Section 3.3: UCB1, Thompson Sampling).
 *   UCB1: an arm never played is chosen first (lowest index); otherwise
 *     argmax_a  mean_a + sqrt(2 ln t / N_a),  t = 1 + sum_a N_a, lowest index
 *     on exact ties.  fp64.
 *   UCB_TUNED: as UCB1 with the bonus sqrt((ln t / N_a) min(1/4, V_a)),
 *     V_a = var_a + sqrt(2 ln t / N_a), var_a = Q_a/N_a - (S_a/N_a)^2 the
 *     empirical variance from the running sums of r and r^2.  fp64.
 *   TS_GAUSS: theta_a ~ N(S_a/(N_a+1), 1/(N_a+1)) (prior N(0,1), unit noise
 *     variance: the paper names the family, not the values); theta_a = mean +
 *     z / sqrt(N_a+1), z = sqrt(-2 ln u1) cos(2 pi u2) from u_ts[b][a][0..1]
 *     (u1 = 0 read as 2^-25).  fp64.
 *   TS_BETA: theta_a ~ Beta(1 + S_a, 1 + N_a - S_a) (S_a = summed rewards),
 *     argmax_a theta_a.  The draw is G1/(G1+G2), G ~ Gamma(shape) by
 *     Marsaglia-Tsang driven by u_ts[b][a][0..47]: 8 attempts x (2 Box-Muller
 *     uniforms, 1 acceptance uniform) for G1, then the same for G2; u = 0 is
 *     read as 2^-25; if all attempts reject, G = shape and
 *     TAPOUT_FLAG_SAMPLER_EXHAUSTED is set.  fp64.
 * u_ts    [B, n_arms, 48] f32 in [0,1), required for TS_BETA and TS_GAUSS,
 *         ignored for UCB1 and UCB_TUNED
 * arm_out [B] i32
 * flags   [B] u32 or NULL (overwritten)
 * With a shared bandit (n_bandits == 1) every sequence gets the arm drawn for
 * sequence 0.  TOKEN_LEVEL: one draw per position, arm_out [B, max_k], u_ts
 * [B, max_k, n_arms, 48]; flags[b] ORs the positions.
 */
TAPOUT_API tapout_status tapout_bandit_select(tapout_ctx *ctx, int32_t B, const float *u_ts,
                                   int32_t *arm_out, uint32_t *flags, void *stream);

/*
 * Signals of the draft distributions and the stop position (Appendix A.1,
 * Table 1; Algorithm 1 lines 2-8).  For every row (b,k), k < k_len[b], of the
 * draft logits x, with p = softmax(x):
 *   lse      = ln sum_j exp(x_j)
 *   entropy  = -sum_j p_j ln p_j          (nats, 0 ln 0 = 0)
 *   p_top1   = max_j p_j,  top1_id = smallest argmax index
 *   p_top2   = second largest p_j counting duplicates (a tie at the top gives
 *              p_top2 = p_top1), margin = p_top1 - p_top2
 *   logq_tok = x[draft_tok] - lse
 * and per sequence n_stop = (first k at which the rule of arm[b] fires) + 1,
 * else k_len[b]: the token drafted at the firing step is kept.  The rule is
 * evaluated on the returned binary32 signals, widened to double (SVIP compares
 * sqrt(entropy)).  Rows k >= k_len[b] are not streamed and their outputs are
 * not written (the [B,K,V] tensor and draft_tok must still be addressable there:
 * single elements of such rows may be read ahead of k_len and are discarded).
 * SVIP_DIFF and ADAEDL arms read the context's rule state (previous entropy,
 * lambda) and, when the configuration holds such an arm, the call keeps the
 * entropies of this draft in the context for tapout_bandit_update.
 *
 * Draft-token sampling (Algorithm 1, "sample x_i from the draft model"): with
 * u_draft given, the token of every live row is drawn first, as the inverse CDF
 * of softmax(row) at u_draft[b,k] with the conventions of the final token of
 * tapout_verify (smallest j whose inclusive prefix sum exceeds u * total, in
 * double), written to sampled_tok, and logq_tok refers to it.  A bad row gets
 * token -1 (BAD_ROW and BAD_TOKEN are both flagged).  Needs a context created
 * with tapout_config.draft_sampling = 1.
 *
 * draft_tok [B,K] i32 or NULL (then logq_tok is not written, unless u_draft is
 *           given); draft_tok and u_draft exclude each other
 * u_draft   [B,K] f32 in [0,1) or NULL;  sampled_tok [B,K] i32, required with
 *           u_draft (rows k >= k_len[b] untouched)
 * k_len     [B] i32 or NULL (= K for all)
 * arm       [B] i32 ([B, max_k] for TOKEN_LEVEL: step k is decided by the rule
 *           of arm[b, k]) or NULL (then n_stop / stop_fired are not written)
 * lse, entropy, p_top1, p_top2, margin, logq_tok [B,K] f32, each or NULL
 * top1_id   [B,K] i32 or NULL
 * n_stop    [B] i32 or NULL;  stop_fired [B,K] u8 or NULL
 * flags     [B] u32 or NULL (overwritten): BAD_ROW, BAD_TOKEN.  A bad row
 *           yields NaN signals (its rule does not fire); a bad token NaN
 *           logq_tok.
 */
TAPOUT_API tapout_status tapout_draft_stats(tapout_ctx *ctx, const tapout_logits *draft,
                                 int32_t B, int32_t K, int32_t V,
                                 const int32_t *draft_tok, const int32_t *k_len, const int32_t *arm,
                                 const float *u_draft,
                                 float *lse, float *entropy, float *p_top1, float *p_top2, float *margin,
                                 int32_t *top1_id, float *logq_tok, int32_t *sampled_tok,
                                 int32_t *n_stop, uint8_t *stop_fired, uint32_t *flags, void *stream);

/*
 * Verification of the drafted tokens and the final token (Algorithm 1 lines
 * 10-11, with "verify" meaning speculative sampling as in the works the
 * paper's introduction cites).  n = n_draft[b] tokens were drafted; target
 * rows 0..n are read (row n is the distribution after all n tokens).
 *   sampled sequence: token k is accepted iff
 *       u_accept[b,k] < exp(logp_tok[b,k] - logq_tok[b,k]),
 *     logp_tok = target[b,k,tok] - lse(target[b,k]) rounded to binary32, the
 *     comparison in double.  accept_len m = number of leading accepts.
 *     Final token: m < n: inverse CDF of max(0, p_m - q_m) (softmaxes of
 *     target / draft row m) at u_sample[b]; m = n: inverse CDF of p_n.
 *     Inverse CDF = smallest j whose inclusive prefix sum exceeds u * total;
 *     accumulated in double.  An all-zero residual falls back to p_m.
 *   greedy sequence (greedy[b] != 0): accepted iff tok == argmax target row k
 *     (smallest index); final token = argmax of target row m.
 *   out_tok[b] = accepted tokens, the final token, then -1 up to K+1 entries;
 *   n_out = m + 1.  (The paper's acceptance length m excludes the final token.)
 * A sequence with BAD_NDRAFT, BAD_TOKEN or BAD_ROW (any target row 0..n, or
 * the draft row it would resample from) gets accept_len 0 and the argmax of
 * target row 0 as its token, except that a bad draft row found only at the
 * residual step falls back to sampling from p_m.
 *
 * target     [B,K+1,V], draft [B,K,V]
 * draft_lse  [B,K] f32: lse from tapout_draft_stats (exponent reference of
 *            the draft row when the residual is formed)
 * logq_tok   [B,K] f32 from tapout_draft_stats
 * draft_tok  [B,K] i32;  n_draft [B] i32 in [1,K]
 * greedy     [B] u8 or NULL (all sampled)
 * u_accept   [B,K] f32 in [0,1);  u_sample [B] f32 in [0,1)
 * accept_len [B] i32;  out_tok [B,K+1] i32;  n_out [B] i32
 * target_lse [B,K+1] f32 or NULL;  logp_tok [B,K] f32 or NULL;
 * target_top1 [B,K+1] i32 or NULL  (rows > n_draft[b] untouched)
 * flags      [B] u32 or NULL (overwritten)
 */
TAPOUT_API tapout_status tapout_verify(tapout_ctx *ctx, const tapout_logits *target, const tapout_logits *draft,
                            int32_t B, int32_t K, int32_t V,
                            const float *draft_lse, const float *logq_tok,
                            const int32_t *draft_tok, const int32_t *n_draft, const uint8_t *greedy,
                            const float *u_accept, const float *u_sample,
                            int32_t *accept_len, int32_t *out_tok, int32_t *n_out,
                            float *target_lse, float *logp_tok, int32_t *target_top1,
                            uint32_t *flags, void *stream);

/*
 * tapout_draft_stats for callers that cannot allocate device memory or hold a
 * context: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  No context: the call computes the same signals and stop
 * positions with the same kernels and the launch shape of a context with
 * default options, and keeps the slice partials of its streaming pass in a
 * fixed array in the library's device image (TAPOUT_STATIC_MAX_PARTIALS 32-byte
 * records, 4 MiB per GPU, held until the process ends) on the CURRENT HIP
 * device, whose logits and arrays the pointers must refer to.  It calls no
 * allocating routine; the first call on a device looks the array's address up
 * once.  Inputs with B * K * slices-per-row beyond the array (slices per row =
 * max(ceil(4096 / (B K)), row bytes / 65536), at most V / 4096) are refused
 * with TAPOUT_EINVAL before anything is launched.
 *   All calls on one GPU share the array, which keeps the previous call's
 *   records: calls that overlap in time on one GPU (different streams, or
 *   different threads) race; issue them in stream order on one stream.
 * Arguments as tapout_draft_stats, except:
 *   no u_draft / sampled_tok (draft-token sampling needs a context);
 *   n_arms, rule, threshold: HOST arrays [n_arms] describing the arm pool that
 *     `arm` indexes (required with arm; only the rules that carry no state
 *     between drafts: SVIP, MAXCONF, MARGIN; others: TAPOUT_EUNSUPPORTED);
 *   arm is [B] (sequence-level).
 * Errors are described by tapout_last_error(NULL) on the calling thread.
 */
#define TAPOUT_STATIC_MAX_PARTIALS 131072
TAPOUT_API tapout_status tapout_draft_stats_static(const tapout_logits *draft, int32_t B, int32_t K, int32_t V,
                                 const int32_t *draft_tok, const int32_t *k_len, const int32_t *arm,
                                 int32_t n_arms, const int32_t *rule, const float *threshold,
                                 float *lse, float *entropy, float *p_top1, float *p_top2, float *margin,
                                 int32_t *top1_id, float *logq_tok,
                                 int32_t *n_stop, uint8_t *stop_fired, uint32_t *flags, void *stream);

/*
 * Vocabulary-sharded operation (the lm_head is tensor-parallel and this GPU holds
 * columns [vocab_offset, vocab_offset + Vs) of every row).  tapout_shard_stats
 * reduces the local slice of every live row to one 32-byte record; the caller
 * exchanges the records of all G shards (an all-gather of 32 bytes per row and
 * GPU) and hands them, shard-major, to tapout_draft_stats_sharded, which returns
 * what tapout_draft_stats returns for the unsplit rows.  Records combine with
 * the associative rule the library uses between the slices of a row.
 *   max     largest logit of the slice (-inf for a fully masked slice)
 *   sum     sum_j 2^(x_j log2(e) - R), R = ceil(max log2(e)) (0 if max = -inf),
 *           over every element of the slice EXCEPT the first maximum (the one
 *           at `argmax`): the entropy of a peaked row is made of small terms,
 *           which a binary32 sum that also held the dominant one would round
 *           away; whoever merges the records adds the maximum's own term
 *           2^(max log2(e) - R) back in double
 *   ent     sum_j 2^(x_j log2(e) - R) (x_j log2(e) - R), over the same elements
 *   second  second largest logit of the slice, duplicates counted
 *   argmax  GLOBAL index (vocab_offset + local) of the first maximum
 *   x_tok   logit of the row's drafted token if its id lies in this slice,
 *           else NaN
 */
typedef struct {
    float max, sum, ent, second;
    int32_t argmax;
    float x_tok;
    int32_t reserved[2];
} tapout_shard_stat;

/*
 * shard     [B, KK, Vs] logits of this GPU's vocabulary slice
 * len       [B] i32 or NULL;  rows_mode 0: rows k < len[b] are live (draft rows,
 *           len = k_len, NULL = all); 1: rows k <= len[b] (target rows, len =
 *           n_draft, required)
 * tok       [B, KK - rows_mode] i32 GLOBAL token ids or NULL (x_tok = NaN)
 * out       [B * KK] records; rows that are not live are left untouched
 */
TAPOUT_API tapout_status tapout_shard_stats(tapout_ctx *ctx, const tapout_logits *shard,
                                 int32_t B, int32_t KK, int32_t Vs, int32_t vocab_offset,
                                 const int32_t *len, int32_t rows_mode, const int32_t *tok,
                                 tapout_shard_stat *out, void *stream);

/*
 * stats     [G, B * K] records of the G shards (shard g of row (b,k) at
 *           stats[g * B * K + b * K + k]), 1 <= G <= 256
 * V         size of the whole vocabulary (token ids are checked against it)
 * Everything else as tapout_draft_stats, which this call equals on the unsplit
 * rows up to the rounding of the binary32 records; u_draft is not supported.
 */
TAPOUT_API tapout_status tapout_draft_stats_sharded(tapout_ctx *ctx, const tapout_shard_stat *stats, int32_t G,
                                 int32_t B, int32_t K, int32_t V,
                                 const int32_t *draft_tok, const int32_t *k_len, const int32_t *arm,
                                 float *lse, float *entropy, float *p_top1, float *p_top2, float *margin,
                                 int32_t *top1_id, float *logq_tok,
                                 int32_t *n_stop, uint8_t *stop_fired, uint32_t *flags, void *stream);

/*
 * Acceptance step of tapout_verify from shard records of the target rows
 * (tapout_shard_stats with rows_mode = 1, tok = draft_tok, len = n_draft,
 * exchanged as for the draft side).  Writes what tapout_verify writes, except
 * the final token of a sampled sequence, for which out_tok[b, accept_len[b]]
 * is -1 and final_jobs[b] describes the draw that the two calls below make
 * (greedy and flagged sequences get their token, the argmax of the merged
 * records, and a job of kind 0).
 * stats      [G, B * (K + 1)] records, shard-major; V the whole vocabulary
 * draft_lse  [B,K] f32 from tapout_draft_stats(_sharded), or NULL if final_jobs
 *            is NULL
 * final_jobs [B] or NULL
 */
typedef struct {
    int32_t kind;     /* 0 nothing to draw, 1 residual max(0, p - q) of row `row`, 2 target row `row` alone */
    int32_t row;
    float ref_p;      /* exponent reference of the target row: its maximum over the whole vocabulary        */
    float ref_q;      /* exponent reference of the draft row: its lse                                       */
    double lam_est;   /* binary32-grade estimate of sum exp(t - ref_p) / sum exp(d - ref_q)                 */
} tapout_final_job;

TAPOUT_API tapout_status tapout_verify_accept_sharded(tapout_ctx *ctx, const tapout_shard_stat *stats, int32_t G,
                                 int32_t B, int32_t K, int32_t V,
                                 const float *logq_tok, const int32_t *draft_tok, const int32_t *n_draft,
                                 const uint8_t *greedy, const float *u_accept, const float *draft_lse,
                                 int32_t *accept_len, int32_t *out_tok, int32_t *n_out,
                                 float *target_lse, float *logp_tok, int32_t *target_top1,
                                 tapout_final_job *final_jobs, uint32_t *flags, void *stream);

/*
 * Final token of the sampled sequences over vocabulary shards, two calls with
 * one exchange between them (and a second exchange in the rare case below).
 *
 * tapout_shard_final_sums: this shard's sums of the job's row pair, in double:
 *   sums[b] = { A, B, R~, D, U } as defined for the unsplit path (A = sum of
 *   exp(t - ref_p), B = sum of exp(d - ref_q), R~ / D / U with lam_est); the
 *   per-slice sums stay in the context for the second call.
 * The caller all-gathers sums to sums_all [G, B, 5] (shard-major).
 *
 * tapout_shard_final_token: every shard forms the exact normaliser ratio and
 * the residual mass of every shard from sums_all, so all agree on the shard
 * that holds u * Z; that shard locates the token in its slice and writes its
 * GLOBAL id to tok_out[b], the others write -1.  If the sums cannot settle the
 * masses to 2e-10 (a heavy token with p = q to 1e-5, p == q, ...), every shard
 * instead writes its exact residual mass to exact_mass[b], sets need_exact[b]
 * and tok_out[b] = -1; the caller all-gathers exact_mass to exact_all [G, B]
 * and calls again with it (sequences that did not need it ignore it).
 * Both calls must follow tapout_shard_final_sums on the same context with the
 * same shards and jobs.
 *
 * target_shard [B,K+1,Vs], draft_shard [B,K,Vs]: this GPU's column slices
 * jobs [B] from tapout_verify_accept_sharded;  g: this shard's index in 0..G-1
 * u_sample [B] f32;  tok_out [B] i32;  exact_mass [B] f64;  need_exact [B] u8
 */
TAPOUT_API tapout_status tapout_shard_final_sums(tapout_ctx *ctx, const tapout_logits *target_shard, const tapout_logits *draft_shard,
                                 int32_t B, int32_t K, int32_t Vs, const tapout_final_job *jobs,
                                 double *sums, void *stream);
TAPOUT_API tapout_status tapout_shard_final_token(tapout_ctx *ctx, const tapout_logits *target_shard, const tapout_logits *draft_shard,
                                 int32_t B, int32_t K, int32_t Vs, int32_t vocab_offset, int32_t G, int32_t g,
                                 const tapout_final_job *jobs, const double *sums_all, const double *exact_all,
                                 const float *u_sample, int32_t *tok_out, double *exact_mass, uint8_t *need_exact,
                                 void *stream);

/*
 * Bandit update after verification (Algorithm 1 line 12; Section 3.2):
 *   r = alpha * m / gamma + (1 - alpha) * m / n,  m = accept_len, n = n_draft,
 *   evaluated in double as (alpha*m)/gamma + ((1-alpha)*m)/n without fused
 *   multiply-add (REWARD_SIMPLE: r = m / gamma); then N[arm] += 1,
 *   S[arm] += r, Q[arm] += r*r.
 * Sequences with active[b] == 0, an arm outside [0, n_arms), n_draft < 1 or
 * gamma < 1 are skipped.  With a shared bandit the B rewards are applied in
 * index order, each as one play.
 * If the configuration holds a SVIP_DIFF or ADAEDL arm, the rule state of every
 * active sequence with 1 <= n_draft <= K (K of the preceding tapout_draft_stats
 * call) is advanced as well, whatever arm was played: previous entropy <-
 * entropy of row n_draft - 1 of that call; AdaEDL rate and lambdas as described
 * at tapout_config.
 * TOKEN_LEVEL: arm is [B, max_k]; for k < min(n_draft, max_k): position k < m
 * plays arm[b,k] with reward 1, position m (if m < n_draft) with reward 0, later
 * positions are not played; gamma is only checked (>= 1).
 * arm, accept_len, n_draft, gamma [B] i32;  active [B] u8 or NULL
 */
TAPOUT_API tapout_status tapout_bandit_update(tapout_ctx *ctx, int32_t B, const int32_t *arm,
                                   const int32_t *accept_len, const int32_t *n_draft,
                                   const int32_t *gamma, const uint8_t *active, void *stream);

/*
 * tapout_bandit_update followed by tapout_bandit_select for the next drafting
 * session (Algorithm 1 line 12, then line 1 of the next round), in ONE launch
 * where every sequence has a sequence-level bandit of its own (n_bandits ==
 * max_batch, SEQUENCE_LEVEL): the thread that applies a sequence's reward picks
 * its next arm from the state it has just written.  Shared and token-level
 * bandits run the two kernels one after the other.  Results are bit-identical
 * to the two separate calls.
 * arm .. active as tapout_bandit_update;  u_ts, arm_out, flags as
 * tapout_bandit_select (u_ts: the uniforms of the NEXT selection).  arm_out may
 * be the same array as arm (each sequence's entry is read before it is written).
 */
TAPOUT_API tapout_status tapout_bandit_update_select(tapout_ctx *ctx, int32_t B, const int32_t *arm,
                                   const int32_t *accept_len, const int32_t *n_draft,
                                   const int32_t *gamma, const uint8_t *active,
                                   const float *u_ts, int32_t *arm_out, uint32_t *flags, void *stream);

/*
 * One whole round of Algorithm 1 in one call: tapout_draft_stats, tapout_verify,
 * tapout_bandit_update_select with the arguments below, in that order and with
 * the same decisions (statistics to the rounding of the binary32 slice sums:
 * the slice count may differ).  What the single call adds: when n_draft is
 * given by the caller (not this round's stop position), the streaming pass over
 * the target rows depends on nothing the draft side computes, and ONE launch
 * streams the draft rows and the target rows together: a launch over a few
 * hundred rows spends a fifth of its time filling and draining the chip, and
 * the pair pays that once.  Nor does verification then wait for the draft
 * epilogue: the accept decisions form log q(tok) from the draft pass's slice
 * sums themselves (binary32 precision: a decision can differ from the separate
 * calls' only if its uniform lies within ~1e-6, relative, of p/q) and the
 * epilogue runs in the same launch as the final-token search (option
 * "defer_epilogue"; contexts without a stateful stop rule).  The logq_tok and lse
 * written are the epilogue's own.
 *   draft [B,K,V], target [B,K+1,V]
 *   draft_tok [B,K];  k_len [B] or NULL;  greedy [B] or NULL
 *   n_draft   [B] tokens submitted to verification, or NULL: this round's stop
 *             position n_stop (Algorithm 1 as written; then nothing overlaps)
 *   arm       [B] IN: the arms of this round (from tapout_bandit_select or the
 *             previous tapout_round); OUT: the arms of the next round.
 *             SEQUENCE_LEVEL contexts; TOKEN_LEVEL: [B, max_k]
 *   u_ts_next uniforms of the next selection (Thompson Sampling), else NULL
 *   u_accept [B,K], u_sample [B]
 *   gamma [B], active [B] or NULL: as tapout_bandit_update
 *   outputs of tapout_draft_stats: lse, logq_tok (required: verification reads
 *             them), entropy, p_top1, p_top2, margin, top1_id, n_stop,
 *             stop_fired, draft_flags (each or NULL)
 *   outputs of tapout_verify: accept_len, out_tok, n_out (required), target_lse,
 *             logp_tok, target_top1, verify_flags (each or NULL)
 *   select_flags [B] or NULL: flags of the next selection
 * Draft-token sampling (u_draft) is not offered here.
 */
typedef struct {
    const tapout_logits *draft, *target;
    int32_t B, K, V;
    const int32_t *draft_tok, *k_len, *n_draft;
    const uint8_t *greedy;
    const float *u_accept, *u_sample, *u_ts_next;
    int32_t *arm;
    const int32_t *gamma;
    const uint8_t *active;
    float *lse, *entropy, *p_top1, *p_top2, *margin;
    int32_t *top1_id;
    float *logq_tok;
    int32_t *n_stop;
    uint8_t *stop_fired;
    uint32_t *draft_flags;
    int32_t *accept_len, *out_tok, *n_out;
    float *target_lse, *logp_tok;
    int32_t *target_top1;
    uint32_t *verify_flags, *select_flags;
} tapout_round_args;
TAPOUT_API tapout_status tapout_round(tapout_ctx *ctx, const tapout_round_args *args, void *stream);

/* Bandit state read-out (the arm values of Section 4.3 are sum_r / count) and
 * restore.  sum_r, sum_r2 (or NULL), count: HOST arrays [n_bandits, n_arms]
 * ([n_bandits, max_k, n_arms] for TOKEN_LEVEL) (f64, f64, i64); sum_r2 = summed squared rewards (UCB_TUNED), set to
 * sum_r^2 / count when NULL on restore.  Both calls synchronise `stream`.     */
TAPOUT_API tapout_status tapout_bandit_get_state(tapout_ctx *ctx, double *sum_r, double *sum_r2, int64_t *count, void *stream);
TAPOUT_API tapout_status tapout_bandit_set_state(tapout_ctx *ctx, const double *sum_r, const double *sum_r2, const int64_t *count, void *stream);

/* State of the stateful stop rules (Appendix A.1: SVIP-Difference, AdaEDL)
 * read-out and restore.  HOST arrays, each or NULL: prev_entropy [max_batch]
 * f32 (NaN = no previous draft), accept_rate [max_batch] f64, lambda
 * [max_batch, n_arms] f64 (only the columns of ADAEDL arms are used).  A new
 * context starts with NaN, adaedl_rate0 and the arms' thresholds.  Both calls
 * synchronise `stream`.                                                       */
TAPOUT_API tapout_status tapout_rule_state_get(tapout_ctx *ctx, float *prev_entropy, double *accept_rate, double *lambda, void *stream);
TAPOUT_API tapout_status tapout_rule_state_set(tapout_ctx *ctx, const float *prev_entropy, const double *accept_rate, const double *lambda, void *stream);

/*
 * Launch-shape tuning (host; takes effect from the next call).  Names:
 *   "wgs_target"  workgroups a streaming launch aims for (rows are cut into
 *                 slices until the launch has about this many), default 4096
 *   "slice_bytes" slice size aimed for when the rows alone already give that
 *                 many workgroups (long rows are still cut), default 65536,
 *                 at least 16384; for bfloat16 rows, binary32 rows take slices
 *                 of as many elements (twice the bytes)
 *   "min_slice"   smallest slice of a row, in elements, default 4096
 *   "fuse_head"   tapout_verify only: 1 = no launch of its own for the accept
 *                 decisions, every workgroup of the final-token slice kernel
 *                 takes them again for its sequence (pays while that kernel
 *                 is a few workgroups per compute unit); 0 = separate launch;
 *                 -1 (default) = decide per call from the launch size
 *   "defer_epilogue"  tapout_round only: 1 (default) = when n_draft comes
 *                 from the caller (and no arm carries rule state), the accept
 *                 decisions form log q(tok) from the draft pass's slice sums
 *                 themselves (binary32 precision) and the draft epilogue
 *                 runs beside the final-token locate kernel in one launch;
 *                 0 = the epilogue keeps its own launch ahead of the
 *                 verification, which then reads the logq_tok it wrote
 *   "exp_lookup"  final token: 1 (default) = where the target row and the
 *                 draft row are both bfloat16, the slice kernel takes
 *                 exp(logit) from a table of the 2 x 2302 bfloat16 values
 *                 with 2^-12 <= |x| < 63.5 (correctly rounded doubles, built
 *                 at tapout_create, held in LDS) and applies the rows'
 *                 references to the slice sums; rows whose references fall
 *                 outside the table's range, and other element types,
 *                 compute each exponential; 0 = always compute
 *   "profile_stride"  kernel timing (below) attaches events to every n-th
 *                 launch of a selected kernel only, default 1: an event pair
 *                 costs a few microseconds of the stream's time per launch
 * Results do not depend on these values except through the rounding of the
 * binary32 partial sums ("fuse_head", "profile_stride": not at all;
 * "defer_epilogue": an accept decision whose uniform lies within 1e-6
 * (relative) of p/q may fall the other way; "exp_lookup": the slice sums
 * agree to 2e-13 relative, so a final token whose inverse-CDF target lies that
 * close to a cell edge may move to the neighbouring cell).
 */
TAPOUT_API tapout_status tapout_set_option(tapout_ctx *ctx, const char *name, int32_t value);

/*
 * Kernel timing for benchmarks (host).  tapout_profile_enable makes the
 * library attach a pair of HIP events to each launch of the selected kernels;
 * the runtime stamps them with the begin and end of the kernel's execution
 * (kind_mask: bit k = kernel k below; at most max_records launches per kernel
 * between two reads; 0 switches timing off and releases the events).  tapout_profile_read synchronises `stream`, returns the
 * summed elapsed time and the number of launches recorded for one kernel since
 * the last read, and rewinds that kernel's records.  No device memory is
 * involved; timing is off by default.
 */
enum {
    TAPOUT_PROFILE_SELECT = 0,          /* bandit select                                            */
    TAPOUT_PROFILE_DRAFT_PASS = 1,      /* streaming pass over the draft logits                     */
    TAPOUT_PROFILE_DRAFT_FINALIZE = 2,  /* signals + stop scan                                      */
    TAPOUT_PROFILE_TARGET_PASS = 3,     /* streaming pass over the target logits                    */
    TAPOUT_PROFILE_VERIFY_HEAD = 4,     /* accept tests, first rejection, emitted prefix            */
    TAPOUT_PROFILE_VERIFY_SLICES = 5,   /* final token: slice sums of the row pair                  */
    TAPOUT_PROFILE_VERIFY_LOCATE = 6,   /* final token: normalisers, slice, token                   */
    TAPOUT_PROFILE_UPDATE = 7,          /* bandit update                                            */
    TAPOUT_PROFILE_SAMPLE_HEAD = 8,     /* draft-token sampling: one job per draft row              */
    TAPOUT_PROFILE_SAMPLE_SLICES = 9,   /* draft-token sampling: slice sums of every draft row      */
    TAPOUT_PROFILE_SAMPLE_LOCATE = 10,  /* draft-token sampling: slice, token                       */
    TAPOUT_PROFILE_STREAM_PAIR = 11,    /* tapout_round: draft and target rows in one streaming pass */
    TAPOUT_PROFILE_KINDS = 12
};
TAPOUT_API tapout_status tapout_profile_enable(tapout_ctx *ctx, uint32_t kind_mask, int32_t max_records);
TAPOUT_API tapout_status tapout_profile_read(tapout_ctx *ctx, int32_t kind, double *total_ms, int32_t *launches, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TAPOUT_H */
