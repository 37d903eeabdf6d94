// Internal declarations shared by the translation units of libtapout (gfx950).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "tapout.h"

namespace tapout {

constexpr int kBlock = 256;          // threads per workgroup of the streaming kernels (4 wavefronts)
constexpr int kStreamU = 4;          // 16-byte vectors a thread of the streaming kernels has in flight (one batch)
constexpr int kWave = 64;
constexpr float kLog2e = 1.44269504088896340736f;   // binary32 nearest to log2(e); also used (widened) by the finalisers
constexpr double kLn2 = 0.693147180559945309417232121458;

// Partial statistics of one (row, split) slice, written by row_reduce and
// merged by the finalisers.  Sums are kept in the base-2 domain relative to an
// integer reference R = ceil(v1 * log2 e):  S = sum 2^(x*log2e - R),
// T = sum 2^(x*log2e - R) * (x*log2e - R).  Changing the reference by an
// integer is an exact power-of-two scaling, so merging loses nothing.
// Target rows: S runs over the whole slice.  Draft rows: S and T leave out the batch of vectors in which the
// slice's first maximum was met (see the streaming kernel); the epilogue adds that batch's elements back from the
// logits, the first maximum itself as an exact term.  Shard records: S and T leave out the first maximum element only.
struct Partial {
    float v1;        // slice maximum (NaN entries ignored), -inf for an empty slice
    float S;
    float T;         // draft rows only
    float v2;        // second largest value of the slice counting duplicates (draft rows only)
    int32_t cand;    // element index at which the 8- (bf16) / 4- (f32) element vector holding the first maximum starts
                     // (shard records: the global index of the first maximum itself)
    int32_t pad[3];  // pad[0]: bits of the logit of the row's token if the slice / shard holds it, else NaN
                     // pad[1]: draft rows: the left-out batch's own sum (binary32, same reference): S + it covers the slice
};
static_assert(sizeof(Partial) == 32, "Partial is one 32-byte record");
static_assert(sizeof(tapout_shard_stat) == sizeof(Partial), "shard records are staged and merged as partials");

// Final-token job of one sequence, produced by the verify finaliser and
// consumed by the residual sampler.
struct SampleJob {
    int32_t kind;    // 0: nothing to sample (greedy / flagged: token already written), 1: residual max(0,p-q), 2: target row only
    int32_t row;     // m: target row (and draft row for kind 1) to sample from
    float ref_p;     // exponent reference of the target row (its maximum)
    float ref_q;     // exponent reference of the draft row (its lse)
    double lam;      // binary32-grade estimate of S_p / S_q in those references (kind 1)
};


static_assert(sizeof(tapout_final_job) == sizeof(SampleJob), "the public job record is the internal one");

constexpr int kExpBf16Doubles = 4608;   // exp(x) of the bfloat16 values with 2^-12 <= |x| < 63.5, both signs, and two stand-in pairs (see the final-token slice kernel)

constexpr int kBandCap = 32;         // band elements per job the locate kernel settles one by one; more: exact slow path

// The job as it lies in memory, together with the list of elements of its row pair whose sign of a - L b is
// open until L is exact (appended by the slice kernel, read by the locate kernel).  One record, so that the
// locate kernel finds everything about its job in two neighbouring cache lines of one page.
struct JobRecord {
    SampleJob job;
    int32_t band_cnt;              // appended so far; entries beyond kBandCap are dropped (the count still grows)
    int32_t pad;
    int32_t band_idx[kBandCap];    // element indices, any order
};
static_assert(sizeof(JobRecord) == 160, "job record layout");

__host__ __device__ inline float ref_of_max(float v1)
{
    // integer-valued reference >= v1*log2e; 0 for a slice without finite maximum
    return (v1 == -INFINITY) ? 0.0f : ceilf(v1 * kLog2e);
}

// Optional timing of one launch: when both events are set the kernel is launched through
// hipExtLaunchKernelGGL, which stamps them with the begin / end of the kernel's execution itself.
struct Timing {
    hipEvent_t start = nullptr, stop = nullptr;
};

struct RowReduceArgs {
    const void *base;
    int64_t stride_b, stride_k;   // elements
    int32_t V;
    int32_t KK;                   // rows per sequence in this tensor (K for draft, K+1 for target)
    int32_t nsplit;               // workgroups per row
    int32_t per;                  // 16-byte vectors per slice (multiple of 64; nsplit * per covers any row)
    int32_t n_rows;               // B * KK
    const int32_t *len;           // draft: k_len (or NULL); target: n_draft
    int32_t len_mode;             // 0: row k active iff k < len[b] (NULL: all); 1: iff k <= clamp(len[b], 1, KK-1)
    Partial *out;                 // [n_rows, nsplit]
    JobRecord *clear_jobs;        // NULL, or [B]: the first workgroup of sequence b empties the band list of its job record
    const int32_t *tok;           // NULL, or [B, tok_rows]: row k < tok_rows of sequence b has a token whose logit the
    int32_t tok_rows;             //   slice holding it puts into its partial (pad[0]; NaN bits in all other partials)
    const int32_t *arm_src;       // NULL, or [B] with arm_dst [B]: the first workgroup of sequence b copies the sequence's arm
    int32_t *arm_dst;             //   (a later launch overwrites the caller's array while another of its workgroups still wants the old value)
};
// Streaming pass: one Partial per (row, slice).  Returns hipGetLastError() after enqueueing.
hipError_t launch_row_reduce(const RowReduceArgs &a, int dtype, bool full, hipStream_t st, Timing tm);
// Draft pass (all statistics) and target pass of the same sequences in one launch.
hipError_t launch_row_reduce_pair(const RowReduceArgs &d, int d_dtype, const RowReduceArgs &t, int t_dtype, hipStream_t st, Timing tm);

struct DraftFinalArgs {
    const void *base; int32_t dtype; int64_t stride_b, stride_k;
    int32_t B, K, V, nsplit;
    int32_t per;                  // 16-byte vectors per slice of the streaming pass that wrote `part`
    const Partial *part;
    const int32_t *draft_tok, *k_len, *arm;
    int32_t arm_stride;           // 0: arm[b] decides every step; > 0 (token-level bandits): step k uses arm[b * arm_stride + k]
    int32_t n_arms; int32_t rule[TAPOUT_MAX_ARMS]; float threshold[TAPOUT_MAX_ARMS];
    float *lse, *entropy, *p_top1, *p_top2, *margin, *logq_tok;
    int32_t *top1_id, *n_stop; uint8_t *stop_fired; uint32_t *flags;
    // stateful rules (SVIP-Difference, AdaEDL); all NULL when the configuration has no such arm
    const float *prev_entropy;    // [B] entropy of the last drafted position of the previous draft, NaN = none
    const double *lambda;         // [B, n_arms] AdaEDL thresholds
    double adaedl_gamma;
    float *round_entropy;         // [B, K] entropies of this draft, kept for the state update
    // vocabulary-sharded input: part holds the records of `shards` vocabulary shards, shard-major [shards, B*K], instead
    // of slice partials [B*K, nsplit] (then nsplit = shards; the argmax of a record is exact and global, the logit of
    // the drafted token travels in the record, and base is not used)
    int32_t shards;
};
hipError_t launch_draft_finalize(const DraftFinalArgs &a, hipStream_t st, Timing tm);

// One record per live row of a vocabulary shard from its slice partials (see tapout_shard_stats).
struct ShardMergeArgs {
    const void *base; int32_t dtype; int64_t stride_b, stride_k;
    int32_t B, KK, Vs, nsplit, per, vocab_offset, rows_mode;
    const Partial *part; const int32_t *len, *tok;
    Partial *out;
};
hipError_t launch_shard_merge(const ShardMergeArgs &a, hipStream_t st, Timing tm);

struct BanditArgs {
    int32_t policy, n_bandits, n_arms, B;
    int32_t positions;            // bandits per slot: 1 (sequence-level) or max_k (token-level, one per draft position)
    int32_t reward;               // tapout_reward
    double alpha;
    double *sum_r, *sum_r2; int64_t *count;
    // stateful stop rules (all NULL when the configuration has no such arm)
    int32_t rule[TAPOUT_MAX_ARMS];
    float *prev_entropy; double *accept_rate; double *lambda;
    const float *round_entropy; int32_t round_K;      // entropies of the last draft_stats call, [B, round_K]; round_K = 0: none
    double ad_alpha, ad_beta1, ad_beta2, ad_eps;
    int32_t ad_steer;             // tapout_config.adaedl_steer
};
// Kernel arguments sit in device memory and reach a wavefront through the scalar cache, one 64-byte line per miss,
// and the compiler loads a field where the code first wants it: a kernel that is a chain of round trips anyway takes
// a miss of this kind at several points along the chain (with the arguments in host memory instead, the final-token
// launches of a Llama-3-vocabulary round take 4.6 and 6.5 us longer).  Reading one word of every line first thing
// makes them one round trip; the later loads hit.  (The hidden arguments behind the declared ones, grid and
// workgroup sizes, are one more line: the kernels on the round's critical path do not read them.)
template <class T>
__device__ inline int32_t arg_lines(const T &a)
{
    const int32_t *w = reinterpret_cast<const int32_t *>(&a);
    int32_t acc = w[sizeof(T) / 4 - 1];
#pragma unroll
    for (size_t i = 0; i < sizeof(T) / 4; i += 16) acc |= w[i];
    return acc;
}
template <class... Ts>
__device__ inline void warm_args(const Ts &...as)
{
    const int32_t acc = (arg_lines(as) | ...);
    asm volatile("" :: "s"(acc));
}

// Verification + final token: the head kernel merges the target partials of each sequence, takes the
// accept decisions and describes the final-token draw (SampleJob); the slice kernel sums the row pair
// per slice; the locate kernel finds the token.
constexpr int32_t kVerifyOwnQ = 1;          // accept decisions form log q(tok) from the draft partials (see dpart)
constexpr int32_t kVerifyNoExpTable = 2;    // final-token slice kernel: computed exponentials also for bfloat16 row pairs
// (Kept at 512 bytes or less: past that the compiler reaches the arguments differently and the fused slice kernel
// takes 107 vector registers instead of 95, one wavefront per SIMD fewer.  vflags and d_nsplit sit in what would be
// alignment padding.)
struct VerifyArgs {
    const void *tbase; int32_t t_dtype; int32_t vflags; int64_t t_stride_b, t_stride_k;   // vflags: kVerify* bits
    const void *dbase; int32_t d_dtype; int32_t d_nsplit; int64_t d_stride_b, d_stride_k;
    int32_t B, K, V, nsplit;      // nsplit: slices per row of the streaming pass
    int32_t nsl;                  // slices per row of the final-token passes (kSampleSlice elements each)
    // The slice and locate kernels work on "jobs": one per sequence for verification (jps = 1, job j belongs to
    // sequence j), one per draft row for draft-token sampling (jps = K, job j = row j % K of sequence j / K).
    // jobs, part1, part2 and u_sample are indexed by job; the rows of a job are rows job.row of its sequence.
    int32_t jps, n_jobs;
    int32_t *tok_direct;          // draft-token sampling: token of job j goes to tok_direct[j] instead of out_tok
    int32_t shards;               // > 0: part holds records of vocabulary shards, shard-major [shards, B*(K+1)] (head kernel only)
    int32_t fused_head;           // 1: no head launch; every workgroup of the slice kernel works out its sequence's job itself
    SampleJob *final_jobs;        // sharded head: the job of every sequence for the caller (or NULL)
    const Partial *part;
    const float *draft_lse, *logq_tok; const int32_t *draft_tok, *n_draft; const uint8_t *greedy;
    const float *u_accept, *u_sample;
    int32_t *accept_len, *out_tok, *n_out;
    float *target_lse, *logp_tok; int32_t *target_top1; uint32_t *flags;
    uint32_t *flags_ws;           // internal copy of the flags (always present)
    JobRecord *jobs;              // [jobs]
    double *part1;                // [jobs, nsl, 5]  A, B, R~, D, U of each slice
    double *part2;                // [B, nsl]     exact weight of each slice (slow path)
    const double *exp_table;      // 2^(k/256), k = 0..255, then the kExpBf16Doubles entries of the bfloat16 table
    // tapout_round (jps = 1): the locate kernel also ends the round of its sequence: reward into the sequence's bandit
    // (arm b_arm_in[b], accept_len, n_draft, b_gamma, b_active as tapout_bandit_update) and the arm of the next round
    // (b_arm_out, b_flags as tapout_bandit_select).  Sequence-level UCB bandits, one per sequence.
    int32_t bandit_tail;
    BanditArgs bandit;
    const int32_t *b_arm_in, *b_gamma; const uint8_t *b_active; const float *b_u_ts; int32_t *b_arm_out; uint32_t *b_flags;
    // tapout_round with n_draft from the caller: the accept decisions form log q(tok) and the draft rows' lse themselves
    // from the draft pass's partials (kVerifyOwnQ; dpart [B*K, d_nsplit], whose token slots the draft pass filled), so the
    // draft epilogue can run beside the locate kernel, in the same launch (B more workgroups, ahead of the others).
    const Partial *dpart;
};
static_assert(sizeof(VerifyArgs) <= 512, "see the note above the struct");
// fin: the draft epilogue's arguments when kVerifyOwnQ is set (pass 2 then runs it too), else NULL.
hipError_t launch_verify(const VerifyArgs &a, int pass /*0 head, 1 slices, 2 locate*/, hipStream_t st, Timing tm,
                         const DraftFinalArgs *fin = nullptr);
// The accept decisions can take log q(tok) from the draft partials themselves (kVerifyOwnQ) for these shapes.
inline bool own_q_shape(int K, int nsplit_target, int nsplit_draft)
{
    auto fits = [](int rows, int nsplit) {
        if (nsplit > 16 || rows > 64) return false;
        int sh = 0;
        while ((1 << sh) < nsplit) ++sh;
        return (rows << sh) <= 512;
    };
    return fits(K + 1, nsplit_target) && fits(K, nsplit_draft);
}

// Draft-token sampling (Algorithm 1, the sampling step of the draft loop): one job per live draft row with the
// row's maximum as exponent reference; bad live rows get token -1 at once.  The slice and locate kernels of
// the final token then draw the tokens.  Arguments as VerifyArgs with the draft tensor in the target slots:
// tbase/t_* = draft logits, part = draft partials [B*K, nsplit], n_draft = k_len (or NULL), jps = K.
hipError_t launch_sample_head(const VerifyArgs &a, hipStream_t st, Timing tm);

// Final token over vocabulary shards (see tapout_shard_final_sums / tapout_shard_final_token).  The VerifyArgs
// describe this shard's column slices (V = its width, nsl = its slices, jobs / part1 / part2 of the context).
struct ShardFinalArgs {
    VerifyArgs v;
    const SampleJob *jobs_in;     // [B] jobs as the caller holds them
    double *sums_out;             // [B, 5]                       (sums)
    const double *sums_all;       // [G, B, 5]                    (token)
    const double *exact_all;      // [G, B] or NULL               (token)
    int32_t G, g, vocab_offset;
    int32_t *tok_out; double *exact_mass; uint8_t *need_exact;
};
hipError_t launch_shard_final_sums(const ShardFinalArgs &a, hipStream_t st);
hipError_t launch_shard_final_token(const ShardFinalArgs &a, hipStream_t st);

constexpr int kSampleSlice = 2048;   // elements per slice of the final-token passes

hipError_t launch_bandit_select(const BanditArgs &a, const float *u_ts, int32_t *arm_out, uint32_t *flags, hipStream_t st, Timing tm);
hipError_t launch_bandit_update(const BanditArgs &a, const int32_t *arm, const int32_t *accept_len,
                                const int32_t *n_draft, const int32_t *gamma, const uint8_t *active, hipStream_t st, Timing tm);
hipError_t launch_bandit_update_select(const BanditArgs &a, const int32_t *arm, const int32_t *accept_len,
                                       const int32_t *n_draft, const int32_t *gamma, const uint8_t *active,
                                       const float *u_ts, int32_t *arm_out, uint32_t *flags, hipStream_t st, Timing tm);

// ---- device helpers --------------------------------------------------------
#ifdef __HIPCC__

template <class F, class... Args>
inline void launch_kernel(F kernel, dim3 grid, dim3 block, hipStream_t st, Timing tm, Args... args)
{
    if (tm.start && tm.stop) hipExtLaunchKernelGGL(kernel, grid, block, 0, st, tm.start, tm.stop, 0, args...);
    else hipLaunchKernelGGL(kernel, grid, block, 0, st, args...);
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int DT> struct Elem;
template <> struct Elem<TAPOUT_F32>  { static constexpr int size = 4, vec = 4; };
template <> struct Elem<TAPOUT_BF16> { static constexpr int size = 2, vec = 8; };

__device__ inline float bf16_to_float(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

template <int DT>
__device__ inline float load_elem(const void *row, int64_t j)
{
    if constexpr (DT == TAPOUT_F32) return ((const float *)row)[j];
    else return bf16_to_float(((const uint16_t *)row)[j]);
}

__device__ inline float load_elem_rt(const void *row, int dtype, int64_t j)
{
    return dtype == TAPOUT_F32 ? ((const float *)row)[j] : bf16_to_float(((const uint16_t *)row)[j]);
}

// Split a row into an unaligned head, 16-byte vectors and a tail.
template <int DT>
__device__ inline void row_geometry(const void *row, int32_t V, int &head, int &nvec, int &tail)
{
    constexpr int VEC = Elem<DT>::vec;
    int mis = (int)(((uintptr_t)row & 15u) / Elem<DT>::size);
    head = (VEC - mis) % VEC;
    if (head > V) head = V;
    nvec = (V - head) / VEC;
    tail = V - head - nvec * VEC;
}

template <int DT>
__device__ inline void unpack(const u32x4 &w, float (&x)[Elem<DT>::vec])
{
    if constexpr (DT == TAPOUT_F32) {
        x[0] = __uint_as_float(w.x); x[1] = __uint_as_float(w.y);
        x[2] = __uint_as_float(w.z); x[3] = __uint_as_float(w.w);
    } else {
        x[0] = __uint_as_float(w.x << 16); x[1] = __uint_as_float(w.x & 0xffff0000u);
        x[2] = __uint_as_float(w.y << 16); x[3] = __uint_as_float(w.y & 0xffff0000u);
        x[4] = __uint_as_float(w.z << 16); x[5] = __uint_as_float(w.z & 0xffff0000u);
        x[6] = __uint_as_float(w.w << 16); x[7] = __uint_as_float(w.w & 0xffff0000u);
    }
}

__device__ inline const void *row_address(const void *base, int dtype, int64_t stride_b, int64_t stride_k, int b, int k)
{
    int64_t off = (int64_t)b * stride_b + (int64_t)k * stride_k;
    return (const char *)base + off * (dtype == TAPOUT_F32 ? 4 : 2);
}

constexpr int kStageCap = 256;     // partials staged in LDS at a time by an epilogue (8 KB)
constexpr int kScanCap = 4096;     // largest K: one stop / accept decision byte per draft position fits LDS

// All threads of the workgroup copy `count` partials (count <= kStageCap) into LDS; the loads of
// all threads are in flight together, so the copy costs one memory round trip.
__device__ inline void stage_partials(Partial *sh, const Partial *src, int count)
{
    const u32x4 *s = (const u32x4 *)src;
    u32x4 *d = (u32x4 *)sh;
    for (int i = threadIdx.x; i < 2 * count; i += kBlock) d[i] = s[i];      // (256-thread workgroups)
    __syncthreads();
}

// The same copy in two steps for a 256-thread workgroup, so that a caller can put other independent loads
// into the same memory round trip: stage_issue requests (at most two 16-byte words per thread, count <=
// kStageCap), stage_commit stores to LDS and synchronises.
struct StageRegs { u32x4 w0, w1; };
__device__ inline StageRegs stage_issue(const Partial *src, int count)
{
    const u32x4 *s = (const u32x4 *)src;
    StageRegs r;
    r.w0 = r.w1 = u32x4{0u, 0u, 0u, 0u};
    const int i = threadIdx.x;
    if (i < 2 * count) r.w0 = s[i];
    if (i + 256 < 2 * count) r.w1 = s[i + 256];
    return r;
}
__device__ inline void stage_commit(Partial *sh, const StageRegs &r, int count)
{
    u32x4 *d = (u32x4 *)sh;
    const int i = threadIdx.x;
    if (i < 2 * count) d[i] = r.w0;
    if (i + 256 < 2 * count) d[i + 256] = r.w1;
    __syncthreads();
}

// The same for records of vocabulary shards: src is shard-major [shards, rows_total]; the `count` = rows * shards
// records of rows row0 .. land in LDS row-major ([row][shard]), where merge_partials expects the slices of a row.
__device__ inline StageRegs stage_issue_shards(const Partial *src, int64_t rows_total, int64_t row0, int shards, int count)
{
    StageRegs r;
    r.w0 = r.w1 = u32x4{0u, 0u, 0u, 0u};
    const u32x4 *s = (const u32x4 *)src;
    const int i = threadIdx.x;                                 // 16-byte word i of the LDS image: record i/2, half i%2
    if (i < 2 * count) { const int rec = i >> 1; r.w0 = s[2 * ((int64_t)(rec % shards) * rows_total + row0 + rec / shards) + (i & 1)]; }
    if (i + 256 < 2 * count) { const int rec = (i + 256) >> 1; r.w1 = s[2 * ((int64_t)(rec % shards) * rows_total + row0 + rec / shards) + (i & 1)]; }
    return r;
}

// v[i] for a small array that lives in scalar registers (kernel arguments): selects instead of a load from
// the argument buffer, which would be one more memory round trip.
template <class T>
__device__ inline T pick8(const T (&v)[TAPOUT_MAX_ARMS], int i)
{
    T r = v[0];
#pragma unroll
    for (int q = 1; q < TAPOUT_MAX_ARMS; ++q) r = (i == q) ? v[q] : r;
    return r;
}

// ---- merging the statistics of the pieces of a row ---------------------------------------------------
// A piece is one slice of a row (a Partial) or one vocabulary shard of it (a shard record).  Two kinds:
//   EXCL = false  S, T run over every element of the piece (target rows of the unsharded path);
//   EXCL = true   S, T leave the piece's first maximum element out (draft rows and all shard records): the entropy of a
//                 peaked row is made of small terms, and they must not share a binary32 sum with the dominant one.
//                 When two pieces meet, the maximum of the one that does not hold the row's maximum is an ordinary
//                 term again and is added in (binary32 exponential: it is either negligible or the row is not peaked);
//                 the row's own first maximum is added at the very end as an exact double term.
struct Piece {
    float M;          // maximum (-inf: no finite element)
    double S, T;      // base-2 sums relative to ref_of_max(M)
    float v2;         // second largest, duplicates counted
    int32_t idx;      // EXCL: index of the first maximum; else: start of the vector that holds it
    float xt;         // logit of the row's token if this piece holds it, else NaN
};

__device__ inline bool piece_empty(const Piece &e) { return e.M == -INFINITY && !(e.S != e.S); }

__device__ inline Piece empty_piece()
{
    Piece e;
    e.M = -INFINITY; e.S = 0.0; e.T = 0.0; e.v2 = -INFINITY; e.idx = 0x7fffffff; e.xt = NAN;
    return e;
}

__device__ inline Piece piece_from_words(const u32x4 &w0, const u32x4 &w1)
{
    Piece e;
    e.M = __uint_as_float(w0.x); e.S = (double)__uint_as_float(w0.y); e.T = (double)__uint_as_float(w0.z);
    e.v2 = __uint_as_float(w0.w); e.idx = (int32_t)w1.x; e.xt = __uint_as_float(w1.y);
    if (piece_empty(e)) { e.S = 0.0; e.T = 0.0; e.v2 = -INFINITY; e.idx = 0x7fffffff; }       // one image for every empty piece
    return e;
}
__device__ inline Piece piece_from_partial(const Partial &p)
{
    const u32x4 *w = (const u32x4 *)&p;
    return piece_from_words(w[0], w[1]);
}

// Commutative: both partners of an exchange compute the same bits.
template <bool EXCL>
__device__ inline Piece merge_pair(const Piece &a, const Piece &b)
{
    const bool a_wins = a.M > b.M || (a.M == b.M && a.idx <= b.idx);            // the piece with the row's first maximum
    const float Mw = a_wins ? a.M : b.M, Ml = a_wins ? b.M : a.M;
    const double Sw = a_wins ? a.S : b.S, Sl = a_wins ? b.S : a.S;
    const double Tw = a_wins ? a.T : b.T, Tl = a_wins ? b.T : a.T;
    const float Rw = ref_of_max(Mw);
    const double d = (double)Rw - (double)ref_of_max(Ml);                       // integer; >= 0 unless the other piece is empty
    const int di = d > 4000.0 ? 4000 : (d < -4000.0 ? -4000 : (int)d);          // 2^-4000 underflows to 0 as it should
    Piece o;
    o.M = Mw;
    o.S = Sw + ldexp(Sl, -di);                                                  // exact power-of-two scaling
    o.T = Tw + ldexp(Tl - d * Sl, -di);
    if constexpr (EXCL) {
        if (Ml > -INFINITY) {                                                   // the other piece's maximum: an ordinary term here
            const float y = __builtin_fmaf(Ml, kLog2e, -Rw);
            const float e = __builtin_amdgcn_exp2f(y);
            o.S += (double)e;
            o.T += (double)e * (double)fmaxf(y, -200.0f);
        }
    }
    o.v2 = fmaxf(fmaxf(fminf(a.M, b.M), a.v2), b.v2);                           // second largest of the union, duplicates counted
    o.idx = a_wins ? a.idx : b.idx;
    o.xt = (a.xt == a.xt) ? a.xt : b.xt;                                        // at most one piece holds the token
    return o;
}

// Merged statistics of a whole row, in double.
struct RowTotal {
    float M;          // row maximum
    double R;         // integer reference of M
    double Sx, Tx;    // the merged base-2 sums relative to R as the pieces carry them: EXCL: without the row's first maximum
    double yM;        // M log2e - R, in (-1, 0]
    double eM;        // EXCL: 2^yM to binary32 precision, the term of the first maximum; else 0
    double S;         // sum over ALL elements: Sx + eM
    float v2;
    int32_t cand;     // EXCL: index of the first maximum; else: start of the vector that holds it
    bool bad;
};

template <bool EXCL>
__device__ inline RowTotal row_total(const Piece &p)
{
    RowTotal r;
    r.M = p.M;
    r.R = (double)ref_of_max(p.M);
    const bool finite = p.M > -INFINITY && p.M < INFINITY;
    r.yM = finite ? (double)p.M * (double)kLog2e - r.R : 0.0;
    r.eM = (EXCL && finite) ? (double)__builtin_amdgcn_exp2f((float)r.yM) : 0.0;
    r.Sx = p.S; r.Tx = p.T;
    r.S = p.S + r.eM;
    r.v2 = p.v2; r.cand = p.idx;
    r.bad = !(r.S > 0.0) || !(r.S < INFINITY) || !finite;
    return r;
}

// Signals of a row whose sums leave the first maximum out (EXCL), written so that the binary32 error of eM and of the
// sums enters every result as a RELATIVE error, however peaked the row: with eps = Sx / eM (everything but the maximum,
// relative to it),
//   log2 sum_j 2^(x_j log2e) = R + yM + log2(1 + eps)          exactly: no eM in it
//   H / ln 2 = log2(1 + eps) + (yM eps - Tx / eM) / (1 + eps)
//   p_top1 = 1 / (1 + eps),  p_top2 = r2 p_top1,  margin = (1 - r2) p_top1,  r2 = 2^((v2 - M) log2e)  (double: a margin
//   between near-tied logits is the small difference 1 - r2)
struct RowSignals { double lse, H, p1, p2, margin; };
__device__ inline RowSignals row_signals(const RowTotal &r, bool has_second)
{
    RowSignals o;
    const double inv = 1.0 / r.eM, eps = r.Sx * inv;
    const double l2 = log2(1.0 + eps);
    o.p1 = 1.0 / (1.0 + eps);
    o.lse = (r.R + r.yM + l2) * kLn2;
    const double Hd = (l2 + (r.yM * eps - r.Tx * inv) * o.p1) * kLn2;
    o.H = Hd > 0.0 ? Hd : 0.0;
    const double r2 = has_second ? exp2(((double)r.v2 - (double)r.M) * (double)kLog2e) : 0.0;
    o.p2 = r2 * o.p1;
    o.margin = (1.0 - r2) * o.p1;
    return o;
}

// The batch of vectors (or the single head / tail element) of the draft pass in which a slice met its first
// maximum, as the streaming kernel laid its work out: thread t of the slice's workgroup takes vectors
// v0 + t + q * kBlock, q = 0, 1, ..., in batches of kStreamU.  `cand` is the element index at which the vector with the
// first maximum starts (or the index of a head / tail element).  All addresses are checked against the slice.
struct BatchRegs {
    u32x4 w[kStreamU];
    uint32_t valid;       // bit u: vector u is wanted (the others hold stand-in data); bit 8: a single element, in `single`
    uint32_t single;      // bits of the single head / tail element
    int32_t first;        // element index of vector 0 (or of the single element)
    int32_t ucand;        // which vector of the batch the candidate is: the one that holds the first maximum
};

// Written so that the four requests are straight-line code at the end: where the branches above them only choose
// addresses (`safe`, any readable 16-byte aligned address, stands in for a vector that is not wanted; the valid bits
// tell), the compiler has no loaded registers to merge between branches.  With the requests inside the branches it
// merged them with the zeros of the other paths and waited for the data right there: a second memory round trip in a
// kernel that is nothing but round trips.
__device__ inline BatchRegs batch_issue(const void *row, int dtype, int32_t V, int32_t cand, int split, int per, const void *safe)
{
    const int esz = dtype == TAPOUT_F32 ? 4 : 2, vsh = dtype == TAPOUT_F32 ? 2 : 3, VEC = 1 << vsh;
    BatchRegs b;
    b.valid = 0; b.first = 0; b.ucand = 0; b.single = 0;
    // (device memory, and said so: chosen among several pointers the compiler would otherwise treat them as generic
    // addresses, whose loads also count as LDS traffic)
    typedef const __attribute__((address_space(1))) u32x4 *GlobalVec;
    GlobalVec p[kStreamU];
#pragma unroll
    for (int u = 0; u < kStreamU; ++u) p[u] = (GlobalVec)safe;
    if (cand >= 0 && cand < V) {
        // the row's unaligned head, 16-byte vectors and tail (as row_geometry)
        const int mis = (int)(((uintptr_t)row & 15u) / (unsigned)esz);
        int head = (VEC - mis) & (VEC - 1);
        if (head > V) head = V;
        const int nvec = (V - head) >> vsh;
        if (cand < head || cand >= head + (nvec << vsh)) {
            b.single = __float_as_uint(load_elem_rt(row, dtype, cand));
            b.valid = 0x100u; b.first = cand;
        } else {
            const int i = (cand - head) >> vsh;
            const int v0 = min(split * per, nvec), v1e = min(v0 + per, nvec);
            if (i >= v0 && i < v1e) {                                           // else: not a candidate of this slice: stale record
                const int rel = i - v0, t = rel % kBlock, q0 = (rel / kBlock) / kStreamU * kStreamU;
                GlobalVec vp = (GlobalVec)((const char *)row + (int64_t)head * esz);
                b.first = head + ((v0 + t + q0 * kBlock) << vsh);
                b.ucand = rel / kBlock - q0;
#pragma unroll
                for (int u = 0; u < kStreamU; ++u) {
                    const int iu = v0 + t + (q0 + u) * kBlock;
                    p[u] = vp + min(iu, v1e - 1);                               // v0 <= i <= v1e - 1: inside the slice
                    b.valid |= iu < v1e ? 1u << u : 0u;
                }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < kStreamU; ++u) b.w[u] = *p[u];
    return b;
}

// The elements of a piece's left-out batch, except the first one equal to the piece's maximum M: their two sums
// relative to ref_of_max(M) (binary32 terms as in the streaming pass: they are small, or the row is not peaked) and
// the index of that first maximum (0x7fffffff if the batch does not hold it).
struct BatchExtra { float sa, ta; int32_t idx; };

// The first maximum lies in the candidate vector (the thread's running maximum reached M there: the vectors before it
// in the batch are below M, equal values after it are duplicates and count as ordinary terms), so only that vector is
// searched.  The entropy terms are formed without looking at them; a masked (-inf) logit makes their sum NaN
// (0 * -inf), and only then they are formed again with the exponent clamped.
template <int DT>
__device__ inline BatchExtra batch_extra_t(float M, const BatchRegs &b)
{
    constexpr int VEC = Elem<DT>::vec;
    const float R = ref_of_max(M);
    BatchExtra o;
    o.sa = 0.0f; o.ta = 0.0f; o.idx = 0x7fffffff;
    auto sums = [&](bool clamp) {
        float sa = 0.0f, ta = 0.0f;
        int32_t idx = 0x7fffffff;
        if (b.valid & 0x100u) {
            const float x = __uint_as_float(b.single);
            if (x == M) idx = b.first;
            else {
                const float y = __builtin_fmaf(x, kLog2e, -R), e = __builtin_amdgcn_exp2f(y);
                sa = e; ta = e * (clamp ? fmaxf(y, -200.0f) : y);
            }
        }
#pragma unroll
        for (int u = 0; u < kStreamU; ++u) {
            if (!((b.valid >> u) & 1u)) continue;
            float x[VEC];
            unpack<DT>(b.w[u], x);
            const bool search = u == b.ucand;
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                const bool first = search && x[j] == M && idx == 0x7fffffff;
                const float y = __builtin_fmaf(x[j], kLog2e, -R);
                const float e = first ? 0.0f : __builtin_amdgcn_exp2f(y);
                if (search) idx = first ? b.first + u * kBlock * VEC + j : idx;
                sa += e;
                ta = __builtin_fmaf(e, clamp ? fmaxf(y, -200.0f) : y, ta);
            }
        }
        o.sa = sa; o.ta = ta; o.idx = idx;
    };
    sums(false);
    if (o.ta != o.ta) sums(true);
    return o;
}
__device__ inline BatchExtra batch_extra(const Piece &p, const BatchRegs &b, int dtype)
{
    if (piece_empty(p) || !b.valid) { BatchExtra o; o.sa = 0.0f; o.ta = 0.0f; o.idx = 0x7fffffff; return o; }
    return dtype == TAPOUT_F32 ? batch_extra_t<TAPOUT_F32>(p.M, b) : batch_extra_t<TAPOUT_BF16>(p.M, b);
}

// Completes a piece of the draft pass: the left-out batch back in, all but the first maximum, whose index becomes idx.
__device__ inline void batch_fix(Piece &p, const BatchRegs &b, int dtype)
{
    const BatchExtra x = batch_extra(p, b, dtype);
    p.S += (double)x.sa; p.T += (double)x.ta;
    p.idx = x.idx;
}

// Sequential merge of the `n` pieces of one row held as Partials (LDS or memory) at stride `stride` records.
// EXCL pieces must have been completed (batch_fix) before: idx exact, only the first maximum left out.
template <bool EXCL>
__device__ inline RowTotal merge_partials(const Partial *p, int n, int stride = 1)
{
    Piece acc = empty_piece();
    for (int s = 0; s < n; ++s) acc = merge_pair<EXCL>(acc, piece_from_partial(p[(int64_t)s * stride]));
    return row_total<EXCL>(acc);
}

// ---- lane-parallel merge ------------------------------------------------------------------------
// A sequential merge walks the slices of a row one after the other: eight dependent LDS reads and rescalings, about
// 1.4 us of a per-sequence kernel whose every other step is one memory round trip.  When the rows of a sequence
// times the slice count rounded up to a power of two (P <= 16) fit two passes of one workgroup, thread t instead
// takes partial (row t / P, slice t % P) straight from memory (and the partial 256 / P rows further on in the
// second pass), and the P lanes of a row combine their records with DPP exchanges in log2 P steps.  The combination
// is commutative, so both partners of an exchange, and in the end all lanes of a group, hold the same bits; the
// first lane of the group puts the row's total into LDS.
struct RowSlot { RowTotal r; float xt; };

template <int CTRL>
__device__ inline Piece piece_dpp(const Piece &e)
{
    auto mv = [](int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true); };
    Piece o;
    o.M = __int_as_float(mv(__float_as_int(e.M)));
    o.S = __hiloint2double(mv(__double2hiint(e.S)), mv(__double2loint(e.S)));
    o.T = __hiloint2double(mv(__double2hiint(e.T)), mv(__double2loint(e.T)));
    o.v2 = __int_as_float(mv(__float_as_int(e.v2)));
    o.idx = mv(e.idx);
    o.xt = __int_as_float(mv(__float_as_int(e.xt)));
    return o;
}

// log2 of the group size P (1, 2, 4, 8 or 16) the lane-parallel merge would use for `rows` rows of `nsplit` slices,
// or -1 if it does not apply (then the staged, sequential merge is used).
__device__ inline int lane_merge_shift(int rows, int nsplit)
{
    if (nsplit > 16 || rows > 64) return -1;
    const int sh = nsplit <= 1 ? 0 : 32 - __clz(nsplit - 1);
    return (rows << sh) <= 512 ? sh : -1;
}

// Request this thread's partials: row `t >> sh` (first pass) and row `(t >> sh) + (256 >> sh)` (second pass),
// slice `t & (P - 1)`, of `rows` rows at `part` ([rows][nsplit]).  Threads without a partial get zeros.
// (256-thread workgroups.)
struct LaneRegs { StageRegs p[2]; };
__device__ inline LaneRegs lane_merge_issue(const Partial *part, int rows, int nsplit, int sh)
{
    // Every thread requests something (one without a partial re-reads partial 0; lane_piece ignores what it got): a
    // request under a condition is merged with the other branch's zeros, and the compiler waits for the data at the
    // merge, ahead of whatever the caller wanted to request next.
    LaneRegs r;
    const int sl = threadIdx.x & ((1 << sh) - 1);
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        // pass 2 only where one pass does not cover the rows (uniform); its registers are left unset otherwise and
        // nothing reads them (setting them would be the merge described above)
        if (q == 1 && (256 >> sh) >= rows) break;
        const int row = (threadIdx.x >> sh) + q * (256 >> sh);
        const bool mine = row < rows && sl < nsplit;
        const u32x4 *s = (const u32x4 *)(part + (mine ? (int64_t)row * nsplit + sl : 0));
        r.p[q].w0 = s[0]; r.p[q].w1 = s[1];
    }
    return r;
}

// Holds the requested partials' registers until here: placed after the caller's other requests, it keeps the compiler
// from handing a register of a still outstanding request to something else (it would have to wait for the request
// first); the wait for the data then happens here, behind all requests.
__device__ inline void lane_merge_pin(const LaneRegs &r, int rows, int sh)
{
    asm volatile("" :: "v"(r.p[0].w0), "v"(r.p[0].w1));
    if ((256 >> sh) < rows) asm volatile("" :: "v"(r.p[1].w0), "v"(r.p[1].w1));
}

// This thread's piece of pass q (an empty piece where the thread has none).
__device__ inline Piece lane_piece(const LaneRegs &w, int q, int rows, int nsplit, int sh)
{
    const int sl = threadIdx.x & ((1 << sh) - 1), row = (threadIdx.x >> sh) + q * (256 >> sh);
    if (q == 1 && (256 >> sh) >= rows) return empty_piece();       // uniform: no second pass was requested
    return (row < rows && sl < nsplit) ? piece_from_words(w.p[q].w0, w.p[q].w1) : empty_piece();
}

// The pieces of the 2^sh lanes of a group combined; every lane of the group returns the same bits.
template <bool EXCL>
__device__ inline Piece lane_group_merge(Piece e, int sh)
{
    // quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror, row_mirror: each pairs groups that already agree
    if (sh >= 1) e = merge_pair<EXCL>(e, piece_dpp<0xB1>(e));
    if (sh >= 2) e = merge_pair<EXCL>(e, piece_dpp<0x4E>(e));
    if (sh >= 3) e = merge_pair<EXCL>(e, piece_dpp<0x141>(e));
    if (sh >= 4) e = merge_pair<EXCL>(e, piece_dpp<0x140>(e));
    return e;
}

template <bool EXCL>
__device__ inline void lane_merge_pass(RowSlot *sh_rows, const Piece &e0, int row, int rows, int sh)
{
    const int sl = threadIdx.x & ((1 << sh) - 1);
    const Piece e = lane_group_merge<EXCL>(e0, sh);
    if (row < rows && sl == 0) {
        RowSlot o;
        o.r = row_total<EXCL>(e);
        o.xt = e.xt;
        sh_rows[row] = o;
    }
}

// Combine and publish: sh_rows[row] for row < rows; ends with a barrier.  e0, e1: this thread's pieces of the two passes.
template <bool EXCL>
__device__ inline void lane_merge_commit(RowSlot *sh_rows, const Piece &e0, const Piece &e1, int rows, int sh)
{
    lane_merge_pass<EXCL>(sh_rows, e0, threadIdx.x >> sh, rows, sh);
    if ((256 >> sh) < rows) lane_merge_pass<EXCL>(sh_rows, e1, (threadIdx.x >> sh) + (256 >> sh), rows, sh);   // uniform
    __syncthreads();
}

// First index j in [cand, cand + window) with x_j == M (the lowest argmax index of the row), in two steps so
// that a caller can put other work between the request and the use of the window.
struct ArgmaxProbe { u32x4 w; bool loaded; };
__device__ inline ArgmaxProbe argmax_issue(const void *row, int dtype, int32_t V, int32_t cand)
{
    ArgmaxProbe pr;
    pr.w = u32x4{0u, 0u, 0u, 0u};
    pr.loaded = false;
    if (cand < 0 || cand >= V) return pr;
    const int window = dtype == TAPOUT_F32 ? 4 : 8;
    const char *p = (const char *)row + (int64_t)cand * (dtype == TAPOUT_F32 ? 4 : 2);
    if ((((uintptr_t)p) & 15u) == 0 && cand + window <= V) {
        // the usual case: the window is one of the 16-byte vectors the streaming pass loaded; one load
        pr.w = *(const u32x4 *)p;
        pr.loaded = true;
    }
    return pr;
}
__device__ inline int32_t argmax_finish(const ArgmaxProbe &pr, const void *row, int dtype, int32_t V, int32_t cand, float M)
{
    if (cand < 0 || cand >= V) return 0;
    const int window = dtype == TAPOUT_F32 ? 4 : 8;
    float x[8];
    if (pr.loaded) {
        const u32x4 w = pr.w;
        const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (dtype == TAPOUT_F32) { x[i] = __uint_as_float(ww[i]); x[4 + i] = NAN; }
            else { x[2 * i] = __uint_as_float(ww[i] << 16); x[2 * i + 1] = __uint_as_float(ww[i] & 0xffff0000u); }
        }
    } else {
        // unaligned head / tail elements of a row
#pragma unroll
        for (int i = 0; i < 8; ++i)
            x[i] = (i < window && cand + i < V) ? load_elem_rt(row, dtype, cand + i) : NAN;
    }
    int32_t hit = cand;
#pragma unroll
    for (int i = 7; i >= 0; --i)
        if (x[i] == M) hit = cand + i;
    return hit;
}
__device__ inline int32_t resolve_argmax(const void *row, int dtype, int32_t V, int32_t cand, float M)
{
    return argmax_finish(argmax_issue(row, dtype, V, cand), row, dtype, V, cand, M);
}

#endif  // __HIPCC__

}  // namespace tapout
