// Verification of the drafted tokens and the final token (Algorithm 1, lines
// 10-11; "verify" = speculative sampling as in the works the paper cites).
//
// After the streaming pass over the target rows (row_reduce.hip) three small
// launches finish the job:
//
//   head    one workgroup per sequence merges the target partials, forms
//           log p(tok), takes the accept decisions u < p(tok)/q(tok), finds the
//           first rejection m, emits the accepted tokens and describes the draw
//           of the final token (row pair (m, m), or target row n alone)
//   slices  per 2048-element slice of the row pair, in double: A = sum a_j,
//           B = sum b_j (a = exp(t - ref_p), b = exp(d - ref_q)) and, with the
//           head's binary32-grade estimate L~ of L = S_p / S_q:
//           R~ = sum max(0, a_j - L~ b_j), D = sum of b_j over a_j > L~ b_j,
//           U = sum of b_j over the band |a_j - L~ b_j| <= eta L~ b_j; the
//           indices of the band elements (a handful: the band is 1e-5 wide) go
//           to a short per-sequence list
//   locate  one workgroup per sequence: exact L = sum A / sum B; the slice
//           weights of the residual max(0, a - L b) are R~ - (L - L~) D, which
//           is exact for every element whose sign of a - L b is the same at L~
//           and at L; an element can change sign only inside the band (given
//           |L - L~| <= eta L~, which is checked), where it is off by at most
//           |L - L~| b_j: in total at most |L - L~| * sum U.  If that bound is
//           below 2e-10 of the total weight (typically it is 1e-12) the sums
//           are used as they are.  If a heavy token sits in the band, the
//           listed elements are evaluated one by one with the exact L and
//           their slices corrected.  Then the slice holding u * Z is found
//           from the slice weights and the token by an exact scan inside it.
//           If the list overflowed (ratios tied inside the band, p == q), L~ is
//           off or Z vanishes, the slice weights are recomputed exactly first
//           (slow path).
//
// token = smallest j whose inclusive prefix sum exceeds u * Z.  Everything is
// double precision: with ~1e5 CDF cell edges in [0,1) a binary32 evaluation
// would move an edge across u for about one draw in a hundred; in double the
// chance is ~1e-10, so the token agrees with a sequential fp64 evaluation.
// Only one row pair per sequence is touched (2/(2K+1) of the round's logits),
// with two exponentials per element.  exp() is 2^(n/256) * (1 + r + r^2/2 +
// r^3/6), |r| <= ln2/512, with a 256-entry table in LDS: relative error
// < 2e-13, far inside what the 1e-9 decision margin needs, at a third of the
// instructions of a correctly rounded exp; row pairs of bfloat16 logits take
// exp(x) itself from a table of all bfloat16 values a softmax row can hold.
#include "common.h"
#include "bandit_device.h"
#include "finalize_device.h"

namespace tapout {

// Per-workgroup time stamps (a build with -DTAPOUT_WG_STAMPS only: `python -m paper_2511_02017_amd.build --stamps`
// makes libtapout_stamps.so beside the library proper, `python -m paper_2511_02017_amd.wg_stamps` runs it).  The first
// thread of a workgroup stores the 100 MHz wall clock at a few points of the final-token kernels; the table a stamp goes
// to and its slots are listed with the reader at the end of this file.  Stamps stretch what they measure (each is a scalar
// memory instruction the wavefront waits for: a few tenths of a microsecond); the library proper has none of this.
#ifdef TAPOUT_WG_STAMPS
constexpr int kStampWgs = 1 << 16;
__device__ unsigned long long g_stamps_slices[kStampWgs * 8];      // slice kernel, by linear workgroup index
__device__ unsigned long long g_stamps_head[kStampWgs * 4];        // accept decisions inside it, same index
__device__ unsigned long long g_stamps_locate[4096 * 8];           // locate kernel (and the draft epilogue's workgroups in its launch)
#define WG_LINEAR() ((int)(((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) & (kStampWgs - 1)))
#define WG_STAMP(table, per, wg, slot) do { if (threadIdx.x == 0) table[(wg) * (per) + (slot)] = wall_clock64(); } while (0)
#define WG_STAMP_LANE0(table, per, wg, slot) do { if ((threadIdx.x & (kWave - 1)) == 0) table[(wg) * (per) + (slot)] = wall_clock64(); } while (0)
#else
#define WG_LINEAR() 0
#define WG_STAMP(table, per, wg, slot) do {} while (0)
#define WG_STAMP_LANE0(table, per, wg, slot) do {} while (0)
#endif
#define HEAD_STAMP(slot) WG_STAMP(g_stamps_head, 4, WG_LINEAR(), slot)
#define LOCATE_STAMP(slot) WG_STAMP(g_stamps_locate, 8, (int)(blockIdx.x & 4095), slot)

namespace {

constexpr int kVBlock = 256;
static_assert(kVBlock == kBlock, "stage_partials strides by kBlock");
constexpr int kPer = 8;                       // elements per 16-byte (bf16) / 32-byte (f32) run



// ---- double-precision helpers ---------------------------------------------------
constexpr double kExpC = 369.3299304675746;            // 256 / ln 2
constexpr double kExpC1 = 0.0027076061740622863;       // ln2/256
constexpr double kExpC2 = kExpC1 * kExpC1 / 2.0;
constexpr double kExpC3 = kExpC1 * kExpC1 * kExpC1 / 6.0;
constexpr double kMagic = 6755399441055744.0;          // 1.5 * 2^52: adding it rounds to an integer held in the low mantissa bits

// exp(x - ref) for x <= ref + small.  neg_ref_c = -ref * 256/ln2; lo = ref - 700 as binary32: inputs
// below it (masked -inf logits, NaN) are treated as ref - 700, i.e. as weight 1e-304.
// c2 is kExpC2 and top is +inf: a caller with many exponentials in a row keeps them in vector registers (an
// instruction takes one scalar constant only, and the compiler would otherwise move c2 into a register before
// every use; with a top it cannot see through, the clamp stays a med3, which unlike fmaxf needs no quieting of
// its input first).
__device__ inline double exp_fast(float x, double neg_ref_c, float lo, const double *T, double c2 = kExpC2, float top = INFINITY)
{
    const double xd = (double)__builtin_amdgcn_fmed3f(x, lo, top);      // max(x, lo) for numbers, lo for NaN
    const double t = fma(xd, kExpC, neg_ref_c);          // (x - ref) * 256/ln2
    const double tm = t + kMagic;
    const int ni = __double2loint(tm);                   // round(t) in two's complement
    const double rs = t - (tm - kMagic);                 // remainder in units of ln2/256, |rs| <= 1/2
    const double q = rs * fma(rs, fma(rs, kExpC3, c2), kExpC1);
    const double tk = T[ni & 255];
    const double e = fma(tk, q, tk);                     // in [1, 2): scale by 2^(ni >> 8) through the exponent field
    int hi;                                              // high word + ((ni >> 8) << 20), as mask and one shift-add
    asm("v_lshl_add_u32 %0, %1, 12, %2" : "=v"(hi) : "v"(ni & (int)0xffffff00), "v"(__double2hiint(e)));
    return __hiloint2double(hi, __double2loint(e));
}

// exp(x) for a double argument (not NaN; clamped to [-700, 700]), same table and polynomial: relative error < 2e-13.
__device__ inline double exp_fast_d(double x, const double *T)
{
    const double t = fmin(fmax(x, -700.0), 700.0) * kExpC;
    const double tm = t + kMagic;
    const int ni = __double2loint(tm);
    const double rs = t - (tm - kMagic);
    const double q = rs * fma(rs, fma(rs, kExpC3, kExpC2), kExpC1);
    const double tk = T[ni & 255];
    return ldexp(fma(tk, q, tk), ni >> 8);
}

struct ExpRef {
    double neg_ref_c; float lo;
    __device__ inline void set(double ref) { neg_ref_c = -ref * kExpC; lo = (float)(ref - 700.0); }
};

// ---- wavefront reductions and scans of doubles with DPP (no LDS round trips) ---------------
// quad_perm [1,0,3,2] = 0xB1, quad_perm [2,3,0,1] = 0x4E, row_half_mirror = 0x141, row_mirror = 0x140,
// row_shr:n = 0x110 + n (lanes without a source inside their 16-lane row read 0).
template <int CTRL>
__device__ inline double dpp_d(double v)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}
__device__ inline double lane_d(double v, int lane)
{
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), lane), __builtin_amdgcn_readlane(__double2loint(v), lane));
}
// Sum over the 64 lanes, same value in every lane, fixed order.
__device__ inline double wave_sum_d(double v)
{
    v += dpp_d<0xB1>(v); v += dpp_d<0x4E>(v); v += dpp_d<0x141>(v); v += dpp_d<0x140>(v);
    return (lane_d(v, 0) + lane_d(v, 16)) + (lane_d(v, 32) + lane_d(v, 48));
}
// Inclusive prefix sum over the 64 lanes (lane order); *total = sum of all lanes.
__device__ inline double wave_incl_scan_d(double v, double *total)
{
    v += dpp_d<0x111>(v); v += dpp_d<0x112>(v); v += dpp_d<0x114>(v); v += dpp_d<0x118>(v);   // inside each 16-lane row
    const double t0 = lane_d(v, 15), t1 = lane_d(v, 31), t2 = lane_d(v, 47), t3 = lane_d(v, 63);
    const int rowid = (threadIdx.x & (kWave - 1)) >> 4;
    const double t01 = t0 + t1, t012 = t01 + t2;
    v += rowid == 0 ? 0.0 : (rowid == 1 ? t0 : (rowid == 2 ? t01 : t012));
    *total = t012 + t3;
    return v;
}

// ---- lse and token logit of the draft rows from the draft pass's partials ----------------
// For accept decisions that do not wait for the draft epilogue.  A draft partial's S leaves out the batch with the
// slice's first maximum; pad[1] holds that batch's own sum in the same reference, so S + pad[1] is the sum over the
// whole slice (binary32 precision).  Same lane layout as the lane-parallel merge: thread t takes the partial of
// (row t >> sh, slice t & (P - 1)) and of the row 256 >> sh further on; the P lanes of a row combine (max, sum) with
// DPP exchanges (commutative: all lanes of a group end with the same bits) and the first writes the row's entry.
struct DraftRowLse { double lse; float xt; };     // xt: the logit of the row's token (NaN: the token is out of range)

struct QPiece { float M; double S; float xt; };

template <int CTRL>
__device__ inline QPiece qpiece_dpp(const QPiece &e)
{
    auto mv = [](int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true); };
    QPiece o;
    o.M = __int_as_float(mv(__float_as_int(e.M)));
    o.S = __hiloint2double(mv(__double2hiint(e.S)), mv(__double2loint(e.S)));
    o.xt = __int_as_float(mv(__float_as_int(e.xt)));
    return o;
}
__device__ inline QPiece qpiece_merge(const QPiece &a, const QPiece &b)
{
    QPiece o;
    o.M = fmaxf(a.M, b.M);                                        // slice maxima are never NaN
    const float Rw = ref_of_max(o.M);
    const int da = (int)fminf(fmaxf(Rw - ref_of_max(a.M), -4000.0f), 4000.0f), db = (int)fminf(fmaxf(Rw - ref_of_max(b.M), -4000.0f), 4000.0f);
    o.S = ldexp(a.S, -da) + ldexp(b.S, -db);                      // an empty piece has S = 0 whatever its shift
    o.xt = (a.xt == a.xt) ? a.xt : b.xt;                          // at most one slice holds the token
    return o;
}
// In two steps, so that the caller can put these requests beside its own and wait for all of them once: the requests ...
struct DraftLseRegs { float pm[2], ps[2], px[2], ph[2]; };       // maximum, sum, token logit, left-out sum: the words wanted
__device__ inline int draft_lse_tid(int rows, int sh)
{
    // when they fit, on the upper two wavefronts: the lower two merge the target rows meanwhile
    return (rows << sh) <= 128 ? (int)threadIdx.x - 128 : (int)threadIdx.x;
}
__device__ inline DraftLseRegs draft_rows_lse_issue(const Partial *part, int rows, int nsplit, int sh)
{
    const int tid = draft_lse_tid(rows, sh), sl = tid & ((1 << sh) - 1);
    DraftLseRegs r;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        if (q == 1 && (256 >> sh) >= rows) break;                              // uniform; pass 2 stays unset and unread
        // unconditional requests (a thread without a partial re-reads partial 0 and ignores it): see lane_merge_issue
        const int row = tid < 0 ? rows : (tid >> sh) + q * (256 >> sh);        // rows: none
        const bool mine = row < rows && sl < nsplit;
        const Partial *s = part + (mine ? (int64_t)row * nsplit + sl : 0);
        r.pm[q] = s->v1; r.ps[q] = s->S; r.px[q] = __int_as_float(s->pad[0]); r.ph[q] = __int_as_float(s->pad[1]);
    }
    return r;
}
// ... and the merge, which writes out[row] for row < rows (published by the caller's next barrier).
__device__ inline void draft_rows_lse_finish(const DraftLseRegs &r, int rows, int nsplit, int sh, DraftRowLse *out)
{
    const int tid = draft_lse_tid(rows, sh), sl = tid & ((1 << sh) - 1);
    asm volatile("" :: "v"(r.pm[0]), "v"(r.ps[0]), "v"(r.px[0]), "v"(r.ph[0]));     // see lane_merge_pin
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        if (q == 1 && (256 >> sh) >= rows) break;                 // uniform
        const int row = tid < 0 ? rows : (tid >> sh) + q * (256 >> sh);
        QPiece e;
        e.M = -INFINITY; e.S = 0.0; e.xt = NAN;
        if (row < rows && sl < nsplit) {
            e.M = r.pm[q];
            e.S = (double)r.ps[q] + (double)r.ph[q];
            e.xt = r.px[q];
            if (e.M == -INFINITY && !(e.S != e.S)) e.S = 0.0;     // empty slice
        }
        if (sh >= 1) e = qpiece_merge(e, qpiece_dpp<0xB1>(e));
        if (sh >= 2) e = qpiece_merge(e, qpiece_dpp<0x4E>(e));
        if (sh >= 3) e = qpiece_merge(e, qpiece_dpp<0x141>(e));
        if (sh >= 4) e = qpiece_merge(e, qpiece_dpp<0x140>(e));
        if (row < rows && sl == 0) {
            const bool bad = !(e.S > 0.0) || !(e.S < INFINITY) || !(e.M > -INFINITY && e.M < INFINITY);
            DraftRowLse o;
            o.lse = bad ? (double)NAN : ((double)ref_of_max(e.M) + log2(e.S)) * kLn2;
            o.xt = e.xt;
            out[row] = o;
        }
    }
}

// Eight consecutive elements j .. j+7 of a row as they lie in memory (one 16-byte vector of bfloat16, two of binary32;
// -inf beyond V), so that a kernel can hold several requests in flight in few registers and widen them, exactly, when
// their turn comes.
template <int DT> struct Raw8 { u32x4 w[DT == TAPOUT_F32 ? 2 : 1]; };
template <int DT>
__device__ inline Raw8<DT> load_raw8(const char *rowp, bool aligned, int j, int V)
{
    Raw8<DT> r;
    if (aligned && j + kPer <= V) {
        if constexpr (DT == TAPOUT_BF16) {
            r.w[0] = *(const u32x4 *)(rowp + (int64_t)j * 2);
        } else {
            r.w[0] = *(const u32x4 *)(rowp + (int64_t)j * 4); r.w[1] = *(const u32x4 *)(rowp + (int64_t)j * 4 + 16);
        }
    } else if (j >= V) {
        // beyond the row: nothing to load (the usual case in a row's last slice)
        constexpr uint32_t ninf = DT == TAPOUT_BF16 ? 0xff80ff80u : 0xff800000u;
#pragma unroll
        for (int h = 0; h < (DT == TAPOUT_F32 ? 2 : 1); ++h) r.w[h] = u32x4{ninf, ninf, ninf, ninf};
    } else {
        uint32_t e[kPer];
#pragma unroll
        for (int i = 0; i < kPer; ++i) e[i] = __float_as_uint((j + i < V) ? load_elem<DT>(rowp, j + i) : -INFINITY);
        if constexpr (DT == TAPOUT_BF16) {
            r.w[0] = u32x4{(e[0] >> 16) | (e[1] & 0xffff0000u), (e[2] >> 16) | (e[3] & 0xffff0000u),
                           (e[4] >> 16) | (e[5] & 0xffff0000u), (e[6] >> 16) | (e[7] & 0xffff0000u)};
        } else {
            r.w[0] = u32x4{e[0], e[1], e[2], e[3]}; r.w[1] = u32x4{e[4], e[5], e[6], e[7]};
        }
    }
    return r;
}
template <int DT>
__device__ inline void widen8(const Raw8<DT> &r, float (&x)[kPer])
{
    if constexpr (DT == TAPOUT_BF16) {
        unpack<TAPOUT_BF16>(r.w[0], x);
    } else {
        float lo[4], hi[4];
        unpack<TAPOUT_F32>(r.w[0], lo); unpack<TAPOUT_F32>(r.w[1], hi);
#pragma unroll
        for (int i = 0; i < 4; ++i) { x[i] = lo[i]; x[4 + i] = hi[i]; }
    }
}

// ---- head: accept decisions of one sequence -----------------------------------------
// Called by all threads of a workgroup.  Returns the sequence's job (identical in every
// workgroup of the sequence); with `writer` also writes the sequence's outputs.
// Accept decisions exist for rows k < n <= K <= kScanCap, so the LDS byte buffer always holds them.
//
// kVerifyOwnQ (whole-round calls, lane-merge shapes only): log q(tok) and the draft rows' lse are not read from the draft
// epilogue's outputs, which then need not exist yet, but formed here from the draft pass's partials: the slice sums
// with their left-out batch's own sum added back (binary32 precision, which a ratio p/q compared with a uniform
// needs no more than) and the token's logit, which the draft pass left in the partial of the slice that holds it.
//
// shT: 256 doubles of LDS for the table of exp_fast, which this function fills (each thread requests its entry with the
// first requests and stores it ahead of the first barrier): the two exponentials on the critical path take 13
// instructions each instead of a call into the device library.  256-thread workgroups.
//
// more_requests(): called once, right after this function's own first requests are out: a caller with bulk loads of its
// own (the slice kernel's table) puts them there, behind the few words the decisions wait for (loads return in order).
struct NoRequests { __device__ void operator()() const {} };
template <bool SHARDED, class MoreRequests = NoRequests>
__device__ inline SampleJob verify_head(const VerifyArgs &a, int b, bool writer,
                                        Partial *sh_part, uint8_t *sh_dec, uint32_t *sh_flags, int32_t *sh_bcast, double *sh_lse,
                                        DraftRowLse *sh_qrows, double *shT, MoreRequests more_requests = MoreRequests())
{
    const int K = a.K;
    // few rows and slices: one partial per thread, merged across lanes (see lane_merge_commit); else staged in LDS
    const int msh = SHARDED ? -1 : lane_merge_shift(K + 1, a.nsplit);
    // The lane-parallel merge leaves the totals of all K + 1 <= 64 rows in LDS at once and row k with thread k: it is
    // one stage whatever the slice count.  The staged merge takes kStageCap partials at a time.
    const int rows_per_stage = msh >= 0 ? kWave : kStageCap / a.nsplit;
    // Everything whose address does not depend on n_draft is requested before n_draft is looked at, so that
    // the first memory round trip carries n_draft, the tokens, the uniforms and the partials together.
    // (Rows beyond n_draft hold stale partials and unused tokens: read, never used.)
    int32_t tok0 = -1;
    float u0 = 0.0f, lq0 = 0.0f, dl0 = 0.0f;
    // n_draft and greedy are requested here too, as vector loads (the index carries a zero the compiler cannot
    // see through): a scalar load would share its counter with the loads of kernel arguments, and the first wait
    // for one of those would wait for memory.  Their first use comes after the staging barrier.
    int zero;
    asm volatile("v_mov_b32 %0, 0" : "=v"(zero));
    int n = a.n_draft[b + zero];
    uint8_t greedy_raw = a.greedy ? a.greedy[b + zero] : (uint8_t)0;
    const double tv = a.exp_table[threadIdx.x];
    const bool own_q = !SHARDED && (a.vflags & kVerifyOwnQ) != 0 && msh >= 0 && lane_merge_shift(K, a.d_nsplit) >= 0;   // (the host offers own_q for lane-merge shapes only)
    if ((int)threadIdx.x < K) {
        const int64_t i = (int64_t)b * K + threadIdx.x;
        tok0 = a.draft_tok[i];
        u0 = a.u_accept[i];
        if (!own_q) {
            lq0 = a.logq_tok[i];
            if (a.draft_lse) dl0 = a.draft_lse[i];  // the final token's job wants it for row m: no dependent load later
        }
    }
    if (threadIdx.x == 0) { *sh_flags = 0; sh_bcast[4] = 0; }     // ahead of the staging barrier: rows of other wavefronts OR into the flags
    RowSlot *sh_rows = (RowSlot *)sh_part;
    static_assert(sizeof(RowSlot) * 64 <= sizeof(Partial) * kStageCap, "the row totals reuse the staging buffer");
    if constexpr (SHARDED) {
        const int c0 = min(K + 1, rows_per_stage) * a.nsplit;
        const StageRegs st = stage_issue_shards(a.part, (int64_t)a.B * (K + 1), (int64_t)b * (K + 1), a.nsplit, c0);
        more_requests();
        shT[threadIdx.x] = tv;
        stage_commit(sh_part, st, c0);
    } else if (__builtin_expect(msh >= 0, 1)) {
        // target partials run over every element of their slice: plain pieces, nothing left out
        // all requests first, then one wait for the lot (see lane_merge_pin)
        const LaneRegs ln = lane_merge_issue(a.part + (int64_t)b * (K + 1) * a.nsplit, K + 1, a.nsplit, msh);
        const int qsh = own_q ? lane_merge_shift(K, a.d_nsplit) : -1;            // >= 0: the host offers own_q for such shapes only
        DraftLseRegs lq;
        if (qsh >= 0) lq = draft_rows_lse_issue(a.dpart + (int64_t)b * K * a.d_nsplit, K, a.d_nsplit, qsh);
        more_requests();
        lane_merge_pin(ln, K + 1, msh);
        HEAD_STAMP(0);                                           // first requests answered
        shT[threadIdx.x] = tv;
        if (qsh >= 0) draft_rows_lse_finish(lq, K, a.d_nsplit, qsh, sh_qrows);     // published by the barrier below
        lane_merge_commit<false>(sh_rows, lane_piece(ln, 0, K + 1, a.nsplit, msh), lane_piece(ln, 1, K + 1, a.nsplit, msh), K + 1, msh);
        HEAD_STAMP(1);                                           // rows merged, barrier passed
    } else {
        const int c0 = min(K + 1, rows_per_stage) * a.nsplit;
        const StageRegs st = stage_issue(a.part + (int64_t)b * (K + 1) * a.nsplit, c0);
        more_requests();
        shT[threadIdx.x] = tv;
        stage_commit(sh_part, st, c0);
    }
    uint32_t f0 = 0;
    n = __builtin_amdgcn_readfirstlane(n);
    if (__builtin_expect(n < 1 || n > K, 0)) { f0 |= TAPOUT_FLAG_BAD_NDRAFT; n = n < 1 ? 1 : K; }
    const bool greedy = __builtin_amdgcn_readfirstlane((int)greedy_raw) != 0;
    SampleJob job;
    job.kind = 0; job.row = 0; job.ref_p = 0.0f; job.ref_q = 0.0f; job.lam = 0.0;
    if (threadIdx.x == 0 && f0) atomicOr(sh_flags, f0);
    const bool need_top1 = writer || greedy;
    int last_k = -1; float last_M = 0.0f, last_dl = 0.0f; int32_t last_top1 = 0; double last_lse = 0.0;   // the last row this thread merged
    bool acc_mine = false; uint32_t f_mine = 0;      // its accept decision and flags (used on the lane-merge path)
    for (int k0 = 0; k0 <= n; k0 += rows_per_stage) {
        const int k1 = min(n + 1, k0 + rows_per_stage);
        const int kmine = k0 + threadIdx.x;
        if (__builtin_expect(k0 > 0, 0)) {                               // further stages (K + 1 > rows_per_stage): load late
            tok0 = -1;
            if (kmine < k1 && kmine < n) {
                const int64_t i = (int64_t)b * K + kmine;
                tok0 = a.draft_tok[i]; u0 = a.u_accept[i]; lq0 = a.logq_tok[i];
                if (a.draft_lse) dl0 = a.draft_lse[i];
            }
            __syncthreads();
            if constexpr (SHARDED) {
                const int c1 = (k1 - k0) * a.nsplit;
                stage_commit(sh_part, stage_issue_shards(a.part, (int64_t)a.B * (K + 1), (int64_t)b * (K + 1) + k0, a.nsplit, c1), c1);
            } else {
                stage_partials(sh_part, a.part + ((int64_t)b * (K + 1) + k0) * a.nsplit, (k1 - k0) * a.nsplit);
            }
        }
        for (int k = kmine; k < k1; k += kVBlock) {
            const int64_t it = (int64_t)b * (K + 1) + k;
            const void *row = SHARDED ? nullptr : row_address(a.tbase, a.t_dtype, a.t_stride_b, a.t_stride_k, b, k);
            // shard records leave their first maximum out of the sums (and carry its exact index), slice partials of
            // target rows do not
            const RowTotal r = msh >= 0 ? sh_rows[k].r : merge_partials<SHARDED>(sh_part + (k - k0) * a.nsplit, a.nsplit);
            // the argmax window is requested here and looked at after the logarithm (greedy sequences need the
            // argmax for their decisions, the others only for the outputs)
            int32_t top1 = 0;
            ArgmaxProbe probe;
            if constexpr (SHARDED) top1 = (r.cand >= 0 && r.cand < a.V) ? r.cand : 0;                // a shard's argmax is exact and global
            else if (need_top1) probe = argmax_issue(row, a.t_dtype, a.V, r.cand);
            uint32_t f = 0;
            double lse_d = NAN;
            if (__builtin_expect(r.bad, 0)) f |= TAPOUT_FLAG_BAD_ROW;
            else lse_d = (r.R + log2(r.S)) * kLn2;
            // greedy sequences decide on the argmax; the others only report it: they look at the window last
            if constexpr (!SHARDED)
                if (greedy) top1 = argmax_finish(probe, row, a.t_dtype, a.V, r.cand, r.M);
            if (k < n) {
                const int64_t i = (int64_t)b * K + k;
                int32_t t = tok0;
                float u = u0, lq = lq0;
                last_dl = dl0;
                if (own_q) {                                   // one row per thread on this path: k == kmine
                    const double lse_q = sh_qrows[k].lse;
                    lq = (float)((double)sh_qrows[k].xt - lse_q);
                    last_dl = (float)lse_q;
                } else if (__builtin_expect(k != kmine, 0)) {                       // more rows than threads: load late
                    t = a.draft_tok[i]; u = a.u_accept[i]; lq = a.logq_tok[i];
                    if (a.draft_lse) last_dl = a.draft_lse[i];
                }
                // the slice (or vocabulary shard) that holds the token put its logit into its partial, the others NaN
                float xt = NAN;
                if (msh >= 0) xt = sh_rows[k].xt;
                else
                    for (int g = 0; g < a.nsplit; ++g) {
                        const float v = __int_as_float(sh_part[(k - k0) * a.nsplit + g].pad[0]);
                        if (v == v) xt = v;
                    }
                bool acc = false;
                float lp = NAN;
                if (__builtin_expect(t < 0 || t >= a.V, 0)) f |= TAPOUT_FLAG_BAD_TOKEN;
                else if (!r.bad) {
                    lp = (float)((double)xt - lse_d);
                    if (greedy) acc = (t == top1);
                    else {
                        const double arg = (double)lp - (double)lq;
                        acc = arg == arg && (double)u < exp_fast_d(arg, shT);
                    }
                }
                if (writer && a.logp_tok) a.logp_tok[i] = lp;
                acc_mine = acc;
                if (msh < 0) sh_dec[k] = acc ? 1 : 0;
            }
            if constexpr (!SHARDED)
                if (need_top1 && !greedy) top1 = argmax_finish(probe, row, a.t_dtype, a.V, r.cand, r.M);
            if (writer) {
                if (a.target_lse) a.target_lse[it] = (float)lse_d;
                if (a.target_top1) a.target_top1[it] = top1;
            }
            last_k = k; last_M = r.M; last_top1 = top1; last_lse = lse_d;
            f_mine = f;
            if (msh < 0 && f) atomicOr(sh_flags, f);
        }
    }
    constexpr uint32_t kFatal = TAPOUT_FLAG_BAD_NDRAFT | TAPOUT_FLAG_BAD_TOKEN | TAPOUT_FLAG_BAD_ROW;
    HEAD_STAMP(2);                                               // every row's lse, log p(tok), accept decision
    if (__builtin_expect(msh >= 0, 1)) {
        // Lane-merge path: row k was thread k's, so the rows are lanes of the first wavefront.  Ballots give the
        // first rejection and the flags, lane m hands over what the job needs of row m, one barrier publishes it.
        if (threadIdx.x < kWave) {
            const uint64_t acc_mask = __builtin_amdgcn_ballot_w64((int)threadIdx.x < n && acc_mine);
            uint32_t fa = f0;
            if (__builtin_amdgcn_ballot_w64((f_mine & TAPOUT_FLAG_BAD_TOKEN) != 0)) fa |= TAPOUT_FLAG_BAD_TOKEN;
            if (__builtin_amdgcn_ballot_w64((f_mine & TAPOUT_FLAG_BAD_ROW) != 0)) fa |= TAPOUT_FLAG_BAD_ROW;
            // first draft position that was not accepted, n if there is none (n <= 63 here)
            const int mm = (fa & kFatal) ? 0 : __builtin_ctzll(~acc_mask | (1ull << n));
            const int Mb = __builtin_amdgcn_readlane(__float_as_int(last_M), mm);
            const int tb = __builtin_amdgcn_readlane(last_top1, mm);
            const int db = __builtin_amdgcn_readlane(__float_as_int(last_dl), mm);
            const int lh = __builtin_amdgcn_readlane(__double2hiint(last_lse), mm);
            const int ll = __builtin_amdgcn_readlane(__double2loint(last_lse), mm);
            if (threadIdx.x == 0) {
                sh_bcast[0] = mm; sh_bcast[1] = (fa & kFatal) ? 1 : 0; sh_bcast[2] = (int32_t)fa;
                sh_bcast[4] = 1; sh_bcast[5] = Mb; sh_bcast[6] = tb; sh_bcast[7] = db;
                *sh_lse = __hiloint2double(lh, ll);
            }
        }
        __syncthreads();
    } else {
        __syncthreads();
        if (threadIdx.x == 0) {
            const uint32_t f = *sh_flags;
            int m = 0;
            if (!(f & kFatal))
                while (m < n && sh_dec[m] != 0) ++m;
            sh_bcast[0] = m;
            sh_bcast[1] = (f & kFatal) ? 1 : 0;
            sh_bcast[2] = (int32_t)f;
        }
        __syncthreads();
        // maximum and argmax of row m: from the thread that merged it, if it still holds them
        if (last_k == sh_bcast[0]) { sh_bcast[4] = 1; sh_bcast[5] = __float_as_int(last_M); sh_bcast[6] = last_top1; sh_bcast[7] = __float_as_int(last_dl); *sh_lse = last_lse; }
        __syncthreads();
    }
    HEAD_STAMP(3);                                               // first rejection published
    const int m = sh_bcast[0];                   // a flagged sequence has m = 0 and emits the argmax of row 0
    const bool flagged = sh_bcast[1] != 0;
    const uint32_t f = (uint32_t)sh_bcast[2];
    float Mm, dl_m = 0.0f; int32_t top1m; double lse_m;
    if (__builtin_expect(sh_bcast[4] != 0, 1)) {
        Mm = __int_as_float(sh_bcast[5]); top1m = sh_bcast[6]; dl_m = __int_as_float(sh_bcast[7]); lse_m = *sh_lse;
    } else {                                     // more rows than threads: merge row m once more
        __syncthreads();
        if constexpr (SHARDED) stage_commit(sh_part, stage_issue_shards(a.part, (int64_t)a.B * (K + 1), (int64_t)b * (K + 1) + m, a.nsplit, a.nsplit), a.nsplit);
        else stage_partials(sh_part, a.part + ((int64_t)b * (K + 1) + m) * a.nsplit, a.nsplit);
        RowTotal r = merge_partials<SHARDED>(sh_part, a.nsplit);
        Mm = r.M;
        lse_m = (r.R + log2(r.S)) * kLn2;
        if constexpr (SHARDED) top1m = (r.cand >= 0 && r.cand < a.V) ? r.cand : 0;
        else top1m = need_top1 ? resolve_argmax(row_address(a.tbase, a.t_dtype, a.t_stride_b, a.t_stride_k, b, m), a.t_dtype, a.V, r.cand, r.M) : 0;
        if (m < n && a.draft_lse) dl_m = a.draft_lse[(int64_t)b * K + m];
    }
    if (!flagged && !greedy) {
        job.kind = m < n ? 1 : 2;
        job.row = m;
        job.ref_p = Mm;                          // exponent references: the target row's maximum, the draft row's lse
        job.ref_q = (m < n && (a.draft_lse || own_q)) ? dl_m : 0.0f;
        // binary32-grade estimate of S_p / S_q in these references (S_q = sum exp(d - lse_q) = 1): lets the
        // slice pass form the residual before the exact normalisers exist
        job.lam = exp_fast_d(lse_m - (double)Mm, shT);
    }
    if (writer) {
        const int32_t final_tok = (flagged || greedy) ? top1m : -1;   // sampled sequences: written by pass 3
        if (threadIdx.x == 0) {
            a.accept_len[b] = m;
            a.n_out[b] = m + 1;
            if constexpr (!SHARDED) {
                a.jobs[b].job = job;
                // the slice kernel appends to the sequence's band list; fused into that kernel, this workgroup
                // cannot empty the list under the others' appends: the target pass has done it
                if (!a.fused_head) a.jobs[b].band_cnt = 0;
                a.flags_ws[b] = f;
            } else if (a.final_jobs) {
                a.final_jobs[b] = job;
            }
            if (a.flags) a.flags[b] = f;
        }
        int32_t *o = a.out_tok + (int64_t)b * (K + 1);
        for (int k = threadIdx.x; k <= K; k += kVBlock) {
            // (lane-merge path: thread k still holds row k's token from the first round trip)
            o[k] = k < m ? ((msh >= 0 && k == (int)threadIdx.x) ? tok0 : a.draft_tok[(int64_t)b * K + k]) : (k == m ? final_tok : -1);
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

// ---- head kernel: one workgroup per sequence ------------------------------------------
template <bool SHARDED>
__global__ __launch_bounds__(kVBlock) void verify_head_kernel(VerifyArgs a)
{
    warm_args(a);
    __shared__ Partial sh_part[kStageCap];
    __shared__ uint8_t sh_dec[kScanCap];
    __shared__ uint32_t sh_flags;
    __shared__ int32_t sh_bcast[8];
    __shared__ double sh_lse;
    __shared__ DraftRowLse sh_qrows[SHARDED ? 1 : kWave];
    __shared__ double shT[256];
    static_assert(kVBlock == 256, "one table entry per thread");
    verify_head<SHARDED>(a, blockIdx.x, true, sh_part, sh_dec, &sh_flags, sh_bcast, &sh_lse, sh_qrows, shT);
}

// ---- slice kernel -----------------------------------------------------------------------
// A slice is kSampleSlice = 2048 elements.
constexpr double kEta = 1.0e-5;        // half-width (relative) of the band around L~ in which a sign may be wrong
constexpr int kSliceVals = 5;          // A, B, R~, D, U

constexpr int kWavesPerWG = kVBlock / kWave;                    // 4 slices per workgroup, one per wavefront
constexpr int kChunks = kSampleSlice / (kWave * kPer);          // a wavefront takes its slice in 4 chunks of 512 elements

// ---- exponentials of bfloat16 logits from a table -----------------------------------------
// A bfloat16 logit has 2^16 possible values, and those between 2^-12 and 2^6 in magnitude (all a softmax row holds
// besides masked entries and the odd tiny one) are 2 * 2302 of them: exp(x) itself, correctly rounded on the host,
// comes from a table of 36 KB in LDS with four integer instructions and one LDS read instead of the thirteen
// instructions of exp_fast.  The row's exponent reference is applied once per slice, to the sums:
//   a_j = exp(t_j - ref_p) = E[t_j] c_t,  b_j = exp(d_j - ref_q) = E[d_j] c_d,   c_t = exp(-ref_p), c_d = exp(-ref_q)
//   a_j - L~ b_j = c_t (E[t_j] - L' E[d_j]),  L' = L~ c_d / c_t
// so the slice kernel sums E[t], E[d], max(0, E[t] - L' E[d]), ... and scales A, R~ by c_t and B, D, U by c_d at the
// end.  A row of another element type keeps exp_fast and c = 1.
// Layout: T[idx] for positive values, T[kTabTop + 1 + idx] for negative ones (kept apart: with the two signs of a
// magnitude side by side a wavefront's 64 reads fall on half as many LDS banks).  Entry idx = 1 .. kTabTop - 1 is
// the magnitude with bfloat16 bits kTabLo15 + idx - 1.
// Entry kTabTop stands for every magnitude from 63.5 up (and NaN): 0 for either sign.  That is exact for -inf (a
// masked entry) and an error below e^-49 of the row's largest term for any other logit <= -63.5 given the condition
// on the references that tab_job_ok checks (row maxima in [-14, 63)); a job outside it takes the computed
// exponentials.  Entry 0 stands for the magnitudes below 2^-12 (and zeros), which are not in the table, and holds
// NaN: a chunk's sums show that it met one, and the slice kernel forms that chunk again with tab_exp_any, which
// evaluates 1 + x + x^2/2 + x^3/6 for them (error < 2e-16).
constexpr int kTabTop = 18 * 128 - 1;
constexpr uint32_t kTabLo15 = (uint32_t)(127 - 12) << 7;            // bfloat16 magnitude bits of 2^-12
constexpr int kTabDoubles = 2 * (kTabTop + 1);                       // 4608 doubles = 36,864 bytes
constexpr int kTabVecs = kTabDoubles / 2;                            // 16-byte vectors
static_assert(kTabVecs % kVBlock == 0, "the table is copied to LDS in whole rounds of the workgroup");
static_assert(kTabDoubles == kExpBf16Doubles, "the host builds the table");
static_assert(8 * (2 * kTabTop + 1) < 65536, "an entry's byte offset fits sixteen bits");

// Two bfloat16 values as they lie in one word -> the byte offsets of their entries, again as two halves of a word.
// Both halves are worked on at once with the packed 16-bit integer instructions: eight instructions for two
// look-ups, the two that take the word apart included (one value at a time it was nine each).
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
__device__ inline uint32_t tab_offsets2(uint32_t w)
{
    const uint32_t mag = w & 0x7fff7fffu;
    u16x2 d = __builtin_elementwise_sub_sat(__builtin_bit_cast(u16x2, mag), (u16x2)(unsigned short)(kTabLo15 - 1));   // 0: below the table
    d = __builtin_elementwise_min(d, (u16x2)(unsigned short)kTabTop);
    d = d << (u16x2)(unsigned short)3;
    typedef short i16x2 __attribute__((ext_vector_type(2)));
    const i16x2 neg = __builtin_bit_cast(i16x2, w) >> (i16x2)(short)15;           // all ones in the half of a negative value
    d += __builtin_bit_cast(u16x2, neg) & (u16x2)(unsigned short)(8 * (kTabTop + 1));
    return __builtin_bit_cast(uint32_t, d);
}
// x: a bfloat16 value widened to binary32 (low 16 bits zero); same entry as tab_offsets2 finds.
__device__ inline double tab_lookup(float x, const double *T)
{
    const uint32_t u = __float_as_uint(x);
    const uint32_t m = (u >> 16) & 0x7fffu;
    const uint32_t d = min(max(m, kTabLo15 - 1) - (kTabLo15 - 1), (uint32_t)kTabTop);
    return T[d + (u >> 31) * (uint32_t)(kTabTop + 1)];
}
// Any binary32-widened bfloat16 value, with the same bits as the table wherever it applies.
__device__ inline double tab_exp_any(float x, const double *T)
{
    const uint32_t u = __float_as_uint(x);
    if (((u >> 16) & 0x7fffu) < kTabLo15) {
        const double t = (double)x;
        return fma(t, fma(t, fma(t, 1.0 / 6.0, 0.5), 1.0), 1.0);
    }
    return tab_lookup(x, T);
}
__device__ inline bool tab_job_ok(const SampleJob &job)
{
    // ref_p: the target row's maximum; ref_q: the draft row's lse, at most ln V above its maximum
    return job.ref_p >= -14.0f && job.ref_p < 63.0f && (job.kind != 1 || (job.ref_q >= 0.0f && job.ref_q < 63.0f));
}
// Scales of a job's two rows (see above); identical code, hence identical bits, in the slice and the locate kernel.
struct TabScale { double ct, cd, Lp; };
__device__ inline TabScale tab_scale(const SampleJob &job, bool tab_t, bool tab_d, const double *shT)
{
    TabScale o;
    const double st = tab_t ? -(double)job.ref_p : 0.0, sd = tab_d ? -(double)job.ref_q : 0.0;
    o.ct = tab_t ? exp_fast_d(st, shT) : 1.0;
    o.cd = tab_d ? exp_fast_d(sd, shT) : 1.0;
    o.Lp = (tab_t || tab_d) ? job.lam * exp_fast_d(sd - st, shT) : job.lam;
    return o;
}

// Adds the sums of one chunk (8 elements per lane) of a row pair to cA .. cDs.  TABT / TABD: that row's exponentials come from the
// table, through tab_exp_any (the chunks that chunk_pair_tab cannot take: tiny magnitudes; band elements).
template <bool TABT, bool TABD>
__device__ inline void chunk_pair(const float (&ct)[kPer], const float (&cd)[kPer], const ExpRef &rp, const ExpRef &rq,
                                  const double *shT, const double *shE, double c2, float top, double Lp, double band,
                                  double &cA, double &cB, double &cR, double &cDs, uint64_t &any_band)
{
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        double av, bv;
        if constexpr (!TABT) av = exp_fast(ct[i], rp.neg_ref_c, rp.lo, shT, c2, top);
        else av = tab_exp_any(ct[i], shE);
        if constexpr (!TABD) bv = exp_fast(cd[i], rq.neg_ref_c, rq.lo, shT, c2, top);
        else bv = tab_exp_any(cd[i], shE);
        const double diff = fma(-Lp, bv, av);
        cA += av;
        cB += bv;
        cR += fmax(diff, 0.0);
        cDs += copysign(bv, diff);
        // band test: the comparison's lane mask is ORed up over the chunk in scalar registers; one branch
        // per chunk instead of one per element (a branch on a fresh vector comparison stalls the wavefront)
        any_band |= __builtin_amdgcn_ballot_w64(fabs(diff) < band * bv);      // strict: an entry with b = 0 (masked, beyond V) is no band element
    }
}
// The same sums for a chunk of two bfloat16 rows as it lies in memory (four words of two values each), every
// exponential straight from the table in LDS; same order of additions.  A value below the table's range makes
// the sums NaN (entry 0).
__device__ inline void chunk_pair_tab(const u32x4 &wt, const u32x4 &wd, const double *shE, double Lp, double band,
                                      double &cA, double &cB, double &cR, double &cDs, uint64_t &any_band)
{
    const char *E = (const char *)shE;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t ot = tab_offsets2(wt[k]), od = tab_offsets2(wd[k]);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const double av = *(const double *)(E + (h ? ot >> 16 : ot & 0xffffu));
            const double bv = *(const double *)(E + (h ? od >> 16 : od & 0xffffu));
            const double diff = fma(-Lp, bv, av);
            cA += av;
            cB += bv;
            cR += fmax(diff, 0.0);
            cDs += copysign(bv, diff);
            any_band |= __builtin_amdgcn_ballot_w64(fabs(diff) < band * bv);
        }
    }
}
// One row alone: the sum of its exponentials over a chunk.
__device__ inline double chunk_one_tab(const u32x4 &wt, const double *shE)
{
    const char *E = (const char *)shE;
    double cA = 0.0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t ot = tab_offsets2(wt[k]);
        cA += *(const double *)(E + (ot & 0xffffu));
        cA += *(const double *)(E + (ot >> 16));
    }
    return cA;
}

// One wavefront per slice, four slices per workgroup.  A wavefront takes its slice in chunks of one 8-element run per
// lane; its five sums need no LDS and no barrier.  The requests run ahead of the arithmetic (see kAhead): with one
// chunk ahead the launch was bound by memory latency.  Four wavefronts per SIMD: the bfloat16 table limits a CU to
// four workgroups anyway, and under a tighter register limit the loop spills.
template <int TD, int DD, bool FUSED>
__global__ __launch_bounds__(kVBlock) __attribute__((amdgpu_waves_per_eu(4))) void verify_slices(VerifyArgs a)
{
    // The table serves row pairs of bfloat16 only: with one row computed and one looked up the compiler's schedule
    // of the mixed loop wants 160-170 registers (two wavefronts per SIMD), and held to four wavefronts it spills
    // inside the loop (V = 256000, 512 sequences, binary32 target rows: 210 us against 139 us all computed; at three
    // wavefronts per SIMD, 154 registers and no spills, 147 us).
    constexpr bool kTabT = TD == TAPOUT_BF16 && DD == TAPOUT_BF16, kTabD = kTabT;
    // LDS: the accept decisions' buffers (FUSED) are dead once the job is known; the table takes their place
    constexpr size_t kHeadBytes = sizeof(Partial) * kStageCap + sizeof(DraftRowLse) * kWave + 8 + 32 + 8 + kScanCap;
    constexpr size_t kTabBytes = (kTabT || kTabD) ? sizeof(double) * kTabDoubles : 0;
    constexpr size_t kRaw = (FUSED && kHeadBytes > kTabBytes) ? kHeadBytes : (kTabBytes > 0 ? kTabBytes : 16);
    __shared__ double shT[256];
    __shared__ __align__(16) unsigned char sh_raw[kRaw];
    warm_args(a);
    // (the grid's shape from the arguments, not from the hidden ones: see warm_args)
    const int j = blockIdx.z * min(a.n_jobs, 65535) + blockIdx.y;
    [[maybe_unused]] const int wg = WG_LINEAR();
    WG_STAMP(g_stamps_slices, 8, wg, 0);                         // entry
    if (j >= a.n_jobs) return;
    const int b = j / a.jps;
    const int wave = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
    // FUSED: the sequence's last workgroup writes the sequence's outputs, from its first wavefront, which therefore
    // takes the group's last slice: most often none at all, or the row's short last one
    const bool writer = FUSED && (int)blockIdx.x == (a.nsl + kWavesPerWG - 1) / kWavesPerWG - 1;
    const int s = blockIdx.x * kWavesPerWG + (writer ? kWavesPerWG - 1 - wave : wave);
    // The tables are requested early: nothing of them depends on the job, and a wavefront's loads return in order, so
    // requested after the rows they would hold the barrier below until the whole slice has arrived.  When the accept
    // decisions run in this kernel they fill the small table themselves and the large one is requested right behind
    // their own first requests; else both are requested here.
    static_assert(kVBlock == 256, "one entry of the small table per thread");
    constexpr int kRounds = (kTabT || kTabD) ? kTabVecs / kVBlock : 1;
    u32x4 tw[kRounds];
    double tv = 0.0;
    if constexpr (!FUSED) tv = a.exp_table[threadIdx.x];
    auto request_table = [&]() {
        if constexpr (kTabT || kTabD) {
            const u32x4 *src = (const u32x4 *)(a.exp_table + 256);
#pragma unroll
            for (int q = 0; q < kRounds; ++q) tw[q] = src[q * kVBlock + threadIdx.x];
        }
    };
    if constexpr (!FUSED) request_table();
    SampleJob job;
    if constexpr (FUSED) {
        // Small batches: a head launch of its own costs more (launch, hand-over of the job record through
        // memory) than taking the accept decisions again in each of the sequence's workgroups.  All of them run
        // the same code on the same inputs and reach the same job; one of them writes the sequence's outputs.
        unsigned char *q = sh_raw;
        Partial *sh_part = (Partial *)q;            q += sizeof(Partial) * kStageCap;
        DraftRowLse *sh_qrows = (DraftRowLse *)q;   q += sizeof(DraftRowLse) * kWave;
        double *sh_lse = (double *)q;               q += 8;
        int32_t *sh_bcast = (int32_t *)q;           q += 32;
        uint32_t *sh_flags = (uint32_t *)q;         q += 8;
        uint8_t *sh_dec = q;
        job = verify_head<false>(a, b, writer, sh_part, sh_dec, sh_flags, sh_bcast, sh_lse, sh_qrows, shT, request_table);
    } else {
        job = a.jobs[j].job;
    }
    WG_STAMP(g_stamps_slices, 8, wg, 1);                         // job known
    if (job.kind == 0) return;
    const Rows r = job_rows<TD, DD>(a, b, job);
    const bool live = s < a.nsl;
    const bool resid = job.kind == 1;
    const int base = s * kSampleSlice + lane * kPer;
    // The wavefront's requests run kAhead chunks ahead of its arithmetic.  With one chunk ahead the kernel was bound by
    // memory latency, not by arithmetic: 2 KB in flight per wavefront, 8 MB over the chip, is 2.5 TB/s at 3 us.
    // bfloat16 pairs request the whole slice at once (32 registers), others two chunks ahead.
    constexpr int kAhead = (TD == TAPOUT_BF16 && DD == TAPOUT_BF16) ? kChunks : 2;
    // whole workgroup, uniform: which rows take their exponentials from the table
    const bool tab_ok = (kTabT || kTabD) && !(a.vflags & kVerifyNoExpTable) && tab_job_ok(job);
    const bool tab_t = kTabT && tab_ok, tab_d = kTabD && tab_ok && resid;
    const double *shE = (const double *)sh_raw;
    // the tables into LDS before the rows are requested: the wait for them then has nothing younger behind it
    if constexpr (!FUSED) shT[threadIdx.x] = tv;
    if constexpr (kTabT || kTabD) {
        if constexpr (FUSED) __syncthreads();                    // every thread is done with the accept decisions' LDS
        if (tab_t || tab_d) {
#pragma unroll
            for (int q = 0; q < kRounds; ++q) ((u32x4 *)sh_raw)[q * kVBlock + threadIdx.x] = tw[q];
        }
    }
    Raw8<TD> qt[kChunks];
    Raw8<DD> qd[kChunks];
    // A slice that lies wholly inside aligned rows (all but a row's last one) is requested in straight-line code:
    // the per-request checks of the general path are branches, and across branches the compiler waits for every
    // outstanding request where the first chunk's would do.
    const bool whole = live && r.t_al && (r.d_al || !resid) && (s + 1) * kSampleSlice <= a.V;       // wavefront-uniform
    if (__builtin_expect(whole, 1)) {
        const char *tp = r.trow + (int64_t)base * Elem<TD>::size;
        const char *dp = r.drow + (int64_t)base * Elem<DD>::size;
#pragma unroll
        for (int c = 0; c < kChunks; ++c) {
            qt[c] = Raw8<TD>{}; qd[c] = Raw8<DD>{};
            if (c < kAhead) {
#pragma unroll
                for (int h = 0; h < (TD == TAPOUT_F32 ? 2 : 1); ++h)
                    qt[c].w[h] = *(const u32x4 *)(tp + (int64_t)c * kWave * kPer * Elem<TD>::size + 16 * h);
            }
        }
        if (resid) {
#pragma unroll
            for (int c = 0; c < kAhead; ++c)
#pragma unroll
                for (int h = 0; h < (DD == TAPOUT_F32 ? 2 : 1); ++h)
                    qd[c].w[h] = *(const u32x4 *)(dp + (int64_t)c * kWave * kPer * Elem<DD>::size + 16 * h);
        }
    } else {
#pragma unroll
        for (int c = 0; c < kChunks; ++c) {
            qt[c] = Raw8<TD>{}; qd[c] = Raw8<DD>{};
            if (c < kAhead && live) {
                qt[c] = load_raw8<TD>(r.trow, r.t_al, base + c * kWave * kPer, a.V);
                if (resid) qd[c] = load_raw8<DD>(r.drow, r.d_al, base + c * kWave * kPer, a.V);
            }
        }
    }
    __syncthreads();
    WG_STAMP(g_stamps_slices, 8, wg, 2);                         // tables in LDS, rows requested
    if (!live) return;
    ExpRef rp, rq;
    rp.set((double)job.ref_p); rq.set((double)job.ref_q);
    const TabScale sc = tab_scale(job, tab_t, tab_d, shT);
    const double lam = sc.Lp, band = kEta * sc.Lp;
    double c2 = kExpC2;
    float top = INFINITY;
    asm volatile("" : "+v"(c2), "+v"(top));               // stay in vector registers through the loop
    // Ds = sum of b carrying the sign of a - L~ b, so that D = (B + Ds) / 2 without a select per element (an
    // element with a == L~ b lands in D; it is in the band, so U covers it).  Elements inside the band are a
    // handful per row at most: their sum and their list are kept under a branch a wavefront almost never enters.
    double A = 0.0, Bs = 0.0, R = 0.0, Ds = 0.0, U = 0.0;
    // one pass over the slice with the rows' exponentials from the table (TT, TD_) or computed
    auto pass = [&](auto tt, auto td) {
        constexpr bool TT = decltype(tt)::value, TD_ = decltype(td)::value;
#pragma unroll
        for (int c = 0; c < kChunks; ++c) {
            if (c + kAhead < kChunks) {
                const int jn = base + (c + kAhead) * kWave * kPer;
                qt[c + kAhead] = load_raw8<TD>(r.trow, r.t_al, jn, a.V);
                if (resid) qd[c + kAhead] = load_raw8<DD>(r.drow, r.d_al, jn, a.V);
            }
            float ct[kPer], cd[kPer];
            widen8<TD>(qt[c], ct);
            widen8<DD>(qd[c], cd);
            if (resid) {
                uint64_t any_band = 0;
                if constexpr (TT && TD_) {
                    double cA = 0.0, cB = 0.0, cR = 0.0, cDs = 0.0;
                    chunk_pair_tab(qt[c].w[0], qd[c].w[0], shE, lam, band, cA, cB, cR, cDs, any_band);
                    // a chunk that holds a magnitude below the table's range is formed again, the slow way
                    if (__builtin_expect(__builtin_amdgcn_ballot_w64(cA != cA || cB != cB) != 0, 0)) {
                        asm volatile("" ::: "memory");
                        any_band = 0;
                        cA = 0.0; cB = 0.0; cR = 0.0; cDs = 0.0;
                        chunk_pair<true, true>(ct, cd, rp, rq, shT, shE, c2, top, lam, band, cA, cB, cR, cDs, any_band);
                    }
                    A += cA; Bs += cB; R += cR; Ds += cDs;
                } else {
                    static_assert(!TT && !TD_, "the table serves both rows or neither");
                    chunk_pair<false, false>(ct, cd, rp, rq, shT, shE, c2, top, lam, band, A, Bs, R, Ds, any_band);
                }
                if (__builtin_expect(any_band != 0, 0)) {
                    asm volatile("" ::: "memory");                  // keep this a branch: a select would cost every element
                    // almost never taken: form the chunk's exponentials again and treat its band elements one by one
#pragma unroll 1
                    for (int i = 0; i < kPer; ++i) {
                        const double av = TT ? tab_exp_any(ct[i], shE) : exp_fast(ct[i], rp.neg_ref_c, rp.lo, shT, c2, top);
                        const double bv = TD_ ? tab_exp_any(cd[i], shE) : exp_fast(cd[i], rq.neg_ref_c, rq.lo, shT, c2, top);
                        const double diff = fma(-lam, bv, av);
                        if (fabs(diff) < band * bv) {
                            U += bv;
                            const int pos = atomicAdd(&a.jobs[j].band_cnt, 1);
                            if (pos < kBandCap) a.jobs[j].band_idx[pos] = base + c * kWave * kPer + i;
                        }
                    }
                }
            } else {
                double cA = 0.0;
                if constexpr (TT) {
                    cA = chunk_one_tab(qt[c].w[0], shE);
                    if (__builtin_expect(__builtin_amdgcn_ballot_w64(cA != cA) != 0, 0)) {
                        asm volatile("" ::: "memory");
                        cA = 0.0;
#pragma unroll
                        for (int i = 0; i < kPer; ++i) cA += tab_exp_any(ct[i], shE);
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < kPer; ++i) cA += exp_fast(ct[i], rp.neg_ref_c, rp.lo, shT, c2, top);
                }
                A += cA;
            }
        }
    };
    using std::false_type; using std::true_type;
    static_assert(kTabT == kTabD, "the table serves both rows or neither");
    if constexpr (kTabT) {
        // (a job on one row, the bonus position, has no draft row: the pass then sums the target row alone)
        if (__builtin_expect(tab_t, 1)) pass(true_type{}, true_type{}); else pass(false_type{}, false_type{});
    } else {
        pass(false_type{}, false_type{});
    }
    WG_STAMP_LANE0(g_stamps_slices, 8, wg, 3 + wave);            // this wavefront's loop done (slots 3..6)
    double D = 0.5 * (Bs + Ds);
    A = wave_sum_d(A) * sc.ct;
    if (resid) { Bs = wave_sum_d(Bs) * sc.cd; R = wave_sum_d(R) * sc.ct; D = wave_sum_d(D) * sc.cd; U = wave_sum_d(U) * sc.cd; }
    if (lane == 0) {
        double *o = a.part1 + ((int64_t)j * a.nsl + s) * kSliceVals;
        o[0] = A; o[1] = Bs; o[2] = R; o[3] = D; o[4] = U;
    }
    WG_STAMP(g_stamps_slices, 8, wg, 7);                         // first wavefront's sums stored
}

// ---- locate kernel: one workgroup per sequence --------------------------------------------
constexpr int kThreadPer = kSampleSlice / kVBlock;     // 8 consecutive elements per thread inside a slice

struct Weights {
    int kind;          // 1 residual max(0, a - L b), 2 target row only (a)
    double lam;        // exact S_p / S_q
    ExpRef rp, rq;
};

// Exclusive scan of one double per thread over the workgroup (thread order); *total = sum.  One barrier;
// sh4 must not be in use by a previous call that other wavefronts may still be reading.
__device__ inline double block_excl_scan_d(double v, double *sh4, double *total)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    double wtot;
    const double inc = wave_incl_scan_d(v, &wtot);
    if (lane == 0) sh4[wave] = wtot;
    __syncthreads();
    double base = 0.0;
#pragma unroll
    for (int w2 = 0; w2 < kVBlock / kWave; ++w2) base += (w2 < wave) ? sh4[w2] : 0.0;
    *total = ((sh4[0] + sh4[1]) + sh4[2]) + sh4[3];
    return base + (inc - v);
}

// Weights of the kThreadPer consecutive elements this thread owns in slice s.
template <int TD, int DD>
__device__ inline void thread_weights(const Weights &w, const Rows &r, int s, int V, const double *T, double (&wv)[kThreadPer])
{
    const int j0 = s * kSampleSlice + threadIdx.x * kThreadPer;
#pragma unroll
    for (int g = 0; g < kThreadPer / kPer; ++g) {
        // both rows' requests side by side where the run lies inside aligned rows (the usual case): the checks of the
        // general path are branches, and the compiler waits for the target row's data before it requests the draft row's
        const int j = j0 + g * kPer;
        const bool pair = w.kind == 1;
        Raw8<TD> qt;
        Raw8<DD> qd = Raw8<DD>{};
        if (r.t_al && (r.d_al || !pair) && j + kPer <= V) {
#pragma unroll
            for (int h = 0; h < (TD == TAPOUT_F32 ? 2 : 1); ++h) qt.w[h] = *(const u32x4 *)(r.trow + (int64_t)j * Elem<TD>::size + 16 * h);
            if (pair) {
#pragma unroll
                for (int h = 0; h < (DD == TAPOUT_F32 ? 2 : 1); ++h) qd.w[h] = *(const u32x4 *)(r.drow + (int64_t)j * Elem<DD>::size + 16 * h);
            }
        } else {
            qt = load_raw8<TD>(r.trow, r.t_al, j, V);
            if (pair) qd = load_raw8<DD>(r.drow, r.d_al, j, V);
        }
        float xt[kPer], xd[kPer];
        widen8<TD>(qt, xt);
        widen8<DD>(qd, xd);
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            double v = exp_fast(xt[i], w.rp.neg_ref_c, w.rp.lo, T);
            if (w.kind == 1) {
                v = fma(-w.lam, exp_fast(xd[i], w.rq.neg_ref_c, w.rq.lo, T), v);
                v = v > 0.0 ? v : 0.0;
            }
            // masked (-inf) logits carry a stand-in weight of ~1e-304: exactly zero for the scan
            wv[g * kPer + i] = (j0 + g * kPer + i < V && v > 1.0e-290) ? v : 0.0;
        }
    }
}

struct LocateShared {
    double scan[2][4];      // alternating buffers of block_excl_scan_d
    double bc[4];           // broadcasts
    int hits[2][4];         // alternating per-wavefront results of locate_in_slice
    int last, slice;
    int band_key[kBandCap];     // band elements of the sequence, sorted by index ...
    double band_val[kBandCap];  // ... and their residual weights with the exact L
};

__device__ inline int wave_min_i32(int v)
{
    v = min(v, __builtin_amdgcn_update_dpp(0x7fffffff, v, 0xB1, 0xf, 0xf, false));
    v = min(v, __builtin_amdgcn_update_dpp(0x7fffffff, v, 0x4E, 0xf, 0xf, false));
    v = min(v, __builtin_amdgcn_update_dpp(0x7fffffff, v, 0x141, 0xf, 0xf, false));
    v = min(v, __builtin_amdgcn_update_dpp(0x7fffffff, v, 0x140, 0xf, 0xf, false));
    return min(min(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
               min(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}

// First element of slice s whose running sum (starting at cum) exceeds target, or -1.
// With track_last, sh->last collects the largest index with positive weight seen (fallback only).
// *slice_total: the slice's weight as scanned.  `phase` alternates between calls so that consecutive
// scans use different LDS buffers.
template <int TD, int DD>
__device__ inline int locate_in_slice(const Weights &w, const Rows &r, int s, int V, const double *T,
                                      double cum, double target, LocateShared *sh, int phase, double *slice_total,
                                      bool track_last = false)
{
    double wv[kThreadPer];
    thread_weights<TD, DD>(w, r, s, V, T, wv);
    double sum = 0.0;
#pragma unroll
    for (int i = 0; i < kThreadPer; ++i) sum += wv[i];
    const double excl = block_excl_scan_d(sum, sh->scan[phase & 1], slice_total);
    const int j0 = s * kSampleSlice + threadIdx.x * kThreadPer;
    double c = cum + excl;
    int hit = 0x7fffffff, lp = -1;
#pragma unroll
    for (int i = 0; i < kThreadPer; ++i) {
        c += wv[i];
        if (wv[i] > 0.0) lp = j0 + i;
        if (hit == 0x7fffffff && j0 + i < V && c > target) hit = j0 + i;
    }
    // one LDS word per wavefront instead of one atomic per thread
    hit = wave_min_i32(hit);
    const int wave = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0) sh->hits[phase & 1][wave] = hit;
    if (track_last) {
        const int neg = wave_min_i32(-lp);                         // max of lp
        if ((threadIdx.x & (kWave - 1)) == 0 && -neg >= 0) atomicMax(&sh->last, -neg);
    }
    __syncthreads();
    const int *hh = sh->hits[phase & 1];
    const int h = min(min(hh[0], hh[1]), min(hh[2], hh[3]));
    return h == 0x7fffffff ? -1 : h;
}

// Band elements of a sequence (see the slice kernel).  Each listed element is evaluated with the exact L; what it
// contributed to the slice sums under L~ (recomputed here with the slice kernel's own arithmetic, hence the same
// number) is taken back: correction = max(0, a - L b) - (max(0, a - L~ b) - delta [a > L~ b] b).  The list is
// sorted by index, so that sums over it do not depend on the order in which the slice kernel's workgroups
// appended.  Leaves the sorted (index, correction) pairs in sh and returns their total.  Whole workgroup.
// E: the table of bfloat16 exponentials (memory), sc / tab_t / tab_d: the job's scales as the slice kernel formed them
// (tab_scale): the side of L~ an element was counted on is decided here on the very numbers the slice kernel compared.
template <int TD, int DD>
__device__ __noinline__ double settle_band(const Weights &w, const Rows &r, int V, const double *T, const double *E,
                                           const TabScale &sc, bool tab_t, bool tab_d,
                                           double delta, int n_band, int band_i, LocateShared *sh)
{
    const int tid = threadIdx.x;
    double wv = 0.0;
    if (tid < n_band && band_i < V) {
        const float xt = load_elem<TD>(r.trow, band_i), xd = load_elem<DD>(r.drow, band_i);
        const double avp = tab_t ? tab_exp_any(xt, E) : exp_fast(xt, w.rp.neg_ref_c, w.rp.lo, T);
        const double bvp = tab_d ? tab_exp_any(xd, E) : exp_fast(xd, w.rq.neg_ref_c, w.rq.lo, T);
        const double av = avp * sc.ct, bv = bvp * sc.cd;       // (scales of 1 where the row's exponentials are computed)
        const double v = fma(-w.lam, bv, av);
        const double exact = v > 1.0e-290 ? v : 0.0;           // same rule as thread_weights (masked logits weigh nothing)
        const double dt = fma(-sc.Lp, bvp, avp);
        wv = exact - (sc.ct * fmax(dt, 0.0) - delta * (dt >= 0.0 ? bv : 0.0));
    }
    if (tid < kBandCap) { sh->band_key[tid] = tid < n_band ? band_i : 0x7fffffff; sh->band_val[tid] = wv; }
    __syncthreads();
    int rank = 0;
    if (tid < n_band)
        for (int q = 0; q < n_band; ++q) rank += sh->band_key[q] < band_i ? 1 : 0;     // indices are distinct
    __syncthreads();
    if (tid < n_band) { sh->band_key[rank] = band_i; sh->band_val[rank] = wv; }
    __syncthreads();
    double total = 0.0;
    for (int q = 0; q < n_band; ++q) total += sh->band_val[q];
    return total;
}

// TAIL: the workgroup also ends its sequence's round for the UCB policies (a logarithm and a square root per arm, one
// thread).  Thompson Sampling is not offered here: its Gamma / Gaussian draws are long double-precision chains that
// want 178 registers and scratch memory, which this kernel would then pay for at every launch (measured: twice as long).
//
// FIN (whole-round calls whose accept decisions did not wait for the draft epilogue): the launch carries
// that epilogue's workgroups too, one per sequence, ahead of the locate workgroups: two latency-bound kernels of a
// few dozen workgroups each run side by side instead of one after the other.
template <int TD, int DD, bool TAIL, bool FIN>
__global__ __launch_bounds__(kVBlock) void verify_locate(VerifyArgs a, DraftFinalArgs fin)
{
    if constexpr (FIN) warm_args(a, fin); else warm_args(a);
    static_assert(kVBlock == kFinalBlock, "the draft epilogue runs in this kernel's workgroups");
    LOCATE_STAMP(0);                                             // entry
    // Thompson Sampling (tapout_round, bandit_tail == 2): the end of the round needs nothing of this launch, only the
    // accepted lengths of an earlier one, so it rides along as workgroups of its own behind the others, sixteen
    // sequences each (sixteen lanes per sequence), instead of taking a launch after this one.
    if (a.bandit_tail == 2) {
        const int first = (FIN ? a.B : 0) + a.n_jobs;
        if ((int)blockIdx.x >= first) {
            update_select_ts_lanes(a.bandit, ((int)blockIdx.x - first) * (kVBlock / 16) + (int)(threadIdx.x >> 4), threadIdx.x & 15,
                                   a.b_arm_in, a.accept_len, a.n_draft, a.b_gamma, a.b_active, a.b_u_ts, a.b_arm_out, a.b_flags);
            return;
        }
    }
    if constexpr (FIN)
        if ((int)blockIdx.x < a.B) {
            draft_finalize_body<false>(fin, blockIdx.x);
#ifdef TAPOUT_WG_STAMPS
            __syncthreads();
#endif
            LOCATE_STAMP(7);                                     // the epilogue's workgroup: done
            return;
        }
    __shared__ double shT[256];
    __shared__ double sh_red[kSliceVals][kVBlock / kWave];
    __shared__ LocateShared shl;
    const int j = FIN ? blockIdx.x - a.B : blockIdx.x;               // job; its sequence is b
    const int b = j / a.jps;
    const int tid = threadIdx.x;
    // the slice sums, the table and the uniform are requested before the job is looked at (one round trip)
    const double *ps = a.part1 + (int64_t)j * a.nsl * kSliceVals;
    double *zs = a.part2 + (int64_t)j * a.nsl;                       // exact slice weights (slow path only)
    // First all loads that do not depend on each other, then their uses: written so that no wait separates the
    // requests (the first slice of each thread without a loop; 256 threads fetch the 256 table entries).
    static_assert(kVBlock == 256, "one table entry per thread");
    double acc[kSliceVals] = {0.0, 0.0, 0.0, 0.0, 0.0};
    const bool has_first = tid < a.nsl;
    const double *pf = ps + (has_first ? tid : 0) * kSliceVals;
    const double f0 = pf[0], f1 = pf[1], f2 = pf[2], f3 = pf[3], f4 = pf[4];     // slot 0 always exists: harmless when unused
    const double tv = a.exp_table[tid];
    const float u32v = a.u_sample[j];
    const int band_n = a.jobs[j].band_cnt;
    const int band_i = a.jobs[j].band_idx[tid & (kBandCap - 1)];                                  // stale beyond band_n: unused
    const SampleJob job = a.jobs[j].job;
    // TAIL: the first thread also requests what the end of the round reads (bandit state of the sequence, its arm,
    // lengths; the accepted length is the head's, written by an earlier launch)
    UcbLane ucb;
    int32_t acc_len = 0;
    if constexpr (TAIL)
        if (tid < TAPOUT_MAX_ARMS) {                                  // one arm per lane
            ucb = ucb_lane_prefetch(a.bandit, b, tid, a.b_arm_in, a.n_draft, a.b_gamma, a.b_active);
            acc_len = a.accept_len[b];
            asm volatile("" :: "v"(ucb.S), "v"(ucb.Q), "v"(ucb.N), "v"(ucb.arm), "v"(ucb.n_draft), "v"(ucb.gamma), "v"(acc_len));
        }
    // the compiler would otherwise sink these loads below the early exit and pay a second round trip for them
    asm volatile("" :: "v"(f0), "v"(f1), "v"(f2), "v"(f3), "v"(f4), "v"(tv), "v"(u32v), "v"(band_n), "v"(band_i));
    shT[tid] = tv;
    // tapout_round: this workgroup also ends the sequence's round (the accepted length is the head's, written by an
    // earlier launch): reward into its bandit, next arm.
    auto end_round = [&]() {
        if constexpr (TAIL)
            if (tid < TAPOUT_MAX_ARMS) ucb_lane_finish(a.bandit, b, tid, ucb, acc_len, a.b_arm_out, a.b_flags);
    };
    if (__builtin_expect(job.kind == 0, 0)) { end_round(); return; }                       // the slice sums of such a sequence are stale: unused
    if (has_first) { acc[0] = f0; acc[1] = f1; acc[2] = f2; acc[3] = f3; acc[4] = f4; }
    for (int s = tid + kVBlock; s < a.nsl; s += kVBlock)              // vocabularies beyond 256 slices
#pragma unroll
        for (int q = 0; q < kSliceVals; ++q) acc[q] += ps[s * kSliceVals + q];
    if (tid == 0) { shl.last = -1; shl.slice = 0x7fffffff; }

    LOCATE_STAMP(1);                                             // first requests answered
    // totals of the five slice quantities, fixed order
    double tot[kSliceVals];
    {
#pragma unroll
        for (int q = 0; q < kSliceVals; ++q) acc[q] = wave_sum_d(acc[q]);
        if ((tid & (kWave - 1)) == 0)
#pragma unroll
            for (int q = 0; q < kSliceVals; ++q) sh_red[q][tid / kWave] = acc[q];
        __syncthreads();                                               // also publishes the table and the inits
#pragma unroll
        for (int q = 0; q < kSliceVals; ++q) tot[q] = (sh_red[q][0] + sh_red[q][1]) + (sh_red[q][2] + sh_red[q][3]);
    }
    const double Sp = tot[0], Sq = tot[1];
    Weights w;
    w.kind = job.kind;
    w.rp.set((double)job.ref_p); w.rq.set((double)job.ref_q);
    bool draft_bad = false;
    if (job.kind == 1 && (!(Sq > 0.0) || !(Sq < INFINITY))) {          // NaN / empty draft row: draw from the target row alone
        w.kind = 2;
        draft_bad = true;
    }
    w.lam = w.kind == 1 ? Sp / Sq : 0.0;
    const double delta = w.lam - job.lam;
    const Rows r = job_rows<TD, DD>(a, b, job);
    const double u = (double)u32v;
    int phase = 0;

    // slice weights: target row alone -> A_s; residual -> R~_s - delta D_s if the bound on the sign flips allows,
    // else with the listed band elements corrected one by one
    double Z = w.kind == 2 ? Sp : tot[2] - delta * tot[3];
    bool exact_sums = false;
    int n_band = 0;
    if (w.kind == 1) {
        const bool close = fabs(delta) <= kEta * job.lam;
        bool certified = close && Z > 0.0 && fabs(delta) * tot[4] <= 2.0e-10 * Z;
        if (__builtin_expect(!certified && close && band_n <= kBandCap, 0)) {
            n_band = band_n;
            const bool tab_ok = TD == TAPOUT_BF16 && DD == TAPOUT_BF16 && !(a.vflags & kVerifyNoExpTable) && tab_job_ok(job);    // as in the slice kernel
            const bool tab_t = tab_ok, tab_d = tab_ok;
            Z += settle_band<TD, DD>(w, r, a.V, shT, a.exp_table + 256, tab_scale(job, tab_t, tab_d, shT), tab_t, tab_d,
                                     delta, band_n, band_i, &shl);
            certified = Z > 0.0;
        }
        if (__builtin_expect(!certified, 0)) {
            n_band = 0;
            // slow path: exact slice weights with the exact L (also the p == q case: then Z may vanish)
            double ztot = 0.0;
            for (int s = 0; s < a.nsl; ++s) {
                double st;
                locate_in_slice<TD, DD>(w, r, s, a.V, shT, 0.0, INFINITY, &shl, phase++, &st);
                if (tid == 0) zs[s] = st;
                ztot += st;
            }
            Z = ztot;
            if (!(Z > 0.0)) {
                // the residual vanished (p == q up to rounding): draw from the target row itself
                w.kind = 2;
                ztot = 0.0;
                for (int s = 0; s < a.nsl; ++s) {
                    double st;
                    locate_in_slice<TD, DD>(w, r, s, a.V, shT, 0.0, INFINITY, &shl, phase++, &st);
                    if (tid == 0) zs[s] = st;
                    ztot += st;
                }
                Z = ztot;
            }
            exact_sums = true;
            if (tid == 0) shl.last = -1;
            __threadfence_block();
            __syncthreads();
        }
    }
    auto slice_weight = [&](int s) -> double {
        if (exact_sums) return zs[s];
        if (w.kind == 2) return ps[s * kSliceVals + 0];
        double v = ps[s * kSliceVals + 2] - delta * ps[s * kSliceVals + 3];
        v = v > 0.0 ? v : 0.0;
        for (int q = 0; q < n_band; ++q)
            if (shl.band_key[q] / kSampleSlice == s) v += shl.band_val[q];
        return v;
    };

    LOCATE_STAMP(2);                                             // total weight known (certified, settled or recomputed)
    int token = -1;
    if (Z > 0.0) {
        const double target = u * Z;
        // slice whose inclusive prefix (slice order) first exceeds the target
        double cum_at = 0.0;
        int s_found = -1;
        if (__builtin_expect(a.nsl <= kVBlock, 1)) {
            // this thread's slice is the one whose sums it fetched with the first round trip: no second look at memory
            double z_mine = 0.0;
            if (tid < a.nsl) {
                if (exact_sums) z_mine = zs[tid];
                else if (w.kind == 2) z_mine = f0;
                else {
                    z_mine = f2 - delta * f3;
                    z_mine = z_mine > 0.0 ? z_mine : 0.0;
                    for (int q = 0; q < n_band; ++q)
                        if (shl.band_key[q] / kSampleSlice == tid) z_mine += shl.band_val[q];
                }
            }
            double ztot;
            const double excl = block_excl_scan_d(z_mine, shl.scan[phase++ & 1], &ztot);
            const int cand = wave_min_i32((tid < a.nsl && excl + z_mine > target) ? tid : 0x7fffffff);
            if ((tid & (kWave - 1)) == 0) shl.hits[phase & 1][tid / kWave] = cand;
            __syncthreads();
            const int *hh = shl.hits[phase & 1];
            const int sf = min(min(hh[0], hh[1]), min(hh[2], hh[3]));
            ++phase;
            s_found = sf == 0x7fffffff ? -1 : sf;
            if (tid == s_found) shl.bc[0] = excl;
            __syncthreads();
            if (s_found >= 0) cum_at = shl.bc[0];
        } else {
            // very large vocabularies: the first thread walks the slice weights
            if (tid == 0) {
                double c = 0.0; int sf = -1;
                for (int s = 0; s < a.nsl; ++s) { const double v = slice_weight(s); if (c + v > target) { sf = s; break; } c += v; }
                shl.bc[0] = c; shl.slice = sf;
            }
            __syncthreads();
            cum_at = shl.bc[0]; s_found = shl.slice;
            __syncthreads();
        }
        LOCATE_STAMP(3);                                         // slice found
        // slice sums and the in-slice scan round differently: if the crossing is not inside the chosen
        // slice, continue into the following ones
        if (s_found >= 0) {
            double cum = cum_at;
            for (int s = s_found; s < a.nsl && token < 0; ++s) {
                double slice_total;
                token = locate_in_slice<TD, DD>(w, r, s, a.V, shT, cum, target, &shl, phase++, &slice_total);
                cum += slice_total;
            }
        }
        if (__builtin_expect(token < 0, 0)) {
            // rounding left no crossing: the largest index with positive weight
            {
                for (int s = 0; s < a.nsl; ++s) {
                    double slice_total;
                    locate_in_slice<TD, DD>(w, r, s, a.V, shT, 0.0, INFINITY, &shl, phase++, &slice_total, true);
                }
                __syncthreads();
            }
            token = shl.last;
        }
    }
    LOCATE_STAMP(4);                                             // token found
    if (tid == 0) {
        if (token < 0) token = 0;
        if (a.tok_direct) a.tok_direct[j] = token;
        else a.out_tok[(int64_t)b * (a.K + 1) + job.row] = token;
        if (__builtin_expect(draft_bad, 0)) {
            uint32_t f = a.flags_ws[b] | TAPOUT_FLAG_BAD_ROW;
            a.flags_ws[b] = f;
            if (a.flags) a.flags[b] = f;
        }
    }
    end_round();
    LOCATE_STAMP(5);                                             // round ended (bandit update, next arm)
}

// ---- draft-token sampling: one job per draft row --------------------------------------------
// One thread per row (b, k): merges the row's slice partials straight from memory (a few dozen bytes) for
// the maximum, the exponent reference of the draw.
__global__ __launch_bounds__(kVBlock) void sample_head_kernel(VerifyArgs a)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= a.n_jobs) return;
    const int b = j / a.K, k = j - b * a.K;
    int kb = a.n_draft ? a.n_draft[b] : a.K;
    kb = kb > a.K ? a.K : kb;
    SampleJob job;
    job.kind = 0; job.row = k; job.ref_p = 0.0f; job.ref_q = 0.0f; job.lam = 0.0;
    if (k < kb) {
        // the row's maximum, and the finaliser's bad-row rule: a NaN anywhere poisons a slice's sum (also from inside
        // the batch the draft pass leaves out of it), an infinite maximum has no softmax
        float M = -INFINITY;
        bool bad = false;
        for (int sl = 0; sl < a.nsplit; ++sl) {
            const Partial p = a.part[(int64_t)j * a.nsplit + sl];
            M = fmaxf(M, p.v1);
            bad |= !(p.S >= 0.0f) || p.S == INFINITY;
        }
        bad |= M == -INFINITY || M == INFINITY;
        if (bad) a.tok_direct[j] = -1;           // NaN in the row or no finite maximum: nothing to draw from
        else { job.kind = 2; job.ref_p = M; }
    }
    a.jobs[j].job = job;
    a.jobs[j].band_cnt = 0;
}

// ---- final token over vocabulary shards ---------------------------------------------------------
// Copies the caller's jobs into the context's job records (the slice kernel reads them there and appends band
// elements, which the sharded path counts but does not use).
__global__ void shard_jobs_kernel(ShardFinalArgs a)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= a.v.B) return;
    a.v.jobs[b].job = a.jobs_in[b];
    a.v.jobs[b].band_cnt = 0;
}

// This shard's five sums per sequence: the slice sums in slice order (fixed order, one thread per value).
__global__ void shard_sums_kernel(ShardFinalArgs a)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= a.v.B * kSliceVals) return;
    const int b = i / kSliceVals, q = i - b * kSliceVals;
    double s = 0.0;
    if (a.jobs_in[b].kind != 0 && (q == 0 || a.jobs_in[b].kind == 1)) {
        const double *ps = a.v.part1 + (int64_t)b * a.v.nsl * kSliceVals;
        for (int sl = 0; sl < a.v.nsl; ++sl) s += ps[sl * kSliceVals + q];
    }
    a.sums_out[i] = s;
}

// One workgroup per sequence.  Every shard runs this on the same sums_all, so all of them derive the same
// normaliser ratio, the same masses and the same owner; only the owner scans its slices for the token.
template <int TD, int DD>
__global__ __launch_bounds__(kVBlock) void shard_locate(ShardFinalArgs a)
{
    __shared__ double shT[256];
    __shared__ LocateShared shl;
    const VerifyArgs &v = a.v;
    const int b = blockIdx.x, tid = threadIdx.x;
    const SampleJob job = a.jobs_in[b];
    if (tid == 0) { a.tok_out[b] = -1; a.need_exact[b] = 0; a.exact_mass[b] = NAN; }
    if (job.kind == 0) return;
    shT[tid] = v.exp_table[tid];
    if (tid == 0) { shl.last = -1; shl.slice = 0x7fffffff; }
    __syncthreads();
    // totals over all shards, shard order
    double tot[kSliceVals] = {0.0, 0.0, 0.0, 0.0, 0.0};
    for (int h = 0; h < a.G; ++h)
#pragma unroll
        for (int q = 0; q < kSliceVals; ++q) tot[q] += a.sums_all[((int64_t)h * v.B + b) * kSliceVals + q];
    const double Sp = tot[0], Sq = tot[1];
    Weights w;
    w.kind = job.kind;
    w.rp.set((double)job.ref_p); w.rq.set((double)job.ref_q);
    if (job.kind == 1 && (!(Sq > 0.0) || !(Sq < INFINITY))) w.kind = 2;       // unusable draft row: draw from the target row alone
    w.lam = w.kind == 1 ? Sp / Sq : 0.0;
    const double delta = w.lam - job.lam;
    const Rows r = job_rows<TD, DD>(v, b, job);
    const double *ps = v.part1 + (int64_t)b * v.nsl * kSliceVals;
    double *zs = v.part2 + (int64_t)b * v.nsl;
    int phase = 0;
    // mass of shard h under the current weights
    bool exact = false;                       // masses and own slice weights are exact recomputations
    auto shard_mass = [&](int h) -> double {
        const double *sh = a.sums_all + ((int64_t)h * v.B + b) * kSliceVals;
        if (w.kind == 2) return sh[0];
        if (exact) return a.exact_all[(int64_t)h * v.B + b];
        const double m = sh[2] - delta * sh[3];
        return m > 0.0 ? m : 0.0;
    };
    double Z = w.kind == 2 ? Sp : tot[2] - delta * tot[3];
    if (w.kind == 1) {
        const bool certified = fabs(delta) <= kEta * job.lam && Z > 0.0 && fabs(delta) * tot[4] <= 2.0e-10 * Z;
        if (!certified) {
            // exact weights of this shard's slices with the exact ratio (every shard does this for its own slices)
            double ztot = 0.0;
            for (int s = 0; s < v.nsl; ++s) {
                double st;
                locate_in_slice<TD, DD>(w, r, s, v.V, shT, 0.0, INFINITY, &shl, phase++, &st);
                if (tid == 0) zs[s] = st;
                ztot += st;
            }
            __threadfence_block();
            __syncthreads();
            if (!a.exact_all) {                                                // first call: hand the exact mass to the caller
                if (tid == 0) { a.exact_mass[b] = ztot; a.need_exact[b] = 1; }
                return;
            }
            exact = true;
            Z = 0.0;
            for (int h = 0; h < a.G; ++h) Z += a.exact_all[(int64_t)h * v.B + b];
            if (!(Z > 0.0)) {                                                   // p == q up to rounding: draw from the target row itself
                w.kind = 2; exact = false; Z = Sp;
            }
        }
    }
    if (!(Z > 0.0)) {                                                           // nothing to draw from anywhere: the first shard answers token 0
        if (tid == 0 && a.g == 0) a.tok_out[b] = a.vocab_offset;
        return;
    }
    // owner: the first shard whose inclusive prefix of masses exceeds u * Z; the last one with mass if rounding leaves none
    const double target = (double)v.u_sample[b] * Z;
    double prefix = 0.0, mine_prefix = 0.0;
    int owner = -1, last_pos = -1;
    for (int h = 0; h < a.G; ++h) {
        const double m = shard_mass(h);
        if (h == a.g) mine_prefix = prefix;
        if (m > 0.0) last_pos = h;
        if (owner < 0 && prefix + m > target) owner = h;
        prefix += m;
    }
    const bool fallback = owner < 0;
    if (fallback) owner = last_pos;
    if (owner != a.g) return;
    auto slice_weight = [&](int s) -> double {
        if (w.kind == 2) return ps[s * kSliceVals + 0];
        if (exact) return zs[s];
        const double x = ps[s * kSliceVals + 2] - delta * ps[s * kSliceVals + 3];
        return x > 0.0 ? x : 0.0;
    };
    int token = -1;
    if (!fallback) {
        const double local = target - mine_prefix;
        // the first thread walks the slice weights (a few hundred at most; this kernel is rare-path simple)
        if (tid == 0) {
            double c = 0.0; int sf = -1;
            for (int s = 0; s < v.nsl; ++s) { const double x = slice_weight(s); if (c + x > local) { sf = s; break; } c += x; }
            shl.bc[0] = c; shl.slice = sf;
        }
        __syncthreads();
        double cum = shl.bc[0];
        const int s_found = shl.slice;
        __syncthreads();
        if (s_found >= 0)
            for (int s = s_found; s < v.nsl && token < 0; ++s) {
                double slice_total;
                token = locate_in_slice<TD, DD>(w, r, s, v.V, shT, cum, local, &shl, phase++, &slice_total);
                cum += slice_total;
            }
    }
    if (token < 0) {                                                            // rounding left no crossing: the last positive weight here
        if (tid == 0) shl.last = -1;
        __syncthreads();
        for (int s = 0; s < v.nsl; ++s) {
            double slice_total;
            locate_in_slice<TD, DD>(w, r, s, v.V, shT, 0.0, INFINITY, &shl, phase++, &slice_total, true);
        }
        __syncthreads();
        token = shl.last;
    }
    if (tid == 0) a.tok_out[b] = a.vocab_offset + (token < 0 ? 0 : token);
}

template <int TD, int DD>
hipError_t launch_shard_typed(const ShardFinalArgs &a, int pass, hipStream_t st)
{
    if (pass == 0) {
        hipLaunchKernelGGL(shard_jobs_kernel, dim3((a.v.B + 63) / 64), dim3(64), 0, st, a);
        const unsigned gy = a.v.n_jobs < 65535 ? a.v.n_jobs : 65535, gz = (a.v.n_jobs + gy - 1) / gy;
        hipLaunchKernelGGL((verify_slices<TD, DD, false>), dim3((a.v.nsl + kWavesPerWG - 1) / kWavesPerWG, gy, gz), dim3(kVBlock), 0, st, a.v);
        hipLaunchKernelGGL(shard_sums_kernel, dim3((a.v.B * kSliceVals + 63) / 64), dim3(64), 0, st, a);
    } else {
        hipLaunchKernelGGL((shard_locate<TD, DD>), dim3(a.v.B), dim3(kVBlock), 0, st, a);
    }
    return hipGetLastError();
}

hipError_t launch_shard_dispatch(const ShardFinalArgs &a, int pass, hipStream_t st)
{
    if (!a.v.exp_table) return hipErrorInvalidValue;
    if (a.v.t_dtype == TAPOUT_F32)
        return a.v.d_dtype == TAPOUT_F32 ? launch_shard_typed<TAPOUT_F32, TAPOUT_F32>(a, pass, st) : launch_shard_typed<TAPOUT_F32, TAPOUT_BF16>(a, pass, st);
    return a.v.d_dtype == TAPOUT_F32 ? launch_shard_typed<TAPOUT_BF16, TAPOUT_F32>(a, pass, st) : launch_shard_typed<TAPOUT_BF16, TAPOUT_BF16>(a, pass, st);
}

template <int TD, int DD>
hipError_t launch_typed(const VerifyArgs &a, const DraftFinalArgs &fin, bool with_fin, int pass, hipStream_t st, Timing tm)
{
    const unsigned gy = a.n_jobs < 65535 ? a.n_jobs : 65535, gz = (a.n_jobs + gy - 1) / gy;
    dim3 grid12((a.nsl + kWavesPerWG - 1) / kWavesPerWG, gy, gz), block(kVBlock);
    if (pass == 1) {
        if (a.fused_head) launch_kernel(verify_slices<TD, DD, true>, grid12, block, st, tm, a);
        else launch_kernel(verify_slices<TD, DD, false>, grid12, block, st, tm, a);
    }
    else {
        // bandit_tail 1: the locate workgroups end the round (UCB); 2: workgroups of their own do (Thompson Sampling)
        const unsigned extra = a.bandit_tail == 2 ? (unsigned)((a.B + kVBlock / 16 - 1) / (kVBlock / 16)) : 0u;
        const bool tail = a.bandit_tail == 1;
        if (with_fin) {
            if (!tail) launch_kernel(verify_locate<TD, DD, false, true>, dim3(a.n_jobs + a.B + extra), block, st, tm, a, fin);
            else launch_kernel(verify_locate<TD, DD, true, true>, dim3(a.n_jobs + a.B), block, st, tm, a, fin);
        }
        else if (!tail) launch_kernel(verify_locate<TD, DD, false, false>, dim3(a.n_jobs + extra), block, st, tm, a, fin);
        else launch_kernel(verify_locate<TD, DD, true, false>, dim3(a.n_jobs), block, st, tm, a, fin);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_shard_final_sums(const ShardFinalArgs &a, hipStream_t st) { return launch_shard_dispatch(a, 0, st); }
hipError_t launch_shard_final_token(const ShardFinalArgs &a, hipStream_t st) { return launch_shard_dispatch(a, 1, st); }

hipError_t launch_sample_head(const VerifyArgs &a, hipStream_t st, Timing tm)
{
    launch_kernel(sample_head_kernel, dim3((a.n_jobs + kVBlock - 1) / kVBlock), dim3(kVBlock), st, tm, a);
    return hipGetLastError();
}

hipError_t launch_verify(const VerifyArgs &a, int pass, hipStream_t st, Timing tm, const DraftFinalArgs *fin)
{
    static const DraftFinalArgs no_fin{};
    const bool with_fin = fin != nullptr;
    if (!a.exp_table) return hipErrorInvalidValue;           // every pass reads it
    if (((a.vflags & kVerifyOwnQ) != 0) != with_fin || (fin && (a.jps != 1 || a.n_jobs != a.B || a.shards > 0 || fin->shards > 0 || fin->B != a.B)))
        return hipErrorInvalidValue;
    if (!fin) fin = &no_fin;
    if (pass == 0) {
        if (a.fused_head) return hipErrorInvalidValue;       // the slice kernel is the head then
        if (a.shards > 0) launch_kernel(verify_head_kernel<true>, dim3(a.B), dim3(kVBlock), st, tm, a);
        else launch_kernel(verify_head_kernel<false>, dim3(a.B), dim3(kVBlock), st, tm, a);
        return hipGetLastError();
    }
    if (a.t_dtype == TAPOUT_F32)
        return a.d_dtype == TAPOUT_F32 ? launch_typed<TAPOUT_F32, TAPOUT_F32>(a, *fin, with_fin, pass, st, tm) : launch_typed<TAPOUT_F32, TAPOUT_BF16>(a, *fin, with_fin, pass, st, tm);
    return a.d_dtype == TAPOUT_F32 ? launch_typed<TAPOUT_BF16, TAPOUT_F32>(a, *fin, with_fin, pass, st, tm) : launch_typed<TAPOUT_BF16, TAPOUT_BF16>(a, *fin, with_fin, pass, st, tm);
}

}  // namespace tapout

#ifdef TAPOUT_WG_STAMPS
// Copies one stamp table to the host (synchronises the device).  table 0: slice kernel, 8 slots per workgroup
// (0 entry, 1 job known, 2 tables in LDS and rows requested, 3..6 each wavefront's loop done, 7 sums stored);
// table 1: accept decisions inside the slice kernel, 4 slots (0 first requests answered, 1 rows merged, 2 decisions
// taken, 3 first rejection published); table 2: locate kernel, 8 slots by blockIdx.x (0 entry, 1 first requests
// answered, 2 total weight known, 3 slice found, 4 token found, 5 round ended; 7: a draft epilogue workgroup is done).
// Units: 10 ns.  Not part of the library's interface.
extern "C" __attribute__((visibility("default"))) int tapout_debug_wg_stamps(int table, unsigned long long *host, int n_wg)
{
    if (!host || n_wg < 0) return -1;
    if (hipDeviceSynchronize() != hipSuccess) return -2;
    if (table == 0 && n_wg <= tapout::kStampWgs)
        return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(tapout::g_stamps_slices), (size_t)n_wg * 8 * sizeof(unsigned long long));
    if (table == 1 && n_wg <= tapout::kStampWgs)
        return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(tapout::g_stamps_head), (size_t)n_wg * 4 * sizeof(unsigned long long));
    if (table == 2 && n_wg <= 4096)
        return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(tapout::g_stamps_locate), (size_t)n_wg * 8 * sizeof(unsigned long long));
    return -1;
}
#endif
