// Streaming pass over logits rows: the one read of the vocabulary that feeds
// every signal of Table 1 / Appendix A.1 (entropy, top-1 probability,
// top-1/top-2 margin) and the normalisers the verification step needs.
//
// One launch covers all rows of a [B, KK, V] tensor.  A row is cut into
// `nsplit` slices of whole 16-byte vectors; one 256-thread workgroup reduces
// one slice to a 32-byte Partial.  Every element is loaded exactly once, with
// 16-byte non-temporal loads that are contiguous across the wavefront, four
// vectors per thread in flight; six (draft) or eight (target) wavefronts per
// SIMD hide the latency (explicit double buffering was measured: slower).
// Batches that lie wholly inside the slice are loaded without bounds checks.
//
// Per thread the softmax sums are kept online in the base-2 domain against an
// integer reference R >= max * log2 e: y = fma(x, log2e, -R) has a single
// rounding, 2^y comes from the hardware exp2, and moving to a larger reference
// is an exact ldexp.  Top-2 values are tracked with max3 / med3 on pairs
// (second largest of {v1, a, b, v2} = max(med3(v1, a, b), v2) while v2 <= v1).
// Only the 16-byte window in which the thread's maximum first appeared is
// remembered; the exact argmax index is recovered later from that window.
//
// Draft rows: the entropy of a peaked row is a small number made of small
// terms, and a binary32 sum that also holds the row's dominant term rounds
// them away.  So the batch of vectors in which a thread met its maximum is
// summed apart from the rest, and the workgroup leaves the batch that holds the
// slice's first maximum out of its partial altogether: the sums of a partial
// then hold "small" terms only, and the epilogue that merges the partials adds
// the few elements of that one batch back from the logits themselves, with the
// row's first maximum as an exact term of its own.
//
// Wavefront reductions use DPP row operations (no LDS traffic).  The partials
// are merged per sequence by a second, small launch (finalize.hip for draft
// rows, the head kernel in verify.hip for target rows): a
// "last workgroup finishes the sequence" scheme was measured and lost, because
// on this chip every cross-workgroup hand-over costs a memory round trip of
// about 3 us under streaming load and four of them chain up.
#include "common.h"

namespace tapout {

namespace {

// max3 / med3 / max as the bare instructions.  fmaxf() and the med3 builtin first quiet every operand the compiler
// cannot prove to be a canonical number (one v_max_f32 x, x per logit, a tenth of the draft pass's vector
// instructions); the instructions themselves already return the other operand when one is a NaN, which is what the
// running maxima want (NaN logits are ignored here and poison the sums instead).
__device__ inline float max3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ inline float med3(float a, float b, float c)
{
    float r;
    asm("v_med3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ inline float max2(float a, float b)
{
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ inline float min2(float a, float b)
{
    float r;
    asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// Headroom (in powers of two) added to a thread's reference when it has to be
// raised, so that a slowly growing running maximum raises it only a few times.
constexpr float kHeadroom = 8.0f;

// Running maximum (and second maximum) over the values of one 16-byte vector, as one block of instructions: a
// statement per instruction makes the compiler put a wait state after each.
template <bool FULL>
__device__ inline void vector_max(float &v1, float &v2, const float (&x)[8])
{
    if constexpr (FULL) {
        float t;
        asm("v_med3_f32 %2, %0, %3, %4\n\tv_max_f32 %1, %1, %2\n\tv_max3_f32 %0, %0, %3, %4\n\t"
            "v_med3_f32 %2, %0, %5, %6\n\tv_max_f32 %1, %1, %2\n\tv_max3_f32 %0, %0, %5, %6\n\t"
            "v_med3_f32 %2, %0, %7, %8\n\tv_max_f32 %1, %1, %2\n\tv_max3_f32 %0, %0, %7, %8\n\t"
            "v_med3_f32 %2, %0, %9, %10\n\tv_max_f32 %1, %1, %2\n\tv_max3_f32 %0, %0, %9, %10"
            : "+v"(v1), "+v"(v2), "=&v"(t)
            : "v"(x[0]), "v"(x[1]), "v"(x[2]), "v"(x[3]), "v"(x[4]), "v"(x[5]), "v"(x[6]), "v"(x[7]));
    } else {
        asm("v_max3_f32 %0, %0, %1, %2\n\tv_max3_f32 %0, %0, %3, %4\n\tv_max3_f32 %0, %0, %5, %6\n\tv_max3_f32 %0, %0, %7, %8"
            : "+v"(v1)
            : "v"(x[0]), "v"(x[1]), "v"(x[2]), "v"(x[3]), "v"(x[4]), "v"(x[5]), "v"(x[6]), "v"(x[7]));
    }
}
template <bool FULL>
__device__ inline void vector_max(float &v1, float &v2, const float (&x)[4])
{
    if constexpr (FULL) {
        float t;
        asm("v_med3_f32 %2, %0, %3, %4\n\tv_max_f32 %1, %1, %2\n\tv_max3_f32 %0, %0, %3, %4\n\t"
            "v_med3_f32 %2, %0, %5, %6\n\tv_max_f32 %1, %1, %2\n\tv_max3_f32 %0, %0, %5, %6"
            : "+v"(v1), "+v"(v2), "=&v"(t)
            : "v"(x[0]), "v"(x[1]), "v"(x[2]), "v"(x[3]));
    } else {
        asm("v_max3_f32 %0, %0, %1, %2\n\tv_max3_f32 %0, %0, %3, %4"
            : "+v"(v1)
            : "v"(x[0]), "v"(x[1]), "v"(x[2]), "v"(x[3]));
    }
}

template <bool FULL>
struct ThreadState {
    float v1 = -INFINITY;   // running maximum
    float v2 = -INFINITY;   // running second largest (FULL only)
    float R = -1.0e30f;     // integer reference: every x seen so far has x*log2e <= R (+ rounding); -1e30: none yet
    float s = 0.0f;         // sum 2^(x*log2e - R); FULL: without the batch in which the running maximum appeared
    float t = 0.0f;         // sum 2^y * y (FULL only), likewise
    float s_hi = 0.0f;      // FULL: the two sums over the batch in which the running maximum appeared
    float t_hi = 0.0f;
    int32_t cand = 0x7fffffff;

    // Raise the reference so that it covers the running maximum (rare after the first few vectors).
    // sb, tb: the sums of the batch in progress (FULL).
    __device__ inline void cover_max(float &sb, float &tb)
    {
        if (__builtin_fmaf(v1, kLog2e, -R) > 0.0f) {          // also the first finite value (nothing is summed yet then)
            float Rn = ceilf(v1 * kLog2e) + kHeadroom;
            float d = Rn - R;
            int di = (int)fminf(fmaxf(d, -1.0e9f), 1.0e9f);
            if constexpr (FULL) {
                t = ldexpf(t - d * s, -di);
                t_hi = ldexpf(t_hi - d * s_hi, -di);
                tb = ldexpf(tb - d * sb, -di);
                s_hi = ldexpf(s_hi, -di);
                sb = ldexpf(sb, -di);
            }
            s = ldexpf(s, -di);
            R = Rn;
        }
    }

    // A batch of U vectors of N values each (vector u starts at element index first + u * stride of the row), vector
    // by vector: maxima (`first + u * stride` is remembered as the argmax candidate when vector u raises the running
    // maximum), reference check, sums.  The entropy sum of a vector is formed without looking at the terms; a masked
    // (-inf) logit gives 0 * -inf = NaN there, and only then the vector is summed again with the exponent clamped (one
    // comparison per vector instead of one clamp per element).
    template <int U, int N>
    __device__ inline void fold_batch(const u32x4 (&w)[U], int32_t first, int32_t stride)
    {
        bool grew = false;                                    // a lane mask in scalar registers
        float sb = 0.0f, tb = 0.0f;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float x[N];
            if constexpr (N == 8) unpack<TAPOUT_BF16>(w[u], x);
            else if constexpr (N == 4) unpack<TAPOUT_F32>(w[u], x);
            else x[0] = __uint_as_float(w[u].x);
            const float old = v1;
            if constexpr (N == 1) {
                if constexpr (FULL) v2 = max2(v2, min2(v1, x[0]));
                v1 = max2(v1, x[0]);
            } else {
                vector_max<FULL>(v1, v2, x);
            }
            const bool g = v1 > old;
            cand = g ? first + u * stride : cand;
            grew |= g;
            cover_max(sb, tb);
            float y[N], e[N];
#pragma unroll
            for (int i = 0; i < N; ++i) {
                y[i] = __builtin_fmaf(x[i], kLog2e, -R);
                e[i] = __builtin_amdgcn_exp2f(y[i]);
            }
            float sv = e[0];
            float tv = FULL ? e[0] * y[0] : 0.0f;
#pragma unroll
            for (int i = 1; i < N; ++i) {
                sv += e[i];
                if constexpr (FULL) tv = __builtin_fmaf(e[i], y[i], tv);
            }
            if constexpr (FULL) {
                if (tv != tv) {
                    tv = 0.0f;
#pragma unroll
                    for (int i = 0; i < N; ++i) tv = __builtin_fmaf(e[i], fmaxf(y[i], -200.0f), tv);
                }
                sb = u == 0 ? sv : sb + sv;                   // (a sum started from 0.0f would cost an addition: -0 + 0)
                tb = u == 0 ? tv : tb + tv;
            } else {
                s += sv;
            }
        }
        if constexpr (FULL) {
            // If the running maximum grew inside the batch, its sums become the set-apart ones and the batch that held
            // the previous maximum joins the rest; else it joins the rest itself.
            s += grew ? s_hi : sb;
            t += grew ? t_hi : tb;
            s_hi = grew ? sb : s_hi;
            t_hi = grew ? tb : t_hi;
        }
    }

    // One element on its own (unaligned head or tail of a row): a batch of one.
    __device__ inline void fold_single(float x0, int32_t j)
    {
        u32x4 w[1];
        w[0] = u32x4{__float_as_uint(x0), 0u, 0u, 0u};
        fold_batch<1, 1>(w, j, 0);
    }
};

// ---- wavefront reductions with DPP -------------------------------------------
// quad_perm [1,0,3,2] = 0xB1, quad_perm [2,3,0,1] = 0x4E, row_half_mirror = 0x141,
// row_mirror = 0x140: after the four steps every lane of a 16-lane row holds the
// row's result; the four rows are then combined through readlane.
template <int CTRL>
__device__ inline float dpp_f(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
template <int CTRL>
__device__ inline int dpp_i(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true); }
__device__ inline float lane_f(float v, int lane) { return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane)); }

__device__ inline float wave_max(float v)
{
    v = fmaxf(v, dpp_f<0xB1>(v)); v = fmaxf(v, dpp_f<0x4E>(v));
    v = fmaxf(v, dpp_f<0x141>(v)); v = fmaxf(v, dpp_f<0x140>(v));
    return fmaxf(fmaxf(lane_f(v, 0), lane_f(v, 16)), fmaxf(lane_f(v, 32), lane_f(v, 48)));
}
__device__ inline float wave_sum(float v)
{
    v += dpp_f<0xB1>(v); v += dpp_f<0x4E>(v); v += dpp_f<0x141>(v); v += dpp_f<0x140>(v);
    return (lane_f(v, 0) + lane_f(v, 16)) + (lane_f(v, 32) + lane_f(v, 48));
}
__device__ inline int wave_min_i(int v)
{
    v = min(v, dpp_i<0xB1>(v)); v = min(v, dpp_i<0x4E>(v)); v = min(v, dpp_i<0x141>(v)); v = min(v, dpp_i<0x140>(v));
    return min(min(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
               min(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}
// (largest, second largest counting duplicates) of the union of two such pairs
__device__ inline void top2_merge(float &a1, float &a2, float b1, float b2)
{
    a2 = max3(fminf(a1, b1), a2, b2);
    a1 = fmaxf(a1, b1);
}
__device__ inline void wave_top2(float &a1, float &a2)
{
    top2_merge(a1, a2, dpp_f<0xB1>(a1), dpp_f<0xB1>(a2));
    top2_merge(a1, a2, dpp_f<0x4E>(a1), dpp_f<0x4E>(a2));
    top2_merge(a1, a2, dpp_f<0x141>(a1), dpp_f<0x141>(a2));
    top2_merge(a1, a2, dpp_f<0x140>(a1), dpp_f<0x140>(a2));
    float r1 = lane_f(a1, 0), r2 = lane_f(a2, 0);
    top2_merge(r1, r2, lane_f(a1, 16), lane_f(a2, 16));
    top2_merge(r1, r2, lane_f(a1, 32), lane_f(a2, 32));
    top2_merge(r1, r2, lane_f(a1, 48), lane_f(a2, 48));
    a1 = r1; a2 = r2;
}

template <int DT> struct NegInfVec;
template <> struct NegInfVec<TAPOUT_F32>  { static constexpr uint32_t word = 0xff800000u; };
template <> struct NegInfVec<TAPOUT_BF16> { static constexpr uint32_t word = 0xff80ff80u; };

template <int DT, int U, bool CHECKED>
__device__ inline void load_batch(u32x4 (&w)[U], const u32x4 *vp, int i, int end)
{
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int idx = i + u * kBlock;
        if (!CHECKED || idx < end) w[u] = __builtin_nontemporal_load(vp + idx);
        else { const uint32_t ni = NegInfVec<DT>::word; w[u] = u32x4{ni, ni, ni, ni}; }   // -inf padding folds to nothing
    }
}

template <int DT, bool FULL, int U>
__device__ inline void fold_batch(ThreadState<FULL> &st, const u32x4 (&w)[U], int i, int head)
{
    constexpr int VEC = Elem<DT>::vec;
    st.template fold_batch<U, VEC>(w, head + i * VEC, kBlock * VEC);
}

// The work of one workgroup: slice `split` of row k of sequence b.
template <int DT, bool FULL>
__device__ inline void stream_pass_body(const RowReduceArgs &a, const int split, const int k, const int b)
{
    constexpr int VEC = Elem<DT>::vec;
    // vectors in flight per thread.  Four is best for both passes: for the draft pass that means 77 registers
    // and six wavefronts per SIMD instead of eight, which still beats two vectors at full occupancy
    // (measured; three, six and eight vectors and an explicit prefetch of the next batch are all slower).
    constexpr int U = kStreamU;
    __shared__ float sh_f[6][kBlock / kWave];
    __shared__ int sh_i[kBlock / kWave];

    const int row = b * a.KK + k;
    const int tid = threadIdx.x;
    int n_active;                                   // rows of sequence b this pass reads
    if (a.len_mode == 0) {                          // draft rows: k < k_len[b]
        n_active = a.len ? a.len[b] : a.KK;
        n_active = n_active > a.KK ? a.KK : (n_active < 0 ? 0 : n_active);
    } else {                                        // target rows: k <= n_draft[b]
        int n = a.len[b];
        n_active = (n < 1 ? 1 : (n > a.KK - 1 ? a.KK - 1 : n)) + 1;
    }
    if (a.clear_jobs && split == 0 && k == 0 && tid == 0) a.clear_jobs[b].band_cnt = 0;
    if (a.arm_dst && split == 0 && k == 0 && tid == 0) a.arm_dst[b] = a.arm_src[b];
    if (k >= n_active) return;
    // The row's token, if it has one.  Requested as a vector load (the index carries a zero the compiler cannot
    // see through): a scalar load from memory would hold up the first wait for the kernel arguments and with it
    // the first logits; this one returns with the first batch.
    int tk = -1;
    if (a.tok && k < a.tok_rows) {                          // target rows, and draft rows when the caller wants log q(tok) early
        int zero;
        asm volatile("v_mov_b32 %0, 0" : "=v"(zero));
        tk = a.tok[(int64_t)b * a.tok_rows + k + zero];
    }
    const char *rowp = (const char *)a.base + ((int64_t)b * a.stride_b + (int64_t)k * a.stride_k) * Elem<DT>::size;
    int head, nvec, tail;
    row_geometry<DT>(rowp, a.V, head, nvec, tail);
    const u32x4 *vp = (const u32x4 *)(rowp + (int64_t)head * Elem<DT>::size);
    // a.per: vectors per slice, chosen on the host as a multiple of 64 (whole 1 KB wavefront loads, so
    // slices of aligned rows start on cache-line boundaries) with nsplit * per >= the vectors of any row
    const int v0 = min(split * a.per, nvec), v1e = min(v0 + a.per, nvec);

    ThreadState<FULL> st;
    // unaligned head (first slice) and tail (last slice): one element per thread
    if (split == 0 && tid < head) st.fold_single(load_elem<DT>(rowp, tid), tid);
    {
        const int nbatch = (v1e - v0 + U * kBlock - 1) / (U * kBlock), nfull = (v1e - v0) / (U * kBlock);
        int i = v0 + tid;
        // A compute unit issues the loads of its oldest wavefront first, so of the eight workgroups that share
        // it the ones dispatched first run ahead and the rest trail by up to a third of the launch; the chip
        // then drains with few loads in flight.  Lowering a wavefront's priority as it gets through its slice
        // keeps the workgroups of a compute unit level (measured: launch 0.6 us shorter for the draft pass).
        const int q1 = nbatch / 4, q2 = nbatch / 2, q3 = (3 * nbatch) / 4;
        __builtin_amdgcn_s_setprio(3);
        for (int bi = 0; bi < nbatch; ++bi, i += U * kBlock) {
            if (bi == q1) __builtin_amdgcn_s_setprio(2);
            if (bi == q2) __builtin_amdgcn_s_setprio(1);
            if (bi == q3) __builtin_amdgcn_s_setprio(0);
            u32x4 w[U];
            if (bi < nfull) load_batch<DT, U, false>(w, vp, i, v1e);      // every vector of the batch lies inside the slice
            else load_batch<DT, U, true>(w, vp, i, v1e);
            fold_batch<DT, FULL, U>(st, w, i, head);
        }
        __builtin_amdgcn_s_setprio(3);      // finish the reduction promptly: the slot is wanted by the next workgroup
    }
    if (split == a.nsplit - 1 && tid < tail) {
        int32_t j = head + nvec * VEC + tid;
        st.fold_single(load_elem<DT>(rowp, j), j);
    }

    // ---- workgroup reduction ----
    const int wave = tid / kWave, lane = tid % kWave;
    float wm = wave_max(st.v1);
    if (lane == 0) sh_f[0][wave] = wm;
    __syncthreads();
    float M = fmaxf(fmaxf(sh_f[0][0], sh_f[0][1]), fmaxf(sh_f[0][2], sh_f[0][3]));
    __syncthreads();
    // bring the thread sums to the workgroup reference (exact scaling), then plain sums
    float Rb = ref_of_max(M);
    float d = Rb - st.R;
    int di = (int)fminf(fmaxf(d, -1.0e9f), 1.0e9f);
    float s = ldexpf(st.s, -di);
    float t = 0.0f, s_hi = 0.0f, t_hi = 0.0f;
    if constexpr (FULL) {
        t = ldexpf(st.t - d * st.s, -di);
        s_hi = ldexpf(st.s_hi, -di);
        t_hi = ldexpf(st.t_hi - d * st.s_hi, -di);
    }
    if (st.v1 == -INFINITY && !(st.s != st.s)) { s = 0.0f; t = 0.0f; s_hi = 0.0f; t_hi = 0.0f; }   // thread saw nothing finite
    float a1 = st.v1, a2 = st.v2;
    if constexpr (FULL) wave_top2(a1, a2);
    // the wavefront's vector with the first maximum; FULL: the thread that met it keeps its set-apart batch out of
    // the wavefront's sums and publishes it on its own (every other thread's set-apart batch is ordinary data)
    const int cw = wave_min_i(st.v1 == M ? st.cand : 0x7fffffff);
    float hs = 0.0f, ht = 0.0f;
    if constexpr (FULL) {
        const bool owner = st.v1 == M && st.cand == cw && cw != 0x7fffffff;
        hs = wave_sum(owner ? s_hi : 0.0f);              // one term and zeros: exact
        ht = wave_sum(owner ? t_hi : 0.0f);
        s += owner ? 0.0f : s_hi;
        t += owner ? 0.0f : t_hi;
    }
    s = wave_sum(s);
    if constexpr (FULL) t = wave_sum(t);
    if (lane == 0) {
        sh_f[0][wave] = s; sh_f[1][wave] = t; sh_f[2][wave] = a1; sh_f[3][wave] = a2; sh_f[4][wave] = hs; sh_f[5][wave] = ht;
        sh_i[wave] = cw;
    }
    __syncthreads();
    if (tid == 0) {
        Partial p;
        p.v1 = M;
        p.S = (sh_f[0][0] + sh_f[0][1]) + (sh_f[0][2] + sh_f[0][3]);
        p.T = (sh_f[1][0] + sh_f[1][1]) + (sh_f[1][2] + sh_f[1][3]);
        float b1 = sh_f[2][0], b2 = sh_f[3][0];
#pragma unroll
        for (int w = 1; w < kBlock / kWave; ++w) top2_merge(b1, b2, sh_f[2][w], sh_f[3][w]);
        p.v2 = b2;
        p.cand = min(min(sh_i[0], sh_i[1]), min(sh_i[2], sh_i[3]));
        if constexpr (FULL) {
            // The batch with the slice's first maximum stays out (the epilogue adds its elements back from the
            // logits); the set-apart batches of the other wavefronts are ordinary data.  A NaN or an infinity
            // inside the left-out batch must still poison the sums: x - x is 0 for finite x only.
            float left_out = 0.0f;
#pragma unroll
            for (int w = 0; w < kBlock / kWave; ++w) {
                const bool holds = sh_i[w] == p.cand;
                p.S += holds ? (sh_f[4][w] - sh_f[4][w]) : sh_f[4][w];
                p.T += holds ? 0.0f : sh_f[5][w];
                left_out = holds ? sh_f[4][w] : left_out;
            }
            // the left-out batch's own sum (same reference): S + this is the slice's sum over every element, to
            // binary32 precision, for a reader that wants the row's lse before the epilogue has run
            p.pad[1] = __float_as_int(left_out);
        }
        p.pad[0] = 0x7fc00000; if constexpr (!FULL) p.pad[1] = 0;
        p.pad[2] = 0;
        // elements of this slice: [e0, e1); every index of the row lies in exactly one slice
        const int e0 = split == 0 ? 0 : head + v0 * VEC, e1 = split == a.nsplit - 1 ? a.V : head + v1e * VEC;
        if (tk >= e0 && tk < e1) {
            // the row's address once more, from scalar registers (the zero is opaque to the compiler): holding the
            // one from the top of the kernel in vector registers through the loop costs the draft pass a wavefront per SIMD
            int zero;
            asm volatile("s_mov_b32 %0, 0" : "=s"(zero));
            const char *rp = (const char *)a.base + ((int64_t)(b + zero) * a.stride_b + (int64_t)k * a.stride_k) * Elem<DT>::size;
            p.pad[0] = __float_as_int(load_elem<DT>(rp, tk));
        }
        a.out[(int64_t)row * a.nsplit + split] = p;
    }
}

// grid = (slice, row of the sequence, sequence): no index arithmetic ahead of the first load.
// At least six wavefronts per SIMD (80 vector registers): the draft pass on bfloat16 sits right at that limit.
template <int DT, bool FULL>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(6))) void stream_pass_kernel(RowReduceArgs a)
{
    warm_args(a);
    stream_pass_body<DT, FULL>(a, blockIdx.x, blockIdx.y, blockIdx.z);
}

// Draft rows and target rows of a round in ONE launch: grid = (slice, row, 2 * sequences), the first half of the
// z range takes the draft tensor, the second half the target tensor (one more row per sequence).  A launch over a
// few hundred rows spends a fifth of its time filling and draining the chip; one launch over both tensors pays
// that once.  Both passes are cut into the same number of slices.
template <int DD, int TD>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(6))) void stream_pair_kernel(RowReduceArgs d, RowReduceArgs t, int n_seq)
{
    warm_args(d, t);
    const int z = blockIdx.z;
    if (z < n_seq) {
        if ((int)blockIdx.y < d.KK && (int)blockIdx.x < d.nsplit) stream_pass_body<DD, true>(d, blockIdx.x, blockIdx.y, z);
    } else {
        if ((int)blockIdx.x < t.nsplit) stream_pass_body<TD, false>(t, blockIdx.x, blockIdx.y, z - n_seq);
    }
}

template <int DT, bool FULL>
hipError_t launch(const RowReduceArgs &a, hipStream_t st, Timing tm)
{
    dim3 grid((unsigned)a.nsplit, (unsigned)a.KK, (unsigned)(a.n_rows / a.KK)), block(kBlock);
    launch_kernel(stream_pass_kernel<DT, FULL>, grid, block, st, tm, a);
    return hipGetLastError();
}

template <int DD, int TD>
hipError_t launch_pair(const RowReduceArgs &d, const RowReduceArgs &t, hipStream_t st, Timing tm)
{
    const int n_seq = t.n_rows / t.KK;
    dim3 grid((unsigned)(d.nsplit > t.nsplit ? d.nsplit : t.nsplit), (unsigned)t.KK, (unsigned)(2 * n_seq)), block(kBlock);
    launch_kernel(stream_pair_kernel<DD, TD>, grid, block, st, tm, d, t, n_seq);
    return hipGetLastError();
}

}  // namespace

// d: the draft tensor ([B, K, V], all statistics), t: the target tensor of the same sequences ([B, K + 1, V]).
hipError_t launch_row_reduce_pair(const RowReduceArgs &d, int d_dtype, const RowReduceArgs &t, int t_dtype, hipStream_t st, Timing tm)
{
    if (d.n_rows / d.KK != t.n_rows / t.KK || d.KK + 1 != t.KK || 2 * (t.n_rows / t.KK) > 65535) return hipErrorInvalidValue;
    if (d_dtype == TAPOUT_F32)
        return t_dtype == TAPOUT_F32 ? launch_pair<TAPOUT_F32, TAPOUT_F32>(d, t, st, tm) : launch_pair<TAPOUT_F32, TAPOUT_BF16>(d, t, st, tm);
    return t_dtype == TAPOUT_F32 ? launch_pair<TAPOUT_BF16, TAPOUT_F32>(d, t, st, tm) : launch_pair<TAPOUT_BF16, TAPOUT_BF16>(d, t, st, tm);
}

hipError_t launch_row_reduce(const RowReduceArgs &a, int dtype, bool full, hipStream_t st, Timing tm)
{
    if (dtype == TAPOUT_F32) return full ? launch<TAPOUT_F32, true>(a, st, tm) : launch<TAPOUT_F32, false>(a, st, tm);
    return full ? launch<TAPOUT_BF16, true>(a, st, tm) : launch<TAPOUT_BF16, false>(a, st, tm);
}

}  // namespace tapout
