// Streaming reduction of logits rows: the one pass over the vocabulary that
// feeds every signal of Table 1 / Appendix A.1 (entropy, top-1 probability,
// top-1/top-2 margin) and the normalisers the verification step needs.
//
// One launch covers all rows of a [B, KK, V] tensor.  A row is cut into
// `nsplit` slices of whole 16-byte vectors; one 256-thread workgroup reduces
// one slice to a 32-byte Partial.  Every element is loaded exactly once, with
// 16-byte loads that are contiguous across the wavefront.
//
// Per thread the softmax sums are kept online in the base-2 domain against an
// integer reference R = ceil(max * log2 e): y = fma(x, log2e, -R) has a single
// rounding, 2^y comes from the hardware exp2, and moving to a larger reference
// is an exact ldexp.  Top-2 values are tracked with max3 / med3 on pairs
// (second largest of {v1, a, b, v2} = max(med3(v1, a, b), v2) while v2 <= v1).
// Only the 16-byte window in which the thread's maximum first appeared is
// remembered; the exact argmax index is recovered later from that window.
#include "common.h"

namespace tapout {

namespace {

__device__ inline float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

// Headroom (in powers of two) added to a thread's reference when it has to be
// raised, so that a slowly growing running maximum raises it only a few times.
constexpr float kHeadroom = 8.0f;

template <bool FULL>
struct ThreadState {
    float v1 = -INFINITY;   // running maximum
    float v2 = -INFINITY;   // running second largest (FULL only)
    float R = 0.0f;         // integer reference: every x seen so far has x*log2e <= R (+ rounding)
    float xlim = -INFINITY; // largest x the current reference covers
    float s = 0.0f;         // sum 2^(x*log2e - R)
    float t = 0.0f;         // sum 2^y * y (FULL only)
    int32_t cand = 0x7fffffff;

    // Fold N values that start at element index `first` of the row; `first` is
    // remembered as the argmax candidate when the running maximum grows.
    template <int N>
    __device__ inline void fold(const float (&x)[N], int32_t first)
    {
        float old = v1;
        if constexpr (N == 1) {
            if constexpr (FULL) v2 = fmaxf(v2, fminf(v1, x[0]));
            v1 = fmaxf(v1, x[0]);
        } else {
#pragma unroll
            for (int i = 0; i < N; i += 2) {
                if constexpr (FULL) v2 = fmaxf(v2, __builtin_amdgcn_fmed3f(v1, x[i], x[i + 1]));
                v1 = max3(v1, x[i], x[i + 1]);
            }
        }
        cand = v1 > old ? first : cand;
        if (v1 > xlim) {                      // rare after the first few vectors
            float Rn = ceilf(v1 * kLog2e) + kHeadroom;
            float d = Rn - R;
            int di = (int)fminf(fmaxf(d, -1.0e9f), 1.0e9f);
            if constexpr (FULL) t = ldexpf(t - d * s, -di);
            s = ldexpf(s, -di);
            R = Rn;
            xlim = Rn * (1.0f / kLog2e);
        }
#pragma unroll
        for (int i = 0; i < N; ++i) {
            float y = __builtin_fmaf(x[i], kLog2e, -R);
            float e = __builtin_amdgcn_exp2f(y);
            s += e;
            if constexpr (FULL) t = __builtin_fmaf(e, fmaxf(y, -200.0f), t);   // clamp keeps 0 * -inf out of T for masked (-inf) logits
        }
    }
};

__device__ inline float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}
__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ inline int wave_min_i(int v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o, kWave));
    return v;
}
// second largest of the union of two (largest, second) pairs, duplicates counted
__device__ inline void wave_top2(float &a1, float &a2)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        float b1 = __shfl_xor(a1, o, kWave), b2 = __shfl_xor(a2, o, kWave);
        a2 = max3(fminf(a1, b1), a2, b2);
        a1 = fmaxf(a1, b1);
    }
}

template <int DT, bool FULL>
__global__ __launch_bounds__(kBlock) void row_reduce_kernel(RowReduceArgs a)
{
    constexpr int VEC = Elem<DT>::vec;
    constexpr int UNROLL = 4;
    const int split = blockIdx.x % a.nsplit;
    const int row = blockIdx.x / a.nsplit;
    const int b = row / a.KK, k = row % a.KK;
    if (a.len_mode == 0) {
        if (a.len && k >= a.len[b]) return;
    } else {
        int n = a.len[b];
        n = n < 1 ? 1 : (n > a.KK - 1 ? a.KK - 1 : n);
        if (k > n) return;
    }
    const char *rowp = (const char *)a.base + ((int64_t)b * a.stride_b + (int64_t)k * a.stride_k) * Elem<DT>::size;
    int head, nvec, tail;
    row_geometry<DT>(rowp, a.V, head, nvec, tail);
    const u32x4 *vp = (const u32x4 *)(rowp + (int64_t)head * Elem<DT>::size);
    const int per = (nvec + a.nsplit - 1) / a.nsplit;
    const int v0 = min(split * per, nvec), v1e = min(v0 + per, nvec);
    const int tid = threadIdx.x;

    ThreadState<FULL> st;
    // unaligned head (first slice) and tail (last slice): one element per thread
    if (split == 0 && tid < head) {
        float x[1] = { load_elem<DT>(rowp, tid) };
        st.template fold<1>(x, tid);
    }
    int i = v0 + tid;
    for (; i + (UNROLL - 1) * kBlock < v1e; i += UNROLL * kBlock) {
        u32x4 w[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) w[u] = __builtin_nontemporal_load(vp + i + u * kBlock);
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            float x[VEC];
            unpack<DT>(w[u], x);
            st.template fold<VEC>(x, head + (i + u * kBlock) * VEC);
        }
    }
    for (; i < v1e; i += kBlock) {
        u32x4 w = __builtin_nontemporal_load(vp + i);
        float x[VEC];
        unpack<DT>(w, x);
        st.template fold<VEC>(x, head + i * VEC);
    }
    if (split == a.nsplit - 1 && tid < tail) {
        int32_t j = head + nvec * VEC + tid;
        float x[1] = { load_elem<DT>(rowp, j) };
        st.template fold<1>(x, j);
    }

    // ---- workgroup reduction ----
    __shared__ float sh_f[4][kBlock / kWave];
    __shared__ int sh_i[kBlock / kWave];
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
    float t = 0.0f;
    if constexpr (FULL) t = ldexpf(st.t - d * st.s, -di);
    if (st.v1 == -INFINITY && !(st.s != st.s)) { s = 0.0f; t = 0.0f; }   // thread saw nothing finite
    s = wave_sum(s);
    if constexpr (FULL) t = wave_sum(t);
    float a1 = st.v1, a2 = st.v2;
    if constexpr (FULL) wave_top2(a1, a2);
    int c = wave_min_i(st.v1 == M ? st.cand : 0x7fffffff);
    if (lane == 0) { sh_f[0][wave] = s; sh_f[1][wave] = t; sh_f[2][wave] = a1; sh_f[3][wave] = a2; sh_i[wave] = c; }
    __syncthreads();
    if (tid == 0) {
        Partial p;
        p.v1 = M;
        p.S = (sh_f[0][0] + sh_f[0][1]) + (sh_f[0][2] + sh_f[0][3]);
        p.T = (sh_f[1][0] + sh_f[1][1]) + (sh_f[1][2] + sh_f[1][3]);
        float b1 = sh_f[2][0], b2 = sh_f[3][0];
#pragma unroll
        for (int w = 1; w < kBlock / kWave; ++w) {
            b2 = max3(fminf(b1, sh_f[2][w]), b2, sh_f[3][w]);
            b1 = fmaxf(b1, sh_f[2][w]);
        }
        p.v2 = b2;
        p.cand = min(min(sh_i[0], sh_i[1]), min(sh_i[2], sh_i[3]));
        p.pad[0] = p.pad[1] = p.pad[2] = 0;
        a.out[(int64_t)row * a.nsplit + split] = p;
    }
}

}  // namespace

hipError_t launch_row_reduce(const RowReduceArgs &a, int dtype, bool full, hipStream_t st)
{
    dim3 grid((unsigned)((int64_t)a.n_rows * a.nsplit)), block(kBlock);
    if (dtype == TAPOUT_F32) {
        if (full) hipLaunchKernelGGL((row_reduce_kernel<TAPOUT_F32, true>), grid, block, 0, st, a);
        else      hipLaunchKernelGGL((row_reduce_kernel<TAPOUT_F32, false>), grid, block, 0, st, a);
    } else {
        if (full) hipLaunchKernelGGL((row_reduce_kernel<TAPOUT_BF16, true>), grid, block, 0, st, a);
        else      hipLaunchKernelGGL((row_reduce_kernel<TAPOUT_BF16, false>), grid, block, 0, st, a);
    }
    return hipGetLastError();
}

}  // namespace tapout
