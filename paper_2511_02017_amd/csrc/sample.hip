// Final token of Algorithm 1 (line 11): for a sequence rejected at position m
// a draw from normalise(max(0, p_m - q_m)); for a fully accepted draft a draw
// from the next target distribution p_n.  The draw is the inverse CDF at the
// caller's uniform: the smallest j whose inclusive prefix sum exceeds u * Z.
//
// Everything here is double precision.  With ~1e5 CDF boundaries in [0,1) a
// binary32 evaluation would move a boundary across u for about one draw in a
// hundred; in double the chance is ~1e-11, so the token agrees with a
// sequential fp64 evaluation.  Only one row pair per sequence is touched
// (2/(2K+1) of the round's bytes), so the cost stays small.
//
// Three launches, the row pair cut into `nsplit` slices of whole 16-byte vectors:
//   pass 1  slice sums of e_p = exp(t - ref_p), e_q = exp(d - ref_q)   -> normalisers
//   pass 2  slice sums of w = max(0, e_p/S_p - e_q/S_q)  (or e_p/S_p)   -> slice weights
//   pass 3  one workgroup per sequence: scan the slice weights, then a
//           block scan inside the slice that contains u * Z.
#include "common.h"

namespace tapout {

namespace {

constexpr int kSampleBlock = 256;

__device__ inline double wave_sum_d(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

__device__ inline double block_sum_d(double v, double *sh4)
{
    v = wave_sum_d(v);
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) sh4[threadIdx.x / kWave] = v;
    __syncthreads();
    return (sh4[0] + sh4[1]) + (sh4[2] + sh4[3]);
}

// Slices are defined on ELEMENT ranges so that target and draft rows (whose
// alignment and element size may differ) are cut at the same indices.
__device__ inline void slice_range(int V, int nsplit, int split, int &j0, int &j1)
{
    int per = (V + nsplit - 1) / nsplit;
    per = (per + 15) & ~15;                    // multiple of 16 elements
    j0 = min(split * per, V);
    j1 = min(j0 + per, V);
}

struct Weights {
    int kind;          // 1 residual, 2 target only
    double ref_p, ref_q, inv_Sp, inv_Sq;
};

template <int TD, int DD>
__device__ inline double weight_at(const Weights &w, const char *trow, const char *drow, int j)
{
    double p = exp((double)load_elem<TD>(trow, j) - w.ref_p) * w.inv_Sp;
    if (w.kind == 2) return p;
    double q = exp((double)load_elem<DD>(drow, j) - w.ref_q) * w.inv_Sq;
    double r = p - q;
    return r > 0.0 ? r : 0.0;
}

// ---- pass 1: normalisers ----------------------------------------------------
template <int TD, int DD>
__global__ __launch_bounds__(kSampleBlock) void sample_pass1(SampleArgs a)
{
    __shared__ double sh4[4];
    const int b = blockIdx.y, split = blockIdx.x;
    const SampleJob job = a.jobs[b];
    if (job.kind == 0) return;
    const char *trow = (const char *)row_address(a.tbase, TD, a.t_stride_b, a.t_stride_k, b, job.row);
    const char *drow = (const char *)row_address(a.dbase, DD, a.d_stride_b, a.d_stride_k, b, job.kind == 1 ? job.row : 0);
    int j0, j1;
    slice_range(a.V, a.nsplit, split, j0, j1);
    const double ref_p = (double)job.ref_p, ref_q = (double)job.ref_q;
    double sp = 0.0, sq = 0.0;
    for (int j = j0 + threadIdx.x; j < j1; j += kSampleBlock) {
        sp += exp((double)load_elem<TD>(trow, j) - ref_p);
        if (job.kind == 1) sq += exp((double)load_elem<DD>(drow, j) - ref_q);
    }
    sp = block_sum_d(sp, sh4);
    sq = block_sum_d(sq, sh4);
    if (threadIdx.x == 0) {
        a.part1[((int64_t)b * a.nsplit + split) * 2 + 0] = sp;
        a.part1[((int64_t)b * a.nsplit + split) * 2 + 1] = sq;
    }
}

__device__ inline Weights make_weights(const SampleArgs &a, const SampleJob &job, int b, bool *draft_bad)
{
    Weights w;
    double Sp = 0.0, Sq = 0.0;
    for (int s = 0; s < a.nsplit; ++s) {
        Sp += a.part1[((int64_t)b * a.nsplit + s) * 2 + 0];
        Sq += a.part1[((int64_t)b * a.nsplit + s) * 2 + 1];
    }
    w.kind = job.kind;
    w.ref_p = (double)job.ref_p; w.ref_q = (double)job.ref_q;
    w.inv_Sp = 1.0 / Sp;
    w.inv_Sq = 1.0 / Sq;
    *draft_bad = false;
    if (job.kind == 1 && (!(Sq > 0.0) || !(Sq < INFINITY))) {     // NaN / empty draft row: sample from the target row
        w.kind = 2;
        *draft_bad = true;
    }
    return w;
}

// ---- pass 2: slice weights ---------------------------------------------------
template <int TD, int DD>
__global__ __launch_bounds__(kSampleBlock) void sample_pass2(SampleArgs a)
{
    __shared__ double sh4[4];
    const int b = blockIdx.y, split = blockIdx.x;
    const SampleJob job = a.jobs[b];
    if (job.kind == 0) return;
    const char *trow = (const char *)row_address(a.tbase, TD, a.t_stride_b, a.t_stride_k, b, job.row);
    const char *drow = (const char *)row_address(a.dbase, DD, a.d_stride_b, a.d_stride_k, b, job.kind == 1 ? job.row : 0);
    bool draft_bad;
    const Weights w = make_weights(a, job, b, &draft_bad);
    int j0, j1;
    slice_range(a.V, a.nsplit, split, j0, j1);
    double z = 0.0;
    for (int j = j0 + threadIdx.x; j < j1; j += kSampleBlock)
        z += weight_at<TD, DD>(w, trow, drow, j);
    z = block_sum_d(z, sh4);
    if (threadIdx.x == 0) a.part2[(int64_t)b * a.nsplit + split] = z;
}

// ---- pass 3: locate ----------------------------------------------------------
// Inclusive scan over the workgroup of one double per thread; returns the
// exclusive prefix of this thread and the total through *total.
__device__ inline double block_excl_scan_d(double v, double *sh_w, double *total)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    double inc = v;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        double up = __shfl_up(inc, o, kWave);
        if (lane >= o) inc += up;
    }
    __syncthreads();
    if (lane == kWave - 1) sh_w[wave] = inc;
    __syncthreads();
    double base = 0.0;
    for (int w2 = 0; w2 < wave; ++w2) base += sh_w[w2];
    *total = ((sh_w[0] + sh_w[1]) + sh_w[2]) + sh_w[3];
    return base + (inc - v);
}

// Locate the first j in [j0, j1) whose running sum (starting from `cum`)
// exceeds `target`; -1 if the slice ends first.  *last_pos tracks the largest
// j with positive weight seen by the workgroup.
template <int TD, int DD>
__device__ inline int locate_in_slice(const Weights &w, const char *trow, const char *drow, int j0, int j1,
                                      double cum, double target, double *sh_w, int *sh_hit, int *last_pos)
{
    constexpr int PER = 4;                                  // consecutive elements per thread and tile
    for (int base = j0; base < j1; base += kSampleBlock * PER) {
        const int jt = base + threadIdx.x * PER;
        double wv[PER], sum = 0.0;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            wv[i] = (jt + i < j1) ? weight_at<TD, DD>(w, trow, drow, jt + i) : 0.0;
            sum += wv[i];
        }
        double tile_total;
        double excl = block_excl_scan_d(sum, sh_w, &tile_total);
        if (threadIdx.x == 0) *sh_hit = 0x7fffffff;
        __syncthreads();
        double c = cum + excl;
        int hit = 0x7fffffff, lp = -1;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            c += wv[i];
            if (wv[i] > 0.0) lp = jt + i;
            if (hit == 0x7fffffff && jt + i < j1 && c > target) hit = jt + i;
        }
        if (hit != 0x7fffffff) atomicMin(sh_hit, hit);
        if (lp >= 0) atomicMax(last_pos, lp);
        __syncthreads();
        int h = *sh_hit;
        __syncthreads();
        if (h != 0x7fffffff) return h;
        cum += tile_total;
    }
    return -1;
}

template <int TD, int DD>
__global__ __launch_bounds__(kSampleBlock) void sample_pass3(SampleArgs a)
{
    __shared__ double sh_w[4];
    __shared__ int sh_hit, sh_last;
    const int b = blockIdx.x;
    const SampleJob job = a.jobs[b];
    if (job.kind == 0) return;
    const char *trow = (const char *)row_address(a.tbase, TD, a.t_stride_b, a.t_stride_k, b, job.row);
    const char *drow = (const char *)row_address(a.dbase, DD, a.d_stride_b, a.d_stride_k, b, job.kind == 1 ? job.row : 0);
    bool draft_bad;
    Weights w = make_weights(a, job, b, &draft_bad);
    if (threadIdx.x == 0) sh_last = -1;
    __syncthreads();
    double Z = 0.0;
    for (int s = 0; s < a.nsplit; ++s) Z += a.part2[(int64_t)b * a.nsplit + s];
    const double u = (double)a.u_sample[b];
    int token = -1;
    if (Z > 0.0) {
        const double target = u * Z;
        double cum = 0.0;
        int s = 0;
        for (; s < a.nsplit; ++s) {
            double nx = cum + a.part2[(int64_t)b * a.nsplit + s];
            if (nx > target) break;
            cum = nx;
        }
        // slice sums and the in-slice scan round differently: if the crossing is not
        // found inside slice s, continue into the following slices
        for (; s < a.nsplit && token < 0; ++s) {
            int j0, j1;
            slice_range(a.V, a.nsplit, s, j0, j1);
            token = locate_in_slice<TD, DD>(w, trow, drow, j0, j1, cum, target, sh_w, &sh_hit, &sh_last);
            cum += a.part2[(int64_t)b * a.nsplit + s];
        }
        if (token < 0) {
            // rounding left no crossing: the largest index with positive weight
            __syncthreads();
            if (sh_last < 0) {
                for (int s2 = 0; s2 < a.nsplit; ++s2) {
                    int j0, j1;
                    slice_range(a.V, a.nsplit, s2, j0, j1);
                    locate_in_slice<TD, DD>(w, trow, drow, j0, j1, 0.0, INFINITY, sh_w, &sh_hit, &sh_last);
                }
                __syncthreads();
            }
            token = sh_last;
        }
    } else if (w.kind == 1) {
        // the residual vanished (p == q up to rounding): draw from the target row itself
        w.kind = 2;
        double z = 0.0;
        for (int j = threadIdx.x; j < a.V; j += kSampleBlock) z += weight_at<TD, DD>(w, trow, drow, j);
        const double Zp = block_sum_d(z, sh_w);
        __syncthreads();
        if (Zp > 0.0)
            token = locate_in_slice<TD, DD>(w, trow, drow, 0, a.V, 0.0, u * Zp, sh_w, &sh_hit, &sh_last);
        if (token < 0) { __syncthreads(); token = sh_last; }
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
hipError_t launch_typed(const SampleArgs &a, int pass, hipStream_t st)
{
    dim3 grid12(a.nsplit, a.B), block(kSampleBlock);
    if (pass == 1) hipLaunchKernelGGL((sample_pass1<TD, DD>), grid12, block, 0, st, a);
    else if (pass == 2) hipLaunchKernelGGL((sample_pass2<TD, DD>), grid12, block, 0, st, a);
    else hipLaunchKernelGGL((sample_pass3<TD, DD>), dim3(a.B), block, 0, st, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_sample(const SampleArgs &a, int pass, hipStream_t st)
{
    if (a.t_dtype == TAPOUT_F32)
        return a.d_dtype == TAPOUT_F32 ? launch_typed<TAPOUT_F32, TAPOUT_F32>(a, pass, st) : launch_typed<TAPOUT_F32, TAPOUT_BF16>(a, pass, st);
    return a.d_dtype == TAPOUT_F32 ? launch_typed<TAPOUT_BF16, TAPOUT_F32>(a, pass, st) : launch_typed<TAPOUT_BF16, TAPOUT_BF16>(a, pass, st);
}

}  // namespace tapout
