// Per-sequence epilogue of the draft pass: merges the slice partials of every
// draft row into the signals of Table 1 / Appendix A.1 (entropy, top-1
// probability, top-1/top-2 margin, lse, log q(tok)) and runs the stop scan of
// Algorithm 1's draft loop: the token drafted at the step where the selected
// rule fires is kept, so n_stop = first firing k + 1.
//
// The partials of the draft pass leave out the batch of vectors in which each
// slice met its first maximum (row_reduce.hip): every (row, slice) piece first
// gets the elements of that batch back from the logits, except the first
// maximum itself, which enters the row's sums at the end as an exact double
// term.  That is what keeps the entropy of a peaked row (a small number made
// of small terms) accurate to binary32 relative precision.
//
// One workgroup per sequence, one thread per row.  The kernel is latency bound
// (O(K * nsplit) work), so it is written to keep dependent memory round trips
// few: the partials are requested by all threads at once, the token gather and
// the left-out batches travel together in a second round trip, and every row decides "fires / does not fire" for itself so that
// the sequential part is a scan over bytes in LDS.  The two rules that look at
// more than the current row's signals (SVIP-Difference: previous row's entropy;
// AdaEDL: the sequence's adaptive threshold) decide in a second sweep, after all
// entropies of the sequence are in LDS.
#include "finalize_device.h"

namespace tapout {

namespace {

template <bool SHARDED>
__global__ __launch_bounds__(kFinalBlock) void draft_finalize_kernel(DraftFinalArgs a)
{
    warm_args(a);
    draft_finalize_body<SHARDED>(a, blockIdx.x);
}

// ---- vocabulary shards -----------------------------------------------------------------------
// One thread per row of the shard: merges the row's slice partials (a few dozen bytes, straight from memory)
// into one record with the exact global argmax and, if this shard owns it, the logit of the drafted token.
__global__ __launch_bounds__(kFinalBlock) void shard_merge_kernel(ShardMergeArgs a)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= a.B * a.KK) return;
    const int b = i / a.KK, k = i - b * a.KK;
    int n_live;
    if (a.rows_mode == 0) {
        n_live = a.len ? a.len[b] : a.KK;
        n_live = n_live > a.KK ? a.KK : n_live;
    } else {
        const int n = a.len[b];
        n_live = (n < 1 ? 1 : (n > a.KK - 1 ? a.KK - 1 : n)) + 1;
    }
    if (k >= n_live) return;
    const void *row = row_address(a.base, a.dtype, a.stride_b, a.stride_k, b, k);
    // every slice partial gets its left-out batch back (all but the first maximum), then the slices are merged; the
    // record leaves the row slice's first maximum out of its two sums
    Piece acc = empty_piece();
    for (int sl = 0; sl < a.nsplit; ++sl) {
        Piece e = piece_from_partial(a.part[(int64_t)i * a.nsplit + sl]);
        const BatchRegs bt = batch_issue(row, a.dtype, a.Vs, e.idx, sl, a.per, a.part);
        batch_fix(e, bt, a.dtype);
        acc = merge_pair<true>(acc, e);
    }
    Partial o;
    o.v1 = acc.M; o.S = (float)acc.S; o.T = (float)acc.T; o.v2 = acc.v2;
    o.cand = a.vocab_offset + ((acc.idx >= 0 && acc.idx < a.Vs) ? acc.idx : 0);
    float xt = NAN;
    const int KT = a.KK - a.rows_mode;                       // tokens per sequence (the last target row has none)
    if (a.tok && k < KT) {
        const int t = a.tok[(int64_t)b * KT + k] - a.vocab_offset;
        if (t >= 0 && t < a.Vs) xt = load_elem_rt(row, a.dtype, t);
    }
    o.pad[0] = __float_as_int(xt); o.pad[1] = o.pad[2] = 0;
    a.out[i] = o;
}

}  // namespace

hipError_t launch_draft_finalize(const DraftFinalArgs &a, hipStream_t st, Timing tm)
{
    if (a.shards > 0) launch_kernel(draft_finalize_kernel<true>, dim3(a.B), dim3(kFinalBlock), st, tm, a);
    else launch_kernel(draft_finalize_kernel<false>, dim3(a.B), dim3(kFinalBlock), st, tm, a);
    return hipGetLastError();
}

hipError_t launch_shard_merge(const ShardMergeArgs &a, hipStream_t st, Timing tm)
{
    const int n = a.B * a.KK;
    launch_kernel(shard_merge_kernel, dim3((n + kFinalBlock - 1) / kFinalBlock), dim3(kFinalBlock), st, tm, a);
    return hipGetLastError();
}

}  // namespace tapout
