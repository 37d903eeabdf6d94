"""Shared helpers of the GPU parity tests: run one round through libtapout and
through the CPU oracle on the same tensors and compare element by element.

Tolerances (written here once, used by every parity test):
  statistics   |gpu - ref| <= TAU * max(|ref|, floor), TAU = 1e-5 for binary32 and
               for bfloat16 logits alike (bfloat16 widens exactly, so the looser
               2e-2 the target statement allows for bfloat16 is not needed).
               floor = 1e-3 for probabilities.
               floor = 1 for log-domain values (lse, log p(tok), log q(tok)): an
               absolute error of a log-probability IS the relative error of the
               probability.
               floor = 1e-3 for entropy and margin as well: the library keeps
               the row maximum's term out of its binary32 sums (it enters as an
               exact double term at the end), so the entropy of a peaked row and
               a margin between near-tied probabilities keep binary32 relative
               precision down to values far below any threshold a stop rule
               compares against (test_peaked_rows_keep_relative_precision
               measures it).
  integers     top-1 ids, stop positions, accepted lengths, emitted tokens are
               bit-exact, except where the ORACLE marks the deciding comparison
               as a near tie: a stop signal within TAU (relative) of its
               threshold, an acceptance uniform within TAU (relative) of
               min(1, p/q), an inverse-CDF target within TAU_S = 1e-9 of a cell
               edge.  Such sequences are counted, not compared.
"""
import numpy as np
import torch

from oracle import oracle as orc

TAU = 1e-5
TAU_S = 1e-9
STAT_KEYS = ("lse", "entropy", "p_top1", "p_top2", "margin", "logq_tok")


def to_host(t):
    return None if t is None else t.detach().cpu()


def host_logits(t):
    return orc.as_logits(t.detach().cpu().contiguous()) if t.is_cuda or not t.is_contiguous() else orc.as_logits(t)


LOG_KEYS = ("lse", "logq_tok", "target_lse", "logp_tok")


def assert_stats_close(name, gpu, ref, mask=None, tau=TAU):
    gpu = np.asarray(gpu, np.float64)
    ref = np.asarray(ref, np.float64)
    if mask is not None:
        gpu, ref = gpu[mask], ref[mask]
    floor = 1.0 if name in LOG_KEYS else 1e-3
    both_nan = np.isnan(gpu) & np.isnan(ref)
    same_inf = np.isinf(ref) & (gpu == ref)
    with np.errstate(invalid="ignore"):
        err = np.abs(gpu - ref)                              # inf - inf: covered by same_inf
    scale = np.maximum(np.abs(ref), floor)
    bad = ~both_nan & ~same_inf & ~(err <= tau * scale)
    assert not bad.any(), (f"{name}: {bad.sum()} of {bad.size} outside tolerance; worst "
                           f"{np.nanmax(np.where(bad, err / scale, 0)):.3e} x scale; first at {np.argwhere(bad)[0]}"
                           f" gpu={gpu[bad][0]!r} ref={ref[bad][0]!r}")


def oracle_round(rnd, arm=None, n_draft=None, rules=(0, 1, 2), thresholds=(0.6, 0.8, 0.2), nthreads=16, seqs=None,
                 prev_entropy=None, lam=None, adaedl_gamma=0.5):
    """Oracle on host copies of a round.  seqs: optional index list (subset of sequences).
    prev_entropy / lam / adaedl_gamma: carried state of the stateful stop rules (oracle.RuleState)."""
    pick = (lambda t: t) if seqs is None else (lambda t: t[seqs])
    draft = host_logits(pick(rnd["draft"]))
    target = host_logits(pick(rnd["target"]))
    tok = pick(rnd["draft_tok"]).cpu().numpy()
    k_len = pick(rnd["k_len"]).cpu().numpy()
    greedy = pick(rnd["greedy"]).cpu().numpy()
    arm_h = None if arm is None else pick(arm).cpu().numpy()
    ds = orc.draft_stats(draft, draft_tok=tok, k_len=k_len, arm=arm_h, rules=rules, thresholds=thresholds, nthreads=nthreads,
                         prev_entropy=prev_entropy, lam=lam, adaedl_gamma=adaedl_gamma)
    if n_draft is None:
        nd = ds["n_stop"] if arm is not None else k_len
    else:
        nd = pick(n_draft).cpu().numpy()
    vf = orc.verify(target, draft, ds["logq_tok"], tok, nd, pick(rnd["u_accept"]).cpu().numpy(),
                    pick(rnd["u_sample"]).cpu().numpy(), greedy=greedy, nthreads=nthreads)
    return ds, vf, nd


def gpu_round(tp, rnd, arm=None, n_draft=None):
    """libtapout on a round: draft_stats then verify (n_draft = n_stop when an arm is given, else k_len)."""
    ds = tp.draft_stats(rnd["draft"], draft_tok=rnd["draft_tok"], k_len=rnd["k_len"], arm=arm)
    if n_draft is None:
        n_draft = ds["n_stop"] if arm is not None else rnd["k_len"]
    vf = tp.verify(rnd["target"], rnd["draft"], ds["lse"], ds["logq_tok"], rnd["draft_tok"], n_draft,
                   rnd["u_accept"], rnd["u_sample"], greedy=rnd["greedy"])
    torch.cuda.synchronize()
    return ds, vf, n_draft


def check_round_call(tp, rnd, arm, truncate, rules=(0, 1, 2), thresholds=(0.6, 0.8, 0.2)):
    """One tapout_round call (the arms in `arm` are played; the call leaves the next round's there) against the oracle.
    truncate: n_draft = this round's stop position, else n_draft = k_len."""
    arm_played = arm.clone()
    launch, outs = tp.prepare_round_call(rnd, arm, truncate)
    launch(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    ods, ovf, o_nd = oracle_round(rnd, arm=arm_played, n_draft=None if truncate else rnd["k_len"], rules=rules, thresholds=thresholds)
    gvf = dict(outs["verify"])
    gvf["n_draft_used"] = outs["n_draft"]
    return compare_round(outs["draft"], gvf, ods, ovf, rnd["k_len"].cpu().numpy(), o_nd)


def compare_round(gds, gvf, ods, ovf, k_len, n_draft_ref, seqs=None, check_stop=True):
    """Element-by-element comparison; returns counts of near-tie (flagged) decisions."""
    pick = (lambda t: t.cpu().numpy()) if seqs is None else (lambda t: t[seqs].cpu().numpy())
    k_len = np.asarray(k_len)
    B, K = ods["lse"].shape
    live = np.arange(K)[None, :] < k_len[:, None]
    for key in STAT_KEYS:
        assert_stats_close(key, pick(gds[key]), ods[key], live)
    g_top1 = pick(gds["top1_id"])
    assert (g_top1[live] == ods["top1_id"][live]).all(), "top1_id differs"
    assert (pick(gds["flags"]).astype(np.uint32) == ods["flags"]).all(), "draft flags differ"
    counts = dict(stop_flagged=0, accept_flagged=0, icdf_flagged=0, sequences=B)
    stop_ok = np.ones(B, bool)
    if check_stop and ods["n_stop"] is not None:
        near = (ods["stop_margin"] <= TAU) & live
        stop_ok = ~near.any(1)
        counts["stop_flagged"] = int((~stop_ok).sum())
        g_ns = pick(gds["n_stop"])
        assert (g_ns[stop_ok] == ods["n_stop"][stop_ok]).all(), "n_stop differs on an unflagged sequence"
        g_sf = pick(gds["stop_fired"])
        assert (g_sf[live & ~near] == ods["stop_fired"][live & ~near]).all(), "stop_fired differs away from the threshold"
    # verification: sequences whose inputs (n_draft) already differ are skipped, they were flagged above
    same_n = pick(gvf["n_draft_used"]) == n_draft_ref if "n_draft_used" in gvf else np.ones(B, bool)
    used = np.arange(K)[None, :] < np.asarray(n_draft_ref)[:, None]
    near_acc = ((ovf["accept_margin"] <= TAU) & used).any(1)
    near_icdf = ovf["icdf_margin"] <= TAU_S
    counts["accept_flagged"] = int(near_acc.sum())
    counts["icdf_flagged"] = int(near_icdf.sum())
    ok = stop_ok & same_n & ~near_acc
    g_len, g_out, g_nout = pick(gvf["accept_len"]), pick(gvf["out_tok"]), pick(gvf["n_out"])
    assert (g_len[ok] == ovf["accept_len"][ok]).all(), \
        f"accept_len differs on unflagged sequences {np.nonzero(ok & (g_len != ovf['accept_len']))[0][:8]}"
    assert (g_nout[ok] == ovf["n_out"][ok]).all()
    ok_tok = ok & ~near_icdf
    bad = ok_tok & (g_out != ovf["out_tok"]).any(1)
    assert not bad.any(), f"out_tok differs on unflagged sequences {np.nonzero(bad)[0][:8]}: " \
                          f"gpu {g_out[bad][0]} ref {ovf['out_tok'][bad][0]}"
    # emitted prefixes agree even where the final draw was a near tie
    pre = np.arange(K + 1)[None, :] < ovf["accept_len"][:, None]
    assert (g_out[ok][pre[ok]] == ovf["out_tok"][ok][pre[ok]]).all()
    rows = np.arange(K + 1)[None, :] <= np.asarray(n_draft_ref)[:, None]
    sel = ok[:, None] & rows
    assert_stats_close("target_lse", pick(gvf["target_lse"]), ovf["target_lse"], sel)
    assert (pick(gvf["target_top1"])[sel] == ovf["target_top1"][sel]).all(), "target_top1 differs"
    sampled_ok = ok[:, None] & used
    assert_stats_close("logp_tok", pick(gvf["logp_tok"]), ovf["logp_tok"], sampled_ok)
    assert (pick(gvf["flags"]).astype(np.uint32)[ok] == ovf["flags"][ok]).all(), "verify flags differ"
    return counts


def check_round(tp, rnd, arm=None, seqs=None, rules=(0, 1, 2), thresholds=(0.6, 0.8, 0.2)):
    """Run both sides on a round and compare.  With `arm`, n_draft = n_stop (Algorithm 1 truncation);
    the oracle then verifies with ITS n_stop and sequences whose stop decision was a near tie are skipped."""
    gds, gvf, g_nd = gpu_round(tp, rnd, arm=arm)
    ods, ovf, o_nd = oracle_round(rnd, arm=arm, rules=rules, thresholds=thresholds, seqs=seqs)
    gvf = dict(gvf)
    gvf["n_draft_used"] = g_nd
    k_len = rnd["k_len"].cpu().numpy() if seqs is None else rnd["k_len"][seqs].cpu().numpy()
    return compare_round(gds, gvf, ods, ovf, k_len, o_nd, seqs=seqs)
