#!/usr/bin/env python3
"""Benchmark of the TapOut logits path on one MI355X.

One "step" is one decode round of the whole hot path over one batch of
synthetic logits already resident in HBM:
    tapout_bandit_select -> tapout_draft_stats -> tapout_verify -> tapout_bandit_update
The headline workload is the Llama-3-vocabulary configuration (V = 128256,
B = 64, K = 8, bfloat16) on which the metric (verified draft tokens/s at a 128k
vocabulary) is quoted.  Inputs rotate through a ring of pre-generated rounds
larger than the 256 MB Infinity Cache, so no step finds its logits cached.

Prints ONE JSON line.
  value                 drafted tokens handed to verification (sum of n_draft over the timed steps) per second of
                        wall time; a step is one tapout_round call (the whole round; four_calls gives the same steps as
                        the four separate calls); the timed region carries no instrumentation at all
  roofline*             after the timed region the same steps run again as four calls, kernel by kernel, with an event
                        pair on every launch (at least 32 steps whatever --steps is): algorithmic bytes per launch over the
                        kernel's average duration against the 8 TB/s HBM peak; then once more as tapout_round calls.
                        roofline = the launch with the most bytes of the timed region (tapout_round's one streaming
                        launch over draft and target rows; the target pass where the round does not pair them),
                        roofline_target_reduce / roofline_draft_reduce = the two passes as launches of their own,
                        roofline_streaming = both weighted by their bytes, roofline_final_token = the final-token
                        slice pass
  roofline_zipf/_ragged the other two configurations with V >= 128k, timed the same way in the same run (no CPU leg)
  parity                decisions of a round of each timed configuration against the CPU oracle: near ties the oracle
                        flags, and mismatches outside them (must be 0)
  cpu_baseline          the CPU oracle on whole rounds of the headline workload
"""
import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
TAU, TAU_S = 1e-5, 1e-9        # near-tie margins of the oracle's decision flags (relative; inverse-CDF cell edges)
METRIC = "verified draft tokens/sec and achieved HBM GB/s (% of peak) at vocab 128k"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="llama3", choices=["tiny", "small", "llama3", "zipf", "ragged"])
    ap.add_argument("--mode", default="full", choices=["full", "truncate"],
                    help="full: verify all K drafted tokens (stop signals still computed); truncate: verify up to the stop position")
    ap.add_argument("--arms", default="three", choices=["three", "five"],
                    help="three: SVIP / Max-Confidence / LogitMargin (the default pool); five: plus SVIPDifference and AdaEDL (Table 1)")
    ap.add_argument("--policy", default=None, choices=["ucb1", "ts", "ucb_tuned", "ts_gauss"], help="bandit policy (default: the workload's)")
    ap.add_argument("--sample-draft", action="store_true",
                    help="let tapout_draft_stats draw the draft tokens (inverse CDF at caller uniforms) instead of reading them")
    ap.add_argument("--ring", type=int, default=0, help="pre-generated rounds to rotate through (0: enough for > 1 GB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="wall-time budget of the CPU-oracle leg")
    ap.add_argument("--kernel-steps", type=int, default=0,
                    help="steps of the instrumented loop behind the roofline figures (0: max(32, min(steps, 200)))")
    ap.add_argument("--opt", action="append", default=[], help="library tuning option name=value")
    ap.add_argument("--no-read-reference", action="store_true", help="skip the plain PyTorch row-sum reference")
    ap.add_argument("--no-extra-workloads", action="store_true", help="headline workload only: no roofline_zipf / roofline_ragged")
    ap.add_argument("--no-parity", action="store_true", help="skip the per-configuration decision check against the oracle")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run 8 plain device copies of 512 MiB (torch copy_): a kernel of known traffic that scales "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    return ap.parse_args()


def kernel_names(w, torch):
    return {"target_pass": f"stream_pass_kernel<{1 if w.target_dtype == torch.bfloat16 else 0}, false>",
            "draft_pass": f"stream_pass_kernel<{1 if w.draft_dtype == torch.bfloat16 else 0}, true>",
            "verify_slices": "verify_slices"}


def committed_traffic(w, kernel_name):
    """HBM bytes per launch (FETCH_SIZE + WRITE_SIZE, copy-kernel calibrated) from the committed rocprofv3 --pmc summary
    of the same workload: not measured in this run."""
    path = os.path.join(ROOT, "profiles", f"stream_pass_{w.name}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    total, seen = 0.0, 0
    for line in open(path):
        if kernel_name in line and "MB per launch" in line:
            total += float(line.split("->")[1].split("MB per launch")[0]) * 1e6
            seen += 1
    return int(total) if seen == 2 else None


def decision_parity(torch, w, rnd, arm, gds, gvf, n_draft, rules, thresholds):
    """The integer decisions of one round against the CPU oracle on host copies of the same tensors.  Returns counts:
    near ties the oracle flags (stop signal within TAU of its threshold, acceptance uniform within TAU of p/q,
    inverse-CDF target within TAU_S of a cell edge) and mismatches outside them."""
    import numpy as np
    from oracle import oracle as orc
    K = w.K
    host = lambda t: orc.as_logits(t.detach().cpu().contiguous())
    tok, k_len = rnd["draft_tok"].cpu().numpy(), rnd["k_len"].cpu().numpy()
    nd = n_draft.cpu().numpy()
    ods = orc.draft_stats(host(rnd["draft"]), draft_tok=tok, k_len=k_len, arm=arm.cpu().numpy(), rules=rules, thresholds=thresholds, nthreads=16)
    ovf = orc.verify(host(rnd["target"]), host(rnd["draft"]), ods["logq_tok"], tok, nd, rnd["u_accept"].cpu().numpy(),
                     rnd["u_sample"].cpu().numpy(), greedy=rnd["greedy"].cpu().numpy(), nthreads=16)
    live = np.arange(K)[None, :] < k_len[:, None]
    used = np.arange(K)[None, :] < nd[:, None]
    stop_f = ((ods["stop_margin"] <= TAU) & live).any(1)
    acc_f = ((ovf["accept_margin"] <= TAU) & used).any(1)
    tok_f = ovf["icdf_margin"] <= TAU_S
    g_stop, g_len, g_out = gds["n_stop"].cpu().numpy(), gvf["accept_len"].cpu().numpy(), gvf["out_tok"].cpu().numpy()
    mism = int((~stop_f & (g_stop != ods["n_stop"])).sum())
    mism += int((~acc_f & (g_len != ovf["accept_len"])).sum())
    mism += int((~acc_f & ~tok_f & (g_len == ovf["accept_len"]) & (g_out != ovf["out_tok"]).any(1)).sum())
    mism += int((gds["top1_id"].cpu().numpy()[live] != ods["top1_id"][live]).sum())
    rel = lambda a, b: float(np.nanmax(np.abs(a[live] - b[live]) / np.maximum(np.abs(b[live]), 1e-3)))
    return {"sequences": int(w.B), "stop_flagged": int(stop_f.sum()), "accept_flagged": int(acc_f.sum()), "token_flagged": int(tok_f.sum()),
            "unflagged_mismatches": mism,
            "worst_rel_err_entropy": rel(gds["entropy"].cpu().numpy().astype(np.float64), ods["entropy"].astype(np.float64)),
            "worst_rel_err_margin": rel(gds["margin"].cpu().numpy().astype(np.float64), ods["margin"].astype(np.float64))}


def run_workload(args, name, steps, warmup, kernel_steps, headline):
    """Times one workload; returns (result dict, objects the CPU leg of the headline needs)."""
    import torch
    from paper_2511_02017_amd import binding, synth
    dev = "cuda:0"
    w = synth.WORKLOADS[name]
    esz = {torch.float32: 4, torch.bfloat16: 2}
    ed, et = esz[w.draft_dtype], esz[w.target_dtype]
    round_bytes = w.V * (w.B * w.K * ed + w.B * (w.K + 1) * et)
    ring_n = (args.ring if headline and args.ring else 0) or max(2, min(8, -(-(1 << 30) // round_bytes)))
    gen = synth.RoundGenerator(w, dev)
    ring = [gen.round(r) for r in range(ring_n)]
    pol_name = (args.policy if headline else None) or w.policy
    policy = {"ucb1": binding.UCB1, "ts": binding.TS_BETA, "ucb_tuned": binding.UCB_TUNED, "ts_gauss": binding.TS_GAUSS}[pol_name]
    needs_u = policy in (binding.TS_BETA, binding.TS_GAUSS)
    rules, thresholds = (0, 1, 2), (0.6, 0.8, 0.2)
    if headline and args.arms == "five":
        rules, thresholds = (0, 1, 2, 3, 4), (0.6, 0.8, 0.2, 0.2, 0.4)
    n_arms = len(rules)
    sample_draft = headline and args.sample_draft
    truncate = headline and args.mode == "truncate"
    mk = lambda: binding.Tapout(w.B, w.K, w.V, policy=policy, rules=rules, thresholds=thresholds, draft_sampling=sample_draft)
    tp = mk()
    if headline:
        for o in args.opt:
            k, v = o.split("=")
            tp.set_option(k, int(v))
    u_ts_ring = [None] * ring_n
    if needs_u:            # uniforms of the Thompson draws, [B, arms, 48]; the generator's are sized for three arms
        g = torch.Generator(device=dev).manual_seed(20251102)
        u_ts_ring = [r["u_ts"] if n_arms == w.n_arms else torch.rand(w.B, n_arms, 48, device=dev, generator=g) for r in ring]
    u_draft_ring = [None] * ring_n
    if sample_draft:
        g = torch.Generator(device=dev).manual_seed(20251103)
        u_draft_ring = [torch.rand(w.B, w.K, device=dev, generator=g) for _ in ring]
    # the four calls of a round, one after the other (select, draft_stats, verify, update) ...
    prepared4 = [tp.prepare_round(r, truncate, u_ts=u, u_draft=ud) for r, u, ud in zip(ring, u_ts_ring, u_draft_ring)]
    sh = torch.cuda.current_stream().cuda_stream

    def run4(n, first=0):
        for i in range(n):
            prepared4[(first + i) % ring_n][0](sh)

    # ... and the whole round as ONE call (tapout_round: update and next selection in one launch, the target pass
    # beside the draft pass when n_draft is given): the headline.  Its arms live in one array that every call
    # reads and overwrites; the uniforms of the next selection are those of the ring slot that follows.
    one_call = not sample_draft
    if one_call:
        arm = torch.zeros(w.B, dtype=torch.int32, device=dev)
        tp.bandit_select(w.B, u_ts=u_ts_ring[0], arm_out=arm)
        prepared = [tp.prepare_round_call(ring[i], arm, truncate, u_ts_next=u_ts_ring[(i + 1) % ring_n]) for i in range(ring_n)]

        def run(n, first=0):
            for i in range(n):
                prepared[(first + i) % ring_n][0](sh)
    else:
        prepared, run = prepared4, run4

    def timed_region(fn):
        fn(warmup)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn(steps, first=warmup)                    # the timed region: no events, no profiling
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    elapsed4 = timed_region(run4) if one_call else None
    elapsed = timed_region(run)
    ms_per_step = elapsed / steps * 1e3

    # work actually done in the timed steps (integer outputs of the last pass over each ring slot)
    n_draft_ring = [p[1]["n_draft"].cpu().long() for p in prepared]
    k_len_ring = [r["k_len"].cpu().long() for r in ring]
    acc_ring = [p[1]["verify"]["accept_len"].cpu().long() for p in prepared]
    slots = [(warmup + i) % ring_n for i in range(steps)]
    verified = sum(int(n_draft_ring[s].sum()) for s in slots)
    emitted = sum(int(acc_ring[s].sum()) + w.B for s in slots)
    draft_rows = sum(int(k_len_ring[s].sum()) for s in slots)
    target_rows = sum(int(n_draft_ring[s].sum()) + w.B for s in slots)
    stream_bytes = w.V * (draft_rows * ed + target_rows * et)          # every logit of a live row once

    # ---- instrumented loop: an event pair on every launch of every kernel, on the stream the kernels run on ----
    kinds = binding.PROFILE_KINDS
    tp.set_option("profile_stride", 1)
    tp.profile_enable(kinds, kernel_steps)
    for k in kinds:
        tp.profile_read(k)
    first_k = warmup + steps
    run4(kernel_steps, first=first_k)              # kernel by kernel: the four calls, nothing overlapped
    torch.cuda.synchronize()
    prof = {k: tp.profile_read(k) for k in kinds}
    prof_round = None
    if one_call:                                   # and the launches of the single call the timed region is made of
        run(kernel_steps, first=first_k)
        torch.cuda.synchronize()
        prof_round = {k: tp.profile_read(k) for k in kinds}
    tp.profile_enable((), 0)
    kslots = [(first_k + i) % ring_n for i in range(kernel_steps)]
    names = kernel_names(w, torch)
    names["stream_pair"] = f"stream_pair_kernel<{1 if w.draft_dtype == torch.bfloat16 else 0}, {1 if w.target_dtype == torch.bfloat16 else 0}>"
    # the final-token slice pass reads one row pair per sampled sequence (draft + target row of the first rejected
    # position, or the last target row alone when nothing was rejected)
    greedy = ring[0]["greedy"].cpu().bool()

    def final_bytes(s):
        m, n = acc_ring[s], n_draft_ring[s]
        pair = ((m < n) & ~greedy).sum().item()
        alone = ((m >= n) & ~greedy).sum().item()
        return w.V * (pair * (ed + et) + alone * et)

    def roof(kind, bytes_of_slot, traffic=False, source=None):
        ms, n = (source or prof)[kind]
        if n == 0:
            return None
        assert n == len(kslots), (kind, n, len(kslots))
        nbytes = sum(bytes_of_slot(s) for s in kslots)
        avg_us = ms / n * 1e3
        gbs = nbytes / n / (avg_us * 1e-6) / 1e9
        d = dict(kernel=names[kind], bound="hbm", achieved=round(gbs, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                 frac=round(gbs / HBM_PEAK_GBS, 4), avg_us=round(avg_us, 2), launches=n, bytes_per_launch=nbytes // n)
        if traffic:
            d["traffic"] = committed_traffic(w, names[kind]) if not truncate else None
            d["traffic_source"] = (f"profiles/stream_pass_{w.name}_hbm_traffic.txt: rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE per launch, "
                                   "copy-kernel calibrated, committed with the sources (not measured in this run)")
        return d

    r_target = roof("target_pass", lambda s: w.V * (int(n_draft_ring[s].sum()) + w.B) * et, traffic=True)
    r_draft = roof("draft_pass", lambda s: w.V * int(k_len_ring[s].sum()) * ed, traffic=True)
    r_final = roof("verify_slices", final_bytes)
    r_stream = None
    if r_target and r_draft:
        us = r_target["avg_us"] + r_draft["avg_us"]
        gbs = (r_target["bytes_per_launch"] + r_draft["bytes_per_launch"]) / (us * 1e-6) / 1e9
        r_stream = dict(kernel="draft pass + target pass", bound="hbm", achieved=round(gbs, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                        frac=round(gbs / HBM_PEAK_GBS, 4), avg_us=round(us, 2), launches=r_target["launches"],
                        bytes_per_launch=r_target["bytes_per_launch"] + r_draft["bytes_per_launch"])
    # The launch with the most bytes in the timed region: the pair launch of tapout_round (draft and target rows in one
    # streaming pass) where the round takes it, else the target pass.
    r_headline, r_pair = r_target, None
    if prof_round and prof_round["stream_pair"][1]:
        r_pair = roof("stream_pair", lambda s: w.V * (int(k_len_ring[s].sum()) * ed + (int(n_draft_ring[s].sum()) + w.B) * et), source=prof_round)
        own = committed_traffic(w, names["stream_pair"])
        if own:
            r_pair["traffic"], r_pair["traffic_source"] = own, r_target["traffic_source"]
        elif r_target and r_draft and r_target.get("traffic") and r_draft.get("traffic"):
            r_pair["traffic"] = r_target["traffic"] + r_draft["traffic"]
            r_pair["traffic_source"] = "sum of the two passes' committed counter figures (same bytes, one launch): " + r_target["traffic_source"]
        r_headline = r_pair
    res = {
        "value": round(verified / elapsed, 1), "unit": "verified draft tokens/s", "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 4),
        "config": {"workload": f"{w.name}: V={w.V} B={w.B} K={w.K} draft={str(w.draft_dtype)[6:]} target={str(w.target_dtype)[6:]}",
                   "mode": "full-K (n_draft = K)" if not truncate else "truncate (n_draft = stop position)",
                   "step": "tapout_round (one call per round)" if one_call else "select, draft_stats, verify, update (four calls)",
                   "policy": pol_name, "arms": args.arms if headline else "three",
                   "draft_tokens": "sampled by the library" if sample_draft else "given",
                   "ring_rounds": ring_n, "ring_bytes": ring_n * round_bytes},
        "emitted_tokens_per_s": round(emitted / elapsed, 1),
        "rows_per_s": round((draft_rows + target_rows) / elapsed, 1),
        "whole_round_GBps": round(stream_bytes / elapsed / 1e9, 1),
        "whole_round_frac_of_hbm_peak": round(stream_bytes / elapsed / 1e9 / HBM_PEAK_GBS, 4),
        "roofline": r_headline, "roofline_target_reduce": r_target, "roofline_draft_reduce": r_draft, "roofline_streaming": r_stream,
        "roofline_final_token": r_final,
        "kernel_avg_us": {k: round(prof[k][0] / prof[k][1] * 1e3, 2) for k in kinds if prof[k][1]},
    }
    if prof_round:
        res["kernel_avg_us_round_call"] = {k: round(prof_round[k][0] / prof_round[k][1] * 1e3, 2) for k in kinds if prof_round[k][1]}
    if elapsed4 is not None:
        res["four_calls"] = {"ms_per_step": round(elapsed4 / steps * 1e3, 4), "value": round(verified / elapsed4, 1),
                             "note": "the same steps as select / draft_stats / verify / update, one after the other on one stream"}
    if not args.no_parity and not sample_draft:
        # one round on a fresh context (the arm pool's first plays), stop rules and all, against the oracle: through the
        # call the timed region makes (tapout_round), with the same options
        tp2 = mk()
        if headline:
            for o in args.opt:
                k, v = o.split("=")
                tp2.set_option(k, int(v))
        rnd = ring[0]
        arm = tp2.bandit_select(w.B, u_ts=u_ts_ring[0])
        arm_played = arm.clone()                      # the call leaves the next round's arms in `arm`
        launch, outs = tp2.prepare_round_call(rnd, arm, truncate, u_ts_next=u_ts_ring[1 % ring_n])
        launch(torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        res["parity"] = decision_parity(torch, w, rnd, arm_played, outs["draft"], outs["verify"], outs["n_draft"], rules, thresholds)
        res["parity"]["call"] = "tapout_round"
        tp2.close()
    keep = dict(w=w, ring=ring, truncate=truncate, policy=policy, rules=rules, thresholds=thresholds, u_ts_ring=u_ts_ring, ed=ed)
    return res, keep


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (sequences are independent, so the path needs no exchange between "
              "GPUs); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    kernel_steps = args.kernel_steps or max(32, min(args.steps, 200))
    res, keep = run_workload(args, args.workload, args.steps, args.warmup, kernel_steps, headline=True)
    w, ring = keep["w"], keep["ring"]
    out = {"metric": METRIC, "value": res.pop("value"), "unit": res.pop("unit"), "n_gpus": 1,
           "steps": res.pop("steps"), "warmup": res.pop("warmup"), "ms_per_step": res.pop("ms_per_step"),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32",                      # arithmetic type of the streaming path (fp64 in the final-token sampler and bandit)
           "data": "synthetic"}
    out.update(res)
    if not args.no_read_reference:
        # A plain read-only streaming kernel on the same box and the same tensors, for scale: PyTorch's row sum of the
        # draft logits of a round (one read of every element, one float per row out), after the timed region.
        flat = [r["draft"].reshape(-1, w.V) for r in ring]
        for i in range(4):
            flat[i % len(ring)].sum(dim=1, dtype=torch.float32)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 24
        e0.record()
        for i in range(reps):
            flat[i % len(ring)].sum(dim=1, dtype=torch.float32)
        e1.record()
        torch.cuda.synchronize()
        ref_us = e0.elapsed_time(e1) / reps * 1e3
        ref_gbs = flat[0].numel() * keep["ed"] / (ref_us * 1e-6) / 1e9
        out["read_only_reference"] = {"kernel": "torch.sum(dim=-1, dtype=float32) over the draft logits of one round",
                                      "avg_us": round(ref_us, 2), "achieved": round(ref_gbs, 1), "unit": "GB/s",
                                      "frac": round(ref_gbs / HBM_PEAK_GBS, 4)}
        del flat
    if args.copy_calibration:
        src = torch.empty(512 << 20, dtype=torch.uint8, device="cuda:0").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(8):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_calibration"] = {"bytes_read_per_copy": src.numel(), "bytes_written_per_copy": src.numel(), "copies": 8}
        del src, dst
    if not args.no_cpu_baseline and not args.sample_draft:
        out["cpu_baseline"] = cpu_baseline(w, ring, keep["truncate"], args.cpu_seconds, keep["policy"], keep["rules"], keep["thresholds"],
                                           [None if u is None else u.cpu().numpy() for u in keep["u_ts_ring"]])
    if not args.no_extra_workloads and args.workload == "llama3":
        # the other two configurations with a vocabulary of 128k or more, in the same run: fewer steps, no CPU leg
        del ring, keep
        for name in ("zipf", "ragged"):
            gc.collect()
            torch.cuda.empty_cache()
            r, k2 = run_workload(args, name, 48, 8, 32, headline=False)
            del k2
            out["roofline_" + name] = {"ms_per_step": r["ms_per_step"], "value": r["value"], "unit": r["unit"], "steps": r["steps"],
                                       "config": r["config"], "whole_round_frac_of_hbm_peak": r["whole_round_frac_of_hbm_peak"],
                                       "round_call": r["roofline"], "target_pass": r["roofline_target_reduce"], "draft_pass": r["roofline_draft_reduce"],
                                       "streaming": r["roofline_streaming"], "final_token": r["roofline_final_token"],
                                       "kernel_avg_us": r["kernel_avg_us"], "kernel_avg_us_round_call": r.get("kernel_avg_us_round_call"),
                                       "four_calls": r.get("four_calls"), "parity": r.get("parity")}
    print(json.dumps(out))


def cpu_baseline(w, ring, truncate, budget_s, policy, rules, thresholds, u_ts_ring):
    """The CPU oracle, as it stands, on whole rounds of the same workload (cycling through the
    pre-generated ring) until about `budget_s` seconds of wall time are spent; all host cores."""
    import numpy as np
    from oracle import oracle as orc
    cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16")))
    host = []
    for rnd in ring:
        host.append(dict(draft=orc.as_logits(rnd["draft"].cpu()), target=orc.as_logits(rnd["target"].cpu()),
                         tok=rnd["draft_tok"].cpu().numpy(), k_len=rnd["k_len"].cpu().numpy(),
                         greedy=rnd["greedy"].cpu().numpy(), ua=rnd["u_accept"].cpu().numpy(),
                         us=rnd["u_sample"].cpu().numpy(), u_ts=u_ts_ring[len(host)]))
    def run(nthreads, seconds):
        bandit = orc.Bandit(policy, w.B, len(rules))          # the policy codes of the oracle and of the boundary coincide
        state = orc.RuleState(w.B, rules, thresholds)
        tokens, rounds = 0, 0
        t0 = time.perf_counter()
        while True:
            h = host[rounds % len(host)]
            arm, _ = bandit.select(w.B, h["u_ts"])
            ds = orc.draft_stats(h["draft"], draft_tok=h["tok"], k_len=h["k_len"], arm=arm, rules=rules, thresholds=thresholds,
                                 prev_entropy=state.prev_entropy, lam=state.lam, nthreads=nthreads)
            nd = ds["n_stop"] if truncate else h["k_len"]
            vf = orc.verify(h["target"], h["draft"], ds["logq_tok"], h["tok"], nd, h["ua"], h["us"], greedy=h["greedy"],
                            nthreads=nthreads)
            bandit.update(arm, vf["accept_len"], nd, h["k_len"])
            state.update(ds["entropy"], nd, vf["accept_len"])
            tokens += int(np.sum(nd))
            rounds += 1
            dt = time.perf_counter() - t0
            if dt >= seconds:
                return tokens, rounds, dt

    tokens, rounds, dt = run(cores, budget_s)
    out = {"value": round(tokens / dt, 1), "unit": "verified draft tokens/s", "cores": cores, "kind": "oracle",
           "sample": f"{rounds} whole rounds of the workload ({tokens} drafted tokens) in {dt:.1f} s"}
    t1, r1, d1 = run(1, min(4.0, budget_s / 3))               # the same on one thread, a shorter sample (at least one round)
    out["single_thread"] = {"value": round(t1 / d1, 1), "sample": f"{r1} whole rounds ({t1} drafted tokens) in {d1:.1f} s"}
    return out


if __name__ == "__main__":
    main()
