#!/usr/bin/env python3
"""Benchmark of the TapOut logits path on one MI355X.

One "step" is one decode round of the whole hot path over one batch of
synthetic logits already resident in HBM:
    tapout_bandit_select -> tapout_draft_stats -> tapout_verify -> tapout_bandit_update
The default workload is the Llama-3-vocabulary configuration (V = 128256,
B = 64, K = 8, bfloat16) on which the headline metric (verified draft tokens/s
at a 128k vocabulary) is quoted.  Inputs rotate through a ring of pre-generated
rounds larger than the 256 MB Infinity Cache, so no step finds its logits cached.

Prints ONE JSON line.  value = drafted tokens handed to verification (sum of n_draft over the timed steps) per
second of wall time; roofline / roofline_draft_reduce = the two streaming launches (target / draft pass):
algorithmic logit bytes per launch over the kernel's average duration, taken from event pairs the library puts on
those launches inside the timed region, against the 8 TB/s HBM peak; traffic = HBM bytes per launch from the
committed rocprofv3 counter summary; cpu_baseline = the CPU oracle on whole rounds of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak


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
    ap.add_argument("--profile-all", action="store_true", help="time every kernel with events (perturbs the step time slightly)")
    ap.add_argument("--opt", action="append", default=[], help="library tuning option name=value")
    ap.add_argument("--no-read-reference", action="store_true", help="skip the plain PyTorch row-sum reference")
    ap.add_argument("--profile-stride", type=int, default=11,
                    help="time the streaming launches of one step in this many (event pairs perturb the step)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run 8 plain device copies of 512 MiB (torch copy_): a kernel of known traffic that scales "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (sequences are independent, so the path needs no exchange between "
              "GPUs); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2511_02017_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = synth.WORKLOADS[args.workload]
    esz = {torch.float32: 4, torch.bfloat16: 2}
    round_bytes = w.V * (w.B * w.K * esz[w.draft_dtype] + w.B * (w.K + 1) * esz[w.target_dtype])
    ring_n = args.ring or max(2, min(8, -(-(1 << 30) // round_bytes)))
    gen = synth.RoundGenerator(w, dev)
    ring = [gen.round(r) for r in range(ring_n)]
    pol_name = args.policy or w.policy
    policy = {"ucb1": binding.UCB1, "ts": binding.TS_BETA, "ucb_tuned": binding.UCB_TUNED, "ts_gauss": binding.TS_GAUSS}[pol_name]
    needs_u = policy in (binding.TS_BETA, binding.TS_GAUSS)
    rules, thresholds = (0, 1, 2), (0.6, 0.8, 0.2)
    if args.arms == "five":
        rules, thresholds = (0, 1, 2, 3, 4), (0.6, 0.8, 0.2, 0.2, 0.4)
    n_arms = len(rules)
    tp = binding.Tapout(w.B, w.K, w.V, policy=policy, rules=rules, thresholds=thresholds, draft_sampling=args.sample_draft)
    for o in args.opt:
        k, v = o.split("=")
        tp.set_option(k, int(v))
    truncate = args.mode == "truncate"
    u_ts_ring = [None] * ring_n
    if needs_u:            # uniforms of the Thompson draws, [B, arms, 48]; the generator's are sized for three arms
        g = torch.Generator(device=dev).manual_seed(20251102)
        u_ts_ring = [r["u_ts"] if n_arms == w.n_arms else torch.rand(w.B, n_arms, 48, device=dev, generator=g) for r in ring]
    u_draft_ring = [None] * ring_n
    if args.sample_draft:
        g = torch.Generator(device=dev).manual_seed(20251103)
        u_draft_ring = [torch.rand(w.B, w.K, device=dev, generator=g) for _ in ring]
    prepared = [tp.prepare_round(r, truncate, u_ts=u, u_draft=ud) for r, u, ud in zip(ring, u_ts_ring, u_draft_ring)]
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream

    def run(n, first=0):
        for i in range(n):
            prepared[(first + i) % ring_n][0](sh)

    kinds = binding.PROFILE_KINDS if args.profile_all else ("draft_pass", "target_pass")
    run(args.warmup)
    torch.cuda.synchronize()
    # The roofline figures come from event pairs on the two streaming launches inside the timed region.  An event
    # pair costs the stream about 4 us per launch, so the default line samples one step in 11 (coprime with every
    # ring length); --profile-all times every launch of every kernel and stretches the step accordingly.
    tp.set_option("profile_stride", 1 if args.profile_all else args.profile_stride)
    tp.profile_enable(kinds, args.steps)
    for k in kinds:
        tp.profile_read(k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps, first=args.warmup)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = {k: tp.profile_read(k) for k in kinds}
    tp.profile_enable((), 0)
    elapsed = t1 - t0
    ms_per_step = elapsed / args.steps * 1e3

    # work actually done in the timed steps (integer outputs of the last pass over each ring slot)
    n_draft_ring = [p[1]["n_draft"].cpu().long() for p in prepared]
    k_len_ring = [r["k_len"].cpu().long() for r in ring]
    acc_ring = [p[1]["verify"]["accept_len"].cpu().long() for p in prepared]
    slots = [(args.warmup + i) % ring_n for i in range(args.steps)]
    verified = sum(int(n_draft_ring[s].sum()) for s in slots)
    emitted = sum(int(acc_ring[s].sum()) + w.B for s in slots)
    draft_rows = sum(int(k_len_ring[s].sum()) for s in slots)
    target_rows = sum(int(n_draft_ring[s].sum()) + w.B for s in slots)
    ed, et = esz[w.draft_dtype], esz[w.target_dtype]
    stream_bytes = w.V * (draft_rows * ed + target_rows * et)          # every logit of a live row once

    def measured_traffic(kernel_name):
        """HBM bytes per launch (FETCH_SIZE + WRITE_SIZE, copy-kernel calibrated) from the committed rocprofv3 --pmc summary."""
        path = os.path.join(ROOT, "profiles", f"stream_pass_{w.name}_hbm_traffic.txt")
        if not os.path.exists(path):
            return None
        total, seen = 0.0, 0
        for line in open(path):
            if kernel_name in line and "MB per launch" in line:
                total += float(line.split("->")[1].split("MB per launch")[0]) * 1e6
                seen += 1
        return int(total) if seen == 2 else None

    kernel_of = {"target_pass": f"stream_pass_kernel<{1 if w.target_dtype == torch.bfloat16 else 0}, false>",
                 "draft_pass": f"stream_pass_kernel<{1 if w.draft_dtype == torch.bfloat16 else 0}, true>"}

    stride = 1 if args.profile_all else args.profile_stride
    timed_slots = slots[::stride]                                       # the steps whose streaming launches carried events

    def roof(kind, bytes_of_slot):
        ms, n = prof[kind]
        if n == 0:
            return None
        assert n == len(timed_slots), (n, len(timed_slots))
        nbytes = sum(bytes_of_slot(s) for s in timed_slots)
        avg_us = ms / n * 1e3
        gbs = nbytes / n / (avg_us * 1e-6) / 1e9
        return dict(kernel=kernel_of[kind], bound="hbm", achieved=round(gbs, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(gbs / HBM_PEAK_GBS, 4), avg_us=round(avg_us, 2), launches=n,
                    bytes_per_launch=nbytes // n, traffic=measured_traffic(kernel_of[kind]) if not truncate else None)

    r_target = roof("target_pass", lambda s: w.V * (int(n_draft_ring[s].sum()) + w.B) * et)
    r_draft = roof("draft_pass", lambda s: w.V * int(k_len_ring[s].sum()) * ed)
    both_ms = prof["target_pass"][0] + prof["draft_pass"][0]
    out = {
        "metric": "verified draft tokens/sec and achieved HBM GB/s (% of peak) at vocab 128k",
        "value": round(verified / elapsed, 1),
        "unit": "verified draft tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32",                               # arithmetic type of the streaming path (fp64 in the final-token sampler and bandit)
        "data": "synthetic",
        "config": {"workload": f"{w.name}: V={w.V} B={w.B} K={w.K} draft={str(w.draft_dtype)[6:]} target={str(w.target_dtype)[6:]}",
                   "mode": "full-K (n_draft = K)" if not truncate else "truncate (n_draft = stop position)",
                   "policy": pol_name, "arms": args.arms, "draft_tokens": "sampled by the library" if args.sample_draft else "given", "ring_rounds": ring_n, "ring_bytes": ring_n * round_bytes},
        "emitted_tokens_per_s": round(emitted / elapsed, 1),
        "rows_per_s": round((draft_rows + target_rows) / elapsed, 1),
        "whole_round_GBps": round(stream_bytes / elapsed / 1e9, 1),
        "whole_round_frac_of_hbm_peak": round(stream_bytes / elapsed / 1e9 / HBM_PEAK_GBS, 4),
        "roofline": r_target,
        "roofline_draft_reduce": r_draft,
        "streaming_kernels_GBps": round((r_target["achieved"] * r_target["avg_us"] + r_draft["achieved"] * r_draft["avg_us"])
                                        / (r_target["avg_us"] + r_draft["avg_us"]), 1) if r_target and r_draft else None,
    }
    if args.profile_all:
        out["kernel_avg_us"] = {k: round(prof[k][0] / max(1, prof[k][1]) * 1e3, 2) for k in kinds}
    if not args.no_read_reference:
        # A plain read-only streaming kernel on the same box and the same tensors, for scale: PyTorch's row sum of the
        # draft logits of a round (one read of every element, one float per row out), after the timed region.
        flat = [r["draft"].reshape(-1, w.V) for r in ring]
        for i in range(4):
            flat[i % ring_n].sum(dim=1, dtype=torch.float32)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 24
        e0.record()
        for i in range(reps):
            flat[i % ring_n].sum(dim=1, dtype=torch.float32)
        e1.record()
        torch.cuda.synchronize()
        ref_us = e0.elapsed_time(e1) / reps * 1e3
        ref_gbs = flat[0].numel() * ed / (ref_us * 1e-6) / 1e9
        out["read_only_reference"] = {"kernel": "torch.sum(dim=-1, dtype=float32) over the draft logits of one round",
                                      "avg_us": round(ref_us, 2), "achieved": round(ref_gbs, 1), "unit": "GB/s",
                                      "frac": round(ref_gbs / HBM_PEAK_GBS, 4)}

    if args.copy_calibration:
        src = torch.empty(512 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(8):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_calibration"] = {"bytes_read_per_copy": src.numel(), "bytes_written_per_copy": src.numel(), "copies": 8}
    if not args.no_cpu_baseline and not args.sample_draft:
        out["cpu_baseline"] = cpu_baseline(w, ring, truncate, args.cpu_seconds, policy, rules, thresholds,
                                           [None if u is None else u.cpu().numpy() for u in u_ts_ring])
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
