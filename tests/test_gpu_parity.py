"""GPU parity: libtapout (through its C ABI) against the CPU oracle, element by
element, on the same seeded inputs.  Tolerances are defined in parity_util."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2511_02017_amd import binding, synth
from tests import parity_util as pu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def announce(msg):
    print(f"[case] {msg}", flush=True)


def make(w, rounds=(0,), fuse=None, **kw):
    gen = synth.RoundGenerator(w, DEV)
    tp = binding.Tapout(w.B, w.K, w.V, **kw)
    if fuse is not None:
        tp.set_option("fuse_head", fuse)
    return gen, tp, [gen.round(r) for r in rounds]


# tapout_verify takes the accept decisions either in a launch of their own (0) or again in every workgroup of the
# final-token slice kernel (1); left alone it picks by launch size, which at test sizes is always (1).
FUSE = pytest.mark.parametrize("fuse", [0, 1])


def random_arms(B, seed=0):
    g = torch.Generator().manual_seed(seed)
    return torch.randint(0, 3, (B,), generator=g, dtype=torch.int32).to(DEV)


# ---- the five workloads, at sizes the oracle finishes in seconds ---------------

@pytest.mark.parametrize("name,kw", [
    ("tiny", {}),
    ("small", {}),
    ("llama3", dict(B=16)),
    ("zipf", dict(B=12)),
    ("ragged", dict(B=12)),
])
@FUSE
def test_workload_parity_full_k(name, kw, fuse):
    w = synth.scaled(synth.WORKLOADS[name], **kw)
    announce(f"full-K {w} fuse_head={fuse}")
    gen, tp, rounds = make(w, rounds=(0, 1), fuse=fuse)
    total = dict(stop_flagged=0, accept_flagged=0, icdf_flagged=0, sequences=0)
    for rnd in rounds:
        c = pu.check_round(tp, rnd)
        for k in total:
            total[k] += c[k]
    announce(f"{name}: near-tie counts {total}")
    assert total["accept_flagged"] + total["icdf_flagged"] <= max(2, total["sequences"] // 50)


@pytest.mark.parametrize("name,kw", [
    ("tiny", {}),
    ("small", {}),
    ("llama3", dict(B=16)),
    ("zipf", dict(B=12)),
    ("ragged", dict(B=12)),
])
@pytest.mark.parametrize("truncate", [False, True])
def test_workload_parity_whole_round_call(name, kw, truncate):
    """The five workloads through tapout_round, the call the benchmark times, against the oracle: draft statistics, stop
    positions, accept decisions, tokens.  With n_draft = k_len (truncate False) the call streams both tensors in one
    launch where their element sizes agree, takes log q(tok) from the draft partials and runs the draft epilogue in the
    locate kernel's launch; the oracle knows none of that."""
    w = synth.scaled(synth.WORKLOADS[name], **kw)
    announce(f"tapout_round {w} truncate={truncate}")
    gen = synth.RoundGenerator(w, DEV)
    tp = binding.Tapout(w.B, w.K, w.V)
    total = dict(stop_flagged=0, accept_flagged=0, icdf_flagged=0, sequences=0)
    for r in (0, 1):
        c = pu.check_round_call(tp, gen.round(r), random_arms(w.B, seed=r), truncate)
        for k in total:
            total[k] += c[k]
    announce(f"{name}: near-tie counts {total}")
    assert total["accept_flagged"] + total["icdf_flagged"] <= max(2, total["sequences"] // 50)


@pytest.mark.parametrize("name,kw", [("tiny", {}), ("small", {}), ("llama3", dict(B=16)), ("ragged", dict(B=8))])
@FUSE
def test_workload_parity_truncated(name, kw, fuse):
    """Algorithm 1 as written: n_draft = stop position of the selected arm."""
    w = synth.scaled(synth.WORKLOADS[name], **kw)
    announce(f"truncate {w} fuse_head={fuse}")
    gen, tp, rounds = make(w, rounds=(2,), fuse=fuse)
    arm = random_arms(w.B, seed=w.index)
    c = pu.check_round(tp, rounds[0], arm=arm)
    announce(f"{name}: near-tie counts {c}")
    # a near tie needs a signal within 1e-5 (relative) of its threshold or a uniform within 1e-5 of p/q: about one
    # decision in 1e5; a count beyond a couple means the flags are hiding mismatches
    assert c["stop_flagged"] + c["accept_flagged"] + c["icdf_flagged"] <= max(2, c["sequences"] // 50)


def test_peaked_rows_separate_the_rules():
    # low-entropy rows: the three rules give different stop positions, none of them trivial
    w = synth.scaled(synth.WORKLOADS["llama3"], B=24, V=32000, sigma_draft=4.5)
    gen, tp, rounds = make(w, rounds=(0,))
    seen = set()
    for a in range(3):
        arm = torch.full((w.B,), a, dtype=torch.int32, device=DEV)
        pu.check_round(tp, rounds[0], arm=arm)
        ds = tp.draft_stats(rounds[0]["draft"], draft_tok=rounds[0]["draft_tok"], arm=arm)
        seen.add(tuple(ds["n_stop"].cpu().tolist()))
    assert len(seen) == 3


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("V,opts", [(32000, ()), (128256, ()), (32000, (("wgs_target", 1),)), (5000, (("wgs_target", 65536), ("min_slice", 256))),
                                    (70001, ())])
def test_peaked_rows_keep_relative_precision(dtype, V, opts):
    """One logit lifted 4 .. 34 above a N(0,1) background: entropies from ~1 down to 1e-9, p_top1 up to 1 - 1e-10.
    Entropy, probabilities and margin must hold |gpu - ref| <= 1e-5 max(|ref|, 1e-3) over the whole sweep, whatever
    the number of slices per row (one workgroup per row, the default, many short slices) and wherever in its slice,
    batch or unaligned row end the maximum sits; the worst ratio to that bound is printed.  Then two near-tied top
    logits (gap 1 .. 1e-7 and an exact tie): the margin goes to 0 with relative precision."""
    g = torch.Generator().manual_seed(V)
    lifts = np.linspace(4.0, 34.0, 96)
    B, K = 12, 8
    x_wide = torch.randn(B, K, V + 3, generator=g)
    x = x_wide[:, :, 3:]                                                  # rows start 3 elements off a 16-byte boundary
    pos = torch.randint(0, V, (B, K), generator=g)
    pos[0, :4] = torch.tensor([0, 1, V - 1, V - 2])                       # unaligned head and tail elements hold the maximum
    for i, a in enumerate(lifts):
        x[i // K, i % K, pos[i // K, i % K]] = float(a)
    xd = x_wide.to(dtype).to(DEV)[:, :, 3:]
    tp = binding.Tapout(B, K, V)
    for k_, v_ in opts:
        tp.set_option(k_, v_)
    o = tp.draft_stats(xd)
    ref = orc.draft_stats(pu.host_logits(xd), nthreads=16)
    worst = {}
    for key in ("entropy", "margin", "p_top1", "p_top2"):
        got, want = o[key].cpu().numpy().astype(np.float64), ref[key].astype(np.float64)
        worst[key] = float((np.abs(got - want) / (pu.TAU * np.maximum(np.abs(want), 1e-3))).max())
        pu.assert_stats_close(key, got, want)
    assert (o["top1_id"].cpu().numpy() == ref["top1_id"]).all()
    H = ref["entropy"]
    assert H.min() < 1e-7 and H.max() > 0.5 and ((H > 1e-4) & (H < 1e-2)).sum() >= 5
    # near ties at the top
    gaps = [10.0 ** (-e / 2) for e in range(0, 15)] + [0.0]
    y = torch.randn(2, len(gaps), V, generator=g)
    for k, d in enumerate(gaps):
        for b_, a in enumerate((6.0, 14.0)):
            y[b_, k, 100] = a
            y[b_, k, V - 37] = float(np.float32(a) - np.float32(d))
    yd = y.to(dtype).to(DEV)
    tp2 = binding.Tapout(2, len(gaps), V)
    for k_, v_ in opts:
        tp2.set_option(k_, v_)
    o2 = tp2.draft_stats(yd)
    ref2 = orc.draft_stats(pu.host_logits(yd), nthreads=16)
    for key in ("entropy", "margin", "p_top1", "p_top2"):
        got, want = o2[key].cpu().numpy().astype(np.float64), ref2[key].astype(np.float64)
        worst["tie_" + key] = float((np.abs(got - want) / (pu.TAU * np.maximum(np.abs(want), 1e-3))).max())
        pu.assert_stats_close(key, got, want)
    assert ref2["margin"][:, -1].tolist() == [0.0, 0.0] and o2["margin"][:, -1].cpu().tolist() == [0.0, 0.0]
    announce(f"peaked rows {dtype} V={V} {opts}: worst error / (1e-5 max(|ref|, 1e-3)) = { {k: round(v, 3) for k, v in worst.items()} }")


# ---- shapes: tails, misalignment, strides, tiny vocabularies --------------------

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("V", [1, 2, 3, 7, 8, 9, 63, 1000, 4097, 12345, 32001])
def test_odd_vocab_sizes_and_misaligned_rows(V, dtype):
    announce(f"odd V={V} {dtype}")
    B, K = 3, 4
    g = torch.Generator(device=DEV).manual_seed(V)
    # rows carved out of a wider buffer at an odd offset: every row start is misaligned differently
    wide_d = (torch.randn(B, K, V + 13, generator=g, device=DEV) * 3).to(dtype)
    wide_t = (torch.randn(B, K + 1, V + 13, generator=g, device=DEV) * 3).to(dtype)
    draft, target = wide_d[:, :, 5:5 + V], wide_t[:, :, 3:3 + V]
    tok = torch.randint(0, V, (B, K), generator=g, device=DEV, dtype=torch.int32)
    rnd = dict(draft=draft, target=target, draft_tok=tok,
               u_accept=torch.rand(B, K, generator=g, device=DEV), u_sample=torch.rand(B, generator=g, device=DEV),
               k_len=torch.full((B,), K, dtype=torch.int32, device=DEV), greedy=torch.zeros(B, dtype=torch.uint8, device=DEV))
    tp = binding.Tapout(B, K, V)
    pu.check_round(tp, rnd)
    pu.check_round(tp, rnd, arm=random_arms(B))
    # the same rows cut into as many slices as the vocabulary allows (slices of 512 elements; the last ones of a row
    # hold only its unaligned tail, or nothing), with tokens at the first and last index: the slice that holds a
    # token's index hands its logit on
    tp.set_option("min_slice", 256)
    tp.set_option("wgs_target", 65536)
    edge = dict(rnd)
    edge["draft_tok"] = tok.clone()
    edge["draft_tok"][:, 0] = 0
    edge["draft_tok"][:, -1] = V - 1
    pu.check_round(tp, edge)
    pu.check_round(tp, edge, arm=random_arms(B))


def test_slice_counts_do_not_change_decisions():
    w = synth.scaled(synth.WORKLOADS["small"], B=6)
    gen, tp, rounds = make(w)
    ref = None
    # slices per row 1 .. 125: one to sixteen take the lane-parallel merge of the per-sequence kernels (groups of
    # 1, 2, 4, 8, 16 lanes, also with empty lanes: 3, 5, 11 slices), more than sixteen the staged sequential one
    for wgs, min_slice in ((1, 4096), (64, 256), (100, 256), (150, 256), (270, 256), (600, 256), (864, 256), (920, 256),
                           (4096, 256), (65536, 256), (4096, 1 << 20)):
        tp.set_option("wgs_target", wgs)
        tp.set_option("min_slice", min_slice)
        pu.check_round(tp, rounds[0])
        ds, vf, _ = pu.gpu_round(tp, rounds[0])
        ints = (ds["top1_id"].cpu(), vf["accept_len"].cpu(), vf["out_tok"].cpu())
        if ref is not None:
            assert all(torch.equal(a, b) for a, b in zip(ints, ref))
        ref = ints


def test_bit_identical_reruns():
    w = synth.scaled(synth.WORKLOADS["llama3"], B=8)
    gen, tp, rounds = make(w)
    a = pu.gpu_round(tp, rounds[0], arm=random_arms(w.B))
    b = pu.gpu_round(tp, rounds[0], arm=random_arms(w.B))
    for x, y in ((a[0], b[0]), (a[1], b[1])):
        for k in x:
            assert torch.equal(x[k].cpu().view(torch.int32) if x[k].dtype == torch.float32 else x[k].cpu(),
                               y[k].cpu().view(torch.int32) if y[k].dtype == torch.float32 else y[k].cpu()), k


@pytest.mark.parametrize("policy", [binding.UCB1, binding.TS_BETA])
def test_rounds_replayed_from_hip_graphs_match_eager_rounds(policy):
    """The four calls of a round capture into a HIP graph (they launch kernels only: no allocation, no memset, no
    host synchronisation).  Nine rounds are run eagerly on one context and replayed from three captured graphs on
    a second one, with eager work and synchronisations between the replays; every replay's outputs and the final
    bandit state must carry the eager run's bits."""
    w = synth.scaled(synth.WORKLOADS["llama3"], B=12)
    gen = synth.RoundGenerator(w, DEV)
    rounds = [gen.round(r) for r in range(3)]
    bits = lambda t: t.cpu().view(torch.int32).clone() if t.dtype == torch.float32 else t.cpu().clone()
    order = [0, 1, 2, 2, 0, 1, 1, 0, 2]

    def context():
        tp = binding.Tapout(w.B, w.K, w.V, policy=policy)
        prep = [tp.prepare_round(r, truncate=True, u_ts=r["u_ts"] if policy == binding.TS_BETA else None) for r in rounds]
        return tp, prep

    def snapshot(outs):
        d = {"arm": bits(outs["arm"])}
        d.update({"d_" + k: bits(v) for k, v in outs["draft"].items()})
        d.update({"v_" + k: bits(v) for k, v in outs["verify"].items()})
        return d

    tp_e, prep_e = context()
    stream = torch.cuda.Stream()
    expect = []
    with torch.cuda.stream(stream):
        for i in order:
            prep_e[i][0](stream.cuda_stream)
            stream.synchronize()
            expect.append(snapshot(prep_e[i][1]))
    state_e = tp_e.bandit_get_state()

    tp_g, prep_g = context()
    graphs = []
    for launch, _ in prep_g:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            launch(torch.cuda.current_stream().cuda_stream)
        graphs.append(g)
    scratch = torch.zeros(1 << 20, device=DEV)
    with torch.cuda.stream(stream):
        for step, i in enumerate(order):
            graphs[i].replay()
            scratch.add_(1.0)                                  # the program's own eager work between replays
            stream.synchronize()
            got = snapshot(prep_g[i][1])
            for k, v in expect[step].items():
                assert torch.equal(got[k], v), (step, i, k)
    for a, b in zip(tp_g.bandit_get_state(), state_e):
        assert (a.view(np.int64) == b.view(np.int64)).all()


@pytest.mark.parametrize("name,B,V", [("llama3", 12, None), ("llama3", 70, 9000), ("zipf", 6, None), ("ragged", 9, 70000), ("small", 32, None), ("llama3", 90, None)])
def test_round_with_the_epilogue_beside_the_locate_kernel(name, B, V):
    """tapout_round with n_draft from the caller: by default the accept decisions form log q(tok) from the draft pass's
    slice sums themselves and the draft epilogue runs in the locate kernel's launch.  Against the same call with the
    epilogue in its own launch ahead of the verification ("defer_epilogue" = 0), on one-launch (equal element sizes)
    and two-launch (ragged: bf16 draft, f32 target) streaming passes, fused and separate accept decisions, ragged
    lengths and greedy sequences: the draft outputs and the target statistics carry the same bits (the epilogue and the
    target merge see the same partials), and so do the decisions: log q(tok) differs by binary32 rounding only, which
    moves a decision only if its uniform lies within ~1e-6 of p/q (the oracle's own near-tie margin is 1e-5)."""
    kw = dict(B=B) if V is None else dict(B=B, V=V)
    w = synth.scaled(synth.WORKLOADS[name], **kw)
    gen = synth.RoundGenerator(w, DEV)
    outs = {}
    for defer in (1, 0):
        tp = binding.Tapout(w.B, w.K, w.V)
        tp.set_option("defer_epilogue", defer)
        arm = tp.bandit_select(w.B)
        res = []
        for r in range(3):
            rnd = gen.round(r)
            launch, o = tp.prepare_round_call(rnd, arm, False)
            launch(torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            snap = {"arm": arm.cpu().clone()}
            snap.update({"d_" + k: v.cpu().clone() for k, v in o["draft"].items()})
            snap.update({"v_" + k: v.cpu().clone() for k, v in o["verify"].items()})
            res.append(snap)
        outs[defer] = (res, tp.bandit_get_state(moments=True))
    for r, (a_, b_) in enumerate(zip(outs[1][0], outs[0][0])):
        assert a_.keys() == b_.keys()
        for k in a_:
            x, y = a_[k], b_[k]
            if x.dtype == torch.float32:
                x, y = x.view(torch.int32), y.view(torch.int32)
            assert torch.equal(x, y), (r, k)
    for a_, b_ in zip(outs[1][1], outs[0][1]):
        assert (a_.view(np.int64) == b_.view(np.int64)).all()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("bad", [False, True])
def test_round_with_the_epilogue_beside_the_locate_kernel_on_degenerate_rows(dtype, bad):
    """The same comparison on rows that are uniform, masked, one-hot, tied at the top, equal in draft and target, and
    (bad) on NaN rows, rows without a finite maximum, tokens out of range and lengths of 0 and K + 1: either place of
    the draft epilogue gives the same bits, flags included."""
    rnd = degenerate_round(dtype)
    B, K, V = rnd["draft"].shape
    if bad:
        rnd["draft"][0, 1, 17] = float("nan")
        rnd["target"][1, 0, 3] = float("nan")
        rnd["target"][2, 2, :] = float("-inf")
        rnd["draft_tok"][3, 0] = V
        rnd["draft_tok"][4, 2] = -1
        rnd["k_len"][5] = 0
        rnd["k_len"][6] = K + 1
    outs = {}
    for defer in (1, 0):
        tp = binding.Tapout(B, K, V)
        tp.set_option("defer_epilogue", defer)
        arm = tp.bandit_select(B)
        launch, o = tp.prepare_round_call(rnd, arm, False)
        launch(torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        snap = {"arm": arm.cpu().clone()}
        snap.update({"d_" + k: v.cpu().clone() for k, v in o["draft"].items()})
        snap.update({"v_" + k: v.cpu().clone() for k, v in o["verify"].items()})
        outs[defer] = snap
    live = (torch.arange(K)[None, :] < rnd["k_len"].cpu().clamp(0, K)[:, None])
    for k in outs[1]:
        x, y = outs[1][k], outs[0][k]
        if k.startswith("d_") and x.dim() == 2 and x.shape == live.shape:
            x, y = x[live], y[live]                       # rows beyond k_len are not written
        if x.dtype == torch.float32:
            x, y = x.view(torch.int32), y.view(torch.int32)
        assert torch.equal(x, y), k
    if bad:
        assert outs[1]["v_flags"].tolist()[1:5] == [orc.FLAG_BAD_ROW, orc.FLAG_BAD_ROW, orc.FLAG_BAD_TOKEN, orc.FLAG_BAD_TOKEN]
        assert outs[1]["d_flags"].tolist()[0] == orc.FLAG_BAD_ROW


@pytest.mark.parametrize("policy", [binding.UCB1, binding.TS_BETA])
@pytest.mark.parametrize("truncate,five", [(False, False), (True, False), (True, True)])
def test_whole_round_in_one_call_gives_the_bits_of_the_separate_calls(policy, truncate, five):
    """tapout_round (with n_draft given: draft and target rows in one streaming launch, the draft epilogue beside the
    locate kernel) against select / draft_stats / verify / update on a second context: every output of every round and the bandit
    state in the end carry the same bits; then the same rounds replayed from HIP graphs, eager work between replays."""
    w = synth.scaled(synth.WORKLOADS["llama3"], B=12, n_arms=5 if five else 3)
    gen = synth.RoundGenerator(w, DEV)
    rounds = [gen.round(r) for r in range(4)]
    ts = policy == binding.TS_BETA
    bits = lambda t: t.cpu().view(torch.int32).clone() if t.dtype == torch.float32 else t.cpu().clone()
    order = [0, 1, 2, 3, 3, 1, 0, 2, 2, 0]
    u_of = lambda i: rounds[i]["u_ts"] if ts else None
    # five: the paper's whole arm pool; SVIPDifference and AdaEDL carry state that the end of a round advances
    kw = dict(policy=policy, rules=FIVE_RULES, thresholds=FIVE_THRESHOLDS) if five else dict(policy=policy)

    def snapshot(outs):
        d = {"arm": bits(outs["arm"])}
        d.update({"d_" + k: bits(v) for k, v in outs["draft"].items()})
        d.update({"v_" + k: bits(v) for k, v in outs["verify"].items()})
        return d

    def same(got, want, where):
        """Bit for bit, except that with n_draft given the single call streams both tensors in one launch with a slice
        count of its own: there the statistics agree to the rounding of the binary32 slice sums, the integers exactly."""
        if truncate or got.dtype != torch.int32 or where[-1] in ("d_top1_id", "d_n_stop", "d_flags", "v_accept_len", "v_out_tok", "v_n_out",
                                                                "v_target_top1", "v_flags"):
            assert torch.equal(got, want), where
        elif got.dtype == torch.int32:                                     # float bits
            g_, w_ = got.view(torch.float32).double().numpy(), want.view(torch.float32).double().numpy()
            floor = 1.0 if where[-1][2:] in pu.LOG_KEYS else 1e-3          # log-domain values: absolute
            ok = (np.isnan(g_) & np.isnan(w_)) | (np.abs(g_ - w_) <= 2e-6 * np.maximum(np.abs(w_), floor))
            assert ok.all(), where

    # reference: the separate calls; the uniforms of round i's selection are rounds[order[i]]["u_ts"]
    tp_ref = binding.Tapout(w.B, w.K, w.V, **kw)
    expect = []
    for step, i in enumerate(order):
        rnd = rounds[i]
        arm = tp_ref.bandit_select(w.B, u_ts=u_of(i))
        ds = tp_ref.draft_stats(rnd["draft"], draft_tok=rnd["draft_tok"], k_len=rnd["k_len"], arm=arm)
        nd = ds["n_stop"] if truncate else rnd["k_len"]
        vf = tp_ref.verify(rnd["target"], rnd["draft"], ds["lse"], ds["logq_tok"], rnd["draft_tok"], nd, rnd["u_accept"], rnd["u_sample"],
                           greedy=rnd["greedy"])
        tp_ref.bandit_update(arm, vf["accept_len"], nd, rnd["k_len"])
        torch.cuda.synchronize()
        expect.append(snapshot(dict(arm=arm, draft=ds, verify=vf)))
    state_ref = tp_ref.bandit_get_state(moments=True)

    def one_call_context():
        tp = binding.Tapout(w.B, w.K, w.V, **kw)
        arm = torch.zeros(w.B, dtype=torch.int32, device=DEV)
        # the next selection's uniforms belong to the round that follows in `order`: one prepared call per (round, next round)
        calls = {}
        for step, i in enumerate(order):
            nxt = order[step + 1] if step + 1 < len(order) else order[0]
            if (i, nxt) not in calls:
                calls[(i, nxt)] = tp.prepare_round_call(rounds[i], arm, truncate, u_ts_next=u_of(nxt))
        return tp, arm, calls

    stream = torch.cuda.Stream()
    tp1, arm1, calls1 = one_call_context()
    with torch.cuda.stream(stream):
        tp1.bandit_select(w.B, u_ts=u_of(order[0]), arm_out=arm1, stream=stream)
        for step, i in enumerate(order):
            nxt = order[step + 1] if step + 1 < len(order) else order[0]
            arm_in = bits(arm1)
            stream.synchronize()
            arm_in = bits(arm1)
            launch, outs = calls1[(i, nxt)]
            launch(stream.cuda_stream)
            stream.synchronize()
            got = snapshot(dict(arm=outs["arm"], draft=outs["draft"], verify=outs["verify"]))
            assert torch.equal(arm_in, expect[step]["arm"]), (step, "arm")
            for k, v in expect[step].items():
                if k != "arm":
                    same(got[k], v, (step, i, k))
    for a_, b_ in zip(tp1.bandit_get_state(moments=True), state_ref):
        assert (a_.view(np.int64) == b_.view(np.int64)).all()
    if five:
        s1, s2 = tp1.rule_state_get(), tp_ref.rule_state_get()
        assert (s1["lam"] == s2["lam"]).all() and (s1["accept_rate"] == s2["accept_rate"]).all()
        assert (s1["prev_entropy"].view(np.int32) == s2["prev_entropy"].view(np.int32)).all()

    # the same from HIP graphs
    tp2, arm2, calls2 = one_call_context()
    graphs = {}
    tp2.bandit_select(w.B, u_ts=u_of(order[0]), arm_out=arm2, stream=stream)
    stream.synchronize()
    arm_start = arm2.clone()
    state_start = tp2.bandit_get_state(moments=True)
    for key, (launch, _) in calls2.items():
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            launch(torch.cuda.current_stream().cuda_stream)
        graphs[key] = g
    # capturing runs nothing, but be independent of that: restore the state the first round starts from
    arm2.copy_(arm_start)
    tp2.bandit_set_state(state_start[0], state_start[2], sum_r2=state_start[1])
    scratch = torch.zeros(1 << 20, device=DEV)
    with torch.cuda.stream(stream):
        for step, i in enumerate(order):
            nxt = order[step + 1] if step + 1 < len(order) else order[0]
            graphs[(i, nxt)].replay()
            scratch.add_(1.0)
            stream.synchronize()
            outs = calls2[(i, nxt)][1]
            got = snapshot(dict(arm=outs["arm"], draft=outs["draft"], verify=outs["verify"]))
            for k, v in expect[step].items():
                if k != "arm":
                    same(got[k], v, ("graph", step, i, k))
    for a_, b_ in zip(tp2.bandit_get_state(moments=True), state_ref):
        assert (a_.view(np.int64) == b_.view(np.int64)).all()


def test_head_inside_the_slice_kernel_gives_the_same_bits():
    """Both placements of the accept decisions run the same code: every output of tapout_verify is bit-identical,
    also when the two alternate on one context (the band list of a job record is emptied by whoever appends next)."""
    w = synth.scaled(synth.WORKLOADS["llama3"], B=24)
    gen, tp, rounds = make(w, rounds=(0, 4))
    bits = lambda t: t.cpu().view(torch.int32) if t.dtype == torch.float32 else t.cpu()
    for rnd in rounds:
        for arm in (None, random_arms(w.B, seed=5)):
            outs = []
            for fuse in (0, 1, 0, 1):
                tp.set_option("fuse_head", fuse)
                _, vf, _ = pu.gpu_round(tp, rnd, arm=arm)
                outs.append({k: bits(v) for k, v in vf.items()})
            for o in outs[1:]:
                assert o.keys() == outs[0].keys()
                for k in o:
                    assert torch.equal(o[k], outs[0][k]), k
    with pytest.raises(binding.TapoutError, match="fuse_head"):
        tp.set_option("fuse_head", 2)


# ---- degenerate rows --------------------------------------------------------------

def degenerate_round(dtype):
    B, K, V = 8, 3, 5000
    g = torch.Generator(device=DEV).manual_seed(77)
    d = (torch.randn(B, K, V, generator=g, device=DEV) * 2).to(dtype)
    t = (torch.randn(B, K + 1, V, generator=g, device=DEV) * 2).to(dtype)
    d[0] = 0.5                                   # uniform rows: H = ln V, every rule fires at once
    t[0] = 0.5
    d[1, :, 100:] = float("-inf")                # masked vocabulary
    t[1, :, 50:] = float("-inf")
    d[2, :, 7] = 40.0                            # one-hot-like rows: H ~ 0, p_top1 ~ 1
    t[2, :, 7] = 40.0
    d[3, :, 11] = 9.0; d[3, :, 4000] = 9.0       # exact tie at the top: margin 0, lowest index wins
    t[4] = d.new_tensor(0.0).expand(K + 1, V)    # flat target against a random draft
    t[5, :K] = d[5]                              # p == q: everything accepted, bonus from row K
    d[6, :, :] = -1e4; d[6, :, V - 1] = 0.0      # maximum at the last element
    t[6, :, :] = -1e4; t[6, :, 0] = 0.0
    tok = torch.randint(0, V, (B, K), generator=g, device=DEV, dtype=torch.int32)
    tok[1] = torch.randint(0, 50, (K,), generator=g, device=DEV, dtype=torch.int32)
    tok[2] = 7
    tok[6] = V - 1
    return dict(draft=d, target=t, draft_tok=tok,
                u_accept=torch.rand(B, K, generator=g, device=DEV), u_sample=torch.rand(B, generator=g, device=DEV),
                k_len=torch.full((B,), K, dtype=torch.int32, device=DEV),
                greedy=torch.tensor([0, 0, 0, 0, 0, 0, 0, 1], dtype=torch.uint8, device=DEV))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@FUSE
def test_degenerate_rows(dtype, fuse):
    rnd = degenerate_round(dtype)
    B, K, V = rnd["draft"].shape
    tp = binding.Tapout(B, K, V)
    tp.set_option("fuse_head", fuse)
    pu.check_round(tp, rnd)
    for a in range(3):
        pu.check_round(tp, rnd, arm=torch.full((B,), a, dtype=torch.int32, device=DEV))
    ds, vf, _ = pu.gpu_round(tp, rnd)
    assert float(ds["margin"][3, 0]) == 0.0 and int(ds["top1_id"][3, 0]) == 11
    assert int(vf["accept_len"][5]) == K
    assert abs(float(ds["entropy"][0, 0]) - np.log(V)) < 1e-4
    assert not ds["flags"].any() and not vf["flags"].any()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_scattered_masked_logits(dtype):
    """A third of the vocabulary masked with -inf at random positions, differently in draft and target: nearly every
    group of eight logits holds a masked one (the entropy sum then takes its clamped path), whole 16-byte vectors are
    masked, drafted tokens can have target probability zero, and the residual lives on a thinned support."""
    B, K, V = 5, 6, 40003
    g = torch.Generator(device=DEV).manual_seed(77)
    d = torch.randn(B, K, V, generator=g, device=DEV) * 2.5
    t = d[:, :, :] + torch.randn(B, K, V, generator=g, device=DEV)
    t = torch.cat([t, torch.randn(B, 1, V, generator=g, device=DEV) * 2.5], 1)
    d[torch.rand(B, K, V, generator=g, device=DEV) < 0.33] = float("-inf")
    t[torch.rand(B, K + 1, V, generator=g, device=DEV) < 0.33] = float("-inf")
    d[0, 0, 4096:8192] = float("-inf")                                   # a whole slice masked
    d, t = d.to(dtype), t.to(dtype)
    tok = torch.multinomial(torch.softmax(d.float().reshape(B * K, V), -1), 1, generator=g).reshape(B, K).to(torch.int32)
    rnd = dict(draft=d, target=t, draft_tok=tok,
               u_accept=torch.rand(B, K, generator=g, device=DEV), u_sample=torch.rand(B, generator=g, device=DEV),
               k_len=torch.full((B,), K, dtype=torch.int32, device=DEV), greedy=torch.zeros(B, dtype=torch.uint8, device=DEV))
    tp = binding.Tapout(B, K, V)
    for wgs, min_slice in ((4096, 4096), (65536, 256)):
        tp.set_option("wgs_target", wgs)
        tp.set_option("min_slice", min_slice)
        c = pu.check_round(tp, rnd)
        assert c["accept_flagged"] + c["icdf_flagged"] <= 1
        pu.check_round(tp, rnd, arm=random_arms(B))
    ds, vf, _ = pu.gpu_round(tp, rnd)
    assert not ds["flags"].any() and not vf["flags"].any()
    assert torch.isfinite(ds["entropy"]).all() and torch.isfinite(ds["logq_tok"]).all()


@pytest.mark.parametrize("seed", list(range(int(os.environ.get("TAPOUT_RANDOM_CONFIGS", "96")))))
def test_random_configurations(seed):
    """Shapes, dtypes, strides, lengths, masks, decoding modes and launch options drawn at random (seeded): whatever
    combination comes out must match the oracle."""
    rs = np.random.RandomState(1000 + seed)
    B, K = int(rs.randint(1, 10)), int(rs.randint(1, 13))
    V = int(rs.choice([rs.randint(2, 600), rs.randint(600, 9000), rs.randint(9000, 70000)]))
    dt_d, dt_t = (torch.float32, torch.bfloat16)[rs.randint(2)], (torch.float32, torch.bfloat16)[rs.randint(2)]
    pad_d, pad_t, off_d, off_t = (int(x) for x in rs.randint(0, 11, 4))
    sigma, noise = float(rs.uniform(0.5, 6.0)), float(rs.uniform(0.2, 2.5))
    g = torch.Generator(device=DEV).manual_seed(seed)
    wide_d = torch.randn(B, K, V + pad_d + off_d, generator=g, device=DEV) * sigma
    d32 = wide_d[:, :, off_d:off_d + V]
    wide_t = torch.randn(B, K + 1, V + pad_t + off_t, generator=g, device=DEV) * noise
    wide_t[:, :K, off_t:off_t + V] += d32
    wide_t[:, K] *= sigma / noise
    if rs.rand() < 0.4:                                                  # masked vocabulary tail or random holes
        if rs.rand() < 0.5:
            cut = int(rs.randint(1, V + 1))
            wide_d[:, :, off_d + cut:] = float("-inf"); wide_t[:, :, off_t + cut:] = float("-inf")
        else:
            wide_d[torch.rand(wide_d.shape, generator=g, device=DEV) < 0.2] = float("-inf")
    wide_d, wide_t = wide_d.to(dt_d), wide_t.to(dt_t)
    draft, target = wide_d[:, :, off_d:off_d + V], wide_t[:, :, off_t:off_t + V]
    q = torch.softmax(draft.float().reshape(B * K, V), -1)
    tok = torch.multinomial(q, 1, generator=g).reshape(B, K).to(torch.int32)
    greedy = torch.from_numpy((rs.rand(B) < 0.3).astype(np.uint8)).to(DEV)
    tok = torch.where(greedy.bool()[:, None], draft.float().argmax(-1).to(torch.int32), tok)
    k_len = torch.from_numpy(rs.randint(1, K + 1, B).astype(np.int32)).to(DEV)
    rnd = dict(draft=draft, target=target, draft_tok=tok, u_accept=torch.rand(B, K, generator=g, device=DEV),
               u_sample=torch.rand(B, generator=g, device=DEV), k_len=k_len, greedy=greedy)
    tp = binding.Tapout(B, K, V)
    tp.set_option("wgs_target", int(rs.choice([1, 64, 300, 4096, 65536])))
    tp.set_option("min_slice", int(rs.choice([256, 1024, 4096])))
    tp.set_option("fuse_head", int(rs.randint(-1, 2)))
    announce(f"random configuration {seed}: B={B} K={K} V={V} {dt_d}/{dt_t} offsets {off_d}/{off_t} greedy={greedy.cpu().tolist()} k_len={k_len.cpu().tolist()}")
    c = pu.check_round(tp, rnd)
    c2 = pu.check_round(tp, rnd, arm=random_arms(B, seed=seed))
    assert c["accept_flagged"] + c["icdf_flagged"] + c2["stop_flagged"] <= 2
    # the same round as one tapout_round call (its own launch order: see the library's "defer_epilogue" option)
    tp.set_option("defer_epilogue", int(rs.randint(0, 2)))
    c3 = pu.check_round_call(tp, rnd, random_arms(B, seed=seed), truncate=bool(seed & 1))
    assert c3["accept_flagged"] + c3["icdf_flagged"] <= 2


def force_slices(tp, rows, P, min_slice=256):
    """Launch options under which a pass over `rows` rows cuts every row into P slices (given V >= P * min_slice and
    rows shorter than P * slice_bytes)."""
    tp.set_option("min_slice", min_slice)
    tp.set_option("wgs_target", min(65536, rows * P))


def lane_round(B, K, V, dtype, seed, greedy_rows=(), sigma=3.0):
    rnd = random_round(B, K, V, dtype, seed=seed, sigma=sigma)
    g = torch.zeros(B, dtype=torch.uint8)
    g[list(greedy_rows)] = 1
    rnd["greedy"] = g.to(DEV)
    tok = rnd["draft_tok"]
    rnd["draft_tok"] = torch.where(rnd["greedy"].bool()[:, None], rnd["draft"].float().argmax(-1).to(torch.int32), tok)
    return rnd


@pytest.mark.parametrize("B,K,V,P", [
    (16, 16, 128256, 0),      # default options: 16 slices per row, 17 target rows > 256 / 16
    (8, 32, 65536, 0),        # default options, draft side: 16 slices, 32 rows
    (16, 20, 70001, 0),
    (3, 63, 4096, 8),         # 64 target rows x 8 slices = 512: the largest lane-merge shape
    (3, 42, 3100, 12),        # 12 slices in groups of 16 lanes with empty lanes; 43 x 16 = 688 > 512 -> staged; draft 42 x 16 too
    (5, 31, 4100, 16),        # 32 x 16 = 512 target rows on the lane path, second pass of every thread in use
    (4, 40, 2100, 5),         # 5 slices in groups of 8: rows 32..40 come from the second pass
    (2, 64, 1100, 4),         # K = 64: draft side on the lane path (64 x 4), target side (65 rows) staged
    (6, 17, 9000, 15),
])
@FUSE
def test_lane_merge_with_more_rows_than_one_stage_of_partials(B, K, V, P, fuse):
    """Per-sequence epilogues on the lane-parallel merge when the sequence has more rows than a staging buffer of
    256 partials holds at the slice count in use (K + 1 > 256 / slices): all rows are still one stage, row k stays
    with thread k.  Full-K (accept decisions far into the draft), greedy and sampled sequences, every stop rule,
    and flags raised at row 0."""
    announce(f"lane merge B={B} K={K} V={V} P={P} fuse_head={fuse}")
    rnd = lane_round(B, K, V, torch.bfloat16 if V > 60000 else torch.float32, seed=K * 1000 + P, greedy_rows=range(0, B, 3))
    tp = binding.Tapout(B, K, V)
    tp.set_option("fuse_head", fuse)
    if P:
        force_slices(tp, B * K, P)
    c = pu.check_round(tp, rnd)
    assert c["accept_flagged"] + c["icdf_flagged"] <= 1
    # a draft equal to the target is accepted to the end: the decisions of rows beyond 256 / slices count
    same = dict(rnd); same["target"] = torch.cat([rnd["draft"], rnd["target"][:, K:]], 1).contiguous()
    _, vf, _ = pu.gpu_round(tp, same)
    assert (vf["accept_len"] == K).all() and (vf["n_out"] == K + 1).all()
    pu.check_round(tp, same)
    # a sequence rejected only at its last position
    late = dict(same); late["u_accept"] = same["u_accept"].clone(); late["target"] = same["target"].clone()
    late["target"][:, K - 1] = rnd["target"][:, K - 1]
    late["u_accept"][:, K - 1] = 1.0 - 2.0 ** -24
    pu.check_round(tp, late)
    for a in range(3):
        c = pu.check_round(tp, rnd, arm=torch.full((B,), a, dtype=torch.int32, device=DEV))
        assert c["stop_flagged"] <= 1
    # bad inputs at row 0 and at the last row: the flags of every row reach the sequence's flag word
    bad = {k: (v.clone() if torch.is_tensor(v) else v) for k, v in rnd.items()}
    bad["draft_tok"][0, 0] = V                          # token out of range at row 0
    if B > 1:
        bad["target"][1, 0, 1] = float("nan")           # NaN in target row 0
    if B > 2:
        bad["draft"][2, K - 1, 0] = float("nan")        # NaN in the last draft row
        bad["draft_tok"][2, K - 1] = -1
    gds, gvf, _ = pu.gpu_round(tp, bad)
    ods, ovf, _ = pu.oracle_round(bad)
    assert gds["flags"].cpu().numpy().astype(np.uint32).tolist() == ods["flags"].tolist()
    assert gvf["flags"].cpu().numpy().astype(np.uint32).tolist() == ovf["flags"].tolist()
    assert ods["flags"][0] & orc.FLAG_BAD_TOKEN and ovf["flags"][0] & orc.FLAG_BAD_TOKEN
    flagged = ovf["flags"] != 0
    assert (gvf["accept_len"].cpu().numpy()[flagged] == ovf["accept_len"][flagged]).all()
    assert (gvf["out_tok"].cpu().numpy()[flagged] == ovf["out_tok"][flagged]).all()


@pytest.mark.parametrize("seed", list(range(int(os.environ.get("TAPOUT_RANDOM_LANE_SHAPES", "40")))))
def test_random_lane_merge_shapes(seed):
    """13 <= K <= 64 with 2 .. 16 slices per row forced through the launch options: every (group size, rows) pair of the
    lane-parallel merge, including rows in (256 / slices, 512 / group] that take each thread's second pass, and the
    shapes just beyond it that fall back to the staged merge."""
    rs = np.random.RandomState(3000 + seed)
    P = int(rs.randint(2, 17))
    K = int(rs.randint(13, 65))
    B = int(rs.randint(1, 5))
    V = int(P * 256 + rs.randint(0, 3000))
    dt = (torch.float32, torch.bfloat16)[rs.randint(2)]
    rnd = lane_round(B, K, V, dt, seed=seed, greedy_rows=[b for b in range(B) if rs.rand() < 0.3], sigma=float(rs.uniform(1.5, 6.0)))
    rnd["k_len"] = torch.from_numpy(np.where(rs.rand(B) < 0.5, K, rs.randint(1, K + 1, B)).astype(np.int32)).to(DEV)
    if rs.rand() < 0.5:                                   # p == q on a prefix: accept decisions deep into the draft
        keep = int(rs.randint(1, K + 1))
        rnd["target"] = rnd["target"].clone()
        rnd["target"][:, :keep] = rnd["draft"][:, :keep]
    if rs.rand() < 0.3:
        rnd["draft_tok"] = rnd["draft_tok"].clone()
        rnd["draft_tok"][0, 0] = -1 if rs.rand() < 0.5 else V
    tp = binding.Tapout(B, K, V)
    force_slices(tp, B * K, P)
    tp.set_option("fuse_head", int(rs.randint(-1, 2)))
    announce(f"random lane shape {seed}: B={B} K={K} V={V} P={P} {dt} k_len={rnd['k_len'].cpu().tolist()} greedy={rnd['greedy'].cpu().tolist()}")
    c = pu.check_round(tp, rnd)
    c2 = pu.check_round(tp, rnd, arm=random_arms(B, seed=seed))
    assert c["accept_flagged"] + c["icdf_flagged"] + c2["stop_flagged"] <= 2


@pytest.mark.parametrize("boost", [8.0, 1e-2, 1e-4])
def test_residual_with_tied_probability_ratios(boost):
    """target = draft except for a few boosted tokens: p/q is the same number for almost every token.  With a
    large boost the ratio is clearly below 1 there (fast path); with a tiny boost it sits inside the band in
    which the sign of p - q cannot be decided from binary32-grade normalisers, which must send the sampler
    down its exact path.  The drafted tokens avoid the boosted ones and u_accept is ~1, so position 0 is
    rejected and the final token is a residual draw."""
    B, K, V = 6, 3, 40000
    g = torch.Generator(device=DEV).manual_seed(int(boost * 1e5) + 1)
    d = (torch.randn(B, K, V, generator=g, device=DEV) * 2).float()
    t = torch.cat([d, torch.randn(B, 1, V, generator=g, device=DEV) * 2], 1).clone()
    hot = torch.randint(0, V, (B, 5), generator=g, device=DEV)
    for b in range(B):
        t[b, :, hot[b]] += boost
    tok = torch.randint(0, V, (B, K), generator=g, device=DEV, dtype=torch.int32)
    for b in range(B):
        clash = (tok[b][:, None] == hot[b][None, :]).any(1)
        tok[b][clash] = (tok[b][clash] + 7) % V
    rnd = dict(draft=d, target=t, draft_tok=tok,
               u_accept=torch.full((B, K), 1.0 - 2.0 ** -24, device=DEV), u_sample=torch.rand(B, generator=g, device=DEV),
               k_len=torch.full((B,), K, dtype=torch.int32, device=DEV), greedy=torch.zeros(B, dtype=torch.uint8, device=DEV))
    tp = binding.Tapout(B, K, V)
    c = pu.check_round(tp, rnd)
    ds, vf, _ = pu.gpu_round(tp, rnd)
    ok = vf["accept_len"].cpu() == 0
    assert ok.sum() >= B - c["accept_flagged"]                       # rejected at once unless the accept test itself was a near tie
    final = vf["out_tok"][:, 0].cpu()
    assert all(int(final[b]) in hot[b].cpu().tolist() for b in range(B) if ok[b])   # the residual lives on the boosted tokens


def test_residual_with_a_few_tokens_where_p_equals_q():
    """A few heavy tokens with p = q to within 1e-6: the sign of p - q there cannot be taken from binary32-grade
    normalisers; the sampler has to settle exactly these tokens with the exact normalisers (and only them)."""
    B, K, V = 5, 2, 30000
    g = torch.Generator().manual_seed(41)
    d = (torch.randn(B, K, V, generator=g) * 2).float()
    t = torch.cat([d + torch.randn(B, K, V, generator=g), torch.randn(B, 1, V, generator=g) * 2], 1).float()
    hot = torch.randint(0, V, (B, 4), generator=g)
    for b in range(B):
        d[b, 0, hot[b]] = d[b, 0].max() + torch.tensor([2.0, 1.5, 1.0, 0.5])        # heavy under q
        # p_h = q_h on the hot set H:  e^{t_h} = q_h R_p / (1 - Q_H),  R_p = sum of e^{t_j} over j outside H, Q_H = sum_H q_h
        q = torch.softmax(d[b, 0].double(), 0)
        mask = torch.ones(V, dtype=torch.bool); mask[hot[b]] = False
        ln_rp = torch.logsumexp(t[b, 0].double()[mask], 0)
        t[b, 0, hot[b]] = (q[hot[b]].log() + ln_rp - torch.log1p(-q[hot[b]].sum())).float()
        p = torch.softmax(t[b, 0].double(), 0); q = torch.softmax(d[b, 0].double(), 0)
        rel = ((p - q) / q)[hot[b]].abs()
        assert (rel < 5e-6).all() and (q[hot[b]] > 1e-3).all()
    tok = torch.randint(0, V, (B, K), generator=g, dtype=torch.int32)
    for b in range(B):
        clash = (tok[b][:, None] == hot[b][None, :]).any(1)
        tok[b][clash] = (tok[b][clash] + 11) % V
    rnd = dict(draft=d.to(DEV), target=t.to(DEV), draft_tok=tok.to(DEV),
               u_accept=torch.full((B, K), 1.0 - 2.0 ** -24, device=DEV), u_sample=torch.rand(B, generator=g).to(DEV),
               k_len=torch.full((B,), K, dtype=torch.int32, device=DEV), greedy=torch.zeros(B, dtype=torch.uint8, device=DEV))
    tp = binding.Tapout(B, K, V)
    c = pu.check_round(tp, rnd)
    assert c["icdf_flagged"] <= 1
    _, vf, _ = pu.gpu_round(tp, rnd)
    assert (vf["accept_len"].cpu() == 0).sum() >= B - c["accept_flagged"] - 1


@pytest.mark.parametrize("shift", [0.0, 70.0, -40.0, 55.0])
@FUSE
def test_bfloat16_final_token_table_and_its_limits(shift, fuse):
    """The final-token pass of bfloat16 row pairs takes exp(x) from a table of the bfloat16 values with 2^-12 <= |x| < 63.5.
    Rows full of what the table does not hold: exact zeros, +-0, magnitudes below 2^-12 (formed by a polynomial in a
    chunk of their own), logits at and below -63.5 (weigh nothing; -63.25 is the table's last entry), masked entries, a vocabulary that ends inside a
    slice; and whole rows shifted so that the row maximum leaves the table's range (+70, -40: such jobs compute their
    exponentials) or sits just inside it (+55).  Against the oracle, and against the same call with the table switched
    off ("exp_lookup" = 0): same tokens, same accepted lengths."""
    B, K, V = 6, 5, 2048 * 5 + 777
    g = torch.Generator(device=DEV).manual_seed(4242)
    d = torch.randn(B, K, V, generator=g, device=DEV) * 3.0
    t = torch.cat([d + torch.randn(B, K, V, generator=g, device=DEV) * 1.2, torch.randn(B, 1, V, generator=g, device=DEV) * 3.0], 1)
    for x in (d, t):
        r = torch.rand(x.shape, generator=g, device=DEV)
        x[r < 0.05] = 0.0
        x[(r >= 0.05) & (r < 0.08)] = -0.0
        x[(r >= 0.08) & (r < 0.14)] *= 1e-5                      # far below 2^-12
        x[(r >= 0.14) & (r < 0.16)] = 2.0 ** -12                 # the table's first entry
        x[(r >= 0.16) & (r < 0.18)] = -(2.0 ** -12) * (1 - 2.0 ** -8)   # the largest magnitude below it
        x[(r >= 0.18) & (r < 0.19)] = -63.75
        x[(r >= 0.19) & (r < 0.195)] = -63.5                     # the first magnitude beyond the table
        x[(r >= 0.195) & (r < 0.20)] = -63.25                    # the table's last entry
        x[(r >= 0.20) & (r < 0.22)] = -64.0
        x[(r >= 0.22) & (r < 0.24)] = -3.0e38
        x[(r >= 0.24) & (r < 0.27)] = float("-inf")
    d, t = (d + shift).to(torch.bfloat16), (t + shift).to(torch.bfloat16)
    gum = -torch.log(-torch.log(torch.rand(B, K, V, generator=g, device=DEV).clamp_min(1e-20)))
    tok = (d.float() + gum).argmax(-1).to(torch.int32)
    rnd = dict(draft=d, target=t, draft_tok=tok, u_accept=torch.rand(B, K, generator=g, device=DEV),
               u_sample=torch.rand(B, generator=g, device=DEV), k_len=torch.full((B,), K, dtype=torch.int32, device=DEV),
               greedy=torch.zeros(B, dtype=torch.uint8, device=DEV))
    rnd["u_accept"][0] = 0.0                                      # every token accepted: the draw comes from target row K alone
    rnd["u_accept"][1] = 1.0                                      # rejected at once: residual of row 0
    outs = {}
    for lookup in (1, 0):
        tp = binding.Tapout(B, K, V)
        tp.set_option("fuse_head", fuse)
        tp.set_option("exp_lookup", lookup)
        c = pu.check_round(tp, rnd)
        assert c["accept_flagged"] + c["icdf_flagged"] <= 1
        _, vf, _ = pu.gpu_round(tp, rnd)
        outs[lookup] = {k: v.cpu().clone() for k, v in vf.items()}
    for k in ("accept_len", "out_tok", "n_out", "flags"):
        assert torch.equal(outs[1][k], outs[0][k]), k


def random_round(B, K, V, dtype, seed, sigma=2.5, k_len=None):
    g = torch.Generator(device=DEV).manual_seed(seed)
    d = (torch.randn(B, K, V, generator=g, device=DEV) * sigma).to(dtype)
    t = torch.cat([d.float() + torch.randn(B, K, V, generator=g, device=DEV), torch.randn(B, 1, V, generator=g, device=DEV) * sigma], 1).to(dtype)
    gum = -torch.log(-torch.log(torch.rand(B, K, V, generator=g, device=DEV).clamp_min(1e-20)))
    tok = (d.float() + gum).argmax(-1).to(torch.int32)
    kl = torch.full((B,), K, dtype=torch.int32, device=DEV) if k_len is None else torch.tensor(k_len, dtype=torch.int32, device=DEV)
    return dict(draft=d, target=t, draft_tok=tok, u_accept=torch.rand(B, K, generator=g, device=DEV),
                u_sample=torch.rand(B, generator=g, device=DEV), k_len=kl, greedy=torch.zeros(B, dtype=torch.uint8, device=DEV))


@pytest.mark.parametrize("K,V,dtype", [(300, 600, torch.float32), (700, 20000, torch.bfloat16), (4096, 50, torch.bfloat16)])
@FUSE
def test_long_drafts(K, V, dtype, fuse):
    """More draft positions than a workgroup has threads, and more rows than one LDS stage of partials holds: the
    per-sequence kernels walk them in stages.  K = 4096 is the largest K a context accepts."""
    B = 2 if K < 4096 else 1
    rnd = random_round(B, K, V, dtype, seed=K, sigma=1.0, k_len=[K, K - 37][:B])
    tp = binding.Tapout(B, K, V)
    tp.set_option("fuse_head", fuse)
    arm = torch.tensor([1, 2][:B], dtype=torch.int32, device=DEV)
    c = pu.check_round(tp, rnd)                                          # full K: accept decisions far into the draft
    assert c["accept_flagged"] + c["icdf_flagged"] <= 1
    c = pu.check_round(tp, rnd, arm=arm)                                 # stop scan over K positions
    assert c["stop_flagged"] <= 1
    # a draft that equals the target is accepted to the end: accept_len = n_draft, bonus token from the last target row
    same = dict(rnd); same["target"] = torch.cat([rnd["draft"], rnd["target"][:, K:]], 1).contiguous()
    ds, vf, nd = pu.gpu_round(tp, same)
    assert torch.equal(vf["accept_len"], same["k_len"]) and torch.equal(vf["n_out"], same["k_len"] + 1)
    pu.check_round(tp, same)
    # the five-arm pool with carried state and token-level arms over a long draft
    tp5 = binding.Tapout(B, K, V, rules=FIVE_RULES, thresholds=FIVE_THRESHOLDS, token_level=True)
    arms = ((torch.arange(B)[:, None] * 3 + torch.arange(K)[None, :]) % 5).to(torch.int32).to(DEV)
    tp5.rule_state_set(prev_entropy=[1.0, float("nan")][:B] if B > 1 else [1.0])
    gds = tp5.draft_stats(rnd["draft"], draft_tok=rnd["draft_tok"], k_len=rnd["k_len"], arm=arms)
    st = orc.RuleState(B, FIVE_RULES, FIVE_THRESHOLDS)
    st.prev_entropy[:] = [1.0, np.nan][:B]
    ods = orc.draft_stats(pu.host_logits(rnd["draft"]), draft_tok=rnd["draft_tok"].cpu().numpy(), k_len=rnd["k_len"].cpu().numpy(),
                          arm=arms.cpu().numpy(), rules=FIVE_RULES, thresholds=FIVE_THRESHOLDS, prev_entropy=st.prev_entropy, lam=st.lam,
                          token_level=True, nthreads=16)
    live = np.arange(K)[None, :] < rnd["k_len"].cpu().numpy()[:, None]
    near = (ods["stop_margin"] <= pu.TAU) & live
    assert near.sum() <= 2
    assert (gds["stop_fired"].cpu().numpy()[live & ~near] == ods["stop_fired"][live & ~near]).all()
    ok = ~near.any(1)
    assert (gds["n_stop"].cpu().numpy()[ok] == ods["n_stop"][ok]).all()


def test_vocabulary_beyond_256_final_token_slices():
    """V = 600001 gives 293 slices of the final-token passes: more than the locate kernel's workgroup scan covers."""
    B, K, V = 3, 2, 600001
    rnd = random_round(B, K, V, torch.float32, seed=5, sigma=3.0)
    rnd["u_accept"][:] = 1.0 - 2.0 ** -24                                 # reject at once: residual draws ...
    rnd["u_accept"][2] = 0.0                                              # ... and one bonus-token draw from the last row
    rnd["u_sample"][:] = torch.tensor([0.0001, 0.9999, 0.5], device=DEV)
    tp = binding.Tapout(B, K, V, draft_sampling=True)
    c = pu.check_round(tp, rnd)
    assert c["icdf_flagged"] <= 1
    ds, vf, _ = pu.gpu_round(tp, rnd)
    assert vf["accept_len"].cpu().tolist()[2] == K
    # draft-token sampling walks the same kernels with one job per row
    u = torch.rand(B, K, generator=torch.Generator().manual_seed(3))
    o = tp.draft_stats(rnd["draft"], u_draft=u.to(DEV))
    osm = orc.draft_sample(pu.host_logits(rnd["draft"]), u.numpy(), nthreads=16)
    near = osm["icdf_margin"] <= pu.TAU_S
    assert (o["sampled_tok"].cpu().numpy()[~near] == osm["tok"][~near]).all()


@FUSE
def test_bad_inputs_set_flags_and_fall_back(fuse):
    rnd = degenerate_round(torch.float32)
    B, K, V = rnd["draft"].shape
    rnd["draft"][0, 1, 17] = float("nan")        # NaN in a draft row
    rnd["target"][1, 0, 3] = float("nan")        # NaN in a target row
    rnd["target"][2, 2, :] = float("-inf")       # target row without finite maximum
    rnd["draft_tok"][3, 0] = V                   # token out of range
    rnd["draft_tok"][4, 2] = -1
    n_draft = torch.full((B,), K, dtype=torch.int32, device=DEV)
    n_draft[5] = 0
    n_draft[6] = K + 1
    tp = binding.Tapout(B, K, V)
    tp.set_option("fuse_head", fuse)
    gds = tp.draft_stats(rnd["draft"], draft_tok=rnd["draft_tok"], k_len=rnd["k_len"])
    gvf = tp.verify(rnd["target"], rnd["draft"], gds["lse"], gds["logq_tok"], rnd["draft_tok"], n_draft,
                    rnd["u_accept"], rnd["u_sample"], greedy=rnd["greedy"])
    torch.cuda.synchronize()
    ods, ovf, _ = pu.oracle_round(rnd, n_draft=n_draft)
    assert gds["flags"].cpu().numpy().astype(np.uint32).tolist() == ods["flags"].tolist()
    assert ods["flags"].tolist()[:5] == [orc.FLAG_BAD_ROW, 0, 0, orc.FLAG_BAD_TOKEN, orc.FLAG_BAD_TOKEN]
    assert gvf["flags"].cpu().numpy().astype(np.uint32).tolist() == ovf["flags"].tolist()
    assert ovf["flags"].tolist()[1:7] == [orc.FLAG_BAD_ROW, orc.FLAG_BAD_ROW, orc.FLAG_BAD_TOKEN, orc.FLAG_BAD_TOKEN,
                                          orc.FLAG_BAD_NDRAFT, orc.FLAG_BAD_NDRAFT]
    assert gvf["accept_len"].cpu().tolist() == ovf["accept_len"].tolist()
    assert gvf["out_tok"].cpu().tolist() == ovf["out_tok"].tolist()
    assert gvf["n_out"].cpu().tolist() == ovf["n_out"].tolist()
    assert np.isnan(gds["entropy"][0, 1].item()) and np.isnan(gds["logq_tok"][3, 0].item())


# ---- full benchmark shapes, launch configuration of bench.py: every sequence of a round against the oracle ----

@pytest.mark.parametrize("name,n_seq", [("llama3", 64), ("zipf", 256), ("ragged", 512)])
def test_full_size_rounds_every_sequence(name, n_seq):
    w = synth.WORKLOADS[name]
    assert n_seq == w.B                     # the oracle takes a whole round of these sizes in a second or two on 16 threads
    announce(f"full size {w}")
    gen, tp, rounds = make(w, rounds=(3,))
    rnd = rounds[0]
    g = torch.Generator().manual_seed(w.index)
    seqs = torch.randperm(w.B, generator=g)[:n_seq].sort().values.tolist()
    c = pu.check_round(tp, rnd, seqs=seqs)
    announce(f"{name} full size, sequences {seqs}: near-tie counts {c}")
    assert c["sequences"] == w.B
    assert c["stop_flagged"] + c["accept_flagged"] + c["icdf_flagged"] <= max(2, w.B // 100)
    # properties that hold for every sequence at any size
    ds, vf, nd = pu.gpu_round(tp, rnd)
    m, n_out, out = vf["accept_len"].cpu(), vf["n_out"].cpu(), vf["out_tok"].cpu()
    k_len, tok = rnd["k_len"].cpu(), rnd["draft_tok"].cpu()
    assert ((0 <= m) & (m <= k_len)).all() and (n_out == m + 1).all()
    pos = torch.arange(w.K + 1)[None]
    assert (out[pos > m[:, None]] == -1).all()
    assert ((out >= 0) & (out < w.V))[pos <= m[:, None]].all()
    assert (out[:, :w.K][pos[:, :w.K] < m[:, None]] == tok[pos[:, :w.K] < m[:, None]]).all()
    live = pos[:, :w.K] < k_len[:, None]
    H, p1, p2, mg = (ds[k].cpu() for k in ("entropy", "p_top1", "p_top2", "margin"))
    assert (H[live] >= 0).all() and (H[live] <= np.log(w.V) + 1e-4).all()
    assert (p1[live] >= p2[live]).all() and (p1[live] <= 1.0).all() and (mg[live] >= 0).all()
    assert (p1[live] >= torch.exp(-H[live]) * (1 - 1e-5)).all()          # H >= -ln p_max
    # the accept decisions are a function of the returned log-probabilities and the uniforms
    lp, lq, ua = vf["logp_tok"].cpu().double(), ds["logq_tok"].cpu().double(), rnd["u_accept"].cpu().double()
    acc = ua < torch.exp(lp - lq)
    greedy = rnd["greedy"].cpu().bool()
    acc = torch.where(greedy[:, None], tok.long() == vf["target_top1"].cpu()[:, :w.K].long(), acc) & live
    first_rej = torch.where(acc, torch.full_like(pos[:, :w.K], w.K + 1), pos[:, :w.K]).min(1).values
    assert (torch.minimum(first_rej, k_len.long()) == m).all()


# ---- bandit -----------------------------------------------------------------------

@pytest.mark.parametrize("policy,reward", [(binding.UCB1, binding.REWARD_BLEND), (binding.TS_BETA, binding.REWARD_BLEND),
                                           (binding.UCB_TUNED, binding.REWARD_BLEND), (binding.TS_GAUSS, binding.REWARD_BLEND),
                                           (binding.UCB1, binding.REWARD_SIMPLE), (binding.UCB_TUNED, binding.REWARD_SIMPLE)])
@pytest.mark.parametrize("shared", [False, True])
def test_bandit_trajectory_matches_oracle(policy, reward, shared):
    B, K, A, rounds = 37, 8, 3, 300
    tp = binding.Tapout(B, K, 1000, policy=policy, shared_bandit=shared, reward=reward)
    ob = orc.Bandit(policy, 1 if shared else B, A, reward_kind=reward)
    needs_u = policy in (binding.TS_BETA, binding.TS_GAUSS)
    g = torch.Generator().manual_seed(5)
    for r in range(rounds):
        u = torch.rand(B, A, 48, generator=g)
        if r % 50 == 7:
            u[:, :, ::3] = 0.0                                           # zero uniforms hit the 2^-25 substitution
        arm = tp.bandit_select(B, u_ts=u.to(DEV) if needs_u else None)
        o_arm, _ = ob.select(B, u.numpy())
        assert arm.cpu().tolist() == o_arm.tolist(), f"round {r}"
        gamma = torch.randint(1, K + 1, (B,), generator=g, dtype=torch.int32)
        n = (torch.rand(B, generator=g) * gamma).floor().to(torch.int32) + 1
        m = (torch.rand(B, generator=g) * (n + 1) * (0.4 + 0.2 * arm.cpu())).floor().clamp(max=n).to(torch.int32)
        active = (torch.rand(B, generator=g) < 0.9).to(torch.uint8)
        tp.bandit_update(arm, m.to(DEV), n.to(DEV), gamma.to(DEV), active=active.to(DEV))
        ob.update(o_arm, m.numpy(), n.numpy(), gamma.numpy(), active=active.numpy())
    s, q, c = tp.bandit_get_state(moments=True)
    assert (c == ob.count).all()
    assert (s == ob.sum_r).all() and (q == ob.sum_r2).all()              # same fp64 operations in the same order
    # restore round trip
    tp2 = binding.Tapout(B, K, 1000, policy=policy, shared_bandit=shared, reward=reward)
    tp2.bandit_set_state(s, c, sum_r2=q)
    u = torch.rand(B, A, 48, generator=g)
    a1 = tp.bandit_select(B, u_ts=u.to(DEV) if needs_u else None)
    a2 = tp2.bandit_select(B, u_ts=u.to(DEV) if needs_u else None)
    assert torch.equal(a1, a2)
    # without the second moments the restored bandit takes every play of an arm to have had its mean reward
    tp2.bandit_set_state(s, c)
    _, q2, _ = tp2.bandit_get_state(moments=True)
    np.testing.assert_allclose(q2, np.where(c > 0, s * s / np.maximum(c, 1), 0.0), rtol=1e-15)


@pytest.mark.parametrize("policy", [binding.UCB1, binding.TS_BETA, binding.UCB_TUNED, binding.TS_GAUSS])
@pytest.mark.parametrize("kind", ["own", "shared", "token", "stateful"])
def test_update_and_next_select_in_one_call(policy, kind):
    """tapout_bandit_update_select against the two separate calls and against the oracle's bandit: the same arms in
    every round (also with the arm array updated in place), bit-equal state in the end; one launch for per-sequence
    bandits, the two kernels back to back for shared and token-level ones."""
    if kind == "token" and policy not in (binding.UCB1, binding.TS_BETA):
        pytest.skip("token-level bandits are UCB1 or Beta Thompson Sampling")
    B, K, rounds = 29, 6, 120
    rules = FIVE_RULES if kind == "stateful" else (0, 1, 2)
    thresholds = FIVE_THRESHOLDS if kind == "stateful" else (0.6, 0.8, 0.2)
    A = len(rules)
    kw = dict(policy=policy, rules=rules, thresholds=thresholds, shared_bandit=kind == "shared", token_level=kind == "token")
    tp_two, tp_one = binding.Tapout(B, K, 500, **kw), binding.Tapout(B, K, 500, **kw)
    ob = orc.Bandit(policy, 1 if kind == "shared" else B, A, positions=K if kind == "token" else 1)
    needs_u = policy in (binding.TS_BETA, binding.TS_GAUSS)
    g = torch.Generator().manual_seed(23)
    ushape = (B, K, A, 48) if kind == "token" else (B, A, 48)
    x = (torch.randn(B, K, 500, generator=g) * 3).to(DEV)
    u = torch.rand(ushape, generator=g)
    arm_one = tp_one.bandit_select(B, u_ts=u.to(DEV) if needs_u else None)
    for r in range(rounds):
        arm_two = tp_two.bandit_select(B, u_ts=u.to(DEV) if needs_u else None)
        o_arm, _ = ob.select(B, u.numpy())
        assert torch.equal(arm_one, arm_two) and (arm_two.cpu().numpy() == o_arm).all(), f"round {r}"
        if kind == "stateful":                                   # the update also advances the carried rule state
            tp_two.draft_stats(x, arm=arm_two)
            tp_one.draft_stats(x, arm=arm_one)
        n = torch.randint(1, K + 1, (B,), generator=g, dtype=torch.int32)
        m = (torch.rand(B, generator=g) * (n + 1)).floor().clamp(max=n).to(torch.int32)
        gamma = torch.full((B,), K, dtype=torch.int32)
        active = (torch.rand(B, generator=g) < 0.9).to(torch.uint8)
        u = torch.rand(ushape, generator=g)                      # the uniforms of the NEXT selection
        tp_two.bandit_update(arm_two, m.to(DEV), n.to(DEV), gamma.to(DEV), active=active.to(DEV))
        fl = torch.full((B,), 7, dtype=torch.int32, device=DEV)
        arm_one = tp_one.bandit_update_select(arm_one, m.to(DEV), n.to(DEV), gamma.to(DEV), active=active.to(DEV),
                                              u_ts=u.to(DEV) if needs_u else None, arm_out=arm_one if r & 1 else None, flags=fl)
        assert (fl.cpu() & ~8 == 0).all()
        ob.update(o_arm, m.numpy(), n.numpy(), gamma.numpy(), active=active.numpy())
    for a_, b_ in zip(tp_one.bandit_get_state(moments=True), tp_two.bandit_get_state(moments=True)):
        assert (a_.view(np.int64) == b_.view(np.int64)).all()
    s, q, c = tp_one.bandit_get_state(moments=True)
    assert (c == ob.count).all() and (s == ob.sum_r).all() and (q == ob.sum_r2).all()
    if kind == "stateful":
        s1, s2 = tp_one.rule_state_get(), tp_two.rule_state_get()
        for k_ in s1:
            assert (s1[k_].view(np.int32 if s1[k_].dtype == np.float32 else np.int64) ==
                    s2[k_].view(np.int32 if s2[k_].dtype == np.float32 else np.int64)).all(), k_
    with pytest.raises(binding.TapoutError, match="arm_out|required"):
        tp_one._check(tp_one._lib.tapout_bandit_update_select(tp_one._ctx, B, None, None, None, None, None, None, None, None, None))


@pytest.mark.parametrize("name", ["tiny", "small", "llama3"])
def test_closed_loop_rounds(name):
    """Algorithm 1 end to end over many rounds: select -> draft_stats -> verify -> update, bandit in the loop
    (llama3: the benchmark's own shape, all 64 sequences, stop rules truncating the drafts)."""
    w = synth.WORKLOADS[name]
    if name != "llama3":
        w = synth.scaled(w, sigma_draft=6.0) if name == "tiny" else synth.scaled(w, B=8, sigma_draft=7.0)
    n_rounds = {"tiny": 24, "small": 10, "llama3": 12}[name]
    policy = binding.UCB1
    gen = synth.RoundGenerator(w, DEV)
    tp = binding.Tapout(w.B, w.K, w.V, policy=policy)
    ob = orc.Bandit(policy, w.B, 3)
    flagged = 0
    for r in range(n_rounds):
        rnd = gen.round(r)
        arm = tp.bandit_select(w.B)
        o_arm, _ = ob.select(w.B)
        assert arm.cpu().tolist() == o_arm.tolist(), f"round {r}"
        gds, gvf, g_nd = pu.gpu_round(tp, rnd, arm=arm)
        ods, ovf, o_nd = pu.oracle_round(rnd, arm=arm)
        gvf = dict(gvf); gvf["n_draft_used"] = g_nd
        c = pu.compare_round(gds, gvf, ods, ovf, rnd["k_len"].cpu().numpy(), o_nd)
        flagged += c["stop_flagged"] + c["accept_flagged"]
        tp.bandit_update(arm, gvf["accept_len"], g_nd, rnd["k_len"])
        # the oracle's bandit follows the GPU's integer decisions so that a near-tie flip cannot cascade
        ob.update(o_arm, gvf["accept_len"].cpu().numpy(), g_nd.cpu().numpy(), rnd["k_len"].cpu().numpy())
    s, c = tp.bandit_get_state()
    assert (c == ob.count).all() and (s == ob.sum_r).all()
    assert flagged <= 2


FIVE_RULES = (binding.RULE_SVIP, binding.RULE_MAXCONF, binding.RULE_MARGIN, binding.RULE_SVIP_DIFF, binding.RULE_ADAEDL)
FIVE_THRESHOLDS = (0.6, 0.8, 0.2, 0.2, 0.4)


@pytest.mark.parametrize("name,shared", [("small", False), ("small", True), ("llama3", False)])
def test_stateful_rules_closed_loop(name, shared):
    """The paper's full pool of five arms (Table 1): SVIP-Difference and AdaEDL carry state from draft to draft
    (previous entropy; smoothed acceptance rate and threshold), so the loop is compared round by round,
    decisions and state."""
    w = synth.WORKLOADS[name]
    w = synth.scaled(w, B=8, sigma_draft=7.0) if name == "small" else synth.scaled(w, B=6, V=20000)
    ad = dict(gamma=0.5, alpha=0.6, beta1=0.5, beta2=0.9, eps=0.05, rate0=0.6)
    tp = binding.Tapout(w.B, w.K, w.V, rules=FIVE_RULES, thresholds=FIVE_THRESHOLDS, shared_bandit=shared, adaedl=ad)
    ob = orc.Bandit(orc.POLICY_UCB1, 1 if shared else w.B, 5)
    st = orc.RuleState(w.B, FIVE_RULES, FIVE_THRESHOLDS, ad_alpha=ad["alpha"], beta1=ad["beta1"], beta2=ad["beta2"],
                       eps=ad["eps"], rate0=ad["rate0"])
    gen = synth.RoundGenerator(w, DEV)
    g0 = tp.rule_state_get()
    assert np.isnan(g0["prev_entropy"]).all() and (g0["accept_rate"] == 0.6).all()
    assert (g0["lam"] == np.float32(FIVE_THRESHOLDS).astype(np.float64)[None, :]).all()
    flagged, fired_by_rule = 0, np.zeros(5, int)
    for r in range(14):
        rnd = gen.round(r)
        arm = tp.bandit_select(w.B)
        o_arm, _ = ob.select(w.B)
        assert arm.cpu().tolist() == o_arm.tolist(), f"round {r}"
        if r >= 10:                                               # late rounds: force the two stateful arms
            arm = torch.full_like(arm, 3 + (r & 1)); o_arm = arm.cpu().numpy()
        gds, gvf, g_nd = pu.gpu_round(tp, rnd, arm=arm)
        ods, ovf, o_nd = pu.oracle_round(rnd, arm=arm, rules=FIVE_RULES, thresholds=FIVE_THRESHOLDS,
                                         prev_entropy=st.prev_entropy, lam=st.lam, adaedl_gamma=ad["gamma"])
        gvf = dict(gvf); gvf["n_draft_used"] = g_nd
        c = pu.compare_round(gds, gvf, ods, ovf, rnd["k_len"].cpu().numpy(), o_nd)
        flagged += c["stop_flagged"] + c["accept_flagged"]
        for b in range(w.B):
            if ods["stop_fired"][b, ods["n_stop"][b] - 1]:
                fired_by_rule[FIVE_RULES[int(o_arm[b])]] += 1
        tp.bandit_update(arm, gvf["accept_len"], g_nd, rnd["k_len"])
        # the oracle's state follows the GPU's integer decisions so that a near-tie flip cannot cascade
        ob.update(o_arm, gvf["accept_len"].cpu().numpy(), g_nd.cpu().numpy(), rnd["k_len"].cpu().numpy())
        st.update(ods["entropy"], g_nd.cpu().numpy(), gvf["accept_len"].cpu().numpy())
        gs = tp.rule_state_get()
        pu.assert_stats_close("entropy", gs["prev_entropy"], st.prev_entropy)
        assert (gs["accept_rate"] == st.accept_rate).all(), f"round {r}"
        assert (gs["lam"] == st.lam).all(), f"round {r}"
    s, c = tp.bandit_get_state()
    assert (c == ob.count).all() and (s == ob.sum_r).all()
    assert flagged <= 2
    assert fired_by_rule[3] > 0 and fired_by_rule[4] > 0, fired_by_rule       # both stateful rules actually stopped drafts
    assert len(np.unique(st.lam[:, 4])) > 1 or st.lam[0, 4] != np.float32(0.4)  # and the AdaEDL threshold moved
    # restore: a fresh context given the state continues identically
    tp2 = binding.Tapout(w.B, w.K, w.V, rules=FIVE_RULES, thresholds=FIVE_THRESHOLDS, shared_bandit=shared, adaedl=ad)
    tp2.rule_state_set(**tp.rule_state_get())
    rnd = gen.round(99)
    arm = torch.full((w.B,), 3, dtype=torch.int32, device=DEV)
    arm[::2] = 4
    d1 = tp.draft_stats(rnd["draft"], draft_tok=rnd["draft_tok"], k_len=rnd["k_len"], arm=arm)
    d2 = tp2.draft_stats(rnd["draft"], draft_tok=rnd["draft_tok"], k_len=rnd["k_len"], arm=arm)
    assert torch.equal(d1["n_stop"], d2["n_stop"]) and torch.equal(d1["stop_fired"], d2["stop_fired"])


@pytest.mark.parametrize("seed", list(range(int(os.environ.get("TAPOUT_RANDOM_LOOPS", "16")))))
def test_random_closed_loops(seed):
    """Random arm pools (1-8 arms drawn from the five rules, thresholds jittered), policy, reward, bandit sharing,
    sequence- or token-level bandits and AdaEDL constants: six rounds of Algorithm 1 with the bandit and the carried
    rule state in the loop, compared round by round with the oracle (arms, signals, stop positions, accepted prefixes,
    tokens) and in the end state."""
    rs = np.random.RandomState(9000 + seed)
    B, K, V = int(rs.randint(1, 9)), int(rs.randint(2, 11)), int(rs.randint(200, 30000))
    n_arms = int(rs.randint(1, 9))
    rules = tuple(int(x) for x in rs.randint(0, 5, n_arms))
    base = {0: 0.6, 1: 0.8, 2: 0.2, 3: 0.2, 4: 0.4}
    thresholds = tuple(float(np.float32(base[r] * rs.uniform(0.6, 1.4))) for r in rules)
    token_level = bool(rs.rand() < 0.35)
    policy = int(rs.choice([binding.UCB1, binding.TS_BETA] if token_level
                           else [binding.UCB1, binding.TS_BETA, binding.UCB_TUNED, binding.TS_GAUSS]))
    reward = int(rs.choice([binding.REWARD_BLEND, binding.REWARD_SIMPLE]))
    shared = bool(rs.rand() < 0.3)
    alpha = float(rs.choice([0.0, 0.25, 0.5, 1.0]))
    ad = dict(gamma=float(rs.uniform(0.3, 0.8)), alpha=float(rs.uniform(0.4, 0.9)), beta1=float(rs.uniform(0.2, 0.9)),
              beta2=float(rs.uniform(0.5, 0.95)), eps=float(rs.uniform(0.005, 0.08)), rate0=float(rs.uniform(0.3, 0.9)),
              steer=int(seed & 1))                      # odd seeds: lambda follows r_t as Appendix A.1 prints the update
    announce(f"random loop {seed}: B={B} K={K} V={V} rules={rules} policy={policy} reward={reward} shared={shared} "
             f"alpha={alpha} token_level={token_level}")
    tp = binding.Tapout(B, K, V, policy=policy, rules=rules, thresholds=thresholds, alpha=alpha, shared_bandit=shared,
                        reward=reward, adaedl=ad, token_level=token_level)
    ob = orc.Bandit(policy, 1 if shared else B, n_arms, alpha=alpha, reward_kind=reward, positions=K if token_level else 1)
    st = orc.RuleState(B, rules, thresholds, ad_alpha=ad["alpha"], beta1=ad["beta1"], beta2=ad["beta2"], eps=ad["eps"], rate0=ad["rate0"],
                       steer_raw=bool(ad["steer"]))
    stateful = any(r in (binding.RULE_SVIP_DIFF, binding.RULE_ADAEDL) for r in rules)
    g = torch.Generator(device=DEV).manual_seed(seed)
    flagged = 0
    for r in range(6):
        rnd = random_round(B, K, V, (torch.float32, torch.bfloat16)[r & 1], seed=seed * 100 + r, sigma=float(rs.uniform(2.0, 8.0)),
                           k_len=[int(x) for x in rs.randint(1, K + 1, B)])
        u_ts = None
        if policy in (binding.TS_BETA, binding.TS_GAUSS):
            u_ts = torch.rand((B, K, n_arms, 48) if token_level else (B, n_arms, 48), generator=g, device=DEV)
        arm = tp.bandit_select(B, u_ts=u_ts)
        o_arm, _ = ob.select(B, None if u_ts is None else u_ts.cpu().numpy())
        assert (arm.cpu().numpy() == o_arm).all(), f"round {r}"
        gds = tp.draft_stats(rnd["draft"], draft_tok=rnd["draft_tok"], k_len=rnd["k_len"], arm=arm)
        g_nd = gds["n_stop"]
        gvf = dict(tp.verify(rnd["target"], rnd["draft"], gds["lse"], gds["logq_tok"], rnd["draft_tok"], g_nd,
                             rnd["u_accept"], rnd["u_sample"], greedy=rnd["greedy"]))
        ods = orc.draft_stats(pu.host_logits(rnd["draft"]), draft_tok=rnd["draft_tok"].cpu().numpy(), k_len=rnd["k_len"].cpu().numpy(),
                              arm=o_arm, rules=rules, thresholds=thresholds, prev_entropy=st.prev_entropy, lam=st.lam,
                              adaedl_gamma=ad["gamma"], token_level=token_level, nthreads=16)
        ovf = orc.verify(pu.host_logits(rnd["target"]), pu.host_logits(rnd["draft"]), ods["logq_tok"], rnd["draft_tok"].cpu().numpy(),
                         ods["n_stop"], rnd["u_accept"].cpu().numpy(), rnd["u_sample"].cpu().numpy(),
                         greedy=rnd["greedy"].cpu().numpy(), nthreads=16)
        gvf["n_draft_used"] = g_nd
        c = pu.compare_round(gds, gvf, ods, ovf, rnd["k_len"].cpu().numpy(), ods["n_stop"])
        flagged += c["stop_flagged"] + c["accept_flagged"] + c["icdf_flagged"]
        # the oracle's bandit and rule state follow the GPU's integer decisions so that a near-tie flip cannot cascade
        tp.bandit_update(arm, gvf["accept_len"], g_nd, rnd["k_len"])
        ob.update(o_arm, gvf["accept_len"].cpu().numpy(), g_nd.cpu().numpy(), rnd["k_len"].cpu().numpy())
        st.update(ods["entropy"], g_nd.cpu().numpy(), gvf["accept_len"].cpu().numpy())
        if stateful:
            gs = tp.rule_state_get()
            pu.assert_stats_close("entropy", gs["prev_entropy"], st.prev_entropy)
            assert (gs["accept_rate"] == st.accept_rate).all() and (gs["lam"] == st.lam).all(), f"round {r}"
    s_, q_, c_ = tp.bandit_get_state(moments=True)
    assert (c_ == ob.count).all() and (s_ == ob.sum_r).all() and (q_ == ob.sum_r2).all()
    assert flagged <= 2


def test_stateful_rules_on_closed_form_rows():
    """Rows uniform over n tokens (entropy ln n): the decisions are known in closed form (Table 1)."""
    V, sizes = 5000, [[2, 3, 4, 8], [8, 4, 3, 2], [3, 4, 8, 16]]
    x = torch.full((3, 4, V), float("-inf"))
    for b, row in enumerate(sizes):
        for k, n in enumerate(row):
            x[b, k, 100 * k + b: 100 * k + b + n] = 0.75
    for dt in (torch.float32, torch.bfloat16):
        tp = binding.Tapout(3, 4, V, rules=(binding.RULE_SVIP_DIFF, binding.RULE_ADAEDL), thresholds=(0.2, 0.3))
        xd = x.to(dt).to(DEV)
        arm = torch.zeros(3, dtype=torch.int32, device=DEV)
        o = tp.draft_stats(xd, arm=arm)
        assert o["stop_fired"].cpu().tolist() == [[0, 1, 0, 1], [0, 0, 0, 0], [0, 0, 1, 1]]
        assert o["n_stop"].cpu().tolist() == [2, 4, 3]
        # carried entropies: 0.3 makes the first step of sequence 0 a jump of 0.2848; NaN means no history
        tp.rule_state_set(prev_entropy=[0.3, float("nan"), 0.9])
        o = tp.draft_stats(xd, arm=arm)
        assert o["stop_fired"].cpu()[:, 0].tolist() == [1, 0, 0] and o["n_stop"].cpu().tolist() == [1, 4, 3]
        # AdaEDL, g = 0.5: 1 - sqrt(0.5 ln n) = 0.4113, 0.2588, 0.1674, -0.0197 for n = 2, 3, 4, 8
        o = tp.draft_stats(xd, arm=arm + 1)
        assert o["stop_fired"].cpu().tolist() == [[0, 1, 1, 1], [1, 1, 1, 0], [1, 1, 1, 1]]
        lam = np.zeros((3, 2)); lam[:, 1] = (0.1, 0.42, -1.0)
        tp.rule_state_set(lam=lam)
        o = tp.draft_stats(xd, arm=arm + 1)
        assert o["stop_fired"].cpu().tolist() == [[0, 0, 0, 1], [1, 1, 1, 1], [0, 0, 0, 0]]
        # the update takes the entropy of the last drafted row and moves lambda by (1 - beta2) eps
        n_draft = torch.tensor([2, 4, 1], dtype=torch.int32, device=DEV)
        acc = torch.tensor([2, 0, 1], dtype=torch.int32, device=DEV)
        tp.bandit_update(arm + 1, acc, n_draft, torch.full_like(n_draft, 4), active=torch.tensor([1, 1, 0], dtype=torch.uint8, device=DEV))
        st = tp.rule_state_get()
        np.testing.assert_allclose(st["prev_entropy"][:2], [math.log(3), math.log(2)], rtol=1e-5)
        assert st["prev_entropy"][2] == np.float32(0.9)                          # inactive: untouched
        assert st["accept_rate"].tolist() == [0.5 * 0.9 + 0.5 * 1.0, 0.5 * 0.9 + 0.5 * 0.0, 0.9]
        np.testing.assert_allclose(st["lam"][:, 1], [0.1 - 0.001, 0.42 + 0.001, -1.0], atol=1e-15)


@pytest.mark.parametrize("steer", [0, 1])
def test_adaedl_threshold_update_both_readings(steer, golden):
    """The four drafts of tests/golden/adaedl_update_two_readings.txt through tapout_bandit_update: lambda steered by
    the smoothed acceptance rate (default) or by the draft's own rate r_t (Appendix A.1 as printed), bit-equal to the
    oracle's state and equal to the hand-worked values."""
    rows = golden("adaedl_update_two_readings.txt")
    B, K = 3, 5
    ad = dict(alpha=0.87, beta1=0.5, beta2=0.9, eps=0.01, rate0=1.0, steer=steer)
    rules, th = (binding.RULE_ADAEDL, binding.RULE_SVIP), (0.4, 0.6)
    tp = binding.Tapout(B, K, 64, rules=rules, thresholds=th, adaedl=ad)
    st = orc.RuleState(B, rules, th, ad_alpha=0.87, beta1=0.5, beta2=0.9, eps=0.01, rate0=1.0, steer_raw=bool(steer))
    x = torch.randn(B, K, 64, generator=torch.Generator().manual_seed(1)).to(DEV)
    arm = torch.zeros(B, dtype=torch.int32, device=DEV)
    for row in rows:
        n_acc, n_dr = int(row[0]), int(row[1])
        ds = tp.draft_stats(x, arm=arm)
        m = torch.tensor([n_acc, n_dr, 0], dtype=torch.int32, device=DEV)     # sequence 0 follows the fixture
        n = torch.full((B,), n_dr, dtype=torch.int32, device=DEV)
        tp.bandit_update(arm, m, n, torch.full((B,), K, dtype=torch.int32, device=DEV))
        st.update(ds["entropy"].cpu().numpy(), n.cpu().numpy(), m.cpu().numpy())
        gs = tp.rule_state_get()
        assert (gs["lam"] == st.lam).all() and (gs["accept_rate"] == st.accept_rate).all()
        assert gs["accept_rate"][0] == pytest.approx(float(row[3]), rel=1e-14)
        assert gs["lam"][0, 0] == pytest.approx(float(row[7 - 2 * steer]) + (float(np.float32(0.4)) - 0.4), abs=1e-12)
        assert (gs["lam"][:, 1] == np.float32(0.6)).all()                      # not an AdaEDL arm: never moved
    with pytest.raises(binding.TapoutError, match="adaedl_steer"):
        binding.Tapout(B, K, 64, rules=rules, thresholds=th, adaedl=dict(steer=2))


def test_several_thresholds_per_rule():
    """Arm lists with several thresholds per rule (the paper's "more arms" ablation, Appendix A.2)."""
    w = synth.scaled(synth.WORKLOADS["llama3"], B=16, V=12000)
    rules = (0, 0, 0, 1, 1, 2, 2, 3)
    thresholds = (0.2, 0.4, 0.6, 0.5, 0.8, 0.1, 0.2, 0.1)
    tp = binding.Tapout(w.B, w.K, w.V, rules=rules, thresholds=thresholds)
    rnd = synth.RoundGenerator(w, DEV).round(3)
    arm = (torch.arange(w.B, dtype=torch.int32) % 8).to(DEV)
    gds = tp.draft_stats(rnd["draft"], draft_tok=rnd["draft_tok"], k_len=rnd["k_len"], arm=arm)
    ods, _, _ = pu.oracle_round(rnd, arm=arm, rules=rules, thresholds=thresholds)
    near = (ods["stop_margin"] <= pu.TAU).any(1)
    assert near.sum() <= 1
    assert (gds["n_stop"].cpu().numpy()[~near] == ods["n_stop"][~near]).all()
    assert len(set(ods["n_stop"].tolist())) > 1
    with pytest.raises(binding.TapoutError):
        binding.Tapout(4, 4, 100, rules=(0,) * 9, thresholds=(0.5,) * 9)
    with pytest.raises(binding.TapoutError):
        binding.Tapout(4, 4, 100, rules=(5,), thresholds=(0.5,))


@pytest.mark.parametrize("policy", [binding.UCB1, binding.TS_BETA])
@pytest.mark.parametrize("shared", [False, True])
def test_token_level_bandit_trajectory_matches_oracle(policy, shared):
    """One bandit per draft position, binary rewards up to the first rejection (Sections 3.1, 3.2)."""
    B, K, A, rounds = 21, 6, 3, 200
    tp = binding.Tapout(B, K, 1000, policy=policy, shared_bandit=shared, token_level=True)
    ob = orc.Bandit(policy, 1 if shared else B, A, positions=K)
    g = torch.Generator().manual_seed(17)
    for r in range(rounds):
        u = torch.rand(B, K, A, 48, generator=g)
        if r % 40 == 3:
            u[:, :, :, ::3] = 0.0
        fl = torch.full((B,), 7, dtype=torch.int32, device=DEV)
        arm = tp.bandit_select(B, u_ts=u.to(DEV) if policy == binding.TS_BETA else None, flags=fl)
        o_arm, o_fl = ob.select(B, u.numpy())
        assert arm.shape == (B, K) and (arm.cpu().numpy() == o_arm).all(), f"round {r}"
        assert (fl.cpu().numpy().astype(np.uint32) == o_fl).all()
        n = torch.randint(1, K + 1, (B,), generator=g, dtype=torch.int32)
        m = (torch.rand(B, generator=g) * (n + 1)).floor().clamp(max=n).to(torch.int32)
        active = (torch.rand(B, generator=g) < 0.9).to(torch.uint8)
        gamma = torch.full((B,), K, dtype=torch.int32)
        tp.bandit_update(arm, m.to(DEV), n.to(DEV), gamma.to(DEV), active=active.to(DEV))
        ob.update(o_arm, m.numpy(), n.numpy(), gamma.numpy(), active=active.numpy())
    s, q, c = tp.bandit_get_state(moments=True)
    assert s.shape == ob.sum_r.shape
    assert (c == ob.count).all() and (s == ob.sum_r).all() and (q == ob.sum_r2).all()
    assert c[:, K - 1].sum() < c[:, 0].sum()                            # late positions are played less often
    tp2 = binding.Tapout(B, K, 1000, policy=policy, shared_bandit=shared, token_level=True)
    tp2.bandit_set_state(s, c, sum_r2=q)
    u = torch.rand(B, K, A, 48, generator=g).to(DEV)
    assert torch.equal(tp.bandit_select(B, u_ts=u if policy == binding.TS_BETA else None),
                       tp2.bandit_select(B, u_ts=u if policy == binding.TS_BETA else None))


def test_token_level_closed_loop():
    """Algorithm 1 with token-level bandits over the five-arm pool: the rule of step k is the arm of position k."""
    w = synth.scaled(synth.WORKLOADS["llama3"], B=6, V=20000)
    tp = binding.Tapout(w.B, w.K, w.V, rules=FIVE_RULES, thresholds=FIVE_THRESHOLDS, token_level=True)
    ob = orc.Bandit(orc.POLICY_UCB1, w.B, 5, positions=w.K)
    st = orc.RuleState(w.B, FIVE_RULES, FIVE_THRESHOLDS)
    gen = synth.RoundGenerator(w, DEV)
    flagged, n_stops = 0, set()
    for r in range(12):
        rnd = gen.round(r)
        arm = tp.bandit_select(w.B)
        o_arm, _ = ob.select(w.B)
        assert (arm.cpu().numpy() == o_arm).all(), f"round {r}"
        if r >= 7:                                               # mixed arms along the draft, every rule somewhere
            arm = ((torch.arange(w.B)[:, None] + torch.arange(w.K)[None, :] + r) % 5).to(torch.int32).to(DEV)
            o_arm = arm.cpu().numpy()
        gds = tp.draft_stats(rnd["draft"], draft_tok=rnd["draft_tok"], k_len=rnd["k_len"], arm=arm)
        g_nd = gds["n_stop"]
        gvf = tp.verify(rnd["target"], rnd["draft"], gds["lse"], gds["logq_tok"], rnd["draft_tok"], g_nd,
                        rnd["u_accept"], rnd["u_sample"], greedy=rnd["greedy"])
        ods = orc.draft_stats(pu.host_logits(rnd["draft"]), draft_tok=rnd["draft_tok"].cpu().numpy(), k_len=rnd["k_len"].cpu().numpy(),
                              arm=o_arm, rules=FIVE_RULES, thresholds=FIVE_THRESHOLDS, prev_entropy=st.prev_entropy, lam=st.lam,
                              token_level=True, nthreads=16)
        ovf = orc.verify(pu.host_logits(rnd["target"]), pu.host_logits(rnd["draft"]), ods["logq_tok"], rnd["draft_tok"].cpu().numpy(),
                         ods["n_stop"], rnd["u_accept"].cpu().numpy(), rnd["u_sample"].cpu().numpy(),
                         greedy=rnd["greedy"].cpu().numpy(), nthreads=16)
        gvf = dict(gvf); gvf["n_draft_used"] = g_nd
        c = pu.compare_round(gds, gvf, ods, ovf, rnd["k_len"].cpu().numpy(), ods["n_stop"])
        flagged += c["stop_flagged"] + c["accept_flagged"]
        n_stops |= set(ods["n_stop"].tolist())
        tp.bandit_update(arm, gvf["accept_len"], g_nd, rnd["k_len"])
        ob.update(o_arm, gvf["accept_len"].cpu().numpy(), g_nd.cpu().numpy(), rnd["k_len"].cpu().numpy())
        st.update(ods["entropy"], g_nd.cpu().numpy(), gvf["accept_len"].cpu().numpy())
        gs = tp.rule_state_get()
        pu.assert_stats_close("entropy", gs["prev_entropy"], st.prev_entropy)
        assert (gs["accept_rate"] == st.accept_rate).all() and (gs["lam"] == st.lam).all()
    s, c = tp.bandit_get_state()
    assert (c == ob.count).all() and (s == ob.sum_r).all()
    assert flagged <= 2 and len(n_stops) >= 3


# ---- draft-token sampling inside tapout_draft_stats ---------------------------------------------

@pytest.mark.parametrize("name", ["tiny", "small", "ragged"])
def test_draft_token_sampling_matches_oracle(name):
    w = synth.WORKLOADS[name]
    if name == "small":
        w = synth.scaled(w, B=8)
    if name == "ragged":
        w = synth.scaled(w, B=6, V=70001)                         # odd V: ragged last slice, misaligned rows
    rnd = synth.RoundGenerator(w, DEV).round(2)
    tp = binding.Tapout(w.B, w.K, w.V, draft_sampling=True)
    g = torch.Generator().manual_seed(77)
    u = torch.rand(w.B, w.K, generator=g)
    u[0, 0] = 0.0
    u[-1, -1] = float(np.nextafter(np.float32(1.0), np.float32(0.0)))
    arm = (torch.arange(w.B, dtype=torch.int32) % 3).to(DEV)
    gds = tp.draft_stats(rnd["draft"], k_len=rnd["k_len"], arm=arm, u_draft=u.to(DEV))
    k_len = rnd["k_len"].cpu().numpy()
    live = np.arange(w.K)[None, :] < k_len[:, None]
    osm = orc.draft_sample(pu.host_logits(rnd["draft"]), u.numpy(), k_len=k_len, nthreads=16)
    g_tok = gds["sampled_tok"].cpu().numpy()
    near = osm["icdf_margin"] <= pu.TAU_S
    assert near.sum() <= 1
    assert (g_tok[live & ~near] == osm["tok"][live & ~near]).all()
    assert (g_tok[~live] == -1).all()                               # rows beyond k_len untouched
    # log q of the sampled token and everything else as with caller-supplied tokens
    ods = orc.draft_stats(pu.host_logits(rnd["draft"]), draft_tok=np.where(live, g_tok, 0), k_len=k_len, arm=arm.cpu().numpy(), nthreads=16)
    for key in pu.STAT_KEYS:
        pu.assert_stats_close(key, gds[key].cpu().numpy(), ods[key], live)
    gd2 = tp.draft_stats(rnd["draft"], draft_tok=gds["sampled_tok"].clamp(min=0), k_len=rnd["k_len"], arm=arm)
    assert torch.equal(gd2["n_stop"], gds["n_stop"])
    assert torch.equal(gd2["logq_tok"][torch.from_numpy(live).to(DEV)], gds["logq_tok"][torch.from_numpy(live).to(DEV)])


@pytest.mark.parametrize("seed", list(range(int(os.environ.get("TAPOUT_RANDOM_SAMPLINGS", "12")))))
def test_random_draft_token_sampling(seed):
    """Draft tokens drawn by the library on random shapes, row offsets, lengths, masks and slice counts: the tokens
    are the oracle's inverse-CDF draws, and the round that follows with them matches the oracle as well."""
    rs = np.random.RandomState(7000 + seed)
    B, K = int(rs.randint(1, 8)), int(rs.randint(1, 10))
    V = int(rs.choice([rs.randint(2, 500), rs.randint(500, 9000), rs.randint(9000, 60000)]))
    dt = (torch.float32, torch.bfloat16)[rs.randint(2)]
    off = int(rs.randint(0, 9))
    g = torch.Generator(device=DEV).manual_seed(seed)
    wide = torch.randn(B, K, V + off + 3, generator=g, device=DEV) * float(rs.uniform(1.0, 6.0))
    if rs.rand() < 0.4:
        wide[torch.rand(wide.shape, generator=g, device=DEV) < 0.3] = float("-inf")
        wide[:, :, off] = 0.5                                             # every row keeps a finite logit
    draft = wide.to(dt)[:, :, off:off + V]
    target = torch.cat([draft.float() + torch.randn(B, K, V, generator=g, device=DEV), torch.randn(B, 1, V, generator=g, device=DEV)], 1).to(dt)
    k_len = rs.randint(1, K + 1, B).astype(np.int32)
    u = torch.rand(B, K, generator=g, device=DEV)
    tp = binding.Tapout(B, K, V, draft_sampling=True)
    tp.set_option("wgs_target", int(rs.choice([1, 64, 4096, 65536])))
    tp.set_option("min_slice", int(rs.choice([256, 4096])))
    announce(f"random sampling {seed}: B={B} K={K} V={V} {dt} offset {off} k_len={k_len.tolist()}")
    kl = torch.from_numpy(k_len).to(DEV)
    arm = random_arms(B, seed=seed)
    gds = tp.draft_stats(draft, k_len=kl, arm=arm, u_draft=u)
    live = np.arange(K)[None, :] < k_len[:, None]
    osm = orc.draft_sample(pu.host_logits(draft), u.cpu().numpy(), k_len=k_len, nthreads=16)
    g_tok = gds["sampled_tok"].cpu().numpy()
    near = (osm["icdf_margin"] <= pu.TAU_S) & live
    assert near.sum() <= 1
    assert (g_tok[live & ~near] == osm["tok"][live & ~near]).all()
    assert (g_tok[~live] == -1).all()
    if not near.any():
        rnd = dict(draft=draft, target=target, draft_tok=gds["sampled_tok"].clamp(min=0), k_len=kl,
                   u_accept=torch.rand(B, K, generator=g, device=DEV), u_sample=torch.rand(B, generator=g, device=DEV),
                   greedy=torch.zeros(B, dtype=torch.uint8, device=DEV))
        tp2 = binding.Tapout(B, K, V)
        pu.check_round(tp2, rnd, arm=arm)


def test_draft_token_sampling_with_more_than_65535_rows():
    """B * K = 65600 draft rows: one final-token job per row is more than one grid dimension holds, the slice kernel's
    jobs spread over two of them."""
    B, K, V = 4100, 16, 300
    g = torch.Generator(device=DEV).manual_seed(11)
    draft = torch.randn(B, K, V, generator=g, device=DEV) * 2.0
    u = torch.rand(B, K, generator=g, device=DEV)
    k_len = torch.randint(1, K + 1, (B,), generator=g, device=DEV, dtype=torch.int32)
    k_len[-8:] = K                                                   # every job beyond the first 65535 is live
    tp = binding.Tapout(B, K, V, draft_sampling=True)
    o = tp.draft_stats(draft, k_len=k_len, u_draft=u)
    torch.cuda.synchronize()
    osm = orc.draft_sample(pu.host_logits(draft), u.cpu().numpy(), k_len=k_len.cpu().numpy(), nthreads=16)
    live = np.arange(K)[None, :] < k_len.cpu().numpy()[:, None]
    near = (osm["icdf_margin"] <= pu.TAU_S) & live
    assert near.sum() <= 2
    g_tok = o["sampled_tok"].cpu().numpy()
    assert (g_tok[live & ~near] == osm["tok"][live & ~near]).all()
    assert (g_tok[~live] == -1).all()
    assert live.sum() > 30000 and live.reshape(-1)[65535:].sum() > 30         # jobs beyond the first grid dimension were live
    ods = orc.draft_stats(pu.host_logits(draft), draft_tok=np.where(live, g_tok, 0), k_len=k_len.cpu().numpy(), nthreads=16)
    pu.assert_stats_close("logq_tok", o["logq_tok"].cpu().numpy(), ods["logq_tok"], live & ~near)


def test_draft_token_sampling_law_edges_and_bad_rows():
    V = 6000
    x = torch.full((3, 2, V), float("-inf"))
    x[0, :, 1000:1010] = 1.5                                        # uniform over 10 tokens: token = 1000 + floor(10 u)
    x[1, 0, :] = torch.randn(V) * 2; x[1, 1, :] = x[1, 0, :]
    x[2, 0, :] = 0.0; x[2, 0, 17] = float("nan")                    # bad row
    x[2, 1, :] = float("-inf")                                      # no finite maximum
    tp = binding.Tapout(3, 2, V, draft_sampling=True)
    with pytest.raises(binding.TapoutError):                        # a context without the scratch for it refuses
        binding.Tapout(3, 2, V).draft_stats(x.to(DEV), u_draft=torch.zeros(3, 2, device=DEV))
    for dt in (torch.float32, torch.bfloat16):
        u = torch.tensor([[0.31, 0.99], [0.0, 0.999999], [0.5, 0.5]])
        o = tp.draft_stats(x.to(dt).to(DEV), u_draft=u.to(DEV))
        tok = o["sampled_tok"].cpu()
        assert tok[0].tolist() == [1003, 1009]
        row = x[1, 0].to(dt).double()
        p = torch.softmax(row, 0)
        c = torch.cumsum(p, 0)
        assert tok[1, 0] == int((c > 0).nonzero()[0])               # u = 0: the first token with positive mass
        assert abs(float(c[tok[1, 1]]) - 0.999999) < 1e-3 and float(c[tok[1, 1]]) > 0.999998
        assert tok[2].tolist() == [-1, -1]
        fl = o["flags"].cpu().tolist()
        assert fl[0] == 0 and fl[1] == 0 and fl[2] == (binding.FLAG_BAD_ROW | binding.FLAG_BAD_TOKEN)
        assert torch.isnan(o["logq_tok"][2]).all()
    with pytest.raises(binding.TapoutError):
        tp.draft_stats(x.to(DEV), draft_tok=torch.zeros(3, 2, dtype=torch.int32, device=DEV), u_draft=u.to(DEV))


# ---- vocabulary-sharded entry points --------------------------------------------------------------

@pytest.mark.parametrize("name,G", [("small", 4), ("ragged", 3), ("llama3", 8)])
def test_vocabulary_sharded_draft_stats_match_oracle(name, G):
    """Each "GPU" reduces its column slice of every row to one 32-byte record; the merged records must give what the
    oracle computes on the unsplit rows (signals, argmax, log q(tok), stop position)."""
    w = synth.WORKLOADS[name]
    w = {"small": synth.scaled(w, B=8), "ragged": synth.scaled(w, B=6, V=70001), "llama3": synth.scaled(w, B=4)}[name]
    rnd = synth.RoundGenerator(w, DEV).round(1)
    B, K, V = w.B, w.K, w.V
    tp = binding.Tapout(B, K, V)
    edges = [round(g * V / G) for g in range(G + 1)]
    if name == "ragged":
        edges[1] += 3                                                      # shards of unequal, odd sizes
    recs = []
    for g in range(G):
        sl = rnd["draft"][:, :, edges[g]:edges[g + 1]]                    # a strided view: rows keep the full-row stride
        recs.append(tp.shard_stats(sl, edges[g], length=rnd["k_len"], rows_mode=0, tok=rnd["draft_tok"]).clone())
    stats = torch.stack(recs)
    arm = (torch.arange(B, dtype=torch.int32) % 3).to(DEV)
    gds = tp.draft_stats_sharded(stats, B, K, V, draft_tok=rnd["draft_tok"], k_len=rnd["k_len"], arm=arm)
    ods, _, _ = pu.oracle_round(rnd, arm=arm)
    k_len = rnd["k_len"].cpu().numpy()
    live = np.arange(K)[None, :] < k_len[:, None]
    for key in pu.STAT_KEYS:
        pu.assert_stats_close(key, gds[key].cpu().numpy(), ods[key], live)
    assert (gds["top1_id"].cpu().numpy()[live] == ods["top1_id"][live]).all()
    near = ((ods["stop_margin"] <= pu.TAU) & live).any(1)
    assert near.sum() <= 1
    assert (gds["n_stop"].cpu().numpy()[~near] == ods["n_stop"][~near]).all()
    assert (gds["flags"].cpu().numpy().astype(np.uint32) == ods["flags"]).all()
    # and the unsplit library call agrees with the sharded one to rounding
    one = tp.draft_stats(rnd["draft"], draft_tok=rnd["draft_tok"], k_len=rnd["k_len"], arm=arm)
    for key in pu.STAT_KEYS:
        pu.assert_stats_close(key, gds[key].cpu().numpy(), one[key].cpu().numpy(), live, tau=2e-6)


@pytest.mark.parametrize("name,G", [("small", 4), ("ragged", 3)])
def test_vocabulary_sharded_accept_step_matches_oracle(name, G):
    """Target rows through shard records: log p(tok), accept decisions, accepted prefix, greedy final tokens."""
    w = synth.WORKLOADS[name]
    w = synth.scaled(w, B=8) if name == "small" else synth.scaled(w, B=8, V=70001)
    rnd = synth.RoundGenerator(w, DEV).round(2)
    B, K, V = w.B, w.K, w.V
    tp = binding.Tapout(B, K, V)
    ods, ovf, nd = pu.oracle_round(rnd)                                   # full-K: n_draft = k_len
    n_draft = rnd["k_len"]
    edges = [round(g * V / G) for g in range(G + 1)]
    recs = torch.stack([tp.shard_stats(rnd["target"][:, :, edges[g]:edges[g + 1]], edges[g], length=n_draft, rows_mode=1,
                                       tok=rnd["draft_tok"]).clone() for g in range(G)])
    gds = tp.draft_stats(rnd["draft"], draft_tok=rnd["draft_tok"], k_len=rnd["k_len"])
    gvf = tp.verify_accept_sharded(recs, B, K, V, gds["logq_tok"], rnd["draft_tok"], n_draft, rnd["u_accept"], greedy=rnd["greedy"])
    used = np.arange(K)[None, :] < nd[:, None]
    near = ((ovf["accept_margin"] <= pu.TAU) & used).any(1)
    assert near.sum() <= 1
    ok = ~near
    g_len = gvf["accept_len"].cpu().numpy()
    assert (g_len[ok] == ovf["accept_len"][ok]).all()
    rows = np.arange(K + 1)[None, :] <= nd[:, None]
    pu.assert_stats_close("target_lse", gvf["target_lse"].cpu().numpy(), ovf["target_lse"], rows)
    pu.assert_stats_close("logp_tok", gvf["logp_tok"].cpu().numpy(), ovf["logp_tok"], used)
    assert (gvf["target_top1"].cpu().numpy()[rows] == ovf["target_top1"][rows]).all()
    g_out = gvf["out_tok"].cpu().numpy()
    greedy = rnd["greedy"].cpu().numpy().astype(bool)
    for b in np.nonzero(ok)[0]:
        m = ovf["accept_len"][b]
        assert (g_out[b, :m] == ovf["out_tok"][b, :m]).all()
        assert g_out[b, m] == (ovf["out_tok"][b, m] if greedy[b] else -1)       # sampled sequences: final token not drawn here
        assert (g_out[b, m + 1:] == -1).all()
    assert (gvf["n_out"].cpu().numpy()[ok] == ovf["n_out"][ok]).all()
    # the unsplit call takes the same decisions
    one = tp.verify(rnd["target"], rnd["draft"], gds["lse"], gds["logq_tok"], rnd["draft_tok"], n_draft, rnd["u_accept"],
                    rnd["u_sample"], greedy=rnd["greedy"])
    assert (one["accept_len"].cpu().numpy()[ok] == g_len[ok]).all()


def sharded_round(rnd, G, V, edges=None):
    """A whole verification over G emulated vocabulary shards (one context each, exchanges done with torch.stack).
    Returns accept_len, out_tok and how many sequences needed the second (exact-mass) exchange."""
    B, K = rnd["draft_tok"].shape
    edges = edges or [round(g * V / G) for g in range(G + 1)]
    tps = [binding.Tapout(B, K, edges[g + 1] - edges[g]) for g in range(G)]
    dsl = [rnd["draft"][:, :, edges[g]:edges[g + 1]] for g in range(G)]
    tsl = [rnd["target"][:, :, edges[g]:edges[g + 1]] for g in range(G)]
    n_draft = rnd["k_len"]
    drec = torch.stack([tps[g].shard_stats(dsl[g], edges[g], length=rnd["k_len"], tok=rnd["draft_tok"]).clone() for g in range(G)])
    trec = torch.stack([tps[g].shard_stats(tsl[g], edges[g], length=n_draft, rows_mode=1, tok=rnd["draft_tok"]).clone() for g in range(G)])
    gds = tps[0].draft_stats_sharded(drec, B, K, V, draft_tok=rnd["draft_tok"], k_len=rnd["k_len"])
    gvf = tps[0].verify_accept_sharded(trec, B, K, V, gds["logq_tok"], rnd["draft_tok"], n_draft, rnd["u_accept"],
                                       greedy=rnd["greedy"], draft_lse=gds["lse"])
    jobs = gvf["final_jobs"]
    sums_all = torch.stack([tps[g].shard_final_sums(tsl[g], dsl[g], jobs) for g in range(G)])
    res = [tps[g].shard_final_token(tsl[g], dsl[g], edges[g], G, g, jobs, sums_all, rnd["u_sample"]) for g in range(G)]
    need = torch.stack([r[2] for r in res])
    assert (need == need[0]).all()                                   # every shard reaches the same verdict
    n_second = int(need[0].sum())
    if n_second:
        exact_all = torch.stack([r[1] for r in res]).nan_to_num(0.0)
        res = [tps[g].shard_final_token(tsl[g], dsl[g], edges[g], G, g, jobs, sums_all, rnd["u_sample"], exact_all=exact_all)
               for g in range(G)]
        assert not torch.stack([r[2] for r in res]).any()
    toks = torch.stack([r[0] for r in res])                          # [G, B]: one shard answers, the others say -1
    assert ((toks >= 0).sum(0) <= 1).all()
    final = toks.max(0).values
    out = gvf["out_tok"].clone()
    m = gvf["accept_len"].long()
    idx = torch.arange(B, device=out.device)
    sampled = out[idx, m] < 0
    assert torch.equal(sampled, final >= 0)
    out[idx[sampled], m[sampled]] = final[sampled]
    return gvf["accept_len"], out, n_second


@pytest.mark.parametrize("name,G", [("small", 4), ("ragged", 3), ("llama3", 8)])
def test_vocabulary_sharded_final_token_matches_oracle(name, G):
    w = synth.WORKLOADS[name]
    w = {"small": synth.scaled(w, B=8), "ragged": synth.scaled(w, B=8, V=70001), "llama3": synth.scaled(w, B=6)}[name]
    rnd = synth.RoundGenerator(w, DEV).round(4)
    acc, out, _ = sharded_round(rnd, G, w.V)
    ods, ovf, nd = pu.oracle_round(rnd)
    used = np.arange(w.K)[None, :] < nd[:, None]
    ok = ~((ovf["accept_margin"] <= pu.TAU) & used).any(1) & ~(ovf["icdf_margin"] <= pu.TAU_S)
    assert ok.sum() >= w.B - 1
    assert (acc.cpu().numpy()[ok] == ovf["accept_len"][ok]).all()
    assert (out.cpu().numpy()[ok] == ovf["out_tok"][ok]).all()


@pytest.mark.parametrize("seed", list(range(int(os.environ.get("TAPOUT_RANDOM_SHARDINGS", "16")))))
def test_random_shardings(seed):
    """Random shapes cut into 2-8 vocabulary shards of uneven width (some a single column wide): the sharded path
    must reproduce the oracle's decisions on the unsplit rows."""
    rs = np.random.RandomState(5000 + seed)
    B, K = int(rs.randint(1, 7)), int(rs.randint(1, 9))
    V = int(rs.choice([rs.randint(16, 400), rs.randint(400, 9000), rs.randint(9000, 50000)]))
    G = int(rs.randint(2, 9))
    cuts = np.sort(rs.choice(np.arange(1, V), size=G - 1, replace=False))
    edges = [0] + [int(c) for c in cuts] + [V]
    dt = (torch.float32, torch.bfloat16)[rs.randint(2)]
    rnd = random_round(B, K, V, dt, seed=seed, sigma=float(rs.uniform(1.0, 5.0)),
                       k_len=[int(x) for x in rs.randint(1, K + 1, B)])
    rnd["greedy"] = torch.from_numpy((rs.rand(B) < 0.25).astype(np.uint8)).to(DEV)
    announce(f"random sharding {seed}: B={B} K={K} V={V} {dt} edges {edges}")
    acc, out, _ = sharded_round(rnd, G, V, edges=edges)
    ods, ovf, nd = pu.oracle_round(rnd)
    used = np.arange(K)[None, :] < nd[:, None]
    ok = ~((ovf["accept_margin"] <= pu.TAU) & used).any(1) & ~(ovf["icdf_margin"] <= pu.TAU_S)
    assert ok.sum() >= B - 1
    assert (acc.cpu().numpy()[ok] == ovf["accept_len"][ok]).all()
    assert (out.cpu().numpy()[ok] == ovf["out_tok"][ok]).all()


def test_vocabulary_sharded_final_token_hard_cases():
    """p = q on heavy tokens (the sums cannot settle the masses: second exchange), p == q everywhere (bonus-like draw
    from the target row), and draws near the ends of the CDF."""
    B, K, V, G = 5, 2, 30000, 4
    g = torch.Generator().manual_seed(43)
    d = (torch.randn(B, K, V, generator=g) * 2).float()
    t = torch.cat([d + torch.randn(B, K, V, generator=g), torch.randn(B, 1, V, generator=g) * 2], 1).float()
    hot = torch.randint(0, V, (B, 4), generator=g)
    for b in range(3):                                               # sequences 0..2: heavy tokens with p_h = q_h
        d[b, 0, hot[b]] = d[b, 0].max() + torch.tensor([2.0, 1.5, 1.0, 0.5])
        q = torch.softmax(d[b, 0].double(), 0)
        mask = torch.ones(V, dtype=torch.bool); mask[hot[b]] = False
        ln_rp = torch.logsumexp(t[b, 0].double()[mask], 0)
        t[b, 0, hot[b]] = (q[hot[b]].log() + ln_rp - torch.log1p(-q[hot[b]].sum())).float()
    t[3, :K] = d[3]                                                  # p == q: accepted to the end, bonus token
    tok = torch.randint(0, V, (B, K), generator=g, dtype=torch.int32)
    for b in range(B):
        clash = (tok[b][:, None] == hot[b][None, :]).any(1)
        tok[b][clash] = (tok[b][clash] + 11) % V
    ua = torch.full((B, K), 1.0 - 2.0 ** -24)
    ua[3] = 0.5
    rnd = dict(draft=d.to(DEV), target=t.to(DEV), draft_tok=tok.to(DEV), u_accept=ua.to(DEV),
               u_sample=torch.tensor([0.3, 1e-4, 0.9999, 0.7, 0.5]).to(DEV),
               k_len=torch.full((B,), K, dtype=torch.int32, device=DEV), greedy=torch.zeros(B, dtype=torch.uint8, device=DEV))
    acc, out, n_second = sharded_round(rnd, G, V)
    assert n_second >= 1                                             # the heavy p = q tokens forced the exact masses
    ods, ovf, nd = pu.oracle_round(rnd)
    used = np.arange(K)[None, :] < nd[:, None]
    ok = ~((ovf["accept_margin"] <= pu.TAU) & used).any(1) & ~(ovf["icdf_margin"] <= pu.TAU_S)
    # u_accept ~ 1 makes every drafted token with p >= q a near tie of the accept test: those sequences are not compared
    assert ok[:3].any() and ok[3] and ok[4]
    assert (acc.cpu().numpy()[ok] == ovf["accept_len"][ok]).all()
    assert (out.cpu().numpy()[ok] == ovf["out_tok"][ok]).all()
    assert acc[3] == K
    # and the unsplit call agrees
    tp = binding.Tapout(B, K, V)
    _, vf, _ = pu.gpu_round(tp, rnd)
    assert (vf["out_tok"].cpu().numpy()[ok] == out.cpu().numpy()[ok]).all()


def test_vocabulary_shard_records_edge_cases():
    B, K, V, G = 2, 2, 4000, 4
    x = torch.randn(B, K, V) * 2
    x[0, 0, 1000:2000] = float("-inf")                                    # a fully masked shard
    x[0, 1, :] = 3.0                                                      # all equal: argmax 0, second = max
    x[1, 0, 2500] = float("nan")                                          # NaN in one shard poisons the row
    x[1, 1, 3999] = 50.0                                                  # maximum in the last column of the last shard
    tok = torch.tensor([[1500, 3999], [10, 3999]], dtype=torch.int32)
    tp = binding.Tapout(B, K, V)
    xd = x.to(DEV)
    recs = torch.stack([tp.shard_stats(xd[:, :, g * 1000:(g + 1) * 1000], g * 1000, tok=tok.to(DEV)).clone() for g in range(G)])
    r = recs.cpu().view(G, B, K, 8)
    assert r[1, 0, 0, 0].view(torch.float32) == float("-inf") and r[1, 0, 0, 1].view(torch.float32) == 0.0
    assert not torch.isnan(r[1, 0, 0, 5].view(torch.float32))             # the masked shard still owns token 1500 (its logit is -inf)
    assert torch.isnan(r[0, 0, 0, 5].view(torch.float32))                 # shard 0 does not
    o = tp.draft_stats_sharded(recs, B, K, V, draft_tok=tok.to(DEV))
    ods = orc.draft_stats(x.numpy(), draft_tok=tok.numpy())
    live = np.ones((B, K), bool)
    for key in pu.STAT_KEYS:
        pu.assert_stats_close(key, o[key].cpu().numpy(), ods[key], live)
    assert o["top1_id"].cpu().tolist() == ods["top1_id"].tolist() and o["top1_id"][1, 1] == 3999 and o["top1_id"][0, 1] == 0
    assert (o["flags"].cpu().numpy().astype(np.uint32) == ods["flags"]).all() and o["flags"][1] == binding.FLAG_BAD_ROW
    with pytest.raises(binding.TapoutError):
        tp.shard_stats(xd[:, :, :1000], -1)
    with pytest.raises(binding.TapoutError):
        tp.shard_stats(torch.zeros(B, 1, 10, device=DEV), 0, rows_mode=1)


# ---- boundary error handling --------------------------------------------------------

def test_argument_errors_leave_outputs_untouched():
    B, K, V = 4, 3, 100
    tp = binding.Tapout(B, K, V)
    d = torch.zeros(B, K, V, device=DEV)
    out = tp.alloc_draft_outputs(B, K)
    before = {k: v.clone() for k, v in out.items()}
    with pytest.raises(binding.TapoutError, match="EINVAL"):
        tp.draft_stats(torch.zeros(B + 1, K, V, device=DEV))
    with pytest.raises(binding.TapoutError, match="EINVAL"):
        tp.draft_stats(torch.zeros(B, K + 1, V, device=DEV))
    with pytest.raises(binding.TapoutError, match="EINVAL"):
        tp.draft_stats(torch.zeros(B, K, V + 1, device=DEV))
    with pytest.raises(ValueError):
        tp.draft_stats(torch.zeros(B, K, V, device=DEV, dtype=torch.float16))
    with pytest.raises(ValueError):
        tp.draft_stats(torch.zeros(B, K, 2 * V, device=DEV)[:, :, ::2])
    with pytest.raises(binding.TapoutError, match="required"):
        tp.bandit_update(torch.zeros(B, dtype=torch.int32, device=DEV), None, None, None)
    with pytest.raises(binding.TapoutError):
        binding.Tapout(B, K, V, rules=(7,), thresholds=(0.1,))
    with pytest.raises(binding.TapoutError):
        binding.Tapout(0, K, V)
    torch.cuda.synchronize()
    for k in out:
        a, b = out[k].cpu(), before[k].cpu()
        assert torch.equal(torch.nan_to_num(a.float(), nan=-7.0), torch.nan_to_num(b.float(), nan=-7.0))
    # B = 0 is a valid empty call
    tp.draft_stats(d[:0])
    tp.bandit_select(0)
