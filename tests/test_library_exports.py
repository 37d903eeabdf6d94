"""CPU-only checks of the boundary: the built library loads without a GPU and
exports every entry point include/tapout.h declares; host-side validation in
tapout_create rejects bad configurations before touching a device."""
import ctypes
import os
import re

import pytest

from paper_2511_02017_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_entry_points():
    text = open(os.path.join(ROOT, "include", "tapout.h")).read()
    return re.findall(r"TAPOUT_API[^;(]*?\b(tapout_\w+)\s*\(", text)


def test_library_exports_every_declared_symbol():
    names = declared_entry_points()
    assert {"tapout_draft_stats", "tapout_verify", "tapout_bandit_select", "tapout_bandit_update"} <= set(names)
    lib = binding.load_library()
    for n in names:
        assert hasattr(lib, n), n
    assert set(binding.EXPORTS) == set(names)


def test_default_config_matches_table1(golden):
    cfg = binding.default_config(4, 8, 1000)
    table = {name: float(h) for name, _sig, _dir, h in golden("table1_stop_rules.txt")}
    assert cfg.n_arms == 3 and list(cfg.rule)[:3] == [binding.RULE_SVIP, binding.RULE_MAXCONF, binding.RULE_MARGIN]
    got = [round(float(x), 6) for x in list(cfg.threshold)[:3]]
    assert got == [table["SVIP"], table["Max-Confidence"], table["LogitMargin"]]
    assert cfg.alpha == 0.5 and cfg.policy == binding.UCB1 and cfg.n_bandits == 4


def test_create_rejects_bad_config_on_the_host():
    lib = binding.load_library()
    ctx = ctypes.c_void_p()
    for mutate, word in ((lambda c: setattr(c, "n_arms", 0), "n_arms"),
                         (lambda c: setattr(c, "max_batch", 0), "positive"),
                         (lambda c: setattr(c, "alpha", 1.5), "alpha"),
                         (lambda c: setattr(c, "n_bandits", 3), "n_bandits"),
                         (lambda c: setattr(c, "policy", 9), "policy"),
                         (lambda c: setattr(c, "reward", 2), "reward"),
                         (lambda c: setattr(c, "granularity", 2), "granularity"),
                         (lambda c: c.rule.__setitem__(1, 5), "rule"),
                         (lambda c: (c.rule.__setitem__(0, binding.RULE_ADAEDL), setattr(c, "adaedl_beta1", 1.5)), "adaedl_beta1"),
                         (lambda c: setattr(c, "max_k", 5000), "max_k")):
        cfg = binding.default_config(4, 8, 1000)
        mutate(cfg)
        st = lib.tapout_create(ctypes.byref(ctx), ctypes.byref(cfg))
        assert st in (1, 2) and ctx.value is None
        assert word in lib.tapout_last_error(None).decode()
    assert lib.tapout_create(None, None) == 1
    assert lib.tapout_draft_stats(None, None, 1, 1, 1, *([None] * 16)) == 1


def test_synthetic_workloads_have_the_stated_shapes():
    import torch
    from paper_2511_02017_amd import synth
    expect = {"tiny": (32000, 1, 5), "small": (32000, 32, 8), "llama3": (128256, 64, 8),
              "zipf": (151936, 256, 16), "ragged": (256000, 512, 16)}
    for name, (V, B, K) in expect.items():
        w = synth.WORKLOADS[name]
        assert (w.V, w.B, w.K) == (V, B, K)
    w = synth.scaled(synth.WORKLOADS["ragged"], V=500, B=40)
    gen = synth.RoundGenerator(w, "cpu")
    r0, r0b, r1 = gen.round(0), synth.RoundGenerator(w, "cpu").round(0), gen.round(1)
    assert torch.equal(r0["draft"], r0b["draft"]) and torch.equal(r0["draft_tok"], r0b["draft_tok"])   # seeded
    assert not torch.equal(r0["draft"], r1["draft"])
    assert r0["draft"].dtype == torch.bfloat16 and r0["target"].dtype == torch.float32
    assert r0["target"].shape == (40, 17, 500) and r0["draft"].shape == (40, 16, 500)
    assert int(r0["k_len"].min()) >= 4 and int(r0["k_len"].max()) <= 16
    g = r0["greedy"].bool()
    assert 0 < int(g.sum()) < 40
    assert torch.equal(r0["draft_tok"][g].long(), r0["draft"][g].float().argmax(-1))
    z = synth.RoundGenerator(synth.scaled(synth.WORKLOADS["zipf"], V=300, B=3, shift_round=2), "cpu")
    early, late = z.round(0), z.round(2)
    spread = lambda r: (r["target"].float()[:, :16] - r["draft"].float()).std().item()
    assert spread(early) == pytest.approx(0.6, rel=0.1) and spread(late) == pytest.approx(2.0, rel=0.1)
