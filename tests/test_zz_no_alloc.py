"""tapout_draft_stats_static, the entry point that allocates nothing (its scratch is a fixed array in the library's
device image), against tapout_draft_stats through the C ABI: same kernels, same launch shape, so every output must
carry the same bits; two calls in a row, the second on a smaller input (the array still holds the first call's
records), then argument errors."""
import pytest
import torch

from paper_2511_02017_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def bits(t):
    return t.cpu().view(torch.int32) if t.dtype == torch.float32 else t.cpu()


def compare(rnd, arm):
    B, K, V = rnd["draft"].shape
    tp = binding.Tapout(B, K, V)
    want = tp.draft_stats(rnd["draft"], draft_tok=rnd["draft_tok"], k_len=rnd["k_len"], arm=arm)
    got = binding.draft_stats_static(rnd["draft"], draft_tok=rnd["draft_tok"], k_len=rnd["k_len"], arm=arm)
    torch.cuda.synchronize()
    assert want.keys() == got.keys()
    for k in want:
        assert torch.equal(bits(want[k]), bits(got[k])), k
    return got


def test_static_scratch_entry_point_matches_the_context_entry_point():
    big = synth.RoundGenerator(synth.scaled(synth.WORKLOADS["llama3"], B=24), DEV).round(0)       # 192 rows x 22 slices
    small = synth.RoundGenerator(synth.scaled(synth.WORKLOADS["small"], B=5, K=3), DEV).round(1)  # 15 rows x 7 slices
    arm_big = (torch.arange(24, dtype=torch.int32) % 3).to(DEV)
    arm_small = (torch.arange(5, dtype=torch.int32) % 3).to(DEV)
    a = compare(big, arm_big)
    b = compare(small, arm_small)
    assert len(set(a["n_stop"].cpu().tolist())) > 1                  # the stop rules did something
    assert torch.isfinite(b["entropy"]).all()
    # the larger input once more: nothing of the smaller call is left behind
    compare(big, arm_big)
    # signals only (no arm, no tokens), ragged lengths
    kl = big["k_len"].clone()
    kl[::2] = 3
    tp = binding.Tapout(24, big["draft"].shape[1], big["draft"].shape[2])
    want = tp.draft_stats(big["draft"], k_len=kl)
    got = binding.draft_stats_static(big["draft"], k_len=kl)
    torch.cuda.synchronize()
    live = torch.arange(big["draft"].shape[1])[None, :] < kl.cpu()[:, None]
    for k in ("lse", "entropy", "p_top1", "p_top2", "margin", "top1_id"):
        assert torch.equal(bits(want[k])[live], bits(got[k])[live]), k


def test_static_scratch_entry_point_refuses_what_it_cannot_hold():
    x = torch.zeros(4, 2, 512, device=DEV)
    arm = torch.zeros(4, dtype=torch.int32, device=DEV)
    with pytest.raises(binding.TapoutError, match="carries state"):
        binding.draft_stats_static(x, arm=arm, rules=(binding.RULE_ADAEDL,), thresholds=(0.4,))
    with pytest.raises(binding.TapoutError, match="n_arms"):
        binding.draft_stats_static(x, arm=arm, rules=(), thresholds=())
    # more rows x slices than the static array holds: refused on the host, nothing launched
    rows = binding.STATIC_MAX_PARTIALS + 8
    wide = torch.zeros(rows // 8, 8, 16, device=DEV)
    with pytest.raises(binding.TapoutError, match="static scratch"):
        binding.draft_stats_static(wide)
    got = binding.draft_stats_static(wide[: rows // 8 - 2])            # just inside the limit
    torch.cuda.synchronize()
    assert (got["p_top1"] == 1.0 / 16).all() and (got["top1_id"] == 0).all()
