"""Pins of the oracle's row statistics and stop rules (CPU only).

Each test checks the oracle against something fixed outside it: a closed form,
a library routine evaluating the textbook definition, or the values Table 1
prints.  None of them re-types the oracle's own loop.
"""
import math

import numpy as np
import pytest
import torch

from oracle import oracle as orc


def bf16_bits(x):
    return torch.tensor(np.asarray(x, np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


# ---- closed forms ----------------------------------------------------------

@pytest.mark.parametrize("V", [2, 7, 32000, 128256, 151936, 256000])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_uniform_row_entropy_is_ln_V(V, dtype):
    row = np.full(V, 1.25, np.float32)
    row = row if dtype == "f32" else bf16_bits(row)
    r = orc.row_stats(row)
    assert r["H"] == pytest.approx(math.log(V), rel=1e-10)    # index-order fp64 sum of V terms
    assert r["p1"] == pytest.approx(1.0 / V, rel=1e-12)
    assert r["p2"] == pytest.approx(1.0 / V, rel=1e-12)
    assert r["margin"] == 0.0
    assert r["lse"] == pytest.approx(1.25 + math.log(V), rel=1e-12)
    assert r["top1"] == 0


def test_two_point_row():
    # p = (3/4, 1/4): H = -(3/4 ln 3/4 + 1/4 ln 1/4)
    V = 1000
    row = np.full(V, -np.inf, np.float32)
    row[17] = math.log(3.0)
    row[400] = 0.0
    r = orc.row_stats(row)
    H = -(0.75 * math.log(0.75) + 0.25 * math.log(0.25))
    assert H == pytest.approx(0.5623351446188083, rel=1e-12)
    assert r["H"] == pytest.approx(H, rel=1e-6)          # ln 3 is rounded to binary32
    assert r["p1"] == pytest.approx(0.75, rel=1e-6)
    assert r["p2"] == pytest.approx(0.25, rel=1e-6)
    assert r["margin"] == pytest.approx(0.5, rel=1e-6)
    assert r["top1"] == 17


def test_three_point_row_with_tied_runners_up():
    row = np.full(64, -np.inf, np.float32)
    row[5] = math.log(2.0)
    row[9] = 0.0
    row[33] = 0.0
    r = orc.row_stats(row)
    assert r["H"] == pytest.approx(1.5 * math.log(2.0), rel=1e-6)   # (1/2, 1/4, 1/4)
    assert r["margin"] == pytest.approx(0.25, rel=1e-6)


def test_geometric_row_closed_form():
    # x_j = -a j  =>  p_j = (1-r) r^j / (1 - r^V), r = e^-a;  for r^V ~ 0:
    # H = -ln(1-r) - r ln r / (1-r),  p1 = 1-r,  p2 = (1-r) r
    a = 0.25
    V = 4096
    j = np.arange(V, dtype=np.float64)
    row = (-a * j).astype(np.float32)          # multiples of 0.25 up to 1024: exact in binary32
    r_ = math.exp(-a)
    H = -math.log(1 - r_) - r_ * math.log(r_) / (1 - r_)
    r = orc.row_stats(row)
    assert r["H"] == pytest.approx(H, rel=1e-12)
    assert r["p1"] == pytest.approx(1 - r_, rel=1e-12)
    assert r["p2"] == pytest.approx((1 - r_) * r_, rel=1e-12)
    assert r["lse"] == pytest.approx(-math.log(1 - r_), rel=1e-12)
    assert r["top1"] == 0
    # reversed row: the maximum is the last element
    r = orc.row_stats(np.ascontiguousarray(row[::-1]))
    assert r["top1"] == V - 1
    assert r["H"] == pytest.approx(H, rel=1e-12)


def test_shift_invariance_and_lse_shift():
    g = np.random.default_rng(3)
    row = g.normal(0, 2, 5000).astype(np.float32)
    r0 = orc.row_stats(row)
    # adding 8 is exact for |x| < 8 only up to rounding: use a power-of-two scale-free shift on a coarse grid
    coarse = np.round(row * 64) / 64
    r1 = orc.row_stats(coarse.astype(np.float32))
    r2 = orc.row_stats((coarse + 16.0).astype(np.float32))
    for k in ("H", "p1", "p2", "margin"):
        assert r2[k] == pytest.approx(r1[k], rel=1e-12)
    assert r2["lse"] == pytest.approx(r1["lse"] + 16.0, rel=1e-12)
    assert r0["top1"] == int(np.argmax(row))


# ---- library cross-checks (textbook definitions evaluated by torch in fp64) --

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V,scale", [(977, 2.0), (32000, 2.5), (128256, 6.0)])
def test_against_torch_fp64(V, scale, dtype):
    g = torch.Generator().manual_seed(V)
    x = torch.randn(V, generator=g) * scale
    if dtype == "bf16":
        x = x.to(torch.bfloat16)
    r = orc.row_stats(x)
    xd = x.to(torch.float64)
    p = torch.softmax(xd, 0)
    assert r["H"] == pytest.approx(torch.special.entr(p).sum().item(), rel=1e-10)
    assert r["lse"] == pytest.approx(torch.logsumexp(xd, 0).item(), rel=1e-12)
    top = torch.topk(p, 2)
    assert r["p1"] == pytest.approx(top.values[0].item(), rel=1e-10)
    assert r["p2"] == pytest.approx(top.values[1].item(), rel=1e-10)
    assert r["margin"] == pytest.approx((top.values[0] - top.values[1]).item(), rel=1e-9, abs=1e-15)
    m = xd.max()
    assert r["top1"] == int(torch.nonzero(xd == m)[0])   # lowest index among the maxima
    assert r["M"] == m.item()


def test_bf16_top_tie_gives_zero_margin_and_lowest_index():
    x = torch.zeros(300, dtype=torch.bfloat16)
    x[250] = 3.0
    x[41] = 3.0
    r = orc.row_stats(x)
    assert r["top1"] == 41 and r["margin"] == 0.0 and r["p1"] == r["p2"]


def test_logq_tok_is_log_softmax():
    g = torch.Generator().manual_seed(11)
    d = (torch.randn(3, 4, 1500, generator=g) * 3).to(torch.bfloat16)
    tok = torch.randint(0, 1500, (3, 4), generator=g)
    o = orc.draft_stats(d, draft_tok=tok.numpy())
    ref = torch.log_softmax(d.double(), -1).gather(-1, tok[..., None])[..., 0]
    np.testing.assert_allclose(o["logq_tok"], ref.numpy(), rtol=1e-6)
    np.testing.assert_allclose(o["lse"], torch.logsumexp(d.double(), -1).numpy(), rtol=1e-6)
    assert (o["top1_id"] == d.double().argmax(-1).numpy()).all()
    assert o["n_stop"] is None and not o["flags"].any()


def test_masked_and_bad_rows():
    row = np.array([0.0, -np.inf, 1.0, -np.inf], np.float32)
    r = orc.row_stats(row)
    assert not r["bad"]
    e = math.e
    assert r["p1"] == pytest.approx(e / (1 + e), rel=1e-12)
    assert r["H"] == pytest.approx(math.log(1 + e) - e / (1 + e), rel=1e-12)
    assert orc.row_stats(np.array([0.0, np.nan, 1.0], np.float32))["bad"]
    assert orc.row_stats(np.full(5, -np.inf, np.float32))["bad"]
    assert orc.row_stats(np.array([0.0, np.inf], np.float32))["bad"]
    d = np.zeros((2, 1, 8), np.float32)
    d[1, 0, 3] = np.nan
    o = orc.draft_stats(d, draft_tok=np.array([[9], [0]]))
    assert o["flags"].tolist() == [orc.FLAG_BAD_TOKEN, orc.FLAG_BAD_ROW]


# ---- Table 1: thresholds, directions, strictness ---------------------------

RULE_ID = {"SVIP": orc.RULE_SVIP, "Max-Confidence": orc.RULE_MAXCONF, "LogitMargin": orc.RULE_MARGIN}


def two_point_rows(p_list, V=50):
    """[1, K, V] rows whose softmax is (p, 1-p, 0, ...)."""
    d = np.full((1, len(p_list), V), -np.inf, np.float32)
    for k, p in enumerate(p_list):
        d[0, k, 0] = math.log(p / (1 - p))
        d[0, k, 1] = 0.0
    return d


def binary_entropy(p):
    return -(p * math.log(p) + (1 - p) * math.log(1 - p))


def solve_binary_entropy(H):
    lo, hi = 0.5, 1.0 - 1e-12       # entropy decreases from ln 2 to 0 on [0.5, 1)
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        lo, hi = (mid, hi) if binary_entropy(mid) > H else (lo, mid)
    return 0.5 * (lo + hi)


def test_table1_threshold_edges(golden):
    table = {name: (sig, direction, float(h)) for name, sig, direction, h in golden("table1_stop_rules.txt")}
    assert table["Max-Confidence"][1:] == ("<", 0.8)
    assert table["SVIP"][1:] == (">", 0.6)
    assert table["LogitMargin"][1:] == ("<", 0.2)
    rules = [RULE_ID[n] for n in ("SVIP", "Max-Confidence", "LogitMargin")]
    ths = [table[n][2] for n in ("SVIP", "Max-Confidence", "LogitMargin")]
    eps = 1e-3
    # Max-Confidence fires strictly below 0.8
    d = two_point_rows([0.8 + eps, 0.8 - eps])
    o = orc.draft_stats(d, arm=[1], rules=rules, thresholds=ths)
    assert o["stop_fired"][0].tolist() == [0, 1] and o["n_stop"][0] == 2
    # SVIP fires strictly above sqrt(H) = 0.6, i.e. H = 0.36
    p_hi = solve_binary_entropy(0.36 * (1 + 2 * eps))     # more entropy -> fires
    p_lo = solve_binary_entropy(0.36 * (1 - 2 * eps))
    d = two_point_rows([p_lo, p_hi])
    o = orc.draft_stats(d, arm=[0], rules=rules, thresholds=ths)
    assert o["stop_fired"][0].tolist() == [0, 1]
    assert math.sqrt(o["entropy"][0, 0]) < 0.6 < math.sqrt(o["entropy"][0, 1])
    # LogitMargin fires strictly below p1 - p2 = 0.2, i.e. p = 0.6
    d = two_point_rows([0.6 + eps, 0.6 - eps])
    o = orc.draft_stats(d, arm=[2], rules=rules, thresholds=ths)
    assert o["stop_fired"][0].tolist() == [0, 1]
    # the (3/4, 1/4) row: SVIP and Max-Confidence stop, LogitMargin continues
    d = two_point_rows([0.75])
    fired = [int(orc.draft_stats(d, arm=[a], rules=rules, thresholds=ths)["stop_fired"][0, 0]) for a in range(3)]
    assert fired == [1, 1, 0]


def test_strict_inequality_at_exact_threshold():
    # thresholds chosen equal to the binary32 signal itself: equality must not fire
    d = two_point_rows([0.75])
    o = orc.draft_stats(d, arm=[0], rules=[0, 1, 2], thresholds=[0.6, 0.8, 0.2])
    p1, mg, H = float(o["p_top1"][0, 0]), float(o["margin"][0, 0]), float(o["entropy"][0, 0])
    for a, h in ((1, p1), (2, mg)):
        th = [0.6, 0.8, 0.2]
        th[a] = h
        assert orc.draft_stats(d, arm=[a], rules=[0, 1, 2], thresholds=th)["stop_fired"][0, 0] == 0
        th[a] = float(np.nextafter(np.float32(h), np.float32(2)))
        assert orc.draft_stats(d, arm=[a], rules=[0, 1, 2], thresholds=th)["stop_fired"][0, 0] == 1
    h = float(np.float32(math.sqrt(H)))
    fired = orc.draft_stats(d, arm=[0], rules=[0, 1, 2], thresholds=[h, .8, .2])["stop_fired"][0, 0]
    assert fired == int(math.sqrt(H) > h)


def test_algorithm1_stop_position():
    # the token of the firing step is kept: n_stop = first firing k + 1; never fires -> k_len
    conf = [0.95, 0.9, 0.7, 0.99, 0.5]
    d = np.repeat(two_point_rows(conf), 4, axis=0)
    d[1, 2] = d[1, 0]                      # sequence 1 first fires at k = 4
    d[2, 2] = d[2, 0]; d[2, 4] = d[2, 0]   # sequence 2 never fires
    d[3, 0] = d[3, 2]                      # sequence 3 fires at the first step
    o = orc.draft_stats(d, arm=[1, 1, 1, 1])
    assert o["n_stop"].tolist() == [3, 5, 5, 1]
    # ragged cap: rows beyond k_len are neither read nor written
    o = orc.draft_stats(d, arm=[1, 1, 1, 1], k_len=[2, 5, 3, 4])
    assert o["n_stop"].tolist() == [2, 5, 3, 1]
    assert np.isnan(o["entropy"][0, 2:]).all() and not np.isnan(o["entropy"][0, :2]).any()
    # uniform rows: every rule fires at step 1
    u = np.zeros((3, 4, 100), np.float32)
    assert orc.draft_stats(u, arm=[0, 1, 2])["n_stop"].tolist() == [1, 1, 1]
