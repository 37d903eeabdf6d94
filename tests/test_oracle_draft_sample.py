"""Pins of the oracle's draft-token sampler (Algorithm 1, "sample x_i from the draft model"): CPU only."""
import numpy as np

from oracle import oracle as orc


def test_law_of_the_drawn_token_is_the_softmax_exactly():
    # probabilities that are multiples of 1/64: a grid of 64 * 50 midpoints must hit every token exactly p * 3200 times
    counts = np.array([1, 7, 0, 24, 16, 0, 12, 4])
    x = np.where(counts > 0, np.log(np.maximum(counts, 1) / 64.0), -np.inf).astype(np.float32)
    n = 64 * 50
    u = ((np.arange(n) + 0.5) / n).astype(np.float32)
    # one row per uniform through the batch axis with stride 0 (the same row for every sequence)
    rows = np.lib.stride_tricks.as_strided(x, shape=(n, 1, len(x)), strides=(0, 0, x.strides[0]))
    o = orc.draft_sample(rows, u[:, None])
    got = np.bincount(o["tok"][:, 0], minlength=len(x))
    assert (got == counts * 50).all()
    assert (np.diff(o["tok"][:, 0]) >= 0).all()                 # the inverse CDF is monotone in u
    assert not o["flags"].any()


def test_uniform_row_closed_form_and_edges():
    V, n, off = 40, 10, 7
    x = np.full((1, 3, V), -np.inf, np.float32)
    x[0, :, off:off + n] = 2.5                                  # uniform over 10 tokens: token = off + floor(10 u)
    for u in (0.0, 0.05, 0.31, 0.55, 0.99, 0.99999994):          # away from the cell edges k/10
        o = orc.draft_sample(x, np.full((1, 3), u, np.float32))
        assert (o["tok"][0] == off + int(np.float32(u) * 10)).all(), u
    # margin = distance to the nearer cell edge over Z: u = 0.31 sits 0.01 above the edge 0.3
    o = orc.draft_sample(x, np.full((1, 3), 0.31, np.float32))
    np.testing.assert_allclose(o["icdf_margin"][0], 0.01, rtol=1e-5)


def test_live_rows_bad_rows_and_agreement_with_the_bonus_token_draw():
    g = np.random.default_rng(3)
    B, K, V = 3, 4, 300
    x = (g.standard_normal((B, K, V)) * 3).astype(np.float32)
    x[1, 2, 5] = np.nan
    x[2, 0, :] = -np.inf
    u = g.random((B, K), np.float32)
    o = orc.draft_sample(x, u, k_len=[4, 3, 2])
    assert o["tok"][0].min() >= 0 and o["tok"][1, 3] == -1 and (o["tok"][2, 2:] == -1).all()      # beyond k_len: untouched
    assert o["tok"][1, 2] == -1 and o["tok"][2, 0] == -1                                            # bad rows
    assert o["flags"].tolist() == [0, orc.FLAG_BAD_ROW, orc.FLAG_BAD_ROW]
    # the same row and uniform through the verification path's bonus-token draw (all drafted tokens accepted:
    # a draft equal to the target accepts with probability 1) gives the same token
    b, k = 0, 1
    tgt = np.repeat(x[b:b + 1, k:k + 1], 2, axis=1)                       # target rows 0 and 1 = that draft row
    drf = x[b:b + 1, k:k + 1]
    tok0 = np.array([[int(np.argmax(x[b, k]))]], np.int32)
    ds = orc.draft_stats(drf, draft_tok=tok0)
    vf = orc.verify(tgt, drf, ds["logq_tok"], tok0, [1], np.zeros((1, 1), np.float32), u[b:b + 1, k])
    assert vf["accept_len"][0] == 1 and vf["out_tok"][0, 1] == o["tok"][b, k]
    # and the plain definition on explicit softmax weights
    p = np.exp(x[b, k].astype(np.float64) - x[b, k].max()); p /= p.sum()
    assert orc.inverse_cdf(p, float(u[b, k]))[0] == o["tok"][b, k]
