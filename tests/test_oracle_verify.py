"""Pins of the oracle's verification and final-token sampling (CPU only).

The central pin is the exactness of speculative sampling: with drafted tokens
drawn from q and uniform acceptance / sampling variables, the emitted tokens
follow the target law p.  It is checked by exhaustive enumeration on tiny
vocabularies with probabilities chosen so that every decision threshold falls
on a cell edge of the uniform grids; the enumeration is then exact, not
statistical.
"""
import itertools
import math

import numpy as np
import pytest

from oracle import oracle as orc


def logits_of(p):
    with np.errstate(divide="ignore"):
        return np.log(np.asarray(p, np.float64)).astype(np.float32)


def enumerate_law(p_rows, q_rows, n_draft, n_grid, greedy=False):
    """Exact law of the emitted token string under the oracle.

    p_rows: K+1 target distributions, q_rows: K draft distributions (over V).
    Returns {emitted tuple: probability}.
    """
    K = len(q_rows)
    V = len(p_rows[0])
    tgt = logits_of(p_rows)[None]                 # [1, K+1, V]
    drf = logits_of(q_rows)[None]                 # [1, K, V]
    mids = (np.arange(n_grid) + 0.5) / n_grid
    toks = np.array(list(itertools.product(range(V), repeat=n_draft)), np.int32)          # [T, n]
    us = np.array(list(itertools.product(mids, repeat=n_draft + 1)), np.float32)           # [U, n+1]
    T, U = len(toks), len(us)
    tok = np.zeros((T, U, K), np.int32)
    tok[:, :, :n_draft] = toks[:, None, :]
    ua = np.zeros((T, U, K), np.float32)
    ua[:, :, :n_draft] = us[None, :, :n_draft]
    usamp = np.broadcast_to(us[None, :, n_draft], (T, U))
    B = T * U
    tok = tok.reshape(B, K)
    weight = np.ones(B)
    for k in range(n_draft):
        weight *= np.asarray(q_rows[k])[tok[:, k]]
    weight /= U
    keep = weight > 0
    tok, weight = tok[keep], weight[keep]
    ua = ua.reshape(B, K)[keep]
    usamp = np.ascontiguousarray(usamp.reshape(B)[keep])
    B = len(tok)
    tgt_b = np.lib.stride_tricks.as_strided(tgt, (B, K + 1, V), (0,) + tgt.strides[1:])
    drf_b = np.lib.stride_tricks.as_strided(drf, (B, K, V), (0,) + drf.strides[1:])
    # log q(tok) for every sequence: chain the oracle's own draft pass (row by row, tiny)
    lq_table = np.stack([[orc.draft_stats(drf, draft_tok=np.full((1, K), v))["logq_tok"][0, k] for v in range(V)]
                         for k in range(K)])                    # [K, V]
    logq = np.zeros((B, K), np.float32)
    for k in range(K):
        logq[:, k] = lq_table[k][tok[:, k]]
    o = orc.verify(tgt_b, drf_b, logq, tok, np.full(B, n_draft), ua, usamp,
                   greedy=np.full(B, 1 if greedy else 0), nthreads=8)
    assert not o["flags"].any()
    assert (o["n_out"] == o["accept_len"] + 1).all()
    pos = np.arange(K + 1)[None, :]
    out = o["out_tok"]
    assert (out[pos >= o["n_out"][:, None]] == -1).all()                 # unused slots are -1
    acc = pos[:, :K] < o["accept_len"][:, None]
    assert (out[:, :K][acc] == tok[acc]).all()                           # accepted prefix is the drafted prefix
    code = ((out + 1) * (V + 1) ** pos).sum(1)                           # base-(V+1) digits, -1 -> 0
    mass = np.bincount(code, weights=weight)
    law = {}
    for c in np.nonzero(mass)[0]:
        digits, x = [], int(c)
        while x:
            digits.append(x % (V + 1) - 1)
            x //= V + 1
        law[tuple(digits)] = mass[c]
    return law


def expected_law(p_rows, q_rows, n_draft):
    """Target law of the emitted string: accepted prefix a_0..a_{m-1} has probability
    prod min(p_k, q_k)(a_k); the string then ends with a token whose marginal, summed
    over stop reasons, makes position k ~ p_k.  Written as P(string) directly:
    P(a_0..a_{m-1}, c) = prod_k<m min(p_k,q_k)(a_k) * [ m<n: max(0, p_m(c) - q_m(c)) ; m=n: p_n(c) ]."""
    V = len(p_rows[0])
    law = {}
    for m in range(n_draft + 1):
        for prefix in itertools.product(range(V), repeat=m):
            w = 1.0
            for k, a in enumerate(prefix):
                w *= min(p_rows[k][a], q_rows[k][a])
            for c in range(V):
                last = p_rows[m][c] if m == n_draft else max(0.0, p_rows[m][c] - q_rows[m][c])
                if w * last > 0:
                    law[prefix + (c,)] = w * last
    return law


P0, Q0 = (.5, .3, .2), (.2, .5, .3)
P1, Q1 = (.1, .6, .3), (.4, .4, .2)
P2 = (.3, .3, .4)


def test_worked_case_single_position():
    # p=(.5,.3,.2), q=(.2,.5,.3): P(accept) = sum min = 0.7, residual mass 0.3, residual = (1,0,0)
    law = enumerate_law([P0, P2], [Q0], n_draft=1, n_grid=60)
    first = np.zeros(3)
    for key, w in law.items():
        first[key[0]] += w
    np.testing.assert_allclose(first, P0, atol=1e-12)            # emitted token ~ target law
    p_accept = sum(w for key, w in law.items() if len(key) == 2)
    assert p_accept == pytest.approx(0.7, abs=1e-9)
    rejected = {k: w for k, w in law.items() if len(k) == 1}
    assert set(rejected) == {(0,)} and rejected[(0,)] == pytest.approx(0.3, abs=1e-9)
    exp = expected_law([P0, P2], [Q0], 1)
    assert set(law) == set(exp)
    for k in exp:
        assert law[k] == pytest.approx(exp[k], abs=1e-9)


@pytest.mark.parametrize("n_draft", [1, 2])
def test_exact_output_law_two_positions(n_draft):
    p_rows, q_rows = [P0, P1, P2], [Q0, Q1]
    law = enumerate_law(p_rows, q_rows, n_draft=n_draft, n_grid=60)
    exp = expected_law(p_rows, q_rows, n_draft)
    assert set(law) == set(exp)
    for k in exp:
        assert law[k] == pytest.approx(exp[k], abs=1e-9)
    assert sum(law.values()) == pytest.approx(1.0, abs=1e-9)
    # marginal of every emitted position, given that it is reached, is the target law there
    for pos in range(n_draft + 1):
        marg = np.zeros(3)
        for key, w in law.items():
            if len(key) > pos:
                marg[key[pos]] += w
        reach = marg.sum()
        np.testing.assert_allclose(marg / reach, p_rows[pos], atol=1e-12)


def test_exact_output_law_spread_residual():
    # residual (.3,.1,0,0)/.4 is not one-hot: the inverse CDF over the residual is exercised
    p0, q0 = (.4, .3, .2, .1), (.1, .2, .3, .4)
    p1 = (.25, .25, .25, .25)
    law = enumerate_law([p0, p1], [q0], n_draft=1, n_grid=60)
    exp = expected_law([p0, p1], [q0], 1)
    assert set(law) == set(exp)
    for k in exp:
        assert law[k] == pytest.approx(exp[k], abs=1e-9)
    assert law[(0,)] == pytest.approx(0.3, abs=1e-9) and law[(1,)] == pytest.approx(0.1, abs=1e-9)


def test_identities_tv_distance_and_p_equals_q():
    g = np.random.default_rng(5)
    V, K, B = 300, 4, 64
    tgt = g.normal(0, 2, (B, K + 1, V)).astype(np.float32)
    drf = tgt[:, :K].copy()
    tok = g.integers(0, V, (B, K)).astype(np.int32)
    ds = orc.draft_stats(drf, draft_tok=tok)
    ua = g.random((B, K), np.float32)
    us = g.random(B, np.float32)
    o = orc.verify(tgt, drf, ds["logq_tok"], tok, np.full(B, K), ua, us)
    assert (o["accept_len"] == K).all()                       # p == q: ratio 1, u < 1 always accepts
    # bonus token = inverse CDF of softmax(target row K)
    for b in range(8):
        p = np.exp(tgt[b, K].astype(np.float64))
        c = np.cumsum(p / p.sum())
        assert o["out_tok"][b, K] == int(np.searchsorted(c, us[b], side="right"))


def test_inverse_cdf_special_cases():
    # u = 0 -> first positive weight; one-hot -> that index for every u; uniform -> floor(u V)
    w = np.array([0, 0, .2, 0, .8])
    assert orc.inverse_cdf(w, 0.0)[0] == 2
    one = np.zeros(11); one[7] = 3.0
    assert all(orc.inverse_cdf(one, u)[0] == 7 for u in (0.0, 0.3, 0.999999))
    V = 64
    for u in (0.0, 0.0156, 0.5, 0.51, 0.99):
        assert orc.inverse_cdf(np.ones(V), u)[0] == math.floor(u * V)
    # edges: C_j > u Z is strict
    assert orc.inverse_cdf(np.array([.25, .25, .5]), 0.25)[0] == 1
    assert orc.inverse_cdf(np.array([.25, .25, .5]), 0.5)[0] == 2
    # zero mass is reported, margin is the distance to the nearer edge over Z
    assert orc.inverse_cdf(np.zeros(4), 0.5)[0] == -1
    j, Z, mg = orc.inverse_cdf(np.array([1., 1., 2.]), 0.30)
    assert (j, Z) == (1, 4.0) and mg == pytest.approx(0.05)


def test_greedy_rows_match_argmax():
    g = np.random.default_rng(8)
    V, K, B = 500, 5, 40
    tgt = g.normal(0, 2, (B, K + 1, V)).astype(np.float32)
    drf = g.normal(0, 2, (B, K, V)).astype(np.float32)
    tok = tgt[:, :K].argmax(-1).astype(np.int32)
    cut = g.integers(0, K + 1, B)                         # first mismatch position (K = none)
    for b in range(B):
        if cut[b] < K:
            tok[b, cut[b]] = (tok[b, cut[b]] + 1) % V
    ds = orc.draft_stats(drf, draft_tok=tok)
    o = orc.verify(tgt, drf, ds["logq_tok"], tok, np.full(B, K), np.zeros((B, K)), np.zeros(B), greedy=np.ones(B))
    assert o["accept_len"].tolist() == cut.tolist()
    assert (o["out_tok"][np.arange(B), cut] == tgt[np.arange(B), cut].argmax(-1)).all()
    assert (o["target_top1"] == tgt.argmax(-1)).all()


def test_truncated_draft_uses_row_n_as_bonus_and_flags():
    g = np.random.default_rng(9)
    V, K, B = 200, 6, 16
    tgt = g.normal(0, 2, (B, K + 1, V)).astype(np.float32)
    drf = tgt[:, :K].copy()
    tok = g.integers(0, V, (B, K)).astype(np.int32)
    nd = g.integers(1, K + 1, B).astype(np.int32)
    ds = orc.draft_stats(drf, draft_tok=tok)
    us = g.random(B, np.float32)
    o = orc.verify(tgt, drf, ds["logq_tok"], tok, nd, g.random((B, K), np.float32), us)
    assert (o["accept_len"] == nd).all() and (o["n_out"] == nd + 1).all()
    for b in range(B):
        p = np.exp(tgt[b, nd[b]].astype(np.float64))
        assert o["out_tok"][b, nd[b]] == int(np.searchsorted(np.cumsum(p / p.sum()), us[b], side="right"))
        assert np.isnan(o["target_lse"][b, nd[b] + 1:]).all()      # rows beyond n_draft are not read
    bad_nd = nd.copy(); bad_nd[0] = 0; bad_nd[1] = K + 1
    bad_tok = tok.copy(); bad_tok[2, 0] = V
    o = orc.verify(tgt, drf, ds["logq_tok"], bad_tok, bad_nd, np.zeros((B, K)), us)
    assert o["flags"][:3].tolist() == [orc.FLAG_BAD_NDRAFT, orc.FLAG_BAD_NDRAFT, orc.FLAG_BAD_TOKEN]
    assert o["accept_len"][:3].tolist() == [0, 0, 0]
    assert (o["out_tok"][:3, 0] == tgt[:3, 0].argmax(-1)).all()


def test_expected_acceptance_of_gaussian_family():
    # target = draft + N(0, s^2) on a diffuse row  =>  E[min(1, p/q)] under q is about 2 Phi(-s/2)
    g = np.random.default_rng(21)
    V, K, B = 32000, 1, 200
    from math import erf, sqrt
    for s, tol in ((0.5, 0.03), (1.0, 0.04)):
        drf = g.normal(0, 2, (B, K, V)).astype(np.float32)
        tgt = np.concatenate([drf + g.normal(0, s, (B, K, V)).astype(np.float32),
                              g.normal(0, 2, (B, 1, V)).astype(np.float32)], 1)
        q = np.exp(drf[:, 0].astype(np.float64)); q /= q.sum(-1, keepdims=True)
        tok = np.array([[g.choice(V, p=q[b])] for b in range(B)], np.int32)
        ds = orc.draft_stats(drf, draft_tok=tok, nthreads=8)
        o = orc.verify(tgt, drf, ds["logq_tok"], tok, np.ones(B), g.random((B, K), np.float32),
                       g.random(B, np.float32), nthreads=8)
        phi = 0.5 * (1 + erf((-s / 2) / sqrt(2)))
        assert o["accept_len"].mean() == pytest.approx(2 * phi, abs=3 * tol)
