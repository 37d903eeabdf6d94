"""Pins of the oracle's reward, UCB1 and Thompson-Sampling code (CPU only)."""
import math

import numpy as np
import pytest
from scipy import stats

from oracle import oracle as orc


def test_reward_hand_cases(golden):
    rows = golden("reward_blend.txt")
    assert rows[0] == ["alpha", "0.5"]
    for m, n, g, r in rows[1:]:
        assert orc.reward(int(m), int(n), int(g), 0.5) == float(r)      # dyadic rationals: exact
    # alpha = 1 is the acceptance-length-only reward |Y| / gamma, alpha = 0 the acceptance rate
    assert orc.reward(3, 4, 8, 1.0) == 3 / 8
    assert orc.reward(3, 4, 8, 0.0) == 3 / 4
    # bounds: 0 <= r <= 1, and r = 1 only when everything drafted up to the cap is accepted
    for g in range(1, 9):
        for n in range(1, g + 1):
            for m in range(n + 1):
                r = orc.reward(m, n, g)
                assert 0.0 <= r <= 1.0 and (r == 1.0) == (m == n == g)


def test_ucb1_plays_every_arm_once_in_index_order():
    s, c = np.zeros(3), np.zeros(3, np.int64)
    for expect in (0, 1, 2):
        a, idx = orc.ucb1_select(s, c)
        assert a == expect and np.isinf(idx[expect])
        c[a] += 1
        s[a] += 0.3


def test_ucb1_hand_values():
    # one play each, t = 4: the bonus sqrt(2 ln 4) is common, so argmax = best mean (lowest index on ties)
    s, c = np.array([0.2, 0.7, 0.7]), np.array([1, 1, 1])
    a, idx = orc.ucb1_select(s, c)
    assert a == 1
    b4 = math.sqrt(2 * math.log(4))
    assert b4 == pytest.approx(1.6651092223153954, rel=1e-15)
    np.testing.assert_allclose(idx, s + b4, rtol=1e-15)
    # N = (2,1,1), t = 5: bonuses sqrt(2 ln5 / 2), sqrt(2 ln 5)
    s, c = np.array([1.8, 0.4, 0.1]), np.array([2, 1, 1])
    a, idx = orc.ucb1_select(s, c)
    assert math.sqrt(math.log(5)) == pytest.approx(1.2686362411795196, rel=1e-15)
    assert math.sqrt(2 * math.log(5)) == pytest.approx(1.7941225779941015, rel=1e-15)
    np.testing.assert_allclose(idx, [0.9 + 1.2686362411795196, 0.4 + 1.7941225779941015, 0.1 + 1.7941225779941015],
                               rtol=1e-15)
    assert a == 1                         # 2.1941 beats 2.1686: exploration outweighs the better mean
    # all equal: lowest index
    assert orc.ucb1_select(np.array([.5, .5, .5]), np.array([4, 4, 4]))[0] == 0


def test_ucb1_bonus_shrinks_with_plays_and_grows_with_time():
    s = np.array([50.0, 5.0])
    a, idx = orc.ucb1_select(s, np.array([100, 10]))
    assert idx[1] - 0.5 > idx[0] - 0.5 > 0            # same mean 0.5: the less played arm has the larger bonus
    assert a == 1
    _, later = orc.ucb1_select(np.array([500.0, 5.0]), np.array([1000, 10]))
    assert later[1] > idx[1]                          # ln t grew, N_1 did not


def uniforms(g, n):
    return g.random(n, np.float32)


@pytest.mark.parametrize("shape", [1.0, 1.7, 4.0, 30.5])
def test_gamma_sampler_law(shape):
    g = np.random.default_rng(int(shape * 10))
    N = 40000
    draws = np.empty(N)
    fails = 0
    for i in range(N):
        draws[i], ex = orc.gamma_draw(shape, uniforms(g, 24))
        fails += ex
    assert fails == 0
    assert draws.mean() == pytest.approx(shape, rel=0.03)
    assert draws.var() == pytest.approx(shape, rel=0.06)
    assert stats.kstest(draws, stats.gamma(shape).cdf).pvalue > 1e-3


@pytest.mark.parametrize("a,b", [(1.0, 1.0), (3.5, 1.25), (20.0, 60.0)])
def test_beta_sampler_law(a, b):
    g = np.random.default_rng(int(a * 7 + b))
    N = 40000
    draws = np.array([orc.beta_draw(a, b, uniforms(g, 48))[0] for _ in range(N)])
    assert draws.mean() == pytest.approx(a / (a + b), abs=0.01)
    assert draws.var() == pytest.approx(a * b / ((a + b) ** 2 * (a + b + 1)), rel=0.08)
    assert stats.kstest(draws, stats.beta(a, b).cdf).pvalue > 1e-3


def test_gamma_sampler_uses_uniforms_in_order_and_reports_exhaustion():
    # u1 = 1 -> z = 0 -> v = 1 -> accepted iff ln u3 < 0: the first attempt returns d = shape - 1/3
    u = np.full(24, 0.5, np.float32)
    u[0] = 1.0
    val, ex = orc.gamma_draw(2.0, u)
    assert val == pytest.approx(2.0 - 1 / 3, rel=1e-15) and not ex
    # z very negative makes v <= 0 on every attempt (u1 -> 2^-25 at u = 0, u2 = 0.5 -> cos = -1)
    u = np.zeros(24, np.float32)
    u[1::3] = 0.5
    val, ex = orc.gamma_draw(1.0, u)
    z = -math.sqrt(-2 * math.log(2.0 ** -25))
    assert 1 + z / math.sqrt(9 * (1 - 1 / 3)) < 0          # indeed rejected
    assert ex and val == 1.0
    # only the second attempt usable: same value as when it comes first
    u2 = np.zeros(24, np.float32); u2[1] = 0.5
    u2[3:6] = (0.3, 0.2, 0.9 * 0 + 1e-9)
    first = np.full(24, 0.5, np.float32); first[0:3] = u2[3:6]
    assert orc.gamma_draw(3.0, u2)[0] == orc.gamma_draw(3.0, first)[0]


def test_ts_select_is_argmax_of_posterior_draws_and_prefers_good_arm():
    g = np.random.default_rng(2)
    s, c = np.array([2.0, 45.0, 10.0]), np.array([50, 50, 50])
    wins = np.zeros(3)
    for _ in range(2000):
        u = g.random((3, 48), np.float32)
        a, th, ex = orc.ts_select(s, c, u)
        assert a == int(np.argmax(th)) and not ex
        for k in range(3):                                   # posterior = Beta(1 + S, 1 + N - S)
            assert th[k] == orc.beta_draw(1 + s[k], 1 + c[k] - s[k], u[k])[0]
        wins[a] += 1
    assert wins[1] > 1990
    # fresh bandit: uniform posteriors, every arm is chosen about a third of the time
    wins = np.zeros(3)
    for _ in range(3000):
        wins[orc.ts_select(np.zeros(3), np.zeros(3, np.int64), g.random((3, 48), np.float32))[0]] += 1
    assert (abs(wins / 3000 - 1 / 3) < 0.04).all()


def test_batched_bandit_state_machine():
    # per-sequence bandits: independent; update adds one play and the blended reward
    bd = orc.Bandit(orc.POLICY_UCB1, n_bandits=2, n_arms=3)
    arms, _ = bd.select(2)
    assert arms.tolist() == [0, 0]
    bd.update(arms, [3, 0], [4, 3], [8, 8])
    assert bd.count.tolist() == [[1, 0, 0], [1, 0, 0]]
    assert bd.sum_r[:, 0].tolist() == [0.5625, 0.0]
    arms, _ = bd.select(2)
    assert arms.tolist() == [1, 1]
    bd.update(arms, [5, 2], [5, 8], [5, 8], active=[0, 1])      # inactive sequence: untouched
    assert bd.count.tolist() == [[1, 0, 0], [1, 1, 0]] and bd.sum_r[1, 1] == 0.25
    # shared bandit: one arm for the round, B plays applied in order
    sh = orc.Bandit(orc.POLICY_UCB1, n_bandits=1, n_arms=3)
    arms, _ = sh.select(4)
    assert arms.tolist() == [0, 0, 0, 0]
    sh.update(arms, [1, 2, 3, 4], [4, 4, 4, 4], [4, 4, 4, 4])
    assert sh.count.tolist() == [[4, 0, 0]] and sh.sum_r[0, 0] == 0.25 + 0.5 + 0.75 + 1.0
    # Thompson: the batched call equals the single call on each bandit's own uniforms
    ts = orc.Bandit(orc.POLICY_TS_BETA, n_bandits=3, n_arms=3)
    ts.sum_r[:] = [[1, 2, 3], [4, 1, 0.5], [0, 0, 0]]
    ts.count[:] = [[5, 5, 5], [6, 2, 9], [0, 0, 0]]
    u = np.random.default_rng(4).random((3, 3, 48), np.float32)
    arms, fl = ts.select(3, u)
    assert arms.tolist() == [orc.ts_select(ts.sum_r[b], ts.count[b], u[b])[0] for b in range(3)]
    assert not fl.any()


def test_ucb1_converges_to_best_arm():
    # the bandit loop as a whole: arm 2 has the highest mean reward and ends up played most
    g = np.random.default_rng(0)
    bd = orc.Bandit(orc.POLICY_UCB1, 1, 3)
    means = (0.3, 0.5, 0.7)
    for _ in range(3000):
        a = int(bd.select(1)[0][0])
        m = int(g.random() < means[a]) * 8
        bd.update([a], [m], [8], [8])
    assert bd.count[0].argmax() == 2 and bd.count[0, 2] > 2000
    np.testing.assert_allclose(bd.sum_r[0] / bd.count[0], means, atol=0.12)


# ---- bandit and reward variants of the ablations (Section 3.2, Section 3.3) ------------------------------

def test_reward_simple_is_the_normalised_acceptance_length():
    assert orc.reward_simple(3, 8) == 0.375 and orc.reward_simple(0, 5) == 0.0 and orc.reward_simple(5, 5) == 1.0
    # it is the alpha = 1 end of the blend, and it ignores how many tokens were drafted
    for m, n, g in ((2, 3, 8), (2, 7, 8), (4, 4, 16)):
        assert orc.reward_simple(m, g) == orc.reward(m, n, g, 1.0)
    bd = orc.Bandit(orc.POLICY_UCB1, 1, 2, reward_kind=orc.REWARD_SIMPLE)
    bd.update([1], [3], [4], [8])
    assert bd.sum_r[0, 1] == 0.375 and bd.sum_r2[0, 1] == 0.375 ** 2


def test_ucb_tuned_hand_cases(golden):
    for N, S, Q, t, want in golden("ucb_tuned_hand_cases.txt"):
        N, t = int(N), int(t)
        # two arms with the same statistics and N + N + 1 = t: both indices equal the hand value, tie -> arm 0
        assert 2 * N + 1 == t
        a, idx = orc.ucb_tuned_select([float(S)] * 2, [float(Q)] * 2, [N, N])
        assert a == 0
        np.testing.assert_allclose(idx, float(want), atol=2e-6)


def test_ucb_tuned_variance_is_the_population_variance_of_the_rewards_played():
    g = np.random.default_rng(11)
    bd = orc.Bandit(orc.POLICY_UCB_TUNED, 1, 3)
    hist = [[], [], []]
    for _ in range(400):
        a = int(g.integers(3))
        n = int(g.integers(1, 9)); m = int(g.integers(0, n + 1))
        bd.update([a], [m], [n], [8])
        hist[a].append(orc.reward(m, n, 8))
    t = 401
    _, idx = orc.ucb_tuned_select(bd.sum_r[0], bd.sum_r2[0], bd.count[0])
    for a in range(3):
        r = np.array(hist[a])
        V = np.var(r) + math.sqrt(2 * math.log(t) / len(r))          # numpy: two-pass, divides by N
        want = r.mean() + math.sqrt(math.log(t) / len(r) * min(0.25, V))
        assert idx[a] == pytest.approx(want, rel=1e-12)
    # more spread at equal mean and plays -> larger index, until the 1/4 cap
    lo = orc.ucb_tuned_select([500.0, 500.0], [250.0, 260.0], [1000, 1000])
    assert lo[0] == 1 and lo[1][1] > lo[1][0]
    capped = orc.ucb_tuned_select([5.0, 5.0], [2.5, 5.0], [10, 10])
    assert capped[0] == 0 and capped[1][0] == capped[1][1]


def test_ucb_tuned_plays_every_arm_once_first_and_explores_less_than_ucb1():
    s, q, c = np.zeros(3), np.zeros(3), np.zeros(3, np.int64)
    for expect in (0, 1, 2):
        a, idx = orc.ucb_tuned_select(s, q, c)
        assert a == expect and np.isinf(idx[expect])
        c[a] += 1; s[a] += 0.3; q[a] += 0.09
    # bonus <= sqrt(ln t / (4 N)) < UCB1's sqrt(2 ln t / N)
    s, q, c = np.array([30.0, 4.0]), np.array([12.0, 2.0]), np.array([60, 10])
    _, tuned = orc.ucb_tuned_select(s, q, c)
    _, plain = orc.ucb1_select(s, c)
    assert ((tuned - s / c) < (plain - s / c)).all() and ((tuned - s / c) > 0).all()


def test_ts_gauss_posterior_and_uniform_use():
    # u2 = 0 -> cos = 1, u1 = exp(-2) -> z = 2;  u2 = 0.5 -> z = -2;  u2 = 0.25 -> z = 0 (to rounding)
    u = np.zeros((3, 48), np.float32)
    u[:, 0] = math.exp(-2.0)
    u[:, 1] = (0.0, 0.5, 0.25)
    z = math.sqrt(-2.0 * math.log(float(np.float32(math.exp(-2.0)))))
    a, th = orc.ts_gauss_select([3.0, 3.0, 3.0], [8, 8, 8], u)
    np.testing.assert_allclose(th, [3 / 9 + z / 3, 3 / 9 - z / 3, 3 / 9], atol=1e-15)
    assert a == 0
    # fresh arm: the prior N(0, 1) itself
    a, th = orc.ts_gauss_select([0.0], [0], u[:1])
    assert th[0] == pytest.approx(z, rel=1e-15)
    # law of the draw: N(S/(N+1), 1/(N+1))
    g = np.random.default_rng(5)
    draws = np.array([orc.ts_gauss_select([6.0], [15], g.random((1, 48), np.float32))[1][0] for _ in range(40000)])
    assert draws.mean() == pytest.approx(6 / 16, abs=0.005)
    assert draws.var() == pytest.approx(1 / 16, rel=0.04)
    assert stats.kstest(draws, stats.norm(6 / 16, 0.25).cdf).pvalue > 1e-3
    # u1 = 0 is read as 2^-25, not as log(0)
    u0 = np.zeros((1, 48), np.float32)
    assert orc.ts_gauss_select([0.0], [0], u0)[1][0] == pytest.approx(math.sqrt(50 * math.log(2)), rel=1e-15)


def test_batched_select_dispatches_the_variants():
    u = np.random.default_rng(9).random((2, 3, 48), np.float32)
    for pol, single in ((orc.POLICY_UCB_TUNED, None), (orc.POLICY_TS_GAUSS, None)):
        bd = orc.Bandit(pol, 2, 3)
        bd.sum_r[:] = [[1.0, 2.5, 0.5], [3.0, 0.2, 0.1]]
        bd.sum_r2[:] = [[0.6, 1.4, 0.2], [1.9, 0.04, 0.01]]
        bd.count[:] = [[4, 5, 2], [6, 1, 1]]
        arms, fl = bd.select(2, u)
        for b in range(2):
            if pol == orc.POLICY_UCB_TUNED:
                want = orc.ucb_tuned_select(bd.sum_r[b], bd.sum_r2[b], bd.count[b])[0]
            else:
                want = orc.ts_gauss_select(bd.sum_r[b], bd.count[b], u[b])[0]
            assert arms[b] == want
        assert not fl.any()


# ---- token-level bandits (Section 3.1: every draft position is its own bandit; Section 3.2: binary reward) -----

def test_token_level_update_plays_only_the_positions_the_target_evaluated():
    bd = orc.Bandit(orc.POLICY_UCB1, n_bandits=2, n_arms=2, positions=4)
    arms = np.array([[0, 1, 1, 0], [1, 1, 0, 0]], np.int32)
    # sequence 0: 4 drafted, 2 accepted -> positions 0, 1 rewarded 1, position 2 (first rejection) rewarded 0, position 3 unplayed
    # sequence 1: 3 drafted, all accepted -> positions 0..2 rewarded 1, position 3 was never drafted
    bd.update(arms, [2, 3], [4, 3], [4, 4])
    assert bd.count[0].tolist() == [[1, 0], [0, 1], [0, 1], [0, 0]]
    assert bd.sum_r[0].tolist() == [[1, 0], [0, 1], [0, 0], [0, 0]]
    assert bd.count[1].tolist() == [[0, 1], [0, 1], [1, 0], [0, 0]]
    assert bd.sum_r[1].tolist() == [[0, 1], [0, 1], [1, 0], [0, 0]]
    assert (bd.sum_r2 == bd.sum_r).all()                       # r in {0, 1}
    # nothing accepted: only position 0 is played, with reward 0; an inactive sequence is skipped
    bd.update(arms, [0, 1], [2, 2], [4, 4], active=[1, 0])
    assert bd.count[0].tolist() == [[2, 0], [0, 1], [0, 1], [0, 0]] and bd.sum_r[0, 0, 0] == 1.0
    assert bd.count[1].sum() == 3
    # shared bandit: the plays of all sequences land in the one table, position by position
    sh = orc.Bandit(orc.POLICY_UCB1, n_bandits=1, n_arms=2, positions=3)
    sh.update(np.array([[0, 0, 0], [0, 1, 1], [1, 1, 1]], np.int32), [3, 1, 0], [3, 3, 2], [3, 3, 3])
    assert sh.count[0].tolist() == [[2, 1], [1, 1], [1, 0]]
    assert sh.sum_r[0].tolist() == [[2, 0], [1, 0], [1, 0]]


def test_token_level_select_is_the_single_bandit_rule_per_position():
    g = np.random.default_rng(21)
    for pol in (orc.POLICY_UCB1, orc.POLICY_TS_BETA):
        bd = orc.Bandit(pol, n_bandits=3, n_arms=3, positions=5)
        bd.count[:] = g.integers(0, 6, bd.count.shape)
        bd.sum_r[:] = np.minimum(bd.count, g.integers(0, 6, bd.count.shape))          # integer successes <= plays
        u = g.random((3, 5, 3, 48), np.float32)
        arms, fl = bd.select(3, u)
        assert arms.shape == (3, 5) and not fl.any()
        for b in range(3):
            for k in range(5):
                if pol == orc.POLICY_UCB1:
                    want = orc.ucb1_select(bd.sum_r[b, k], bd.count[b, k])[0]
                else:                                                             # Beta(1 + successes, 1 + failures)
                    want, th, _ = orc.ts_select(bd.sum_r[b, k], bd.count[b, k], u[b, k])
                    for a in range(3):
                        assert th[a] == orc.beta_draw(1 + bd.sum_r[b, k, a], 1 + bd.count[b, k, a] - bd.sum_r[b, k, a], u[b, k, a])[0]
                assert arms[b, k] == want
    # shared: every sequence gets the arms drawn for sequence 0
    sh = orc.Bandit(orc.POLICY_TS_BETA, n_bandits=1, n_arms=3, positions=5)
    arms, _ = sh.select(3, u)
    assert (arms == arms[0]).all()


def test_token_level_stop_scan_uses_the_arm_of_each_position():
    # rows uniform over n tokens: sqrt(H) = sqrt(ln n); p_top1 = 1/n; margin 0 for n >= 2
    V = 32
    x = np.full((1, 4, V), -np.inf, np.float32)
    for k, n in enumerate((1, 1, 2, 8)):
        x[0, k, :n] = 0.0
    rules, th = [orc.RULE_SVIP, orc.RULE_MAXCONF, orc.RULE_MARGIN], [0.6, 0.8, 0.2]
    # SVIP fires on rows 2, 3 (0.83, 1.44 > 0.6); Max-Confidence on rows 2, 3 (0.5, 0.125 < 0.8); LogitMargin on rows
    # 2, 3 (margin 0) but not on one-hot rows (margin 1)
    for arms, fired in (([0, 0, 0, 0], [0, 0, 1, 1]), ([2, 1, 0, 2], [0, 0, 1, 1]), ([1, 1, 1, 1], [0, 0, 1, 1])):
        o = orc.draft_stats(x, arm=np.array([arms]), rules=rules, thresholds=th, token_level=True)
        assert o["stop_fired"][0].tolist() == fired and o["n_stop"][0] == 3
    # thresholds that make the per-position arm matter: SVIP at 1.0 fires on row 3 only, Max-Confidence at 0.3 on row 3 only,
    # LogitMargin at 0.2 on rows 2 and 3
    th2 = [1.0, 0.3, 0.2]
    o = orc.draft_stats(x, arm=np.array([[0, 0, 0, 0]]), rules=rules, thresholds=th2, token_level=True)
    assert o["stop_fired"][0].tolist() == [0, 0, 0, 1] and o["n_stop"][0] == 4
    o = orc.draft_stats(x, arm=np.array([[0, 0, 2, 0]]), rules=rules, thresholds=th2, token_level=True)
    assert o["stop_fired"][0].tolist() == [0, 0, 1, 1] and o["n_stop"][0] == 3
    o = orc.draft_stats(x, arm=np.array([[2, 2, 1, 1]]), rules=rules, thresholds=th2, token_level=True)
    assert o["stop_fired"][0].tolist() == [0, 0, 0, 1] and o["n_stop"][0] == 4
