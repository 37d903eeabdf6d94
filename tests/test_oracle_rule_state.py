"""Pins of the oracle's stateful stop rules (SVIPDifference, AdaEDL) and of their carried state (CPU only).

The rows are uniform over n tokens with every other token masked, so their entropy is ln n in closed form and the
expected decisions in tests/golden/ were worked out by hand from the paper's Table 1 / Appendix A.1 formulas.
The VALUES of AdaEDL's hyper-parameters and the exact shape of its threshold update are not recoverable from the
paper (printed garbled): those stay parity unpinned; what is pinned here is the arithmetic of both readings the oracle
offers (threshold steered by the smoothed acceptance rate, or by the draft's own rate as the equation is printed).
"""
import math

import numpy as np
import pytest

from oracle import oracle as orc

V = 32


def uniform_rows(sizes):
    x = np.full((1, len(sizes), V), -np.inf, np.float32)
    for k, n in enumerate(sizes):
        x[0, k, 3:3 + n] = 1.25          # any constant: the law is uniform over n tokens
    return x


def test_table1_lists_the_fourth_threshold(golden):
    rows = {r[0]: r for r in golden("table1_stop_rules.txt")}
    assert rows["SVIPDifference"][2:] == [">", "0.2"]


def test_svip_difference_golden(golden):
    for row in golden("svip_difference_uniform_rows.txt"):
        sizes = [int(v) for v in row[0:4]]
        prev = None if row[4] == "none" else np.array([float(row[4])], np.float32)
        fired = [int(v) for v in row[5:9]]
        n_stop = int(row[9])
        x = uniform_rows(sizes)
        o = orc.draft_stats(x, arm=[0], rules=[orc.RULE_SVIP_DIFF], thresholds=[0.2], prev_entropy=prev)
        np.testing.assert_allclose(o["entropy"][0], np.log(sizes), rtol=1e-6)
        assert o["stop_fired"][0].tolist() == fired, row
        assert o["n_stop"][0] == n_stop, row


def test_svip_difference_without_history_cannot_fire_at_the_first_step():
    x = uniform_rows([16, 16])
    for prev in (None, np.array([np.nan], np.float32)):
        o = orc.draft_stats(x, arm=[0], rules=[orc.RULE_SVIP_DIFF], thresholds=[0.2], prev_entropy=prev)
        assert o["stop_fired"][0].tolist() == [0, 0] and o["n_stop"][0] == 2
        assert np.isinf(o["stop_margin"][0, 0])
    # a previous entropy of 0 (one-hot) makes the first step a jump of sqrt(ln 16) = 1.665
    o = orc.draft_stats(x, arm=[0], rules=[orc.RULE_SVIP_DIFF], thresholds=[0.2], prev_entropy=np.zeros(1, np.float32))
    assert o["stop_fired"][0].tolist() == [1, 0] and o["n_stop"][0] == 1
    assert o["stop_margin"][0, 0] == pytest.approx((math.sqrt(math.log(16)) - 0.2) / 0.2, rel=1e-6)


def test_svip_difference_is_strict_and_reads_its_own_threshold():
    x = uniform_rows([4, 4, 8])
    # delta of row 1 is exactly 0: "> 0" is false; row 2's delta 0.2646 fires for h = 0.26, not for h = 0.27
    o = orc.draft_stats(x, arm=[0], rules=[orc.RULE_SVIP_DIFF], thresholds=[0.0])
    assert o["stop_fired"][0].tolist() == [0, 0, 1]
    for h, want in ((0.26, 1), (0.27, 0)):
        o = orc.draft_stats(x, arm=[1], rules=[orc.RULE_SVIP, orc.RULE_SVIP_DIFF], thresholds=[9.0, h])
        assert o["stop_fired"][0, 2] == want


def test_adaedl_golden(golden):
    for row in golden("adaedl_uniform_rows.txt"):
        g, lam = float(row[0]), float(row[1])
        sizes = [int(v) for v in row[2:5]]
        fired = [int(v) for v in row[5:8]]
        n_stop = int(row[8])
        x = uniform_rows(sizes)
        o = orc.draft_stats(x, arm=[0], rules=[orc.RULE_ADAEDL], thresholds=[0.0], lam=np.array([[lam]]), adaedl_gamma=g)
        assert o["stop_fired"][0].tolist() == fired, row
        assert o["n_stop"][0] == n_stop, row


def test_adaedl_reads_the_lambda_of_its_own_arm_and_sequence():
    x = np.concatenate([uniform_rows([2, 4]), uniform_rows([2, 4])])            # 1 - sqrt(0.5 ln n): 0.4113, 0.1674
    rules = [orc.RULE_ADAEDL, orc.RULE_MAXCONF, orc.RULE_ADAEDL]
    lam = np.array([[0.3, 0.0, 0.5], [0.1, 0.0, 0.3]])
    o = orc.draft_stats(x, arm=[0, 0], rules=rules, thresholds=[9, 9, 9], lam=lam)
    assert o["stop_fired"].tolist() == [[0, 1], [0, 0]]
    o = orc.draft_stats(x, arm=[2, 2], rules=rules, thresholds=[9, 9, 9], lam=lam)
    assert o["stop_fired"].tolist() == [[1, 1], [0, 1]]
    # without a state array the configured threshold is the lambda
    o = orc.draft_stats(x, arm=[0, 0], rules=rules, thresholds=[0.3, 9, 9])
    assert o["stop_fired"].tolist() == [[0, 1], [0, 1]]


def test_state_update_takes_the_last_drafted_row_and_skips_inactive_or_invalid():
    B, K = 4, 5
    ent = np.arange(B * K, dtype=np.float32).reshape(B, K) / 7
    st = orc.RuleState(B, [orc.RULE_SVIP_DIFF, orc.RULE_ADAEDL], [0.2, 0.4], ad_alpha=0.9, beta1=0.5, beta2=0.9, eps=0.01, rate0=1.0)
    st.update(ent, n_draft=[3, 5, 0, 2], accept_len=[1, 5, 0, 2], active=[1, 1, 1, 0])
    assert st.prev_entropy[0] == ent[0, 2] and st.prev_entropy[1] == ent[1, 4]
    assert np.isnan(st.prev_entropy[2]) and np.isnan(st.prev_entropy[3])          # n_draft 0 / inactive: untouched
    assert st.accept_rate.tolist() == [0.5 * 1.0 + 0.5 * (1 / 3), 1.0, 1.0, 1.0]
    step = (1 - 0.9) * 0.01
    # only the AdaEDL column moves: up where the smoothed rate fell below alpha, down where it stayed above
    l0 = float(np.float32(0.4))                                                     # thresholds are binary32 at the boundary
    np.testing.assert_allclose(st.lam[:, 1], [l0 + step, l0 - step, l0, l0], rtol=0, atol=1e-15)
    assert (st.lam[:, 0] == np.float32(0.2)).all()


def test_adaedl_state_follows_the_closed_forms():
    """EMA: rate_t = r + beta1^t (rate_0 - r).  lambda moves by exactly (1 - beta2) eps against sign(rate - alpha)."""
    alpha, b1, b2, eps, lam0 = 0.87, 0.5, 0.9, 0.01, 0.4
    st = orc.RuleState(1, [orc.RULE_ADAEDL], [lam0], ad_alpha=alpha, beta1=b1, beta2=b2, eps=eps, rate0=1.0)
    signs = 0
    lam0 = float(np.float32(lam0))
    for t in range(1, 12):
        st.update(None, n_draft=[5], accept_len=[4])                # r = 0.8 every round
        rate = 0.8 + b1 ** t * (1.0 - 0.8)                          # 0.9, 0.85, 0.825, ...
        assert st.accept_rate[0] == pytest.approx(rate, rel=1e-14)
        signs += 1 if alpha > rate else -1                          # first round above alpha, all later ones below
        assert st.lam[0, 0] == pytest.approx(lam0 + signs * (1 - b2) * eps, abs=1e-15)
    assert signs == 9
    # a rate that sits exactly on alpha leaves lambda where it is
    st = orc.RuleState(1, [orc.RULE_ADAEDL], [0.25], ad_alpha=0.75, beta1=0.5, beta2=0.9, eps=0.01, rate0=0.75)
    st.update(None, n_draft=[4], accept_len=[3])
    assert st.accept_rate[0] == 0.75 and st.lam[0, 0] == 0.25
    # everything accepted, rate stays at 1 > alpha: lambda falls linearly (drafts get longer)
    st = orc.RuleState(1, [orc.RULE_ADAEDL], [0.5], ad_alpha=0.9, beta1=0.5, beta2=0.75, eps=0.04, rate0=1.0)
    for t in range(1, 6):
        st.update(None, n_draft=[6], accept_len=[6])
        assert st.lam[0, 0] == pytest.approx(0.5 - t * 0.25 * 0.04, abs=1e-15)


def test_adaedl_update_golden_both_readings(golden):
    """Four drafts worked by hand (tests/golden/adaedl_update_two_readings.txt): the printed form steers lambda by
    sign(alpha - r_t), the other reading by sign(alpha - smoothed rate); the two part ways at the first draft."""
    rows = golden("adaedl_update_two_readings.txt")
    for raw, sign_col, lam_col in ((True, 4, 5), (False, 6, 7)):
        st = orc.RuleState(1, [orc.RULE_ADAEDL], [0.4], ad_alpha=0.87, beta1=0.5, beta2=0.9, eps=0.01, rate0=1.0, steer_raw=raw)
        lam = float(np.float32(0.4))
        for row in rows:
            n_acc, n_dr = int(row[0]), int(row[1])
            st.update(None, n_draft=[n_dr], accept_len=[n_acc])
            assert n_acc / n_dr == pytest.approx(float(row[2]))
            assert st.accept_rate[0] == pytest.approx(float(row[3]), rel=1e-14)     # the average is kept under both readings
            lam += int(row[sign_col]) * (1 - 0.9) * 0.01
            assert st.lam[0, 0] == pytest.approx(lam, abs=1e-15)
            assert st.lam[0, 0] == pytest.approx(float(row[lam_col]) + (float(np.float32(0.4)) - 0.4), abs=1e-12)


def test_adaedl_as_printed_ignores_the_running_average():
    """Steered by r_t, lambda's path does not depend on where the smoothed rate starts or how it is smoothed."""
    paths = []
    for rate0, b1 in ((1.0, 0.5), (0.0, 0.9), (0.5, 0.0)):
        st = orc.RuleState(1, [orc.RULE_ADAEDL], [0.3], ad_alpha=0.7, beta1=b1, beta2=0.8, eps=0.02, rate0=rate0, steer_raw=True)
        path = []
        for m, n in ((3, 4), (2, 4), (7, 10), (4, 4), (0, 3)):       # r = .75, .5, .7 (= alpha: no move), 1, 0
            st.update(None, n_draft=[n], accept_len=[m])
            path.append(st.lam[0, 0])
        paths.append(path)
    assert paths[0] == paths[1] == paths[2]
    step, l0 = (1 - 0.8) * 0.02, float(np.float32(0.3))
    np.testing.assert_allclose(paths[0], [l0 - step, l0, l0, l0 - step, l0], atol=1e-15)
