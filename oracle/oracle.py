"""ctypes front end of the CPU oracle (oracle/tapout_oracle.c).

Test infrastructure only: tests, the smoke check and the benchmark's
CPU-baseline leg import this module; the product package never does.  All
arithmetic lives in the C file; this module marshals numpy arrays.

Logits arrays are numpy float32 (binary32 logits) or uint16 (bfloat16 bit
patterns); `as_logits` turns a CPU torch tensor into such a view.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tapout_oracle.c")
_LIB = os.path.join(_HERE, "libtapout_oracle.so")

TS_UNIFORMS_PER_ARM = 48
RULE_SVIP, RULE_MAXCONF, RULE_MARGIN, RULE_SVIP_DIFF, RULE_ADAEDL = 0, 1, 2, 3, 4
POLICY_UCB1, POLICY_TS_BETA, POLICY_UCB_TUNED, POLICY_TS_GAUSS = 0, 1, 2, 3
REWARD_BLEND, REWARD_SIMPLE = 0, 1
FLAG_BAD_ROW, FLAG_BAD_TOKEN, FLAG_BAD_NDRAFT, FLAG_SAMPLER_EXHAUSTED = 1, 2, 4, 8


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fopenmp", "-fPIC", "-shared",
               "-ffp-contract=off", "-fvisibility=hidden", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.tapout_oracle_reward.restype = C.c_double
        _lib.tapout_oracle_reward.argtypes = [C.c_int, C.c_int, C.c_int, C.c_double]
        _lib.tapout_oracle_gamma.restype = C.c_double
        _lib.tapout_oracle_gamma.argtypes = [C.c_double, C.c_void_p, C.c_void_p]
        _lib.tapout_oracle_beta.restype = C.c_double
        _lib.tapout_oracle_beta.argtypes = [C.c_double, C.c_double, C.c_void_p, C.c_void_p]
        _lib.tapout_oracle_reward_simple.restype = C.c_double
        _lib.tapout_oracle_reward_simple.argtypes = [C.c_int, C.c_int]
        _lib.tapout_oracle_inverse_cdf.restype = C.c_int32
        _lib.tapout_oracle_inverse_cdf.argtypes = [C.c_void_p, C.c_int64, C.c_double, C.c_void_p, C.c_void_p]
    return _lib


def as_logits(t):
    """CPU torch tensor (float32 / bfloat16) or numpy array -> numpy view the oracle reads."""
    if isinstance(t, np.ndarray):
        assert t.dtype in (np.float32, np.uint16)
        return t
    import torch
    assert t.device.type == "cpu"
    if t.dtype == torch.float32:
        return t.numpy()
    assert t.dtype == torch.bfloat16
    return t.view(torch.int16).numpy().view(np.uint16)


def _dtype_code(a: np.ndarray) -> int:
    return 0 if a.dtype == np.float32 else 1


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _strides(a: np.ndarray):
    assert a.ndim == 3 and a.strides[2] == a.itemsize, "vocabulary axis must be contiguous"
    return a.strides[0] // a.itemsize, a.strides[1] // a.itemsize


def _i32(x, shape=None):
    if x is None:
        return None
    a = np.ascontiguousarray(np.asarray(x), dtype=np.int32)
    if shape is not None:
        assert a.shape == shape, (a.shape, shape)
    return a


def _f32(x, shape=None):
    if x is None:
        return None
    a = np.ascontiguousarray(np.asarray(x), dtype=np.float32)
    if shape is not None:
        assert a.shape == shape, (a.shape, shape)
    return a


def _u8(x, shape=None):
    if x is None:
        return None
    a = np.ascontiguousarray(np.asarray(x), dtype=np.uint8)
    if shape is not None:
        assert a.shape == shape, (a.shape, shape)
    return a


def row_stats(row) -> dict:
    row = as_logits(row)
    assert row.ndim == 1 and row.flags.c_contiguous
    out = np.zeros(7, np.float64)
    top1 = C.c_int32(0)
    bad = lib().tapout_oracle_row_stats(_p(row), _dtype_code(row), C.c_int64(row.shape[0]), _p(out), C.byref(top1))
    keys = ("lse", "H", "p1", "p2", "margin", "M", "S")
    d = dict(zip(keys, out.tolist()))
    d["top1"] = top1.value
    d["bad"] = bool(bad)
    return d


def draft_stats(draft, draft_tok=None, k_len=None, arm=None, rules=(0, 1, 2),
                thresholds=(0.6, 0.8, 0.2), nthreads=1, prev_entropy=None, lam=None, adaedl_gamma=0.5,
                token_level=False) -> dict:
    """Signals of every draft row and the stop position of Algorithm 1's draft loop.
    prev_entropy [B] f32 (NaN = none) feeds SVIPDifference at the first position; lam [B, arms] f64 the
    adaptive thresholds of AdaEDL arms.  token_level: arm is [B, K], one arm per draft position (Section 3.1)."""
    draft = as_logits(draft)
    B, K, V = draft.shape
    sb, sk = _strides(draft)
    tok = _i32(draft_tok, (B, K))
    kl = _i32(k_len, (B,))
    ar = _i32(arm, (B, K) if token_level else (B,))
    rl = _i32(rules)
    th = _f32(thresholds)
    f = lambda: np.full((B, K), np.nan, np.float32)
    o = dict(lse=f(), entropy=f(), p_top1=f(), p_top2=f(), margin=f(),
             top1_id=np.full((B, K), -1, np.int32), logq_tok=f(),
             n_stop=np.zeros(B, np.int32), stop_fired=np.zeros((B, K), np.uint8),
             stop_margin=np.full((B, K), np.inf, np.float64), flags=np.zeros(B, np.uint32))
    lib().tapout_oracle_draft_stats(
        _p(draft), _dtype_code(draft), C.c_int64(sb), C.c_int64(sk), B, K, C.c_int64(V),
        _p(tok), _p(kl), _p(ar), len(rl), _p(rl), _p(th),
        _p(o["lse"]), _p(o["entropy"]), _p(o["p_top1"]), _p(o["p_top2"]), _p(o["margin"]),
        _p(o["top1_id"]), _p(o["logq_tok"]) if tok is not None else None,
        _p(o["n_stop"]), _p(o["stop_fired"]), _p(o["stop_margin"]), _p(o["flags"]),
        _p(_f32(prev_entropy, (B,))), _p(None if lam is None else np.ascontiguousarray(lam, np.float64)),
        C.c_double(adaedl_gamma), K if token_level else 0, int(nthreads))
    if ar is None:
        o["n_stop"] = None
    return o


def draft_sample(draft, u_draft, k_len=None, nthreads=1) -> dict:
    """Draft tokens drawn from softmax(draft row) by inverse CDF at the caller's uniforms (Algorithm 1)."""
    draft = as_logits(draft)
    B, K, V = draft.shape
    sb, sk = _strides(draft)
    o = dict(tok=np.full((B, K), -1, np.int32), icdf_margin=np.full((B, K), np.inf, np.float64), flags=np.zeros(B, np.uint32))
    lib().tapout_oracle_draft_sample(_p(draft), _dtype_code(draft), C.c_int64(sb), C.c_int64(sk), B, K, C.c_int64(V),
                                     _p(_i32(k_len, (B,))), _p(_f32(u_draft, (B, K))), _p(o["tok"]), _p(o["icdf_margin"]),
                                     _p(o["flags"]), int(nthreads))
    return o


def verify(target, draft, logq_tok, draft_tok, n_draft, u_accept, u_sample, greedy=None, nthreads=1) -> dict:
    """Speculative-sampling verification and final token of every sequence."""
    target = as_logits(target)
    draft = as_logits(draft)
    B, K1, V = target.shape
    K = K1 - 1
    assert draft.shape == (B, K, V)
    tsb, tsk = _strides(target)
    dsb, dsk = _strides(draft)
    lq = _f32(logq_tok, (B, K))
    tok = _i32(draft_tok, (B, K))
    nd = _i32(n_draft, (B,))
    gr = _u8(greedy, (B,))
    ua = _f32(u_accept, (B, K))
    us = _f32(u_sample, (B,))
    o = dict(accept_len=np.zeros(B, np.int32), out_tok=np.full((B, K + 1), -1, np.int32),
             n_out=np.zeros(B, np.int32), target_lse=np.full((B, K + 1), np.nan, np.float32),
             logp_tok=np.full((B, K), np.nan, np.float32), target_top1=np.full((B, K + 1), -1, np.int32),
             accept_margin=np.full((B, K), np.inf, np.float64), icdf_margin=np.full(B, np.inf, np.float64),
             flags=np.zeros(B, np.uint32))
    lib().tapout_oracle_verify(
        _p(target), _dtype_code(target), C.c_int64(tsb), C.c_int64(tsk),
        _p(draft), _dtype_code(draft), C.c_int64(dsb), C.c_int64(dsk),
        B, K, C.c_int64(V), _p(lq), _p(tok), _p(nd), _p(gr), _p(ua), _p(us),
        _p(o["accept_len"]), _p(o["out_tok"]), _p(o["n_out"]),
        _p(o["target_lse"]), _p(o["logp_tok"]), _p(o["target_top1"]),
        _p(o["accept_margin"]), _p(o["icdf_margin"]), _p(o["flags"]), int(nthreads))
    return o


def reward(m: int, n_drafted: int, gamma: int, alpha: float = 0.5) -> float:
    return lib().tapout_oracle_reward(int(m), int(n_drafted), int(gamma), float(alpha))


def reward_simple(m: int, gamma: int) -> float:
    return lib().tapout_oracle_reward_simple(int(m), int(gamma))


def ucb_tuned_select(sum_r, sum_r2, count):
    s = np.ascontiguousarray(sum_r, np.float64)
    q = np.ascontiguousarray(sum_r2, np.float64)
    c = np.ascontiguousarray(count, np.int64)
    idx = np.zeros(len(s), np.float64)
    a = lib().tapout_oracle_ucb_tuned_select(_p(s), _p(q), _p(c), len(s), _p(idx))
    return a, idx


def ts_gauss_select(sum_r, count, u):
    s = np.ascontiguousarray(sum_r, np.float64)
    c = np.ascontiguousarray(count, np.int64)
    u = _f32(u, (len(s), TS_UNIFORMS_PER_ARM))
    th = np.zeros(len(s), np.float64)
    a = lib().tapout_oracle_ts_gauss_select(_p(s), _p(c), len(s), _p(u), _p(th))
    return a, th


def ucb1_select(sum_r, count):
    s = np.ascontiguousarray(sum_r, np.float64)
    c = np.ascontiguousarray(count, np.int64)
    idx = np.zeros(len(s), np.float64)
    a = lib().tapout_oracle_ucb1_select(_p(s), _p(c), len(s), _p(idx))
    return a, idx


def ts_select(sum_r, count, u):
    s = np.ascontiguousarray(sum_r, np.float64)
    c = np.ascontiguousarray(count, np.int64)
    u = _f32(u, (len(s), TS_UNIFORMS_PER_ARM))
    th = np.zeros(len(s), np.float64)
    ex = C.c_int(0)
    a = lib().tapout_oracle_ts_select(_p(s), _p(c), len(s), _p(u), _p(th), C.byref(ex))
    return a, th, bool(ex.value)


def gamma_draw(shape: float, u) -> tuple:
    u = _f32(u, (24,))
    ex = C.c_int(0)
    g = lib().tapout_oracle_gamma(float(shape), _p(u), C.byref(ex))
    return g, bool(ex.value)


def beta_draw(a: float, b: float, u) -> tuple:
    u = _f32(u, (48,))
    ex = C.c_int(0)
    v = lib().tapout_oracle_beta(float(a), float(b), _p(u), C.byref(ex))
    return v, bool(ex.value)


def inverse_cdf(w, u: float):
    w = np.ascontiguousarray(w, np.float64)
    Z = C.c_double(0)
    mg = C.c_double(0)
    j = lib().tapout_oracle_inverse_cdf(_p(w), C.c_int64(len(w)), float(u), C.byref(Z), C.byref(mg))
    return j, Z.value, mg.value


class Bandit:
    """Host-side bandit state driven by the oracle's select/update (Section 3.3).  positions > 1: token-level
    bandits, one per draft position (Section 3.1), state [n_bandits, positions, arms], binary rewards."""

    def __init__(self, policy: int, n_bandits: int, n_arms: int, alpha: float = 0.5, reward_kind: int = REWARD_BLEND,
                 positions: int = 1):
        self.policy, self.n_bandits, self.A, self.alpha, self.reward_kind = policy, n_bandits, n_arms, alpha, reward_kind
        self.P = positions
        shape = (n_bandits, n_arms) if positions == 1 else (n_bandits, positions, n_arms)
        self.sum_r = np.zeros(shape, np.float64)
        self.sum_r2 = np.zeros(shape, np.float64)
        self.count = np.zeros(shape, np.int64)

    def select(self, B: int, u_ts=None):
        arm = np.zeros(B if self.P == 1 else (B, self.P), np.int32)
        flags = np.zeros(B, np.uint32)
        u = None
        if self.policy in (POLICY_TS_BETA, POLICY_TS_GAUSS):
            u = _f32(u_ts, (B, self.A, TS_UNIFORMS_PER_ARM) if self.P == 1 else (B, self.P, self.A, TS_UNIFORMS_PER_ARM))
        lib().tapout_oracle_bandit_select(self.policy, self.n_bandits, B, self.A, self.P, _p(self.sum_r), _p(self.sum_r2),
                                          _p(self.count), _p(u), _p(arm), _p(flags))
        return arm, flags

    def update(self, arm, accept_len, n_draft, gamma, active=None):
        B = len(arm)
        lib().tapout_oracle_bandit_update(self.n_bandits, B, self.A, self.P, self.reward_kind, C.c_double(self.alpha),
                                          _p(self.sum_r), _p(self.sum_r2), _p(self.count),
                                          _p(_i32(arm, (B,) if self.P == 1 else (B, self.P))), _p(_i32(accept_len, (B,))),
                                          _p(_i32(n_draft, (B,))), _p(_i32(gamma, (B,))), _p(_u8(active)))


class RuleState:
    """Carried state of the stateful stop rules (Appendix A.1): per sequence the entropy of the last drafted
    position of the previous draft (SVIPDifference) and AdaEDL's smoothed acceptance rate; per sequence and
    arm AdaEDL's threshold lambda (it starts at the arm's configured threshold)."""

    def __init__(self, B: int, rules, thresholds, ad_alpha=0.9, beta1=0.5, beta2=0.9, eps=0.01, rate0=None, steer_raw=False):
        """steer_raw: AdaEDL's threshold follows sign(alpha - r_t), this draft's own acceptance rate, as Appendix A.1
        prints it; default: sign(alpha - smoothed rate)."""
        self.steer_raw = bool(steer_raw)
        self.B, self.rules = B, _i32(rules)
        self.A = len(self.rules)
        self.ad_alpha, self.beta1, self.beta2, self.eps = ad_alpha, beta1, beta2, eps
        self.prev_entropy = np.full(B, np.nan, np.float32)
        self.accept_rate = np.full(B, ad_alpha if rate0 is None else rate0, np.float64)
        self.lam = np.tile(np.asarray(thresholds, np.float32).astype(np.float64), (B, 1))

    def update(self, entropy, n_draft, accept_len, active=None):
        B = self.B
        ent = None if entropy is None else _f32(entropy)
        K = 0 if ent is None else ent.shape[1]
        if ent is None:
            K = int(np.max(n_draft)) if len(n_draft) else 0
        lib().tapout_oracle_rule_state_update(
            B, K, self.A, _p(self.rules), _p(ent), _p(_i32(n_draft, (B,))), _p(_i32(accept_len, (B,))),
            _p(_u8(active)), _p(self.prev_entropy), _p(self.accept_rate), _p(self.lam),
            C.c_double(self.ad_alpha), C.c_double(self.beta1), C.c_double(self.beta2), C.c_double(self.eps),
            int(self.steer_raw))
