"""ctypes binding of libtapout.so (include/tapout.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  torch supplies device memory and the stream; nothing here computes.
The binding fails loudly if the built library is missing: there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libtapout.so")

MAX_ARMS = 8
TS_UNIFORMS_PER_ARM = 48
F32, BF16 = 0, 1
RULE_SVIP, RULE_MAXCONF, RULE_MARGIN, RULE_SVIP_DIFF, RULE_ADAEDL = 0, 1, 2, 3, 4
UCB1, TS_BETA, UCB_TUNED, TS_GAUSS = 0, 1, 2, 3
REWARD_BLEND, REWARD_SIMPLE = 0, 1
SEQUENCE_LEVEL, TOKEN_LEVEL = 0, 1
FLAG_BAD_ROW, FLAG_BAD_TOKEN, FLAG_BAD_NDRAFT, FLAG_SAMPLER_EXHAUSTED = 1, 2, 4, 8
STATUS = {0: "TAPOUT_OK", 1: "TAPOUT_EINVAL", 2: "TAPOUT_EUNSUPPORTED", 3: "TAPOUT_ENOMEM", 4: "TAPOUT_EHIP"}

EXPORTS = ("tapout_default_config", "tapout_create", "tapout_destroy", "tapout_last_error",
           "tapout_bandit_select", "tapout_draft_stats", "tapout_draft_stats_static", "tapout_verify", "tapout_bandit_update",
           "tapout_bandit_update_select", "tapout_round", "tapout_bandit_get_state", "tapout_bandit_set_state", "tapout_rule_state_get", "tapout_rule_state_set",
           "tapout_shard_stats", "tapout_draft_stats_sharded", "tapout_verify_accept_sharded",
           "tapout_shard_final_sums", "tapout_shard_final_token",
           "tapout_set_option",
           "tapout_profile_enable", "tapout_profile_read")

PROFILE_KINDS = ("select", "draft_pass", "draft_finalize", "target_pass", "verify_head", "verify_slices", "verify_locate", "update",
                 "sample_head", "sample_slices", "sample_locate", "stream_pair")


class TapoutConfig(C.Structure):
    _fields_ = [("device", C.c_int32), ("max_batch", C.c_int32), ("max_k", C.c_int32), ("vocab", C.c_int32),
                ("n_arms", C.c_int32), ("rule", C.c_int32 * MAX_ARMS), ("threshold", C.c_float * MAX_ARMS),
                ("policy", C.c_int32), ("n_bandits", C.c_int32), ("alpha", C.c_double),
                ("reward", C.c_int32), ("granularity", C.c_int32),
                ("adaedl_gamma", C.c_double), ("adaedl_alpha", C.c_double), ("adaedl_beta1", C.c_double),
                ("adaedl_beta2", C.c_double), ("adaedl_eps", C.c_double), ("adaedl_rate0", C.c_double),
                ("draft_sampling", C.c_int32), ("adaedl_steer", C.c_int32)]


class TapoutLogits(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("dtype", C.c_int32), ("stride_b", C.c_int64), ("stride_k", C.c_int64)]


class TapoutRoundArgs(C.Structure):
    _fields_ = [("draft", C.POINTER(TapoutLogits)), ("target", C.POINTER(TapoutLogits)),
                ("B", C.c_int32), ("K", C.c_int32), ("V", C.c_int32)] + \
               [(n, C.c_void_p) for n in ("draft_tok", "k_len", "n_draft", "greedy", "u_accept", "u_sample", "u_ts_next", "arm", "gamma",
                                          "active", "lse", "entropy", "p_top1", "p_top2", "margin", "top1_id", "logq_tok", "n_stop",
                                          "stop_fired", "draft_flags", "accept_len", "out_tok", "n_out", "target_lse", "logp_tok",
                                          "target_top1", "verify_flags", "select_flags")]


class TapoutError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{STATUS.get(status, status)}: {text}")
        self.status = status


_lib = None


def load_library(path: str = None):
    """Load the in-tree libtapout.so; raises if it has not been built.  `path` (first call only): another build of the
    same sources, such as the one with time stamps that wg_stamps.py measures with."""
    global _lib
    if _lib is None:
        path = path or LIB_PATH
        if not os.path.exists(path):
            raise ImportError(f"{path} is missing: build it with `python -m paper_2511_02017_amd.build`")
        lib = C.CDLL(path)
        vp, i32 = C.c_void_p, C.c_int32
        lib.tapout_default_config.restype = None
        lib.tapout_default_config.argtypes = [C.POINTER(TapoutConfig), i32, i32, i32]
        lib.tapout_create.argtypes = [C.POINTER(vp), C.POINTER(TapoutConfig)]
        lib.tapout_destroy.argtypes = [vp]
        lib.tapout_last_error.restype = C.c_char_p
        lib.tapout_last_error.argtypes = [vp]
        lib.tapout_bandit_select.argtypes = [vp, i32, vp, vp, vp, vp]
        lib.tapout_draft_stats.argtypes = [vp, C.POINTER(TapoutLogits), i32, i32, i32] + [vp] * 16
        lib.tapout_draft_stats_static.argtypes = [C.POINTER(TapoutLogits), i32, i32, i32, vp, vp, vp, i32, vp, vp] + [vp] * 11
        lib.tapout_shard_stats.argtypes = [vp, C.POINTER(TapoutLogits), i32, i32, i32, i32, vp, i32, vp, vp, vp]
        lib.tapout_draft_stats_sharded.argtypes = [vp, vp, i32, i32, i32, i32] + [vp] * 14
        lib.tapout_verify_accept_sharded.argtypes = [vp, vp, i32, i32, i32, i32] + [vp] * 15
        lib.tapout_shard_final_sums.argtypes = [vp, C.POINTER(TapoutLogits), C.POINTER(TapoutLogits), i32, i32, i32, vp, vp, vp]
        lib.tapout_shard_final_token.argtypes = [vp, C.POINTER(TapoutLogits), C.POINTER(TapoutLogits), i32, i32, i32, i32, i32, i32] + [vp] * 8
        lib.tapout_verify.argtypes = [vp, C.POINTER(TapoutLogits), C.POINTER(TapoutLogits), i32, i32, i32] + [vp] * 15
        lib.tapout_bandit_update.argtypes = [vp, i32] + [vp] * 6
        lib.tapout_bandit_update_select.argtypes = [vp, i32] + [vp] * 9
        lib.tapout_round.argtypes = [vp, C.POINTER(TapoutRoundArgs), vp]
        lib.tapout_bandit_get_state.argtypes = [vp] * 5
        lib.tapout_bandit_set_state.argtypes = [vp] * 5
        lib.tapout_rule_state_get.argtypes = [vp] * 5
        lib.tapout_rule_state_set.argtypes = [vp] * 5
        lib.tapout_set_option.argtypes = [vp, C.c_char_p, i32]
        lib.tapout_profile_enable.argtypes = [vp, C.c_uint32, i32]
        lib.tapout_profile_read.argtypes = [vp, i32, C.POINTER(C.c_double), C.POINTER(i32), vp]
        _lib = lib
    return _lib


def default_config(max_batch: int, max_k: int, vocab: int) -> TapoutConfig:
    cfg = TapoutConfig()
    load_library().tapout_default_config(C.byref(cfg), max_batch, max_k, vocab)
    return cfg


def _ptr(t, dtype=None, shape=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name}: expected {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _logits(t, name) -> TapoutLogits:
    if t.dim() != 3 or not t.is_cuda:
        raise ValueError(f"{name} logits must be a 3-d GPU tensor")
    if t.shape[2] > 1 and t.stride(2) != 1:
        raise ValueError(f"{name} logits: the vocabulary axis must be contiguous")
    if t.dtype == torch.float32:
        dt = F32
    elif t.dtype == torch.bfloat16:
        dt = BF16
    else:
        raise ValueError(f"{name} logits: dtype {t.dtype} is not supported (float32 / bfloat16)")
    return TapoutLogits(t.data_ptr(), dt, t.stride(0), t.stride(1))


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


STATIC_MAX_PARTIALS = 131072


def draft_stats_static(draft, draft_tok=None, k_len=None, arm=None, rules=(RULE_SVIP, RULE_MAXCONF, RULE_MARGIN),
                       thresholds=(0.6, 0.8, 0.2), out=None, stream=None):
    """tapout_draft_stats_static: the draft signals and stop positions without a context and without any allocation
    inside the library (its scratch is a fixed array in the library's device image).  `out`: dict of output tensors as
    Tapout.alloc_draft_outputs makes them (allocated here, by torch, when None).  Returns the dict."""
    lib = load_library()
    B, K, V = draft.shape
    dev = draft.device
    f32, i32 = torch.float32, torch.int32
    if out is None:
        f = lambda: torch.full((B, K), float("nan"), dtype=f32, device=dev)
        out = dict(lse=f(), entropy=f(), p_top1=f(), p_top2=f(), margin=f(), logq_tok=f(),
                   top1_id=torch.full((B, K), -1, dtype=i32, device=dev), n_stop=torch.zeros(B, dtype=i32, device=dev),
                   stop_fired=torch.zeros((B, K), dtype=torch.uint8, device=dev), flags=torch.zeros(B, dtype=i32, device=dev))
    lg = _logits(draft, "draft")
    n = len(rules)
    rule_h, th_h = (C.c_int32 * max(n, 1))(*rules), (C.c_float * max(n, 1))(*thresholds)
    with torch.cuda.device(dev):
        st = lib.tapout_draft_stats_static(
            C.byref(lg), B, K, V, _ptr(draft_tok, i32, (B, K), "draft_tok"), _ptr(k_len, i32, (B,), "k_len"),
            _ptr(arm, i32, (B,), "arm"), n, C.cast(rule_h, C.c_void_p), C.cast(th_h, C.c_void_p),
            _ptr(out.get("lse"), f32, (B, K), "lse"), _ptr(out.get("entropy"), f32, (B, K), "entropy"),
            _ptr(out.get("p_top1"), f32, (B, K), "p_top1"), _ptr(out.get("p_top2"), f32, (B, K), "p_top2"),
            _ptr(out.get("margin"), f32, (B, K), "margin"), _ptr(out.get("top1_id"), i32, (B, K), "top1_id"),
            _ptr(out.get("logq_tok"), f32, (B, K), "logq_tok") if draft_tok is not None else None,
            _ptr(out.get("n_stop"), i32, (B,), "n_stop") if arm is not None else None,
            _ptr(out.get("stop_fired"), torch.uint8, (B, K), "stop_fired") if arm is not None else None,
            _ptr(out.get("flags"), i32, (B,), "flags"), _stream(stream))
    if st != 0:
        raise TapoutError(st, lib.tapout_last_error(None).decode())
    return out


class Tapout:
    """One libtapout context (scratch memory + bandit state) on one GPU."""

    def __init__(self, max_batch: int, max_k: int, vocab: int, *, device: int = 0, policy: int = UCB1,
                 rules=(RULE_SVIP, RULE_MAXCONF, RULE_MARGIN), thresholds=(0.6, 0.8, 0.2),
                 alpha: float = 0.5, shared_bandit: bool = False, reward: int = REWARD_BLEND, adaedl: dict | None = None,
                 token_level: bool = False, draft_sampling: bool = False):
        """adaedl: optional dict with any of gamma, alpha, beta1, beta2, eps, rate0, steer (tapout_config.adaedl_*)."""
        self._lib = load_library()
        cfg = default_config(max_batch, max_k, vocab)
        cfg.device = device
        cfg.policy = policy
        cfg.n_arms = len(rules)
        for i, (r, h) in enumerate(list(zip(rules, thresholds))[:MAX_ARMS]):       # more arms: tapout_create rejects n_arms
            cfg.rule[i], cfg.threshold[i] = r, h
        cfg.alpha = alpha
        cfg.reward = reward
        cfg.granularity = TOKEN_LEVEL if token_level else SEQUENCE_LEVEL
        cfg.draft_sampling = 1 if draft_sampling else 0
        for k, v in (adaedl or {}).items():
            setattr(cfg, "adaedl_" + k, int(v) if k == "steer" else float(v))
        cfg.n_bandits = 1 if shared_bandit else max_batch
        self.cfg = cfg
        self.positions = max_k if token_level else 1           # bandits per slot; arm arrays are [B, max_k] when > 1
        self.device = torch.device("cuda", device)
        self._ctx = C.c_void_p()
        st = self._lib.tapout_create(C.byref(self._ctx), C.byref(cfg))
        if st != 0:
            raise TapoutError(st, self._lib.tapout_last_error(None).decode())

    def close(self):
        ctx = getattr(self, "_ctx", None)
        if ctx is not None and ctx.value:
            self._lib.tapout_destroy(ctx)
            self._ctx = None

    __del__ = close

    def _check(self, st):
        if st != 0:
            raise TapoutError(st, self._lib.tapout_last_error(self._ctx).decode())

    def set_option(self, name: str, value: int):
        self._check(self._lib.tapout_set_option(self._ctx, name.encode(), int(value)))

    # -- kernel timing ---------------------------------------------------------
    def profile_enable(self, kinds=(), max_records: int = 0):
        mask = 0
        for k in kinds:
            mask |= 1 << PROFILE_KINDS.index(k)
        self._check(self._lib.tapout_profile_enable(self._ctx, mask, int(max_records)))

    def profile_read(self, kind: str, stream=None):
        """(total milliseconds, launches) recorded for one kernel since the last read."""
        ms, n = C.c_double(0), C.c_int32(0)
        self._check(self._lib.tapout_profile_read(self._ctx, PROFILE_KINDS.index(kind), C.byref(ms), C.byref(n), _stream(stream)))
        return ms.value, n.value

    # -- one decode round with the arguments marshalled once ---------------------
    def prepare_round(self, rnd: dict, truncate: bool, u_ts=None, u_draft=None):
        """Pre-marshals the four calls of one round (Algorithm 1) on fixed tensors and returns
        (launch, outputs): launch(stream_handle) enqueues select -> draft_stats -> verify -> update.
        truncate=True verifies the tokens up to the stop position, False all k_len drafted tokens.
        u_draft [B, K]: the library draws the draft tokens itself instead of reading rnd["draft_tok"]."""
        draft, target, tok = rnd["draft"], rnd["target"], rnd["draft_tok"]
        B, K, V = draft.shape
        f32, i32 = torch.float32, torch.int32
        do, vo = self.alloc_draft_outputs(B, K), self.alloc_verify_outputs(B, K)
        arm = torch.zeros(B if self.positions == 1 else (B, self.positions), dtype=i32, device=self.device)
        n_draft = do["n_stop"] if truncate else rnd["k_len"]
        if u_draft is not None:
            do["sampled_tok"] = torch.full((B, K), -1, dtype=i32, device=self.device)
            tok = do["sampled_tok"]
        dl, tl = _logits(draft, "draft"), _logits(target, "target")
        keep = (dl, tl, do, vo, arm, rnd, u_ts, u_draft)
        lib, ctx = self._lib, self._ctx
        p = lambda t: C.c_void_p(t.data_ptr()) if t is not None else None
        a_sel = (ctx, B, p(u_ts), p(arm), None)
        a_ds = (ctx, C.byref(dl), B, K, V, None if u_draft is not None else p(tok), p(rnd["k_len"]), p(arm), p(u_draft),
                p(do["lse"]), p(do["entropy"]),
                p(do["p_top1"]), p(do["p_top2"]), p(do["margin"]), p(do["top1_id"]), p(do["logq_tok"]), p(do.get("sampled_tok")),
                p(do["n_stop"]), p(do["stop_fired"]), p(do["flags"]))
        a_vf = (ctx, C.byref(tl), C.byref(dl), B, K, V, p(do["lse"]), p(do["logq_tok"]), p(tok), p(n_draft),
                p(rnd.get("greedy")), p(rnd["u_accept"]), p(rnd["u_sample"]), p(vo["accept_len"]), p(vo["out_tok"]),
                p(vo["n_out"]), p(vo["target_lse"]), p(vo["logp_tok"]), p(vo["target_top1"]), p(vo["flags"]))
        a_up = (ctx, B, p(arm), p(vo["accept_len"]), p(n_draft), p(rnd["k_len"]), None)

        def launch(stream_handle):
            st = lib.tapout_bandit_select(*a_sel, stream_handle)
            st = st or lib.tapout_draft_stats(*a_ds, stream_handle)
            st = st or lib.tapout_verify(*a_vf, stream_handle)
            st = st or lib.tapout_bandit_update(*a_up, stream_handle)
            if st:
                self._check(st)

        launch._keep = keep
        return launch, dict(arm=arm, n_draft=n_draft, draft=do, verify=vo)

    # -- tapout_round: a whole round in one call ---------------------------------
    def round_args(self, rnd: dict, arm, truncate: bool, u_ts_next=None, draft_out=None, verify_out=None, active=None):
        """Marshals one round on fixed tensors for tapout_round.  Returns (args, outputs); keep `args` alive while it is in use
        (it holds the tensors).  truncate=True: n_draft = this round's stop position; False: n_draft = k_len (the target
        pass then runs beside the draft pass)."""
        draft, target = rnd["draft"], rnd["target"]
        B, K, V = draft.shape
        do = draft_out or self.alloc_draft_outputs(B, K)
        vo = verify_out or self.alloc_verify_outputs(B, K)
        sel_flags = torch.zeros(B, dtype=torch.int32, device=self.device)
        dl, tl = _logits(draft, "draft"), _logits(target, "target")
        p = lambda t: None if t is None else t.data_ptr()
        a = TapoutRoundArgs()
        a.draft, a.target = C.pointer(dl), C.pointer(tl)
        a.B, a.K, a.V = B, K, V
        a.draft_tok, a.k_len, a.n_draft = p(rnd["draft_tok"]), p(rnd["k_len"]), None if truncate else p(rnd["k_len"])
        a.greedy, a.u_accept, a.u_sample, a.u_ts_next = p(rnd.get("greedy")), p(rnd["u_accept"]), p(rnd["u_sample"]), p(u_ts_next)
        a.arm, a.gamma, a.active = p(arm), p(rnd["k_len"]), p(active)
        for k in ("lse", "entropy", "p_top1", "p_top2", "margin", "top1_id", "logq_tok", "n_stop", "stop_fired"):
            setattr(a, k, p(do[k]))
        a.draft_flags = p(do["flags"])
        for k in ("accept_len", "out_tok", "n_out", "target_lse", "logp_tok", "target_top1"):
            setattr(a, k, p(vo[k]))
        a.verify_flags, a.select_flags = p(vo["flags"]), p(sel_flags)
        a._keep = (dl, tl, rnd, arm, u_ts_next, do, vo, sel_flags, active)
        n_draft = do["n_stop"] if truncate else rnd["k_len"]
        return a, dict(arm=arm, n_draft=n_draft, draft=do, verify=vo, select_flags=sel_flags)

    def round(self, args: TapoutRoundArgs, stream=None):
        self._check(self._lib.tapout_round(self._ctx, C.byref(args), _stream(stream)))

    def prepare_round_call(self, rnd: dict, arm, truncate: bool, u_ts_next=None):
        """As prepare_round, for the single call: launch(stream_handle) enqueues one tapout_round; `arm` [B] holds this
        round's arms on entry and the next round's afterwards (tapout_bandit_select fills it before the first round)."""
        a, outs = self.round_args(rnd, arm, truncate, u_ts_next=u_ts_next)
        lib, ctx, ref = self._lib, self._ctx, C.byref(a)

        def launch(stream_handle):
            st = lib.tapout_round(ctx, ref, stream_handle)
            if st:
                self._check(st)

        launch._keep = a
        return launch, outs

    # -- tapout_bandit_select ------------------------------------------------
    def bandit_select(self, B: int, u_ts=None, arm_out=None, flags=None, stream=None):
        A, P = self.cfg.n_arms, self.positions
        ashape = (B,) if P == 1 else (B, P)
        ushape = (B, A, TS_UNIFORMS_PER_ARM) if P == 1 else (B, P, A, TS_UNIFORMS_PER_ARM)
        if arm_out is None:
            arm_out = torch.empty(ashape, dtype=torch.int32, device=self.device)
        self._check(self._lib.tapout_bandit_select(
            self._ctx, B, _ptr(u_ts, torch.float32, ushape, "u_ts"),
            _ptr(arm_out, torch.int32, ashape, "arm_out"), _ptr(flags, torch.int32, (B,), "flags"), _stream(stream)))
        return arm_out

    # -- tapout_draft_stats --------------------------------------------------
    def draft_stats(self, draft, draft_tok=None, k_len=None, arm=None, u_draft=None, out=None, stream=None):
        """Returns / fills a dict: lse, entropy, p_top1, p_top2, margin, top1_id, logq_tok, n_stop, stop_fired, flags.
        With u_draft [B, K] the draft tokens are drawn by the library (out["sampled_tok"]) and logq_tok refers to them."""
        B, K, V = draft.shape
        if out is None:
            out = self.alloc_draft_outputs(B, K)
        if u_draft is not None and "sampled_tok" not in out:
            out["sampled_tok"] = torch.full((B, K), -1, dtype=torch.int32, device=self.device)
        f32, i32 = torch.float32, torch.int32
        lg = _logits(draft, "draft")
        self._check(self._lib.tapout_draft_stats(
            self._ctx, C.byref(lg), B, K, V,
            _ptr(draft_tok, i32, (B, K), "draft_tok"), _ptr(k_len, i32, (B,), "k_len"),
            _ptr(arm, i32, (B,) if self.positions == 1 else (B, self.positions), "arm"),
            _ptr(u_draft, f32, (B, K), "u_draft"),
            _ptr(out.get("lse"), f32, (B, K), "lse"), _ptr(out.get("entropy"), f32, (B, K), "entropy"),
            _ptr(out.get("p_top1"), f32, (B, K), "p_top1"), _ptr(out.get("p_top2"), f32, (B, K), "p_top2"),
            _ptr(out.get("margin"), f32, (B, K), "margin"), _ptr(out.get("top1_id"), i32, (B, K), "top1_id"),
            _ptr(out.get("logq_tok"), f32, (B, K), "logq_tok") if (draft_tok is not None or u_draft is not None) else None,
            _ptr(out.get("sampled_tok"), i32, (B, K), "sampled_tok") if u_draft is not None else None,
            _ptr(out.get("n_stop"), i32, (B,), "n_stop") if arm is not None else None,
            _ptr(out.get("stop_fired"), torch.uint8, (B, K), "stop_fired") if arm is not None else None,
            _ptr(out.get("flags"), i32, (B,), "flags"), _stream(stream)))
        return out

    # -- vocabulary shards -----------------------------------------------------
    def shard_stats(self, shard, vocab_offset: int, length=None, rows_mode: int = 0, tok=None, out=None, stream=None):
        """One 32-byte record per row of a vocabulary shard [B, KK, Vs]; returns an int32 tensor [B*KK, 8] (raw records)."""
        B, KK, Vs = shard.shape
        if out is None:
            out = torch.zeros((B * KK, 8), dtype=torch.int32, device=self.device)
        lg = _logits(shard, "shard")
        self._check(self._lib.tapout_shard_stats(
            self._ctx, C.byref(lg), B, KK, Vs, int(vocab_offset), _ptr(length, torch.int32, (B,), "len"), int(rows_mode),
            _ptr(tok, torch.int32, (B, KK - rows_mode), "tok"), _ptr(out, torch.int32, (B * KK, 8), "out"), _stream(stream)))
        return out

    def draft_stats_sharded(self, stats, B: int, K: int, V: int, draft_tok=None, k_len=None, arm=None, out=None, stream=None):
        """stats: int32 tensor [G, B*K, 8] of shard records.  Returns the dict tapout_draft_stats returns."""
        G = stats.shape[0]
        if out is None:
            out = self.alloc_draft_outputs(B, K)
        f32, i32 = torch.float32, torch.int32
        self._check(self._lib.tapout_draft_stats_sharded(
            self._ctx, _ptr(stats, i32, (G, B * K, 8), "stats"), G, B, K, V,
            _ptr(draft_tok, i32, (B, K), "draft_tok"), _ptr(k_len, i32, (B,), "k_len"),
            _ptr(arm, i32, (B,) if self.positions == 1 else (B, self.positions), "arm"),
            _ptr(out.get("lse"), f32, (B, K), "lse"), _ptr(out.get("entropy"), f32, (B, K), "entropy"),
            _ptr(out.get("p_top1"), f32, (B, K), "p_top1"), _ptr(out.get("p_top2"), f32, (B, K), "p_top2"),
            _ptr(out.get("margin"), f32, (B, K), "margin"), _ptr(out.get("top1_id"), i32, (B, K), "top1_id"),
            _ptr(out.get("logq_tok"), f32, (B, K), "logq_tok") if draft_tok is not None else None,
            _ptr(out.get("n_stop"), i32, (B,), "n_stop") if arm is not None else None,
            _ptr(out.get("stop_fired"), torch.uint8, (B, K), "stop_fired") if arm is not None else None,
            _ptr(out.get("flags"), i32, (B,), "flags"), _stream(stream)))
        return out

    def verify_accept_sharded(self, stats, B: int, K: int, V: int, logq_tok, draft_tok, n_draft, u_accept, greedy=None,
                              draft_lse=None, out=None, stream=None):
        """stats: int32 tensor [G, B*(K+1), 8] of target-row shard records.  Fills the dict tapout_verify fills; the final
        token of a sampled sequence is left at -1 and described by out["final_jobs"] (uint8 [B, 24]) when draft_lse is given."""
        G = stats.shape[0]
        if out is None:
            out = self.alloc_verify_outputs(B, K)
        if draft_lse is not None and "final_jobs" not in out:
            out["final_jobs"] = torch.zeros((B, 24), dtype=torch.uint8, device=self.device)
        f32, i32 = torch.float32, torch.int32
        self._check(self._lib.tapout_verify_accept_sharded(
            self._ctx, _ptr(stats, i32, (G, B * (K + 1), 8), "stats"), G, B, K, V,
            _ptr(logq_tok, f32, (B, K), "logq_tok"), _ptr(draft_tok, i32, (B, K), "draft_tok"), _ptr(n_draft, i32, (B,), "n_draft"),
            _ptr(greedy, torch.uint8, (B,), "greedy"), _ptr(u_accept, f32, (B, K), "u_accept"), _ptr(draft_lse, f32, (B, K), "draft_lse"),
            _ptr(out["accept_len"], i32, (B,), "accept_len"), _ptr(out["out_tok"], i32, (B, K + 1), "out_tok"),
            _ptr(out["n_out"], i32, (B,), "n_out"),
            _ptr(out.get("target_lse"), f32, (B, K + 1), "target_lse"), _ptr(out.get("logp_tok"), f32, (B, K), "logp_tok"),
            _ptr(out.get("target_top1"), i32, (B, K + 1), "target_top1"),
            _ptr(out.get("final_jobs"), torch.uint8, (B, 24), "final_jobs") if draft_lse is not None else None,
            _ptr(out.get("flags"), i32, (B,), "flags"), _stream(stream)))
        return out

    def shard_final_sums(self, target_shard, draft_shard, jobs, stream=None):
        """This shard's five double-precision sums per sequence for the final-token draw: float64 tensor [B, 5]."""
        B, K1, Vs = target_shard.shape
        sums = torch.zeros((B, 5), dtype=torch.float64, device=self.device)
        tl, dl = _logits(target_shard, "target shard"), _logits(draft_shard, "draft shard")
        self._check(self._lib.tapout_shard_final_sums(self._ctx, C.byref(tl), C.byref(dl), B, K1 - 1, Vs,
                                                      _ptr(jobs, torch.uint8, (B, 24), "jobs"), _ptr(sums, torch.float64, (B, 5), "sums"),
                                                      _stream(stream)))
        return sums

    def shard_final_token(self, target_shard, draft_shard, vocab_offset: int, G: int, g: int, jobs, sums_all, u_sample,
                          exact_all=None, stream=None):
        """(tok [B] int32: global id where this shard holds the draw, else -1; exact_mass [B] float64; need_exact [B] uint8)."""
        B, K1, Vs = target_shard.shape
        d = self.device
        tok = torch.full((B,), -1, dtype=torch.int32, device=d)
        mass = torch.zeros(B, dtype=torch.float64, device=d)
        need = torch.zeros(B, dtype=torch.uint8, device=d)
        tl, dl = _logits(target_shard, "target shard"), _logits(draft_shard, "draft shard")
        self._check(self._lib.tapout_shard_final_token(
            self._ctx, C.byref(tl), C.byref(dl), B, K1 - 1, Vs, int(vocab_offset), int(G), int(g),
            _ptr(jobs, torch.uint8, (B, 24), "jobs"), _ptr(sums_all, torch.float64, (G, B, 5), "sums_all"),
            _ptr(exact_all, torch.float64, (G, B), "exact_all"), _ptr(u_sample, torch.float32, (B,), "u_sample"),
            _ptr(tok, torch.int32, (B,), "tok_out"), _ptr(mass, torch.float64, (B,), "exact_mass"),
            _ptr(need, torch.uint8, (B,), "need_exact"), _stream(stream)))
        return tok, mass, need

    def alloc_draft_outputs(self, B, K):
        d = self.device
        f = lambda: torch.full((B, K), float("nan"), dtype=torch.float32, device=d)
        return dict(lse=f(), entropy=f(), p_top1=f(), p_top2=f(), margin=f(), logq_tok=f(),
                    top1_id=torch.full((B, K), -1, dtype=torch.int32, device=d),
                    n_stop=torch.zeros(B, dtype=torch.int32, device=d),
                    stop_fired=torch.zeros((B, K), dtype=torch.uint8, device=d),
                    flags=torch.zeros(B, dtype=torch.int32, device=d))

    # -- tapout_verify -------------------------------------------------------
    def verify(self, target, draft, draft_lse, logq_tok, draft_tok, n_draft, u_accept, u_sample,
               greedy=None, out=None, stream=None):
        """Returns / fills a dict: accept_len, out_tok, n_out, target_lse, logp_tok, target_top1, flags."""
        B, K1, V = target.shape
        K = K1 - 1
        if tuple(draft.shape) != (B, K, V):
            raise ValueError(f"draft logits must be {(B, K, V)}, got {tuple(draft.shape)}")
        if out is None:
            out = self.alloc_verify_outputs(B, K)
        f32, i32 = torch.float32, torch.int32
        tl, dl = _logits(target, "target"), _logits(draft, "draft")
        self._check(self._lib.tapout_verify(
            self._ctx, C.byref(tl), C.byref(dl), B, K, V,
            _ptr(draft_lse, f32, (B, K), "draft_lse"), _ptr(logq_tok, f32, (B, K), "logq_tok"),
            _ptr(draft_tok, i32, (B, K), "draft_tok"), _ptr(n_draft, i32, (B,), "n_draft"),
            _ptr(greedy, torch.uint8, (B,), "greedy"),
            _ptr(u_accept, f32, (B, K), "u_accept"), _ptr(u_sample, f32, (B,), "u_sample"),
            _ptr(out["accept_len"], i32, (B,), "accept_len"), _ptr(out["out_tok"], i32, (B, K + 1), "out_tok"),
            _ptr(out["n_out"], i32, (B,), "n_out"),
            _ptr(out.get("target_lse"), f32, (B, K + 1), "target_lse"), _ptr(out.get("logp_tok"), f32, (B, K), "logp_tok"),
            _ptr(out.get("target_top1"), i32, (B, K + 1), "target_top1"),
            _ptr(out.get("flags"), i32, (B,), "flags"), _stream(stream)))
        return out

    def alloc_verify_outputs(self, B, K):
        d = self.device
        return dict(accept_len=torch.zeros(B, dtype=torch.int32, device=d),
                    out_tok=torch.full((B, K + 1), -1, dtype=torch.int32, device=d),
                    n_out=torch.zeros(B, dtype=torch.int32, device=d),
                    target_lse=torch.full((B, K + 1), float("nan"), dtype=torch.float32, device=d),
                    logp_tok=torch.full((B, K), float("nan"), dtype=torch.float32, device=d),
                    target_top1=torch.full((B, K + 1), -1, dtype=torch.int32, device=d),
                    flags=torch.zeros(B, dtype=torch.int32, device=d))

    # -- tapout_bandit_update ------------------------------------------------
    def bandit_update(self, arm, accept_len, n_draft, gamma, active=None, stream=None):
        B = arm.shape[0]
        i32 = torch.int32
        self._check(self._lib.tapout_bandit_update(
            self._ctx, B, _ptr(arm, i32, (B,) if self.positions == 1 else (B, self.positions), "arm"),
            _ptr(accept_len, i32, (B,), "accept_len"),
            _ptr(n_draft, i32, (B,), "n_draft"), _ptr(gamma, i32, (B,), "gamma"),
            _ptr(active, torch.uint8, (B,), "active"), _stream(stream)))

    # -- tapout_bandit_update_select -----------------------------------------
    def bandit_update_select(self, arm, accept_len, n_draft, gamma, active=None, u_ts=None, arm_out=None, flags=None, stream=None):
        """Applies the rewards of the round that was played with `arm` and returns the arms of the next round
        (arm_out may be `arm` itself)."""
        B = arm.shape[0]
        i32 = torch.int32
        A, P = self.cfg.n_arms, self.positions
        ashape = (B,) if P == 1 else (B, P)
        ushape = (B, A, TS_UNIFORMS_PER_ARM) if P == 1 else (B, P, A, TS_UNIFORMS_PER_ARM)
        if arm_out is None:
            arm_out = torch.empty(ashape, dtype=i32, device=self.device)
        self._check(self._lib.tapout_bandit_update_select(
            self._ctx, B, _ptr(arm, i32, ashape, "arm"), _ptr(accept_len, i32, (B,), "accept_len"),
            _ptr(n_draft, i32, (B,), "n_draft"), _ptr(gamma, i32, (B,), "gamma"), _ptr(active, torch.uint8, (B,), "active"),
            _ptr(u_ts, torch.float32, ushape, "u_ts"), _ptr(arm_out, i32, ashape, "arm_out"), _ptr(flags, i32, (B,), "flags"),
            _stream(stream)))
        return arm_out

    # -- state read-out / restore (host arrays) ------------------------------
    def _state_shape(self):
        c = self.cfg
        return (c.n_bandits, c.n_arms) if self.positions == 1 else (c.n_bandits, self.positions, c.n_arms)

    def bandit_get_state(self, stream=None, moments: bool = False):
        """(sum_r, count) or, with moments=True, (sum_r, sum_r2, count) as numpy arrays [n_bandits, n_arms]
        ([n_bandits, max_k, n_arms] for token-level bandits)."""
        import numpy as np
        n = self._state_shape()
        s, q, c = np.zeros(n, np.float64), np.zeros(n, np.float64), np.zeros(n, np.int64)
        self._check(self._lib.tapout_bandit_get_state(self._ctx, s.ctypes.data, q.ctypes.data, c.ctypes.data, _stream(stream)))
        return (s, q, c) if moments else (s, c)

    def bandit_set_state(self, sum_r, count, sum_r2=None, stream=None):
        import numpy as np
        n = self._state_shape()
        s = np.ascontiguousarray(sum_r, np.float64).reshape(n)
        c = np.ascontiguousarray(count, np.int64).reshape(n)
        q = None if sum_r2 is None else np.ascontiguousarray(sum_r2, np.float64).reshape(n)
        self._check(self._lib.tapout_bandit_set_state(self._ctx, s.ctypes.data, None if q is None else q.ctypes.data,
                                                      c.ctypes.data, _stream(stream)))

    def rule_state_get(self, stream=None):
        """dict(prev_entropy [max_batch] f32, accept_rate [max_batch] f64, lam [max_batch, n_arms] f64), numpy."""
        import numpy as np
        nb, A = self.cfg.max_batch, self.cfg.n_arms
        pe, ar, lam = np.zeros(nb, np.float32), np.zeros(nb, np.float64), np.zeros((nb, A), np.float64)
        self._check(self._lib.tapout_rule_state_get(self._ctx, pe.ctypes.data, ar.ctypes.data, lam.ctypes.data, _stream(stream)))
        return dict(prev_entropy=pe, accept_rate=ar, lam=lam)

    def rule_state_set(self, prev_entropy=None, accept_rate=None, lam=None, stream=None):
        import numpy as np
        nb, A = self.cfg.max_batch, self.cfg.n_arms
        pe = None if prev_entropy is None else np.ascontiguousarray(prev_entropy, np.float32).reshape(nb)
        ar = None if accept_rate is None else np.ascontiguousarray(accept_rate, np.float64).reshape(nb)
        lm = None if lam is None else np.ascontiguousarray(lam, np.float64).reshape(nb, A)
        d = lambda x: None if x is None else x.ctypes.data
        self._check(self._lib.tapout_rule_state_set(self._ctx, d(pe), d(ar), d(lm), _stream(stream)))
