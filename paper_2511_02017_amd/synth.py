"""Seeded synthetic inputs for the TapOut logits path.

Input generation only: this module holds none of the method's arithmetic and is
the one piece of code that both the GPU tests/benchmark and the CPU oracle's
tests feed from.  The five workloads stand in for the logits of the model pairs
the paper evaluates (Llama-3, Gemma-3, OLMo-2 vocabularies); only vocabulary
sizes and batch / draft-length shapes are taken from those families.

Recipe of a round (every config):
  base      fp32 draft logits of shape [B, K, V] from the config's law
  draft     base rounded to the draft dtype
  target    rows 0..K-1: base + N(0, sigma^2) noise; row K (the position after
            all K drafted tokens): a fresh draw of the base law + noise; rounded
            to the target dtype
  draft_tok sampled rows: Gumbel-max draw from softmax(draft) at temperature 1;
            greedy rows: argmax(draft)
  u_accept  [B, K], u_sample [B], u_ts [B, A, 48]: U[0,1) fp32
  k_len     per-sequence draft cap (ragged config: U{4..16}, else K)
  greedy    per-sequence flag (ragged config: 25 % of the rows, fixed over rounds)
All draws come from torch generators seeded by (config seed, round index), on the
device the tensors live on; the oracle is fed host copies of the same tensors.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import torch

TS_UNIFORMS_PER_ARM = 48
BASE_SEED = 20251102


@dataclass(frozen=True)
class Workload:
    name: str
    index: int
    V: int
    B: int
    K: int
    draft_dtype: torch.dtype
    target_dtype: torch.dtype
    law: str                 # "normal" | "regime" | "zipf"
    sigma_draft: float       # std of the base law (normal / regime), of the additive noise (zipf)
    sigma_target: tuple      # (lo, hi): per-sequence U(lo, hi); equal values = fixed
    rounds: int
    policy: str              # "ucb1" | "ts"
    ragged: bool = False     # per-sequence K_b ~ U{4..K}
    greedy_frac: float = 0.0
    shift_round: int = -1    # zipf: sigma_target switches to sigma_shift from this round on
    sigma_shift: float = 0.0
    n_arms: int = 3

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index


bf16, f32 = torch.bfloat16, torch.float32
WORKLOADS = {
    "tiny": Workload("tiny", 0, 32000, 1, 5, f32, f32, "normal", 2.0, (1.0, 1.0), 64, "ucb1"),
    "small": Workload("small", 1, 32000, 32, 8, bf16, bf16, "normal", 2.5, (0.5, 2.0), 1000, "ucb1"),
    "llama3": Workload("llama3", 2, 128256, 64, 8, bf16, bf16, "regime", 3.0, (1.2, 1.2), 2000, "ucb1"),
    "zipf": Workload("zipf", 3, 151936, 256, 16, bf16, bf16, "zipf", 0.3, (0.6, 0.6), 3000, "ts",
                     shift_round=1500, sigma_shift=2.0),
    "ragged": Workload("ragged", 4, 256000, 512, 16, bf16, f32, "normal", 2.0, (1.0, 1.0), 1000, "ucb1",
                       ragged=True, greedy_frac=0.25),
}


def scaled(w: Workload, **kw) -> Workload:
    """Same recipe at another shape (tests use small V / B)."""
    return replace(w, **kw)


class RoundGenerator:
    """Generates the rounds of one workload on one device, reproducibly."""

    def __init__(self, w: Workload, device="cpu", chunk_rows: int = 64):
        self.w = w
        self.device = torch.device(device)
        self.chunk_rows = max(1, chunk_rows)
        g = self._gen(-1)
        B, V = w.B, w.V
        lo, hi = w.sigma_target
        self.sigma_b = lo + (hi - lo) * torch.rand(B, generator=g, device=self.device)
        if w.ragged:
            self.k_len = torch.randint(4, w.K + 1, (B,), generator=g, device=self.device, dtype=torch.int32)
        else:
            self.k_len = torch.full((B,), w.K, dtype=torch.int32, device=self.device)
        self.greedy = (torch.rand(B, generator=g, device=self.device) < w.greedy_frac).to(torch.uint8)
        self.zipf_base = None
        if w.law == "zipf":
            # -1.1 ln(rank) under one seeded permutation per sequence, fixed over rounds
            base = torch.empty(B, V, dtype=torch.float32, device=self.device)
            ranks = -1.1 * torch.log(torch.arange(1, V + 1, device=self.device, dtype=torch.float32))
            for b in range(B):
                perm = torch.randperm(V, generator=g, device=self.device)
                base[b, perm] = ranks
            self.zipf_base = base

    def _gen(self, round_idx: int) -> torch.Generator:
        g = torch.Generator(device=self.device)
        g.manual_seed((self.w.seed * 1000003 + round_idx + 1) & 0x7FFFFFFFFFFFFFFF)
        return g

    def _base(self, b0, b1, rows, g):
        w = self.w
        shape = (b1 - b0, rows, w.V)
        z = torch.randn(shape, generator=g, device=self.device, dtype=torch.float32)
        if w.law == "normal":
            return z * w.sigma_draft
        if w.law == "regime":
            peaked = torch.rand(shape[:2], generator=g, device=self.device) < 0.5
            scale = torch.where(peaked, torch.tensor(2.0, device=self.device), torch.tensor(1.0 / 1.5, device=self.device))
            return z * (w.sigma_draft * scale)[..., None]
        return self.zipf_base[b0:b1, None, :] + z * w.sigma_draft

    def round(self, round_idx: int) -> dict:
        w = self.w
        B, K, V = w.B, w.K, w.V
        dev = self.device
        g = self._gen(round_idx)
        draft = torch.empty(B, K, V, dtype=w.draft_dtype, device=dev)
        target = torch.empty(B, K + 1, V, dtype=w.target_dtype, device=dev)
        tok = torch.empty(B, K, dtype=torch.int32, device=dev)
        sig = self.sigma_b
        if w.shift_round >= 0 and round_idx >= w.shift_round:
            sig = torch.full_like(sig, w.sigma_shift)
        step = max(1, self.chunk_rows // (K + 1))
        for b0 in range(0, B, step):
            b1 = min(B, b0 + step)
            base = self._base(b0, b1, K + 1, g)                        # row K: the position after the draft
            noise = torch.randn(base.shape, generator=g, device=dev, dtype=torch.float32)
            target[b0:b1] = (base + noise * sig[b0:b1, None, None]).to(w.target_dtype)
            d = base[:, :K].to(w.draft_dtype)
            draft[b0:b1] = d
            u = torch.rand(d.shape, generator=g, device=dev, dtype=torch.float32).clamp_(1e-20, 1.0 - 1e-7)
            gumbel = -torch.log(-torch.log(u))
            sampled = (d.float() + gumbel).argmax(-1)
            greedy_tok = d.float().argmax(-1)
            is_g = self.greedy[b0:b1].bool()[:, None]
            tok[b0:b1] = torch.where(is_g, greedy_tok, sampled).to(torch.int32)
            del base, noise, d, u, gumbel
        out = dict(draft=draft, target=target, draft_tok=tok,
                   u_accept=torch.rand(B, K, generator=g, device=dev, dtype=torch.float32),
                   u_sample=torch.rand(B, generator=g, device=dev, dtype=torch.float32),
                   u_ts=torch.rand(B, w.n_arms, TS_UNIFORMS_PER_ARM, generator=g, device=dev, dtype=torch.float32),
                   k_len=self.k_len, greedy=self.greedy)
        return out


def logits_bytes(w: Workload, n_draft_rows: int, n_target_rows: int) -> int:
    """Bytes of logits one round streams: draft rows + target rows, each element once."""
    esz = {torch.float32: 4, torch.bfloat16: 2}
    return w.V * (n_draft_rows * esz[w.draft_dtype] + n_target_rows * esz[w.target_dtype])
