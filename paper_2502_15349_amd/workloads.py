"""Seeded synthetic workloads shared by the tests, the benchmark and smoke().

This module holds NO arithmetic of the attention method: it only names the
workload shapes and draws the inputs.  Both the CPU oracle's callers and the
HIP path's callers read the same bf16 tensors produced here.

Recipe: Q, K, V are i.i.d. N(0, 1) drawn in fp32 with
torch.Generator('cpu').manual_seed(1000 * config_id + {0: Q, 1: K, 2: V}) and
rounded to bf16 (round to nearest even).  They stand in for the random tensors
of the paper's operator microbenchmark (Table 2 and the batch/sequence grid of
Section 6.1), whose shapes the configurations below take.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Optional, Tuple

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    config_id: int
    B: int
    H_q: int
    H_kv: int
    L_q: int
    L_k: int
    D_qk: int
    D_v: int
    score_mod: str = "none"      # none | bias | head_decay | relu
    norm: str = "softmax"        # softmax | sigmoid | abssum | abs_of_sum | none
    mask: str = "none"           # none | causal | sliding_window
    scale: Optional[float] = None  # default 1/sqrt(D_qk)
    bias: float = 0.0
    decay: bool = False          # per-head gamma_h = 1 - 2^(-5-h)
    window: int = 0              # keys per query of the sliding-window mask

    @property
    def scale_value(self) -> float:
        return self.scale if self.scale is not None else 1.0 / math.sqrt(self.D_qk)

    def gamma(self) -> Optional[Tuple[float, ...]]:
        """Per-query-head decay rates of the retention configuration
        (gamma_h = 1 - 2^(-5-h), h = 0..H_q-1); an input, not derived data."""
        if not self.decay:
            return None
        return tuple(1.0 - 2.0 ** (-5 - h) for h in range(self.H_q))

    def visible_pairs_per_head(self) -> int:
        if self.mask == "none":
            return self.L_q * self.L_k
        off = self.L_k - self.L_q
        if self.mask == "sliding_window":
            return sum(max(0, min(self.L_k, i + off + 1) - max(0, i + off + 1 - self.window)) for i in range(self.L_q))
        return sum(max(0, min(self.L_k, i + off + 1)) for i in range(self.L_q))

    def oracle_mask(self):
        """The mask in the form the oracle's functions take."""
        return ("sliding_window", self.window) if self.mask == "sliding_window" else self.mask

    def mfma_flop(self) -> int:
        """2*(D_qk + D_v) flop per visible (query, key) pair."""
        return 2 * (self.D_qk + self.D_v) * self.visible_pairs_per_head() * self.B * self.H_q

    def compulsory_bytes(self) -> int:
        q = self.B * self.H_q * self.L_q * self.D_qk * 2
        k = self.B * self.H_kv * self.L_k * self.D_qk * 2
        v = self.B * self.H_kv * self.L_k * self.D_v * 2
        o = self.B * self.H_q * self.L_q * self.D_v * 4
        return q + k + v + o

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five benchmark configurations, in the order the benchmark spec lists them.
C1 = Workload("c1_softmax_noncausal", 1, 1, 2, 2, 256, 256, 64, 64)
C2 = Workload("c2_gqa_causal_softmax", 2, 4, 32, 8, 2048, 2048, 128, 128, mask="causal")
C3 = Workload("c3_sigmoid_causal", 3, 8, 16, 16, 4096, 4096, 64, 64,
              score_mod="bias", norm="sigmoid", mask="causal", bias=-math.log(4096.0))
C4 = Workload("c4_retnet", 4, 4, 8, 8, 4096, 4096, 128, 256,
              score_mod="head_decay", norm="abssum", mask="causal", decay=True)
C5 = Workload("c5_mla_causal_softmax", 5, 1, 128, 128, 8192, 8192, 192, 128, mask="causal")

CONFIGS = {w.name: w for w in (C1, C2, C3, C4, C5)}
BY_ID = {w.config_id: w for w in (C1, C2, C3, C4, C5)}


def table2_workloads():
    """The parallel-pattern rows of the paper's operator microbenchmark (Table 2) that the
    tile table covers, over its grid of batch 1 / 8 and sequence 2k / 4k / 8k (Section 6.1).
    The paper does not say which rows are causal: the language-model rows are taken as
    causal, the vision row (ReLU attention, ViT) as unmasked; the sigmoid row gets the
    bias -ln(L) of sigmoid attention; the retention row (256 / 512) gets RetNet's per-head decay
    rates and the abs-sum normalizer of the retention configuration."""
    rows = (
        ("softmax_llama31_8b", 32, 128, 128, dict(mask="causal")),
        ("softmax_dsv2_lite", 16, 192, 128, dict(mask="causal")),
        ("softmax_difftr_3b", 12, 128, 256, dict(mask="causal")),
        ("sigmoid_llama3_8b", 32, 128, 128, dict(mask="causal", norm="sigmoid", score_mod="bias")),
        ("relu_vit_s16", 6, 64, 64, dict(norm="none", score_mod="relu")),
        ("retention_parallel_retnet_6b7", 32, 256, 512, dict(mask="causal", score_mod="head_decay", norm="abssum", decay=True)),
    )
    out = []
    cid = 100
    for name, heads, dqk, dv, kw in rows:
        for batch in (1, 8):
            for seq in (2048, 4096, 8192):
                cid += 1
                extra = dict(kw)
                if extra.get("score_mod") == "bias":
                    extra["bias"] = -math.log(float(seq))
                out.append(Workload(f"t2_{name}_b{batch}_s{seq}", cid, batch, heads, heads, seq, seq, dqk, dv, **extra))
    return out


def make_inputs(w: Workload, seed_base: Optional[int] = None):
    """Return (Q, K, V) as contiguous CPU bf16 tensors [B, H, L, D]."""
    base = 1000 * w.config_id if seed_base is None else seed_base
    out = []
    for idx, shape in enumerate((
            (w.B, w.H_q, w.L_q, w.D_qk),
            (w.B, w.H_kv, w.L_k, w.D_qk),
            (w.B, w.H_kv, w.L_k, w.D_v))):
        g = torch.Generator(device="cpu")
        g.manual_seed(base + idx)
        x = torch.randn(shape, generator=g, dtype=torch.float32)
        out.append(x.to(torch.bfloat16).contiguous())
    return tuple(out)


def make_grad(w: Workload, seed_base: Optional[int] = None):
    """Upstream gradient dO for the backward pass: a contiguous CPU bf16 tensor [B, H_q, L_q, D_v], standard
    normal like the inputs, from a seed of its own."""
    base = 1000 * w.config_id if seed_base is None else seed_base
    g = torch.Generator(device="cpu")
    g.manual_seed(base + 7)
    return torch.randn((w.B, w.H_q, w.L_q, w.D_v), generator=g, dtype=torch.float32).to(torch.bfloat16).contiguous()


def make_bias_tensor(w: Workload, per_batch: bool = True, per_head: bool = True, seed_base: Optional[int] = None):
    """Additive bias for score_mod "bias_tensor": a contiguous CPU bf16 tensor [B or 1, H_q or 1, L_q, L_k], standard
    normal, from a seed of its own."""
    base = 1000 * w.config_id if seed_base is None else seed_base
    g = torch.Generator(device="cpu")
    g.manual_seed(base + 11)
    shape = (w.B if per_batch else 1, w.H_q if per_head else 1, w.L_q, w.L_k)
    return torch.randn(shape, generator=g, dtype=torch.float32).to(torch.bfloat16).contiguous()


def make_gates(B: int, H: int, L: int, seed: int, kind: str = "gated_retention"):
    """Per-token gates of the recurrent pattern, CPU fp32 [B, H, L], from a seed of their own.  Returns (log_decay,
    key_gate or None); the recipes follow how the models of Table 2 produce them from a token projection x ~ N(0, 1):
      gated_retention  decay = sigmoid(x) ** (1 / 16) (a sigmoid gate raised to a small power), no key gate;
      mamba2           dt = softplus(x - 4) (time steps around 0.02 .. 0.2), per-head A = -(1 + h % 16):
                       log_decay = dt * A, key_gate = dt."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    x = torch.randn((B, H, L), generator=g, dtype=torch.float32)
    if kind == "gated_retention":
        return (torch.nn.functional.logsigmoid(x) / 16.0).contiguous(), None
    if kind == "mamba2":
        dt = torch.nn.functional.softplus(x - 4.0)
        A = -(1.0 + (torch.arange(H, dtype=torch.float32) % 16)).view(1, H, 1)
        return (dt * A).contiguous(), dt.contiguous()
    raise ValueError(kind)
