"""Synthetic workloads: the five cache shapes of the benchmark and their seeded generators.

Everything here is *data*: shapes, value distributions, seeds.  The generators draw fp32
values from a seeded torch generator, round them once to bf16 (round-to-nearest-even) and
return bf16 tensors; the very same bits are handed to the HIP path and, converted exactly to
fp64, to the oracle.  The same (workload, layer, device) always yields the same tensors; CPU
and GPU generators give different streams, so a test fixes one device for both sides.

The caches stand in for the long-context prompts the paper evaluates on (Llama-3.1-8B /
Mistral-7B / Qwen-shaped GQA attention at 4K-128K context, Section 4 "Models and Evaluation
Setup"); only the shapes are taken from there.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional, Tuple

import torch

BASE_SEED = 25475

# tensor-kind ids used to derive independent seeds
_KIND = {"params": 1, "k": 2, "v": 3, "q": 4, "aux": 5, "x": 6}


@dataclass(frozen=True)
class Workload:
    """One benchmark configuration (a cache shape plus its eviction schedule)."""

    name: str
    index: int                 # 1-based number of the configuration
    n_q_heads: int             # H
    n_kv_heads: int            # H_kv
    n_layers: int
    batch: int
    context: int               # prompt length L
    budget: int                # kept entries per (batch, KV head) after an eviction event
    decode_steps: int
    dist: str                  # "normal" | "planted" | "mixture" | "walk"
    planted_frac: float = 0.0
    planted_scale: float = 4.0
    prefill_chunk: Optional[int] = None   # None: one-shot eviction after the whole prompt
    head_dim: int = 128
    idx_dim: int = 64          # d_index
    mem_dim: int = 128         # d_mem
    n_sink: int = 4
    n_recent: int = 0
    fold_block: int = 64
    lam: float = 0.999         # decay of the memory state per eviction event
    eta: float = 0.5           # write strength
    param_std: float = 0.02
    # the layer-wide form of the paper's text: indexer keys from hidden states (idx_dim 16), one
    # eviction set and one memory per sequence, shared by all KV heads
    head_shared: bool = False

    def __post_init__(self):
        # the library takes lambda and eta as fp32 arguments: the recipe's values ARE those fp32 values
        # (0.999 -> 0.99900001287...), so that both sides of a parity test decay by the same factor
        # (a relative 1.3e-8 per event adds up to 1.4e-5 of M over configuration 5's 1055 events)
        object.__setattr__(self, "lam", float(torch.tensor(self.lam, dtype=torch.float32).item()))
        object.__setattr__(self, "eta", float(torch.tensor(self.eta, dtype=torch.float32).item()))

    @property
    def n_idx_heads(self) -> int:      # H_index = H / 4 (Section 4, hyper-parameters)
        return self.n_q_heads // 4

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def gate_in_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def capacity(self) -> int:
        """Slots per (batch, KV head) needed to run the schedule."""
        if self.prefill_chunk is None:
            return max(self.context, self.budget + 1)
        return self.budget + self.prefill_chunk

    @property
    def n_tokens(self) -> int:
        return self.context + self.decode_steps

    def scaled(self, **kw) -> "Workload":
        """A reduced copy (same distribution and head shape) for parity tests."""
        return replace(self, **kw)

    def shared(self, **kw) -> "Workload":
        """The same cache shape in the head-shared layout (d_index = d_head / 8)."""
        return replace(self, head_shared=True, idx_dim=self.head_dim // 8, name=self.name + "-shared", **kw)


WORKLOADS: Dict[str, Workload] = {
    "cfg1": Workload("cfg1", 1, 32, 8, 1, 1, 1024, 256, 16, "normal"),
    "cfg2": Workload("cfg2", 2, 32, 8, 32, 8, 4096, 1024, 256, "planted", planted_frac=0.05),
    "cfg3": Workload("cfg3", 3, 32, 8, 32, 4, 16384, 2048, 512, "mixture"),
    "cfg4": Workload("cfg4", 4, 28, 4, 28, 16, 16384, 512, 256, "planted", planted_frac=0.01),
    "cfg5": Workload("cfg5", 5, 32, 8, 32, 1, 131072, 4096, 1024, "walk", prefill_chunk=4096),
}


def _gen(device, w: Workload, layer: int, kind: str) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(BASE_SEED * 1_000_003 + w.index * 100_003 + layer * 1_009 + _KIND[kind])
    return g


def _randn(shape, g: torch.Generator, device) -> torch.Tensor:
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32)


def layer_params(w: Workload, layer: int, device="cpu") -> Dict[str, object]:
    """Random-init slow weights of one layer: every matrix ~ N(0, param_std^2) in bf16,
    norm weights one, gate bias zero."""
    g = _gen(device, w, layer, "params")
    H, D, Hi, di, dm = w.n_q_heads, w.head_dim, w.n_idx_heads, w.idx_dim, w.mem_dim
    s = w.param_std

    def mat(*shape):
        return (_randn(shape, g, device) * s).to(torch.bfloat16)

    return {
        "Uq": mat(Hi * di, H * D),
        "G": mat(Hi, w.gate_in_dim),
        "Uk": mat(di, w.gate_in_dim if w.head_shared else D),
        "norm_q_w": torch.ones(di, device=device, dtype=torch.bfloat16),
        "norm_k_w": torch.ones(di, device=device, dtype=torch.bfloat16),
        "Wtheta": mat(dm, D),
        "wg": mat(D),
        "cg": 0.0,
    }


def token_stream(w: Workload, layer: int, device="cpu",
                 n_tokens: Optional[int] = None) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """All tokens of one layer, prompt followed by the decode tokens.

    Returns (K, V, Q): K, V of shape [batch, H_kv, T, D] and Q of shape [batch, T, H, D], bf16,
    T = context + decode_steps unless n_tokens is given.  Token t has position t.
    """
    T = w.n_tokens if n_tokens is None else n_tokens
    Bz, Hkv, H, D = w.batch, w.n_kv_heads, w.n_q_heads, w.head_dim
    gk, gv, gq, ga = (_gen(device, w, layer, k) for k in ("k", "v", "q", "aux"))

    K = _randn((Bz, Hkv, T, D), gk, device)
    if w.dist == "normal":
        pass
    elif w.dist == "planted":
        # exactly floor(frac * context) prompt positions per (batch, head) get their key row
        # scaled; each decode token is scaled with probability frac
        u = torch.rand((Bz, Hkv, T), generator=ga, device=device)
        n_prompt = min(w.context, T)
        n_planted = int(w.planted_frac * n_prompt)
        mask = torch.zeros((Bz, Hkv, T), dtype=torch.bool, device=device)
        if n_planted > 0:
            idx = torch.topk(u[:, :, :n_prompt], n_planted, dim=-1, largest=False).indices
            mask.scatter_(2, idx, True)
        if T > n_prompt:
            mask[:, :, n_prompt:] = u[:, :, n_prompt:] < w.planted_frac
        K = torch.where(mask.unsqueeze(-1), K * w.planted_scale, K)
    elif w.dist == "mixture":
        # 8 components per (layer, head): means ~ N(0, I), uniform assignment per token
        mu = _randn((Hkv, 8, D), ga, device)
        c = torch.randint(0, 8, (Bz, Hkv, T), generator=ga, device=device)
        head = torch.arange(Hkv, device=device).view(1, Hkv, 1).expand(Bz, Hkv, T)
        K = K + mu[head, c]
    elif w.dist == "walk":
        # slowly drifting mean per (layer, head): mu_t = mu_{t-1} + 0.01 N(0, I), mu_0 = 0
        steps = _randn((Hkv, T, D), ga, device) * 0.01
        steps[:, 0, :] = 0.0
        mu = torch.cumsum(steps, dim=1)
        K = K + mu.unsqueeze(0)
    else:
        raise ValueError(f"unknown distribution {w.dist!r}")
    K = K.to(torch.bfloat16)
    V = _randn((Bz, Hkv, T, D), gv, device).to(torch.bfloat16)
    Q = _randn((Bz, T, H, D), gq, device).to(torch.bfloat16)
    return K, V, Q


def hidden_stream(w: Workload, layer: int, device="cpu", n_tokens: Optional[int] = None) -> torch.Tensor:
    """Hidden states X [batch, T, d_model] ~ N(0, 1) in bf16 (d_model = H * head_dim): the input of the
    head-shared layout's key projection and head gate.  Token t has position t."""
    T = w.n_tokens if n_tokens is None else n_tokens
    return _randn((w.batch, T, w.gate_in_dim), _gen(device, w, layer, "x"), device).to(torch.bfloat16)
