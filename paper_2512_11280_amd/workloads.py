"""Seeded synthetic inputs shaped like the paper's workloads.

The paper decodes with Llama-3 (V = 128256) and Qwen-2.5 (V = 152064) model
pairs on public benchmark suites; neither weights nor datasets are available
here, so logits are drawn from seeded Gaussians with a "peaked mode" spike and a
draft row that is a noisy mix of the target row.  This module holds no part of
the method's arithmetic: it only produces tensors.  Both the GPU library and
the CPU oracle are fed from here, and neither imports the other.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch

DEFAULT_SEED = 0xADA5D


@dataclass
class VerifyBatch:
    target: torch.Tensor          # [B, k+1, V]
    draft: torch.Tensor           # [B, k, V]
    draft_tokens: torch.Tensor    # [B, k] int32
    draft_len: Optional[torch.Tensor] = None   # [B] int32 or None (= k everywhere)
    state: dict = field(default_factory=dict)  # numpy arrays: LA LR nA nR ent_sum ent_cnt T_G
    seed: int = DEFAULT_SEED
    round0: int = 0
    name: str = ""

    @property
    def B(self):
        return self.target.shape[0]

    @property
    def k(self):
        return self.draft.shape[1]

    @property
    def V(self):
        return self.target.shape[2]


def empty_state(B: int, cap: int) -> dict:
    """Algorithm 1's initial state: empty lists, generation threshold 0."""
    return dict(LA=np.zeros((B, cap), np.float32), LR=np.zeros((B, cap), np.float32),
                nA=np.zeros(B, np.int32), nR=np.zeros(B, np.int32),
                ent_sum=np.zeros(B, np.float64), ent_cnt=np.zeros(B, np.int32),
                T_G=np.zeros(B, np.float32))


def threshold_state(B: int, cap: int, gen: torch.Generator, n_hist: int = 64,
                    tau_lo: float = 0.05, tau_hi: float = 0.5) -> dict:
    """History lists whose posterior crosses 1/2 near a per-sequence distance tau_b:
    accepted distances ~ N(tau-0.1, 0.05^2), rejected ~ N(tau+0.1, 0.05^2), clipped into (0,1)."""
    st = empty_state(B, cap)
    tau = tau_lo + (tau_hi - tau_lo) * torch.rand(B, generator=gen, dtype=torch.float64)
    a = (tau[:, None] - 0.1) + 0.05 * torch.randn(B, n_hist, generator=gen, dtype=torch.float64)
    r = (tau[:, None] + 0.1) + 0.05 * torch.randn(B, n_hist, generator=gen, dtype=torch.float64)
    st["LA"][:, :n_hist] = a.clamp(1e-3, 1 - 1e-3).numpy().astype(np.float32)
    st["LR"][:, :n_hist] = r.clamp(1e-3, 1 - 1e-3).numpy().astype(np.float32)
    st["nA"][:] = n_hist
    st["nR"][:] = n_hist
    st["ent_sum"][:] = 4.0
    st["ent_cnt"][:] = 1
    st["T_G"][:] = 4.0
    st["tau"] = tau.numpy()
    return st


def _sample_tokens(draft_rows: torch.Tensor, gen: torch.Generator) -> torch.Tensor:
    """x_i ~ softmax(draft logits), one token per row (rows: [n, V])."""
    probs = torch.softmax(draft_rows.double(), dim=-1)
    return torch.multinomial(probs, 1, generator=gen).squeeze(-1).to(torch.int32)


def mix_logits(B: int, k: int, V: int, dtype: torch.dtype, gen: torch.Generator,
               std, spike, alpha: torch.Tensor, draw_tokens: bool = True):
    """Target rows N(0, std^2) with `spike` added at one random index per row; draft rows
    alpha*target + (1-alpha)*N(0, std^2).  `std`/`spike` are scalars or [k+1] tensors,
    `alpha` is [B, k].  Generated one sequence at a time to bound host memory.  draw_tokens=False leaves
    the token array at 0 (for callers whose tokens come from the drafting call)."""
    std = torch.as_tensor(std, dtype=torch.float32).expand(k + 1).reshape(k + 1, 1)
    spike = torch.as_tensor(spike, dtype=torch.float32).expand(k + 1)
    target = torch.empty(B, k + 1, V, dtype=dtype)
    draft = torch.empty(B, k, V, dtype=dtype)
    tokens = torch.zeros(B, k, dtype=torch.int32)
    for b in range(B):
        t = torch.randn(k + 1, V, generator=gen, dtype=torch.float32) * std
        idx = torch.randint(0, V, (k + 1,), generator=gen)
        t[torch.arange(k + 1), idx] += spike
        noise = torch.randn(k, V, generator=gen, dtype=torch.float32) * std[:k]
        a = alpha[b].to(torch.float32).reshape(k, 1)
        d = a * t[:k] + (1.0 - a) * noise
        target[b] = t.to(dtype)
        draft[b] = d.to(dtype)
        if k and draw_tokens:
            tokens[b] = _sample_tokens(draft[b].float(), gen)
    return target, draft, tokens


def config_tiny(seed: int = DEFAULT_SEED, B: int = 1, k: int = 4, V: int = 32000) -> VerifyBatch:
    """B=1, k=4, V=32000, fp32; per-position alpha ~ U[0.6,0.95]; paper-default (empty) state."""
    g = torch.Generator().manual_seed(seed)
    alpha = 0.6 + 0.35 * torch.rand(B, k, generator=g)
    t, d, x = mix_logits(B, k, V, torch.float32, g, 3.0, 8.0, alpha)
    return VerifyBatch(t, d, x, None, empty_state(B, 64), seed, 0, "tiny")


def config_single_stream(seed: int = DEFAULT_SEED + 1, V: int = 128256,
                         with_state: bool = True) -> VerifyBatch:
    """B=1, k=8, bf16; positions 0-3 low entropy (std 6, spike 10), 4-7 high entropy (std 1)."""
    g = torch.Generator().manual_seed(seed)
    k = 8
    alpha = 0.6 + 0.35 * torch.rand(1, k, generator=g)
    std = torch.tensor([6.0] * 4 + [1.0] * 4 + [1.0])
    spike = torch.tensor([10.0] * 4 + [0.0] * 4 + [0.0])
    t, d, x = mix_logits(1, k, V, torch.bfloat16, g, std, spike, alpha)
    st = threshold_state(1, 128, g) if with_state else empty_state(1, 128)
    return VerifyBatch(t, d, x, None, st, seed, 0, "single_stream")


def config_batched(seed: int = DEFAULT_SEED + 2, B: int = 32, k: int = 8, V: int = 128256,
                   dtype: torch.dtype = torch.bfloat16, cap: int = 128) -> VerifyBatch:
    """Headline shape: B=32, k=8, V=128256, bf16; per-sequence alpha ~ U[0.5,0.98]; per-sequence
    thresholds tau_b ~ U[0.05,0.5] realised as history lists."""
    g = torch.Generator().manual_seed(seed)
    alpha = (0.5 + 0.48 * torch.rand(B, 1, generator=g)).expand(B, k)
    t, d, x = mix_logits(B, k, V, dtype, g, 3.0, 8.0, alpha)
    st = threshold_state(B, cap, g)
    return VerifyBatch(t, d, x, None, st, seed, 0, "batched")


def config_large(seed: int = DEFAULT_SEED + 3, B: int = 128, k: int = 16, V: int = 152064,
                 dtype: torch.dtype = torch.bfloat16, cap: int = 128,
                 indep_frac: float = 0.1) -> VerifyBatch:
    """B=128, k=16, V=152064, bf16; draft = target + N(0, 0.5^2); `indep_frac` of the positions
    get a fully independent draft row so early rejection is frequent."""
    g = torch.Generator().manual_seed(seed)
    target = torch.empty(B, k + 1, V, dtype=dtype)
    draft = torch.empty(B, k, V, dtype=dtype)
    tokens = torch.empty(B, k, dtype=torch.int32)
    indep = torch.rand(B, k, generator=g) < indep_frac
    for b in range(B):
        t = torch.randn(k + 1, V, generator=g, dtype=torch.float32) * 3.0
        idx = torch.randint(0, V, (k + 1,), generator=g)
        t[torch.arange(k + 1), idx] += 8.0
        d = t[:k] + 0.5 * torch.randn(k, V, generator=g, dtype=torch.float32)
        fresh = torch.randn(k, V, generator=g, dtype=torch.float32) * 3.0
        d = torch.where(indep[b].reshape(k, 1), fresh, d)
        target[b] = t.to(dtype)
        draft[b] = d.to(dtype)
        tokens[b] = _sample_tokens(draft[b].float(), g)
    st = threshold_state(B, cap, g)
    return VerifyBatch(target, draft, tokens, None, st, seed, 0, "large")


class ClosedLoopSource:
    """Logit producer for the closed-loop configuration: per sequence an alpha that drifts by a
    +-0.02 random walk clipped to [0.4, 0.99]; each decode round draws fresh target/draft rows
    with the tiny configuration's recipe (std 3, spike 8)."""

    def __init__(self, B: int, V: int, k_max: int, dtype=torch.bfloat16,
                 seed: int = DEFAULT_SEED + 4, draw_tokens: bool = True):
        self.B, self.V, self.k_max, self.dtype = B, V, k_max, dtype
        self.draw_tokens = draw_tokens
        self.gen = torch.Generator().manual_seed(seed)
        self.alpha = 0.5 + 0.4 * torch.rand(B, generator=self.gen)
        self.seed = seed

    def next_round(self):
        step = torch.where(torch.rand(self.B, generator=self.gen) < 0.5, -0.02, 0.02)
        self.alpha = (self.alpha + step).clamp(0.4, 0.99)
        alpha = self.alpha.reshape(self.B, 1).expand(self.B, self.k_max)
        return mix_logits(self.B, self.k_max, self.V, self.dtype, self.gen, 3.0, 8.0, alpha, self.draw_tokens)


class ClosedLoopDeviceSource:
    """The same recipe generated on the GPU (its own random stream): per round target rows [B, k_max+1, V]
    and draft rows [B, k_max, V] in bf16, resident in device memory.  For the sequences of a closed-loop run
    that no host-side check replays."""

    def __init__(self, B: int, V: int, k_max: int, seed: int = DEFAULT_SEED + 4, device: str = "cuda"):
        self.B, self.V, self.k_max, self.device = B, V, k_max, device
        self.gen = torch.Generator(device=device).manual_seed(seed)
        self.alpha = 0.5 + 0.4 * torch.rand(B, generator=self.gen, device=device)

    def next_round(self):
        B, k, V, g, dev = self.B, self.k_max, self.V, self.gen, self.device
        walk = torch.where(torch.rand(B, generator=g, device=dev) < 0.5, -0.02, 0.02)
        self.alpha = (self.alpha + walk).clamp(0.4, 0.99)
        t = torch.randn(B, k + 1, V, generator=g, device=dev) * 3.0
        idx = torch.randint(0, V, (B, k + 1, 1), generator=g, device=dev)
        t.scatter_add_(2, idx, torch.full_like(idx, 8.0, dtype=torch.float32))
        a3 = self.alpha.reshape(B, 1, 1)
        d = (a3 * t[:, :k] + (1 - a3) * 3.0 * torch.randn(B, k, V, generator=g, device=dev)).to(torch.bfloat16)
        return t.to(torch.bfloat16), d
