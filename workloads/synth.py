"""Seeded synthetic rollout batches shaped like the paper's reasoning workloads.

The paper trains Qwen-class models on groups of G = 8 rollouts per prompt with
generation caps of 16K (math) and 32K (code) tokens, sampled at temperature 1
and top-p 1 (appendix tables of shared hyper-parameters).  Neither its
datasets nor its checkpoints are used here: every batch below is drawn from a
seeded generator and only reproduces the *shapes* (hidden size, vocabulary,
group structure, length mix) and the value distributions of such a batch.

This module only produces inputs and is not part of the library (it lives
beside the tests and the benchmark that use it).  It computes nothing of the
OAPL objective.  The one piece of arithmetic it holds is a stand-in for the
*inference engine*:
the lagged policy's log-probabilities of the sampled tokens are an input of
the method (Sec. 3.1, Eq. 3 uses them as given), and in the paper's system they
come from a separate engine with its own numerics.  Here they come from plain
library calls (``torch.matmul`` / ``torch.logsumexp``) plus seeded Gaussian
drift, and are frozen before either the HIP path or the CPU oracle sees them.

Everything is generated on the requested device with a ``torch.Generator`` so
the large configurations take seconds, not minutes; both consumers then read
the very same tensors (the oracle through ``.cpu()``).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional

import torch

BASE_SEED = 20260219


@dataclasses.dataclass(frozen=True)
class RolloutConfig:
    """Shape and distribution recipe of one synthetic batch."""

    name: str
    dtype: str                 # "f32" or "bf16": storage type of H and W
    d: int                     # hidden size
    V: int                     # vocabulary size
    n_prompts: int             # P, number of groups
    n_rollouts: int            # G, rollouts per prompt
    length: str                # "fixed" or "lognormal"
    len_fixed: int = 0         # tokens per rollout when length == "fixed"
    len_median: int = 0        # lognormal median
    len_max: int = 0           # generation cap (truncation point)
    len_min: int = 16
    len_sigma: float = 0.6
    tokens: str = "uniform"    # "uniform" or "policy" (softmax(H W^T / temp))
    token_temp: float = 0.8
    logq: str = "drift"        # "drift": engine lp + N(0, sigma); "lagged_w": lp under W'
    logq_sigma: float = 0.1
    lag_w_var: float = 0.01    # W' = W + N(0, lag_w_var / d)
    rewards: str = "bernoulli"  # "bernoulli" or "beta_prompt"
    reward_p: float = 0.5
    beta: float = 1.0
    backward: bool = True
    seed_index: int = 0

    @property
    def n_seq(self) -> int:
        return self.n_prompts * self.n_rollouts


# The five named configurations.  Index 1 is the small case an fp64 CPU oracle
# finishes in well under a second; the others are one-GPU production shapes.
CONFIGS = {
    "tiny_f32": RolloutConfig(
        name="tiny_f32", dtype="f32", d=64, V=1024, n_prompts=2, n_rollouts=4,
        length="fixed", len_fixed=32, tokens="uniform", logq="drift",
        logq_sigma=0.05, rewards="bernoulli", reward_p=0.5, beta=1.0,
        backward=True, seed_index=1),
    "qwen1p7b_fwd": RolloutConfig(
        name="qwen1p7b_fwd", dtype="bf16", d=2048, V=151936, n_prompts=4,
        n_rollouts=8, length="fixed", len_fixed=1024, tokens="policy",
        token_temp=0.8, logq="drift", logq_sigma=0.1, rewards="bernoulli",
        reward_p=0.3, beta=1.0, backward=False, seed_index=2),
    "qwen7b": RolloutConfig(
        name="qwen7b", dtype="bf16", d=4096, V=151936, n_prompts=8,
        n_rollouts=8, length="lognormal", len_median=2048, len_max=4096,
        tokens="uniform", logq="drift", logq_sigma=0.2, rewards="bernoulli",
        reward_p=0.4, beta=0.5, backward=True, seed_index=3),
    "r1_14b": RolloutConfig(
        name="r1_14b", dtype="bf16", d=5120, V=151936, n_prompts=8,
        n_rollouts=16, length="lognormal", len_median=6000, len_max=16384,
        tokens="uniform", logq="drift", logq_sigma=0.2, rewards="beta_prompt",
        beta=1.0, backward=True, seed_index=4),
    "long_rollout": RolloutConfig(
        name="long_rollout", dtype="bf16", d=4096, V=151936, n_prompts=4,
        n_rollouts=8, length="fixed", len_fixed=32768, tokens="uniform",
        logq="lagged_w", lag_w_var=0.01, rewards="bernoulli", reward_p=0.2,
        beta=2.0, backward=True, seed_index=5),
}


def reduced(cfg: RolloutConfig, **overrides) -> RolloutConfig:
    """Same recipe with some fields replaced (used for oracle-sized slices)."""
    return dataclasses.replace(cfg, **overrides)


@dataclasses.dataclass
class RolloutBatch:
    """One packed batch; all tensors live on ``device``."""

    cfg: RolloutConfig
    H: torch.Tensor            # [T, d] hidden states, cfg.dtype
    W: torch.Tensor            # [V, d] LM-head weights, cfg.dtype
    tokens: torch.Tensor       # [T] int32 sampled token ids
    logq: torch.Tensor         # [T] fp32 inference-policy log-probs of tokens
    seq_offsets: torch.Tensor  # [N+1] int64, packed stream offsets
    rewards: torch.Tensor      # [N] fp32
    group_ids: torch.Tensor    # [N] int32 prompt index of each rollout
    beta: float

    @property
    def T(self) -> int:
        return int(self.H.shape[0])

    @property
    def n_seq(self) -> int:
        return int(self.rewards.shape[0])

    @property
    def n_groups(self) -> int:
        return self.cfg.n_prompts


def _torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def _draw_lengths(cfg: RolloutConfig, gen: torch.Generator, device) -> torch.Tensor:
    n = cfg.n_seq
    if cfg.length == "fixed":
        return torch.full((n,), cfg.len_fixed, dtype=torch.int64)
    # Truncated lognormal: the cap plays the role of the max-generation-length
    # cut-off, so a visible fraction of rollouts sits exactly at the cap.
    xi = torch.randn(n, generator=gen, device=device, dtype=torch.float64).cpu()
    raw = torch.round(cfg.len_median * torch.exp(cfg.len_sigma * xi))
    return raw.clamp(cfg.len_min, cfg.len_max).to(torch.int64)


def _randn_rows(rows: int, cols: int, std: float, dtype, gen, device) -> torch.Tensor:
    """N(0, std^2) drawn in fp32 slab by slab, rounded once (RNE) to ``dtype``."""
    out = torch.empty((rows, cols), dtype=dtype, device=device)
    slab = max(1, (1 << 26) // max(cols, 1))
    for r0 in range(0, rows, slab):
        r1 = min(rows, r0 + slab)
        x = torch.randn((r1 - r0, cols), generator=gen, device=device, dtype=torch.float32)
        out[r0:r1] = (x * std).to(dtype)
    return out


def _matmul_dtype(device) -> Optional[torch.dtype]:
    # CPU half-precision matmuls are slow; widen there.  Values are unchanged.
    return torch.float32 if torch.device(device).type == "cpu" else None


def _engine_logits(Hc: torch.Tensor, W: torch.Tensor) -> torch.Tensor:
    md = _matmul_dtype(Hc.device)
    if md is not None:
        return Hc.to(md) @ W.to(md).T
    return (Hc @ W.T).float()


def _row_chunk(V: int, device) -> int:
    budget = (1 << 31) if torch.device(device).type != "cpu" else (1 << 28)
    return max(1, budget // (4 * V))


def engine_sample_tokens(H, W, temp: float, gen, chunk: Optional[int] = None) -> torch.Tensor:
    """Draw one token per row from softmax(H W^T / temp) by the Gumbel-max trick."""
    T, V = H.shape[0], W.shape[0]
    chunk = chunk or _row_chunk(V, H.device)
    Wm = W.to(_matmul_dtype(H.device)) if _matmul_dtype(H.device) else W
    out = torch.empty(T, dtype=torch.int32, device=H.device)
    for r0 in range(0, T, chunk):
        z = _engine_logits(H[r0:r0 + chunk], Wm) / temp
        u = torch.rand(z.shape, generator=gen, device=H.device, dtype=torch.float32)
        u = u.clamp_(1e-12, 1.0 - 1e-7)
        z -= torch.log(-torch.log(u))
        out[r0:r0 + chunk] = z.argmax(dim=1).to(torch.int32)
    return out


def engine_logprobs(H, W, tokens, chunk: Optional[int] = None) -> torch.Tensor:
    """Inference-engine stand-in: log-softmax of H W^T gathered at ``tokens``.

    Library calls only; its rounding is the engine's own and is part of the
    input, exactly as a real engine's log-probs would be.
    """
    T, V = H.shape[0], W.shape[0]
    chunk = chunk or _row_chunk(V, H.device)
    Wm = W.to(_matmul_dtype(H.device)) if _matmul_dtype(H.device) else W
    out = torch.empty(T, dtype=torch.float32, device=H.device)
    for r0 in range(0, T, chunk):
        z = _engine_logits(H[r0:r0 + chunk], Wm)
        lse = torch.logsumexp(z, dim=1)
        zy = z.gather(1, tokens[r0:r0 + chunk].long().unsqueeze(1)).squeeze(1)
        out[r0:r0 + chunk] = zy - lse
    return out


def make_batch(cfg: RolloutConfig, device="cpu", seed: Optional[int] = None) -> RolloutBatch:
    """Draw one batch.  Draw order is fixed: lengths, H, W, tokens, logq, rewards."""
    device = torch.device(device)
    seed = BASE_SEED + cfg.seed_index if seed is None else seed
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    dt = _torch_dtype(cfg.dtype)

    lengths = _draw_lengths(cfg, gen, device)
    offsets = torch.zeros(cfg.n_seq + 1, dtype=torch.int64)
    offsets[1:] = torch.cumsum(lengths, 0)
    T = int(offsets[-1])

    H = _randn_rows(T, cfg.d, 1.0, dt, gen, device)
    W = _randn_rows(cfg.V, cfg.d, 1.0 / math.sqrt(cfg.d), dt, gen, device)

    if cfg.tokens == "uniform":
        tokens = torch.randint(0, cfg.V, (T,), generator=gen, device=device, dtype=torch.int64).to(torch.int32)
    elif cfg.tokens == "policy":
        tokens = engine_sample_tokens(H, W, cfg.token_temp, gen)
    else:
        raise ValueError(cfg.tokens)

    if cfg.logq == "drift":
        base = engine_logprobs(H, W, tokens)
        noise = torch.randn(T, generator=gen, device=device, dtype=torch.float32)
        logq = base + cfg.logq_sigma * noise
    elif cfg.logq == "lagged_w":
        Wlag = torch.empty_like(W)
        std = math.sqrt(cfg.lag_w_var / cfg.d)
        slab = max(1, (1 << 26) // cfg.d)
        for r0 in range(0, cfg.V, slab):
            r1 = min(cfg.V, r0 + slab)
            e = torch.randn((r1 - r0, cfg.d), generator=gen, device=device, dtype=torch.float32)
            Wlag[r0:r1] = (W[r0:r1].float() + std * e).to(dt)
        logq = engine_logprobs(H, Wlag, tokens)
        del Wlag
    else:
        raise ValueError(cfg.logq)

    n = cfg.n_seq
    group_ids = (torch.arange(n, dtype=torch.int64) // cfg.n_rollouts).to(torch.int32)
    if cfg.rewards == "bernoulli":
        u = torch.rand(n, generator=gen, device=device, dtype=torch.float32).cpu()
        rewards = (u < cfg.reward_p).to(torch.float32)
    elif cfg.rewards == "beta_prompt":
        # Per-prompt solve rate p ~ Beta(1, 2) (inverse CDF: 1 - sqrt(1 - u));
        # prompts 0 and 1 are forced to all-fail / all-pass so that the
        # degenerate all-equal-rewards value estimate is always present.
        up = torch.rand(cfg.n_prompts, generator=gen, device=device, dtype=torch.float32).cpu()
        p = 1.0 - torch.sqrt(1.0 - up)
        u = torch.rand(n, generator=gen, device=device, dtype=torch.float32).cpu()
        rewards = (u < p[group_ids.long()]).to(torch.float32)
        rewards[group_ids == 0] = 0.0
        if cfg.n_prompts > 1:
            rewards[group_ids == 1] = 1.0
    else:
        raise ValueError(cfg.rewards)

    return RolloutBatch(
        cfg=cfg, H=H, W=W, tokens=tokens, logq=logq.contiguous(),
        seq_offsets=offsets.to(device), rewards=rewards.to(device),
        group_ids=group_ids.to(device), beta=cfg.beta)
