"""Seeded synthetic inputs for the DPPO loss hot path.

This module only draws random numbers and shapes them into arrays. It holds none
of the method's arithmetic (no advantages, masks, packing, log-probs or losses):
those live in the HIP library and, separately, in the CPU oracle, and both are
handed the arrays made here.

The five workloads mirror the shapes, length mixes and reward structure of
group-based RL fine-tuning of Qwen3-sized models on verifiable-reward math data
(binary rewards, G completions per prompt, ragged prompt/completion lengths);
they stand in for the paper's training sets, which are not used here.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    Q: int                      # prompts per batch
    G: int                      # completions per prompt
    prompt_len: Tuple[int, int]  # inclusive uniform range
    comp_len: Tuple             # ("uniform", lo, hi) | ("lognormal", median, sigma, lo, hi) | ("bimodal", lo1, hi1, lo2, hi2)
    D: int                      # hidden size
    V: int                      # vocabulary size
    dtype: str                  # "f32" | "bf16"
    w_std: float
    ids: str                    # "uniform" | "zipf"
    reward_p: Tuple             # ("uniform",) | ("beta", a, b) | ("mixture01",)
    r_q: float                  # prompt prune probability  (= 1 - keep-prob)
    r_o: float                  # completion prune probability
    capacity: int               # packing window (tokens per packed row)
    n_win: int                  # candidate-pool size of the packer
    clip_eps: float = 0.2
    kl_beta: float = 0.04
    logp_noise: float = 0.05


WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", 4, 4, (8, 16), ("uniform", 8, 32), 64, 512, "f32", 0.05,
                     "uniform", ("uniform",), 0.5, 0.5, 256, 4),
    "small": Workload("small", 32, 8, (64, 256), ("uniform", 128, 1024), 1024, 32000, "bf16", 0.02,
                      "uniform", ("beta", 0.5, 0.5), 0.4, 0.5, 4096, 32),
    "qwen3_4b": Workload("qwen3_4b", 64, 8, (64, 512), ("lognormal", 1200.0, 0.6, 16, 4096),
                         2560, 151936, "bf16", 0.02, "zipf", ("beta", 0.5, 0.5), 0.5, 0.5, 8192, 32),
    "qwen3_8b": Workload("qwen3_8b", 128, 16, (64, 512), ("lognormal", 2000.0, 0.6, 16, 8192),
                         4096, 151936, "bf16", 0.02, "zipf", ("mixture01",), 0.6, 0.5, 16384, 32),
    "stress": Workload("stress", 256, 16, (16, 2048), ("bimodal", 16, 128, 4096, 16384),
                       4096, 151936, "bf16", 0.02, "zipf", ("beta", 0.3, 0.3), 0.7, 0.7, 32768, 32),
}


@dataclass
class RolloutBatch:
    """Host-side description of one batch after rollout, before selection."""
    wl: Workload
    seed: int
    prompt_len: np.ndarray      # [Q]   int32
    comp_len: np.ndarray        # [Q,G] int32
    rewards: np.ndarray         # [Q,G] float32 in {0,1}
    hist: np.ndarray            # [Q]   float32, stand-in for last epoch's score (has ties)
    u_prompt: np.ndarray        # [Q]   float32 in [0,1)
    u_comp: np.ndarray          # [Q,G] float32 in [0,1)
    extra: dict = field(default_factory=dict)

    @property
    def item_prompt_len(self) -> np.ndarray:
        """Prompt length repeated per completion, [Q*G] int32."""
        return np.repeat(self.prompt_len, self.wl.G).astype(np.int32)

    @property
    def item_comp_len(self) -> np.ndarray:
        return self.comp_len.reshape(-1).astype(np.int32)


def _draw_comp_len(rng: np.random.Generator, spec: Tuple, shape) -> np.ndarray:
    kind = spec[0]
    if kind == "uniform":
        return rng.integers(spec[1], spec[2] + 1, size=shape)
    if kind == "lognormal":
        _, median, sigma, lo, hi = spec
        x = np.rint(rng.lognormal(np.log(median), sigma, size=shape))
        return np.clip(x, lo, hi).astype(np.int64)
    if kind == "bimodal":
        _, lo1, hi1, lo2, hi2 = spec
        short = rng.integers(lo1, hi1 + 1, size=shape)
        long_ = rng.integers(lo2, hi2 + 1, size=shape)
        pick = rng.random(size=shape) < 0.5
        return np.where(pick, short, long_)
    raise ValueError(kind)


def _draw_reward_p(rng: np.random.Generator, spec: Tuple, Q: int) -> np.ndarray:
    kind = spec[0]
    if kind == "uniform":
        return rng.random(Q)
    if kind == "beta":
        return rng.beta(spec[1], spec[2], size=Q)
    if kind == "mixture01":
        # half the groups are all-0 or all-1 (zero-variance groups), the rest Beta(1,1)
        degenerate = rng.random(Q) < 0.5
        which = (rng.random(Q) < 0.5).astype(np.float64)
        return np.where(degenerate, which, rng.beta(1.0, 1.0, size=Q))
    raise ValueError(kind)


def make_rollout(name: str, seed: Optional[int] = None) -> RolloutBatch:
    wl = WORKLOADS[name]
    if seed is None:
        seed = list(WORKLOADS).index(name) + 1
    rng = np.random.default_rng([seed, 0xD990])
    Q, G = wl.Q, wl.G
    prompt_len = rng.integers(wl.prompt_len[0], wl.prompt_len[1] + 1, size=Q).astype(np.int32)
    comp_len = _draw_comp_len(rng, wl.comp_len, (Q, G)).astype(np.int32)
    p = _draw_reward_p(rng, wl.reward_p, Q)
    rewards = (rng.random((Q, G)) < p[:, None]).astype(np.float32)
    # Stand-in for the previous epoch's per-prompt score: non-negative, two decimals
    # (so equal scores occur), and a fifth of the prompts still at the initial 0.
    hist = np.round(rng.random(Q), 2)
    hist[rng.random(Q) < 0.2] = 0.0
    u_prompt = rng.random(Q, dtype=np.float32)
    u_comp = rng.random((Q, G), dtype=np.float32)
    return RolloutBatch(wl, seed, prompt_len, comp_len, rewards, hist.astype(np.float32),
                        u_prompt, u_comp, {"reward_p": p})


# Prompt-length sets for packing a whole dataset before any rollout (Sec. 4.3). The sizes are
# those of the paper's two training sets (8.5 K and 7.5 K problems); the lengths are synthetic:
# log-normal token counts, short word problems and longer competition problems.
PROMPT_DATASETS: Dict[str, Tuple] = {
    "short_8k5": (8500, ("lognormal", 90.0, 0.35, 16, 512)),
    "long_7k5": (7500, ("lognormal", 140.0, 0.6, 16, 2048)),
}


def make_prompt_dataset(name: str, seed: Optional[int] = None) -> np.ndarray:
    n, spec = PROMPT_DATASETS[name]
    if seed is None:
        seed = list(PROMPT_DATASETS).index(name) + 1
    rng = np.random.default_rng([seed, 0xDA7A])
    return _draw_comp_len(rng, spec, n).astype(np.int32)


def zipf_table(V: int, exponent: float, seed: int):
    """CDF over ranks (p_r ~ r^-exponent, r=1..V) and a fixed rank->id permutation."""
    w = np.arange(1, V + 1, dtype=np.float64) ** (-exponent)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    perm = np.random.default_rng([seed, 0x21BF]).permutation(V).astype(np.int32)
    return cdf, perm


def make_ids(wl: Workload, T: int, seed: int) -> np.ndarray:
    """Token ids for T packed positions, int32 in [0, V)."""
    rng = np.random.default_rng([seed, 0x1D5])
    if wl.ids == "uniform":
        return rng.integers(0, wl.V, size=T).astype(np.int32)
    cdf, perm = zipf_table(wl.V, 1.1, seed)
    ranks = np.searchsorted(cdf, rng.random(T), side="right")
    ranks = np.minimum(ranks, wl.V - 1)
    return perm[ranks].astype(np.int32)


def torch_dtype(wl: Workload):
    import torch
    return torch.float32 if wl.dtype == "f32" else torch.bfloat16


def make_hidden(wl: Workload, T: int, seed: int, device="cpu", rows_per_block: int = 1 << 16):
    """H[T,D] ~ N(0,1) rounded to the workload dtype (one row per packed token)."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed * 7919 + 11)
    out = torch.empty((T, wl.D), dtype=torch_dtype(wl), device=device)
    for r0 in range(0, T, rows_per_block):
        r1 = min(T, r0 + rows_per_block)
        out[r0:r1] = torch.randn((r1 - r0, wl.D), generator=gen, device=device,
                                 dtype=torch.float32).to(out.dtype)
    return out


def make_vocab_matrix(wl: Workload, seed: int, device="cpu", rows_per_block: int = 1 << 15):
    """W[V,D] ~ N(0, w_std) rounded to the workload dtype; logits = H @ W^T."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed * 104729 + 5)
    out = torch.empty((wl.V, wl.D), dtype=torch_dtype(wl), device=device)
    for r0 in range(0, wl.V, rows_per_block):
        r1 = min(wl.V, r0 + rows_per_block)
        out[r0:r1] = (torch.randn((r1 - r0, wl.D), generator=gen, device=device,
                                  dtype=torch.float32) * wl.w_std).to(out.dtype)
    return out


def perturb_logp(base: np.ndarray, noise: float, seed: int, which: int) -> np.ndarray:
    """Old-policy (which=0) / reference-policy (which=1) log-probs: base + N(0, noise), float32."""
    rng = np.random.default_rng([seed, 0x0DD + which])
    return (np.asarray(base, dtype=np.float64)
            + rng.normal(0.0, noise, size=np.shape(base))).astype(np.float32)
