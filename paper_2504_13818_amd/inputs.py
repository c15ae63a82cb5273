"""Seeded synthetic inputs for the PODS hot path (rewards, rollout lengths, token ids,
hidden states, lm_head weights, old-policy log-probs).

This module only draws random numbers and converts storage formats.  It holds none of the
method's arithmetic (no sorting, no variance, no softmax, no loss): it is the one piece of
code that both the CPU oracle's tests and the HIP path's tests / benchmark are fed from.

The shapes and value structure follow the paper's workloads: discrete rule-based rewards
(Sec. 4, "Rewards"; App. "Reward functions"), n rollouts down-sampled to m per prompt
(Table 2), completion length capped at 1024 / 2048 tokens (Table 2), and the lm_head shapes of
the model families it trains (Qwen2.5-3B / 7B, Llama-3-8B class).  The datasets and weights
themselves are not used: these tensors stand in for them.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 20250418

# name, B groups, n rollouts, m kept, T padded length, (len_lo, len_hi), d, V, dtype, reward kind
CONFIGS = {
    0: dict(name="tiny-fp32", B=4, n=16, m=4, T=64, len_range=(64, 64), d=256, V=1024,
            dtype="f32", hidden_std=0.02, w_std=0.02, rewards="bernoulli_uniform", clip_eps=0.2),
    1: dict(name="qwen2.5-3b-head", B=32, n=64, m=16, T=1024, len_range=(128, 1024), d=2048,
            V=151936, dtype="bf16", hidden_std=1.0, w_std=0.02, rewards="bernoulli_beta",
            clip_eps=0.2),
    2: dict(name="qwen2.5-7b-head", B=16, n=32, m=8, T=2048, len_range=(256, 2048), d=3584,
            V=152064, dtype="bf16", hidden_std=1.0, w_std=0.02, rewards="correct_plus_format",
            clip_eps=0.2),
    3: dict(name="selector-stress", B=65536, n=256, m=64, T=None, len_range=None, d=None, V=None,
            dtype=None, rewards="bernoulli_noise_ties", clip_eps=None),
    4: dict(name="llama3-8b-head-ties", B=64, n=16, m=8, T=512, len_range=(64, 512), d=4096,
            V=128256, dtype="bf16", hidden_std=1.0, w_std=0.02, rewards="three_level",
            clip_eps=0.2),
}


def seed_for(cfg: int, stream: int = 0) -> int:
    """One seed per (config, purpose): rewards=0, lengths=1, tokens=2, hidden=3, W=4, noise=5."""
    return BASE_SEED + cfg + 1000 * stream


def _rng(cfg: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed_for(cfg, stream)))


def rewards(cfg: int, B: int | None = None, n: int | None = None) -> np.ndarray:
    """rewards[B, n] float32, drawn per the config's reward recipe."""
    c = CONFIGS[cfg]
    B = c["B"] if B is None else B
    n = c["n"] if n is None else n
    g = _rng(cfg, 0)
    kind = c["rewards"]
    if kind == "bernoulli_uniform":
        p = g.random(B)
        r = (g.random((B, n)) < p[:, None]).astype(np.float32)
    elif kind == "bernoulli_beta":
        p = g.beta(0.5, 0.5, B)
        r = (g.random((B, n)) < p[:, None]).astype(np.float32)
    elif kind == "correct_plus_format":
        p = g.random(B)
        correct = (g.random((B, n)) < p[:, None]).astype(np.float32)
        fmt = (g.random((B, n)) < 0.8).astype(np.float32)
        r = (correct + np.float32(0.1) * fmt).astype(np.float32)
    elif kind == "bernoulli_noise_ties":
        p = g.random(B)
        base = (g.random((B, n)) < p[:, None]).astype(np.float32)
        noise = g.normal(0.0, 0.1, (B, n)).astype(np.float32)
        r = (base + noise).astype(np.float32)
        flat = g.random(B) < 0.10            # about 10 % of groups: every rollout the same reward
        dyadic = g.random(B) < 0.5           # half of those 0/1, half a non-dyadic constant
        const = np.where(dyadic, (g.random(B) < 0.5).astype(np.float32),
                         (g.random(B).astype(np.float32) + g.normal(0, 0.1, B).astype(np.float32)))
        r[flat, :] = const[flat, None].astype(np.float32)
    elif kind == "three_level":
        r = (g.integers(0, 3, (B, n)).astype(np.float32) * np.float32(0.5)).astype(np.float32)
    else:
        raise ValueError(kind)
    return np.ascontiguousarray(r, dtype=np.float32)


def lengths(cfg: int, R: int | None = None, T: int | None = None) -> np.ndarray:
    """lengths[R] int32: valid (right-padded) completion length per kept rollout."""
    c = CONFIGS[cfg]
    R = c["B"] * c["m"] if R is None else R
    lo, hi = c["len_range"]
    if T is not None and T != c["T"]:
        lo = max(1, int(round(lo * T / c["T"])))
        hi = T
    g = _rng(cfg, 1)
    return g.integers(lo, hi + 1, R).astype(np.int32)


def tokens(cfg: int, R: int, T: int, V: int) -> np.ndarray:
    """tokens[R, T] int32 uniform over the vocabulary."""
    g = _rng(cfg, 2)
    return g.integers(0, V, (R, T)).astype(np.int32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 (exact)."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def dense(cfg: int, R: int, T: int, d: int, V: int):
    """hidden[R, T, d] and w_lm[V, d] as float32 arrays.

    For a bf16 config the values are already rounded to bf16, so widening the bf16 storage
    handed to the GPU reproduces exactly the float32 arrays handed to the oracle.
    """
    c = CONFIGS[cfg]
    gh, gw = _rng(cfg, 3), _rng(cfg, 4)
    h = gh.standard_normal((R, T, d), dtype=np.float32) * np.float32(c["hidden_std"])
    w = gw.standard_normal((V, d), dtype=np.float32) * np.float32(c["w_std"])
    if c["dtype"] == "bf16":
        h = bf16_bits_to_f32(f32_to_bf16_bits(h))
        w = bf16_bits_to_f32(f32_to_bf16_bits(w))
    return h, w


def old_logp_from(cur_logp: np.ndarray, cfg: int, sigma: float = 0.05) -> np.ndarray:
    """old_logp = current log-prob + N(0, sigma); the current log-prob is supplied by the caller."""
    g = _rng(cfg, 5)
    noise = g.normal(0.0, sigma, cur_logp.shape)
    return (np.asarray(cur_logp, dtype=np.float64) + noise).astype(np.float32)


def advantages_like(cfg: int, R: int) -> np.ndarray:
    """Stand-in advantages[R] float32 (zero-mean, unit-scale) for loss-only runs."""
    g = _rng(cfg, 6)
    return g.standard_normal(R).astype(np.float32)


def dense_torch(cfg: int, device, R: int | None = None, T: int | None = None,
                d: int | None = None, V: int | None = None):
    """Full-size hidden / w_lm generated on `device` with a seeded torch generator.

    Used where the tensors are too large to draw on the host in reasonable time.  Returns torch
    tensors in the config's storage dtype (bf16 or fp32).
    """
    import torch

    c = CONFIGS[cfg]
    R = c["B"] * c["m"] if R is None else R
    T = c["T"] if T is None else T
    d = c["d"] if d is None else d
    V = c["V"] if V is None else V
    dt = torch.bfloat16 if c["dtype"] == "bf16" else torch.float32
    g = torch.Generator(device=device)
    g.manual_seed(seed_for(cfg, 3))
    h = torch.empty((R, T, d), dtype=dt, device=device)
    rows = max(1, (1 << 26) // (T * d))
    for r0 in range(0, R, rows):
        r1 = min(R, r0 + rows)
        blk = torch.randn((r1 - r0, T, d), generator=g, device=device, dtype=torch.float32)
        h[r0:r1] = (blk * c["hidden_std"]).to(dt)
    g.manual_seed(seed_for(cfg, 4))
    w = torch.empty((V, d), dtype=dt, device=device)
    rows = max(1, (1 << 26) // d)
    for v0 in range(0, V, rows):
        v1 = min(V, v0 + rows)
        blk = torch.randn((v1 - v0, d), generator=g, device=device, dtype=torch.float32)
        w[v0:v1] = (blk * c["w_std"]).to(dt)
    return h, w
