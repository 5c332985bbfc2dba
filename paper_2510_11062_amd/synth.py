"""Seeded synthetic rollouts shaped like AT-GRPO training batches.

This module only draws random inputs (ids, lengths, rewards, hidden states, head weights,
and the raw random numbers a rollout engine would consume).  It contains none of the
method's arithmetic: no logits, no softmax, no advantages, no loss.  Both the GPU library's
callers and the CPU oracle's tests read their inputs from here, so the two sides see
identical bits.

Structure follows Alg. 1 of the paper: E environments x N agents x T turns, K sampled
candidates per (e, i, t); every candidate is one response (a token sequence).  Responses
are emitted in shuffled order so that nothing downstream may rely on input order.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional

import numpy as np
import torch

BASE_SEED = 251011062


@dataclass(frozen=True)
class RolloutConfig:
    name: str
    H: int
    V: int
    dtype: str            # "f32" or "bf16"
    n_heads: int          # M policies; agent i -> head i % M when M > 1
    E: int
    N: int
    T: int
    K: int
    len_kind: str         # "uniform" | "lognormal"
    len_lo: int
    len_hi: int
    padded: bool          # responses stored in fixed-length slots with a mask
    reward_kind: str      # "bernoulli" | "mixed" | "uniform" | "turn_bernoulli"
    forced_equal_groups: float  # count (>=1) or fraction (<1) of groups forced all-equal
    old_sigma: float      # std of (old_logp - current logp)
    eps_clip: float
    seed: int
    lognormal_sigma: float = 0.5
    drop_tail_frac: float = 0.0   # fraction of environments that terminate early

    @property
    def n_resp(self) -> int:
        return self.E * self.N * self.T * self.K


CONFIGS = {
    "C1": RolloutConfig("C1", 64, 512, "f32", 1, 4, 2, 2, 4, "uniform", 8, 32, False,
                        "bernoulli", 2, 0.05, 0.2, BASE_SEED + 1),
    "C2": RolloutConfig("C2", 2048, 151936, "bf16", 1, 16, 2, 4, 8, "uniform", 64, 512, True,
                        "mixed", 0.10, 0.1, 0.2, BASE_SEED + 2),
    "C3": RolloutConfig("C3", 4096, 151936, "bf16", 2, 32, 2, 3, 8, "uniform", 128, 1024, False,
                        "uniform", 0, 0.1, 0.2, BASE_SEED + 3),
    "C4": RolloutConfig("C4", 2048, 151936, "bf16", 1, 256, 2, 10, 4, "uniform", 32, 128, False,
                        "turn_bernoulli", 0, 0.1, 0.2, BASE_SEED + 4),
    "C5": RolloutConfig("C5", 4096, 151936, "bf16", 3, 64, 3, 4, 8, "lognormal", 1, 4096, False,
                        "mixed", 0, 0.2, 0.2, BASE_SEED + 5),
}


def mini(cfg: RolloutConfig, E: int, len_lo: int, len_hi: int, K: Optional[int] = None,
         V: Optional[int] = None, H: Optional[int] = None) -> RolloutConfig:
    """A small twin of a config: same heads, reward structure and layout, fewer/shorter responses."""
    return replace(cfg, name=cfg.name + "-mini", E=E, len_lo=len_lo, len_hi=len_hi,
                   K=cfg.K if K is None else K, V=cfg.V if V is None else V,
                   H=cfg.H if H is None else H,
                   len_kind="uniform" if cfg.len_kind == "uniform" else cfg.len_kind)


@dataclass
class RolloutStructure:
    """Host-side (numpy) description of one rollout batch; no floating-point tensors but rewards."""
    cfg: RolloutConfig
    env_id: np.ndarray        # int32 [R]
    agent_id: np.ndarray      # int32 [R]
    turn_id: np.ndarray       # int32 [R]
    sample_id: np.ndarray     # int32 [R]  candidate index c within its (e, i, t)
    reward: np.ndarray        # float32 [R]
    lengths: np.ndarray       # int64 [R]  response lengths in tokens
    cu_seqlens: np.ndarray    # int64 [R+1] row range of each response in the token arrays
    mask: Optional[np.ndarray]  # uint8 [n_tok] (padded layout) or None (packed: all ones)
    head_of_agent: np.ndarray   # int32 [N]
    n_tok: int                # rows of the token arrays (slots, padding included)
    n_valid: int              # response tokens


def make_structure(cfg: RolloutConfig) -> RolloutStructure:
    rng = np.random.Generator(np.random.PCG64(cfg.seed))
    E, N, T, K = cfg.E, cfg.N, cfg.T, cfg.K
    e, i, t, c = np.meshgrid(np.arange(E), np.arange(N), np.arange(T), np.arange(K), indexing="ij")
    e, i, t, c = (a.reshape(-1).astype(np.int32) for a in (e, i, t, c))

    # early termination: environments whose later turns never happened
    if cfg.drop_tail_frac > 0:
        stop = np.where(rng.random(E) < cfg.drop_tail_frac, rng.integers(1, max(T, 2), size=E), T)
        keep = t < stop[e]
        e, i, t, c = e[keep], i[keep], t[keep], c[keep]
    R = e.shape[0]

    # rewards, drawn group by group in canonical order
    gkey = (e.astype(np.int64) * N + i) * T + t
    groups, ginv = np.unique(gkey, return_inverse=True)
    G = groups.shape[0]
    u = rng.random(R)
    if cfg.reward_kind == "bernoulli":
        reward = (u < 0.5).astype(np.float32)
    elif cfg.reward_kind == "uniform":
        reward = u.astype(np.float32)
    elif cfg.reward_kind == "mixed":
        binary_group = rng.random(G) < 0.5
        reward = np.where(binary_group[ginv], (u < 0.5).astype(np.float32), u.astype(np.float32))
    elif cfg.reward_kind == "turn_bernoulli":
        p_t = 0.05 + 0.55 * t.astype(np.float64) / max(T - 1, 1)
        reward = (u < p_t).astype(np.float32)
    else:
        raise ValueError(cfg.reward_kind)
    reward = reward.astype(np.float32)
    n_forced = int(cfg.forced_equal_groups) if cfg.forced_equal_groups >= 1 \
        else int(round(cfg.forced_equal_groups * G))
    if n_forced > 0:
        forced = rng.choice(G, size=n_forced, replace=False)
        for g in forced:
            members = np.nonzero(ginv == g)[0]
            reward[members] = reward[members[0]]

    # response lengths
    if cfg.len_kind == "uniform":
        lengths = rng.integers(cfg.len_lo, cfg.len_hi + 1, size=R).astype(np.int64)
    elif cfg.len_kind == "lognormal":
        raw = np.exp(np.log(256.0) + cfg.lognormal_sigma * rng.standard_normal(R))
        lengths = np.clip(np.rint(raw), max(cfg.len_lo, 1), cfg.len_hi).astype(np.int64)
    else:
        raise ValueError(cfg.len_kind)

    # shuffle the response order
    order = rng.permutation(R)
    e, i, t, c, reward, lengths = (a[order] for a in (e, i, t, c, reward, lengths))

    if cfg.padded:
        Lmax = int(cfg.len_hi)
        cu = (np.arange(R + 1, dtype=np.int64) * Lmax)
        n_tok = R * Lmax
        mask = (np.arange(Lmax)[None, :] < lengths[:, None]).astype(np.uint8).reshape(-1)
    else:
        cu = np.zeros(R + 1, dtype=np.int64)
        cu[1:] = np.cumsum(lengths)
        n_tok = int(cu[-1])
        mask = None
    head_of_agent = (np.arange(N) % cfg.n_heads).astype(np.int32)
    return RolloutStructure(cfg, e, i, t, c, reward, lengths, cu, mask, head_of_agent,
                            n_tok, int(lengths.sum()))


def make_team_local_rewards(cfg: RolloutConfig, n_resp: int, levels: int = 8):
    """Team and local reward of every candidate, as a coder/tester-style workflow produces them:
    pass rates over `levels` unit tests, i.e. multiples of 1/levels in [0, 1] (so equal rewards are
    common).  Returns (r_team[R], r_loc[R]) as fp32; no arithmetic of the method happens here."""
    rng = np.random.default_rng(cfg.seed * 7 + 3)
    r_team = rng.integers(0, levels + 1, size=n_resp).astype(np.float32) / np.float32(levels)
    r_loc = rng.integers(0, levels + 1, size=n_resp).astype(np.float32) / np.float32(levels)
    return r_team, r_loc


def torch_dtype(cfg: RolloutConfig):
    return torch.float32 if cfg.dtype == "f32" else torch.bfloat16


def make_tensors(cfg: RolloutConfig, n_tok: int, device="cpu", w_std: float = 0.02,
                 rows_per_chunk: int = 1 << 16):
    """hidden [n_tok, H] ~ N(0, 1) and n_heads matrices W [V, H] ~ N(0, w_std), in cfg.dtype."""
    gen = torch.Generator(device=device)
    gen.manual_seed(cfg.seed * 7 + 11)
    dt = torch_dtype(cfg)
    hidden = torch.empty((n_tok, cfg.H), dtype=dt, device=device)
    for r0 in range(0, n_tok, rows_per_chunk):
        r1 = min(n_tok, r0 + rows_per_chunk)
        hidden[r0:r1] = torch.randn((r1 - r0, cfg.H), generator=gen, device=device).to(dt)
    W = []
    for _ in range(cfg.n_heads):
        w = torch.empty((cfg.V, cfg.H), dtype=dt, device=device)
        for r0 in range(0, cfg.V, rows_per_chunk):
            r1 = min(cfg.V, r0 + rows_per_chunk)
            w[r0:r1] = (torch.randn((r1 - r0, cfg.H), generator=gen, device=device) * w_std).to(dt)
        W.append(w)
    return hidden, W


def make_rollout_randoms(cfg: RolloutConfig, n_tok: int, device="cpu"):
    """Raw random numbers a rollout engine consumes: one uniform per token (to draw the sampled
    token by inverse CDF) and one N(0, old_sigma) deviate per token (behaviour-policy drift)."""
    gen = torch.Generator(device=device)
    gen.manual_seed(cfg.seed * 13 + 5)
    u = torch.rand((n_tok,), generator=gen, device=device, dtype=torch.float64)
    noise = torch.randn((n_tok,), generator=gen, device=device, dtype=torch.float32) * cfg.old_sigma
    return u, noise
