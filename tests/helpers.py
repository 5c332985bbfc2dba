"""Shared test plumbing: turns seeded synthetic rollouts into oracle-side (numpy) inputs.

The "rollout stand-in" here plays the part of the inference engine that, in the paper's
system, produces the sampled tokens and the behaviour-policy log-probs: on oracle-sized
cases it is driven by the oracle itself (fp64), so no value handed to the oracle ever comes
from the GPU library.
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import at_grpo_oracle as orc
from paper_2510_11062_amd import synth


def to_np(x):
    if x is None:
        return None
    if isinstance(x, torch.Tensor):
        x = x.detach().cpu()
        if x.dtype == torch.bfloat16:
            x = x.float()
        return x.numpy()
    return np.asarray(x)


def oracle_rollout_standin(hidden, W_list, mask, head_of_tok, u, noise):
    """Sample y_t ~ softmax(h_t W^T) by inverse CDF with the given uniforms, and set
    old_logp = logp(y_t) + noise.  Rows that are masked out get token 0 and old_logp 0."""
    n_tok = hidden.shape[0]
    m = np.ones(n_tok, dtype=bool) if mask is None else (mask != 0)
    token_id = np.zeros(n_tok, dtype=np.int32)
    old_logp = np.zeros(n_tok, dtype=np.float32)
    for k, W in enumerate(W_list):
        rows = np.nonzero(m & (head_of_tok == k))[0]
        if rows.size == 0:
            continue
        z = orc.head_logits(hidden[rows], W)
        z = z - z.max(axis=1, keepdims=True)
        p = np.exp(z)
        p /= p.sum(axis=1, keepdims=True)
        cdf = np.cumsum(p, axis=1)
        y = (cdf < u[rows][:, None]).sum(axis=1)
        y = np.minimum(y, W.shape[0] - 1)
        token_id[rows] = y.astype(np.int32)
        logp = np.log(p[np.arange(rows.size), y])
        old_logp[rows] = (logp + noise[rows]).astype(np.float32)
    return token_id, old_logp


class Case:
    """One fully specified batch, host side (numpy), plus the torch tensors it came from."""


def build_case(cfg: synth.RolloutConfig, device="cpu") -> Case:
    st = synth.make_structure(cfg)
    hidden_t, W_t = synth.make_tensors(cfg, st.n_tok, device=device)
    u_t, noise_t = synth.make_rollout_randoms(cfg, st.n_tok, device=device)
    c = Case()
    c.cfg, c.st = cfg, st
    c.hidden_t, c.W_t = hidden_t, W_t
    c.hidden = to_np(hidden_t)
    c.W = [to_np(w) for w in W_t]
    c.u, c.noise = to_np(u_t), to_np(noise_t)
    c.resp_of_tok, c.head_of_tok = orc.token_heads(st.n_tok, st.cu_seqlens, st.agent_id,
                                                   st.head_of_agent if cfg.n_heads > 1 else None)
    c.token_id, c.old_logp = oracle_rollout_standin(c.hidden, c.W, st.mask, c.head_of_tok, c.u, c.noise)
    key = orc.group_key(st.env_id, st.agent_id, st.turn_id, cfg.N, cfg.T)
    c.group_id, c.n_groups, c.seg_offsets, c.perm = orc.group_segments(key)
    c.adv64, c.gmean, c.gstd = orc.group_advantage(st.reward, c.group_id, c.n_groups)
    c.adv = c.adv64.astype(np.float32)
    return c


def oracle_fwd(c: Case, agg="token_mean", old_logp=None, adv=None):
    cfg, st = c.cfg, c.st
    return orc.policy_loss_fwd(c.hidden, c.W, c.token_id, st.mask, st.cu_seqlens,
                               st.agent_id, st.head_of_agent if cfg.n_heads > 1 else None,
                               c.old_logp if old_logp is None else old_logp,
                               c.adv if adv is None else adv, cfg.eps_clip, cfg.eps_clip, agg)


def oracle_bwd(c: Case, agg="token_mean", grad_loss=None):
    cfg, st = c.cfg, c.st
    return orc.policy_loss_bwd(c.hidden, c.W, c.token_id, st.mask, st.cu_seqlens,
                               st.agent_id, st.head_of_agent if cfg.n_heads > 1 else None,
                               c.old_logp, c.adv, cfg.eps_clip, cfg.eps_clip, agg, grad_loss)


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return np.linalg.norm(a - b) / (den if den > 0 else 1.0)


# ------------------------------------------------------------------------------------------------
# Gradient comparison.  A Frobenius ratio over a whole matrix hides one wrong row or one wrong tile
# edge, so gradients are compared row by row and element by element:
#   row check      max_r ||got_r - ref_r|| / max(||ref_r||, floor)          <= tol
#   element check  |got - ref| <= tol * |ref| + tol * rms(ref_r)             for every element
# The element bound carries the row's root-mean-square because an element that is the sum of
# cancelling terms is only accurate relative to the terms, not to itself.  floor keeps rows that are
# numerically zero in the reference (far below the typical row) from dividing rounding noise by ~0.
# ------------------------------------------------------------------------------------------------
def grad_errors(got, ref, floor_frac=1e-6):
    """Returns (worst row error, worst element excess, row index of the worst row)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if got.ndim == 1:
        got, ref = got[None, :], ref[None, :]
    rn = np.linalg.norm(ref, axis=1)
    floor = floor_frac * (rn.max() if rn.size else 0.0)
    row_err = np.linalg.norm(got - ref, axis=1) / np.maximum(np.maximum(rn, floor), 1e-300)
    rms = rn / np.sqrt(ref.shape[1])
    # excess[i, j] = |d| / (|ref| + rms_row): compared against tol by the caller
    den = np.abs(ref) + np.maximum(rms, floor / np.sqrt(ref.shape[1]))[:, None]
    elem = np.abs(got - ref) / np.maximum(den, 1e-300)
    worst = int(np.argmax(row_err)) if row_err.size else -1
    return (float(row_err.max()) if row_err.size else 0.0, float(elem.max()) if elem.size else 0.0, worst)


def assert_grad_close(got, ref, tol, what, fro_tol=None):
    """Row-wise and element-wise gradient parity (see grad_errors), plus the Frobenius bound."""
    row_err, elem_err, worst = grad_errors(got, ref)
    fro = rel_fro(got, ref)
    assert np.all(np.isfinite(np.asarray(got, dtype=np.float64))), f"{what}: non-finite values"
    assert row_err <= tol, f"{what}: row {worst} off by {row_err:.3e} (tol {tol})"
    assert elem_err <= tol, f"{what}: an element exceeds tol*(|ref| + rms of its row) by factor {elem_err / tol:.2f}"
    assert fro <= (tol if fro_tol is None else fro_tol), f"{what}: Frobenius error {fro:.3e}"
    return row_err, elem_err, fro
