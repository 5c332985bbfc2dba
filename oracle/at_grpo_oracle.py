"""Plain fp64 CPU oracle for the AT-GRPO policy-loss path.

TEST INFRASTRUCTURE ONLY.  This module is the slow, obviously-correct statement of
what the GPU library computes.  It is imported by the tests, by the smoke check and
by the CPU-baseline leg of the benchmark, and by nothing else; the product path never
routes through it.  It shares no code with the HIP kernels and does not import the
package that wraps them.

Everything is written straight from the paper's definitions, in fp64, with numpy.
Library primitives (matmul, sort, exp/log) serve as single steps; nothing is blocked,
fused or reordered.  Inputs that live in bf16/fp32 on the device are widened exactly to
fp64 here and are never re-rounded.

Paper passages followed (arXiv 2510.11062):
  * group key  g = hash(e, i, t)                      -- Alg. 1 (Phase 1), Sec. 4.1
                                                        "Agent- and Turn-wise Grouping"
  * the groupings it is compared with                  -- Sec. 4.1 / Fig. 3 (parallel sampling:
                                                        groups of one after the first turn),
                                                        Sec. 5.3 (trajectory-level groups)
  * group-relative advantage                           -- Sec. 3 "Group-based RL", Eq. (1)
  * per-model batch B_m and clipped surrogate          -- Sec. 3, Eq. (2)
  * response-token credit (reward mask)                -- Sec. 4.1, first paragraph
  * pi_theta(token) from the LM head                   -- implicit in r(theta) below Eq. (2)
  * mixed team / local reward                          -- Sec. 4.1 "Agent-wise Credit
                                                        Assignment", Eq. (3)
  * greedy choice of the executed candidate            -- Alg. 1 / Sec. 4.1 "Tree-structured
                                                        Sampling"
  * update of policy m: gradient clipping, Adam        -- Alg. 1 Phase 2; App. C.1 (clip 1.0,
                                                        lr 1e-6, weight decay 0.01)

Readings taken where the paper is silent (all are parameters):
  * F_norm in Eq. (1) is the standard deviation; population (ddof=0) by default; the
    quotient is (R - mean) / (std + eps_std).  A group whose rewards are all the same
    fp32 value (including a singleton group) gets advantage exactly 0.
  * the importance ratio is per token, r_t = exp(logp_t - old_logp_t), and the expectation
    in Eq. (2) is a masked token mean over the per-model batch ("token_mean"), or, read
    literally, a mean over responses of per-response token means ("seq_mean_token_mean").
  * clip flags are decided in log space on the fp32 difference d = fp32(logp) - fp32(old):
    low  <=> d < fp32(log1p(-eps_low)),  high <=> d > fp32(log1p(eps_high)).
"""
from __future__ import annotations

import numpy as np

CLIP_LOW = 1    # bit 0: ratio below 1 - eps_low
CLIP_HIGH = 2   # bit 1: ratio above 1 + eps_high
CLIP_ZERO_GRAD = 4  # bit 2: the clipped branch is the one min() selects (no gradient)


# --------------------------------------------------------------------------------------
# S1: group keys and segments  (Alg. 1, "Define group key g <- hash(e, i, t)")
# --------------------------------------------------------------------------------------
def group_key(env_id, agent_id, turn_id, n_agent: int, n_turn: int) -> np.ndarray:
    """Injective packing of (e, i, t): key = (e * n_agent + i) * n_turn + t.

    Any injective hash gives the same partition of the responses; this one also fixes a
    canonical ORDER of the groups (ascending key) so integer outputs are comparable.
    """
    e = np.asarray(env_id, dtype=np.int64)
    i = np.asarray(agent_id, dtype=np.int64)
    t = np.asarray(turn_id, dtype=np.int64)
    return (e * int(n_agent) + i) * int(n_turn) + t


def group_key_by(env_id, agent_id, turn_id, sample_id, n_agent: int, n_turn: int, n_sample: int,
                 group_by: str = "agent_turn") -> np.ndarray:
    """Keys of the groupings the paper sets its own against.

    "agent_turn"  (e, i, t): AT-GRPO (Alg. 1), the same key as group_key.
    "trajectory"  e alone: every candidate of a task in one group, whichever agent and turn produced
                  it (GRPO applied to the multi-agent system as a whole, Sec. 5.3).
    "parallel"    K trajectories sampled in parallel from the task's start (Sec. 4.1, Fig. 3): the
                  candidates share a state only at the first turn, so the key is (e, i, 0) at t = 0 and
                  (e, i, t, c) with the candidate index c afterwards: groups of one.
    Keys are packed so that ascending key is the lexicographic order of the tuple.
    """
    e = np.asarray(env_id, dtype=np.int64)
    i = np.asarray(agent_id, dtype=np.int64)
    t = np.asarray(turn_id, dtype=np.int64)
    if group_by == "agent_turn":
        return (e * int(n_agent) + i) * int(n_turn) + t
    if group_by == "trajectory":
        return e.copy()
    if group_by == "parallel":
        c = np.asarray(sample_id, dtype=np.int64)
        return ((e * int(n_agent) + i) * int(n_turn) + t) * int(n_sample) + np.where(t > 0, c, 0)
    raise ValueError(group_by)


def group_segments(key: np.ndarray):
    """Dense group numbering, CSR offsets and the stable permutation that sorts by key.

    Returns (group_id[R], n_groups, seg_offsets[G+1], perm[R]).  Keys that do not occur
    (an environment that terminated early) produce no group.
    """
    key = np.asarray(key, dtype=np.int64)
    present = np.unique(key)                      # ascending distinct keys
    group_id = np.searchsorted(present, key).astype(np.int32)
    n_groups = int(present.shape[0])
    counts = np.bincount(group_id, minlength=n_groups)
    seg_offsets = np.zeros(n_groups + 1, dtype=np.int32)
    seg_offsets[1:] = np.cumsum(counts)
    perm = np.argsort(key, kind="stable").astype(np.int32)
    return group_id, n_groups, seg_offsets, perm


# --------------------------------------------------------------------------------------
# S2: group-relative advantage  (Eq. 1)
# --------------------------------------------------------------------------------------
def group_advantage(reward, group_id, n_groups: int, eps_std: float = 1e-6, ddof: int = 0,
                    norm: str = "std"):
    """A = (R - mean_g R) / F_norm, per group.  Returns (adv[R], mean[G], std[G]) in fp64.

    norm="std":  F_norm = std + eps_std (std with the given ddof; 0 if n_g - ddof <= 0)
    norm="none": F_norm = 1
    Groups whose rewards are all bit-identical fp32 values get A = 0 exactly.
    """
    r32 = np.asarray(reward, dtype=np.float32)
    r = r32.astype(np.float64)
    gid = np.asarray(group_id, dtype=np.int64)
    adv = np.zeros(r.shape[0], dtype=np.float64)
    mean = np.zeros(n_groups, dtype=np.float64)
    std = np.zeros(n_groups, dtype=np.float64)
    for g in range(n_groups):
        members = np.nonzero(gid == g)[0]
        x = r[members]
        n = x.shape[0]
        mu = x.sum() / n
        dev = x - mu
        denom = n - ddof
        sigma = np.sqrt((dev * dev).sum() / denom) if denom > 0 else 0.0
        mean[g] = mu
        std[g] = sigma
        if np.all(r32[members] == r32[members[0]]):
            mean[g] = x[0]
            std[g] = 0.0
            continue                               # adv stays exactly 0
        if norm == "std":
            adv[members] = dev / (sigma + eps_std)
        elif norm == "none":
            adv[members] = dev
        else:
            raise ValueError(norm)
    return adv, mean, std


# --------------------------------------------------------------------------------------
# Before S2: agent-wise credit assignment (Eq. 3) and the tree-sampling choice (Alg. 1)
# --------------------------------------------------------------------------------------
def mix_rewards(r_team, r_loc, alpha: float) -> np.ndarray:
    """Eq. (3): r = alpha * r_team + r_loc, per candidate.

    The result is the fp32 reward array that Eq. (1) consumes.  It decides integers further
    down (which group counts as all-equal, which candidate is the arg max), so it is formed
    in the precision the rewards live in: one fp32 multiplication, then one fp32 addition.
    """
    a = np.float32(alpha)
    team = np.asarray(r_team, dtype=np.float32)
    loc = np.asarray(r_loc, dtype=np.float32)
    prod = (a * team).astype(np.float32)
    return (prod + loc).astype(np.float32)


def select_candidates(reward, group_id, n_groups: int) -> np.ndarray:
    """Alg. 1, tree-structured sampling: c* = arg max_c r^(c) inside every group.

    Returns best[G]: the response index of the candidate with the largest reward in each
    group; among equal rewards the candidate that comes first (lowest response index).
    """
    r32 = np.asarray(reward, dtype=np.float32)
    gid = np.asarray(group_id, dtype=np.int64)
    best = np.full(n_groups, -1, dtype=np.int32)
    for g in range(n_groups):
        members = np.nonzero(gid == g)[0]          # ascending response index
        top = members[0]
        for m in members[1:]:
            if r32[m] > r32[top]:
                top = m
        best[g] = top
    return best


# --------------------------------------------------------------------------------------
# S3 + S4: LM-head logits, log-softmax, gather of the sampled token
# --------------------------------------------------------------------------------------
def head_logits(hidden, W) -> np.ndarray:
    """z[t, v] = sum_h hidden[t, h] * W[v, h]   (fp64)."""
    h = np.asarray(hidden, dtype=np.float64)
    w = np.asarray(W, dtype=np.float64)
    return h @ w.T


def token_logprob_single(hidden, W, token_id):
    """log pi(y_t) and log-sum-exp for every row of `hidden` under ONE head.

    Returns (logp[n], lse[n]).
    """
    z = head_logits(hidden, W)
    y = np.asarray(token_id, dtype=np.int64)
    mx = z.max(axis=1)
    lse = mx + np.log(np.exp(z - mx[:, None]).sum(axis=1))
    logp = z[np.arange(z.shape[0]), y] - lse
    return logp, lse


def token_heads(n_tok: int, cu_seqlens, resp_agent=None, head_of_agent=None):
    """resp_of_tok[t] and head_of_tok[t]: the response owning row t and sigma(agent)."""
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    n_resp = cu.shape[0] - 1
    resp_of_tok = np.full(n_tok, -1, dtype=np.int64)
    for r in range(n_resp):
        resp_of_tok[cu[r]:cu[r + 1]] = r
    if resp_agent is None or head_of_agent is None:
        head_of_tok = np.zeros(n_tok, dtype=np.int64)
    else:
        head_of_resp = np.asarray(head_of_agent, dtype=np.int64)[np.asarray(resp_agent, dtype=np.int64)]
        head_of_tok = np.where(resp_of_tok >= 0, head_of_resp[np.maximum(resp_of_tok, 0)], 0)
    head_of_tok = np.where(resp_of_tok >= 0, head_of_tok, -1)
    return resp_of_tok, head_of_tok


def token_logprob(hidden, W_list, token_id, mask, head_of_tok):
    """logp, lse for every row; rows with mask 0 (or owned by no response) give 0, 0."""
    n_tok = np.asarray(hidden).shape[0]
    m = np.ones(n_tok, dtype=bool) if mask is None else (np.asarray(mask) != 0)
    logp = np.zeros(n_tok, dtype=np.float64)
    lse = np.zeros(n_tok, dtype=np.float64)
    y = np.asarray(token_id)
    for k, W in enumerate(W_list):
        rows = np.nonzero(m & (head_of_tok == k))[0]
        if rows.size == 0:
            continue
        lp, ls = token_logprob_single(np.asarray(hidden)[rows], W, y[rows])
        logp[rows] = lp
        lse[rows] = ls
    return logp, lse


def token_entropy_single(hidden, W):
    """Entropy of the policy's next-token distribution at every row, H = - sum_v p_v ln p_v with
    p = softmax(hidden W^T), under ONE head (a monitor: the paper's entropy coefficient is 0)."""
    z = head_logits(hidden, W)
    z = z - z.max(axis=1, keepdims=True)
    e = np.exp(z)
    p = e / e.sum(axis=1, keepdims=True)
    logp = np.where(p > 0, np.log(np.where(p > 0, p, 1.0)), 0.0)
    return -(p * logp).sum(axis=1)


def token_entropy(hidden, W_list, mask, head_of_tok):
    """Entropy for every row; rows with mask 0 (or owned by no response) give 0."""
    n_tok = np.asarray(hidden).shape[0]
    m = np.ones(n_tok, dtype=bool) if mask is None else (np.asarray(mask) != 0)
    ent = np.zeros(n_tok, dtype=np.float64)
    for k, W in enumerate(W_list):
        rows = np.nonzero(m & (head_of_tok == k))[0]
        if rows.size:
            ent[rows] = token_entropy_single(np.asarray(hidden)[rows], W)
    return ent


# --------------------------------------------------------------------------------------
# S5 + S6: clipped surrogate and masked averaging  (Eq. 2)
# --------------------------------------------------------------------------------------
def clip_thresholds(eps_low: float, eps_high: float):
    """fp32 log-space thresholds lo = log1p(-eps_low), hi = log1p(eps_high)."""
    el = float(np.float32(eps_low))
    eh = float(np.float32(eps_high))
    return np.float32(np.log1p(-el)), np.float32(np.log1p(eh))


def token_weights(mask, head_of_tok, resp_of_tok, n_heads: int, agg: str = "token_mean"):
    """w_t such that loss_m = - sum_t w_t * l_t, plus n_valid[m].

    token_mean:           w_t = mask_t / (number of masked-in tokens routed to head m)
    seq_mean_token_mean:  w_t = mask_t / (R_m * len_r), len_r = masked-in tokens of the
                          response, R_m = responses of head m with len_r > 0
    """
    n_tok = head_of_tok.shape[0]
    m = np.ones(n_tok, dtype=bool) if mask is None else (np.asarray(mask) != 0)
    m = m & (head_of_tok >= 0)
    w = np.zeros(n_tok, dtype=np.float64)
    n_valid = np.zeros(n_heads, dtype=np.int64)
    for k in range(n_heads):
        sel = m & (head_of_tok == k)
        n_valid[k] = int(sel.sum())
        if n_valid[k] == 0:
            continue
        if agg == "token_mean":
            w[sel] = 1.0 / n_valid[k]
        elif agg == "seq_mean_token_mean":
            resp = resp_of_tok[sel]
            ids, lens = np.unique(resp, return_counts=True)
            len_of = dict(zip(ids.tolist(), lens.tolist()))
            w[sel] = np.array([1.0 / (ids.shape[0] * len_of[int(r)]) for r in resp])
        else:
            raise ValueError(agg)
    return w, n_valid


def surrogate_terms(logp, old_logp, adv_tok, eps_low: float, eps_high: float):
    """Per-token pieces of Eq. (2).

    Returns (l[n], ratio[n], clip_mask[n] uint8, sel[n] bool) where
      d     = fp32(logp) - fp32(old_logp)               (one fp32 subtraction)
      ratio = exp(d)
      l     = min(ratio * A, clip(ratio, 1 - eps_low, 1 + eps_high) * A)
      clip_mask bits: CLIP_LOW (d < lo), CLIP_HIGH (d > hi), CLIP_ZERO_GRAD
      sel   = the unclipped branch is the one min() takes (ties -> unclipped); d l / d logp
              is ratio * A where sel, 0 elsewhere.
    """
    lo32, hi32 = clip_thresholds(eps_low, eps_high)
    d32 = np.asarray(logp, dtype=np.float64).astype(np.float32) - np.asarray(old_logp, dtype=np.float32)
    d = d32.astype(np.float64)
    A = np.asarray(adv_tok, dtype=np.float64)
    ratio = np.exp(d)
    el = float(np.float32(eps_low))
    eh = float(np.float32(eps_high))
    unclipped = ratio * A
    clipped = np.clip(ratio, 1.0 - el, 1.0 + eh) * A
    l = np.minimum(unclipped, clipped)
    low = d32 < lo32
    high = d32 > hi32
    zero_grad = (high & (A > 0)) | (low & (A < 0))
    clip_mask = (low.astype(np.uint8) * CLIP_LOW) | (high.astype(np.uint8) * CLIP_HIGH) \
        | (zero_grad.astype(np.uint8) * CLIP_ZERO_GRAD)
    sel = ~zero_grad
    return l, ratio, clip_mask, sel


def policy_loss_from_logp(logp, old_logp, adv, mask, head_of_tok, resp_of_tok, n_heads: int,
                          eps_low: float, eps_high: float, agg: str = "token_mean"):
    """S5 + S6 given log-probs.  Returns (loss[M], clip_mask[n], n_valid[M], w[n], ratio, sel)."""
    n_tok = head_of_tok.shape[0]
    w, n_valid = token_weights(mask, head_of_tok, resp_of_tok, n_heads, agg)
    adv64 = np.asarray(adv, dtype=np.float32).astype(np.float64)
    adv_tok = np.where(resp_of_tok >= 0, adv64[np.maximum(resp_of_tok, 0)], 0.0)
    l, ratio, clip_mask, sel = surrogate_terms(logp, old_logp, adv_tok, eps_low, eps_high)
    valid = w > 0
    clip_mask = np.where(valid, clip_mask, 0).astype(np.uint8)
    loss = np.zeros(n_heads, dtype=np.float64)
    for k in range(n_heads):
        rows = valid & (head_of_tok == k)
        loss[k] = -(w[rows] * l[rows]).sum()
    return loss, clip_mask, n_valid, w, ratio, sel, adv_tok


def surrogate_diagnostics(logp, old_logp, adv, mask, head_of_tok, resp_of_tok, n_heads: int,
                          eps_low: float, eps_high: float):
    """Training diagnostics of Eq. (2)'s pieces, per policy, over its participating tokens:

      counts[m] = (n, n_low, n_high, n_zero_grad): tokens, tokens with ratio below 1 - eps_low,
                  above 1 + eps_high, and on the clipped branch (no gradient)
      kl[m]     = mean of ratio - 1 - d: the non-negative sample estimate of KL(pi_old || pi_theta)
                  from tokens drawn under pi_old (d = log ratio)
      ratio[m]  = mean importance ratio
    The paper reports none of these (its entropy coefficient is 0 and Eq. 2 has no KL term); they
    are the usual monitors of a clipped-ratio update.  d is the fp32 difference the clip flags use.
    """
    w, n_valid = token_weights(mask, head_of_tok, resp_of_tok, n_heads, "token_mean")
    adv64 = np.asarray(adv, dtype=np.float32).astype(np.float64)
    adv_tok = np.where(resp_of_tok >= 0, adv64[np.maximum(resp_of_tok, 0)], 0.0)
    _, ratio, clip_mask, _ = surrogate_terms(logp, old_logp, adv_tok, eps_low, eps_high)
    d = (np.asarray(logp, dtype=np.float64).astype(np.float32) - np.asarray(old_logp, dtype=np.float32)).astype(np.float64)
    counts = np.zeros((n_heads, 4), dtype=np.int64)
    kl = np.zeros(n_heads, dtype=np.float64)
    mean_ratio = np.zeros(n_heads, dtype=np.float64)
    for k in range(n_heads):
        rows = (w > 0) & (head_of_tok == k)
        n = int(rows.sum())
        counts[k] = (n, int(((clip_mask[rows] & CLIP_LOW) != 0).sum()), int(((clip_mask[rows] & CLIP_HIGH) != 0).sum()),
                     int(((clip_mask[rows] & CLIP_ZERO_GRAD) != 0).sum()))
        if n > 0:
            kl[k] = (ratio[rows] - 1.0 - d[rows]).sum() / n
            mean_ratio[k] = ratio[rows].sum() / n
    return counts, kl, mean_ratio


def policy_loss_fwd(hidden, W_list, token_id, mask, cu_seqlens, resp_agent, head_of_agent,
                    old_logp, adv, eps_low: float, eps_high: float, agg: str = "token_mean"):
    """S3..S6.  Returns dict(loss, logp, lse, clip_mask, n_valid)."""
    n_tok = np.asarray(hidden).shape[0]
    resp_of_tok, head_of_tok = token_heads(n_tok, cu_seqlens, resp_agent, head_of_agent)
    logp, lse = token_logprob(hidden, W_list, token_id, mask, head_of_tok)
    loss, clip_mask, n_valid, w, ratio, sel, adv_tok = policy_loss_from_logp(
        logp, old_logp, adv, mask, head_of_tok, resp_of_tok, len(W_list), eps_low, eps_high, agg)
    return dict(loss=loss, logp=logp, lse=lse, clip_mask=clip_mask, n_valid=n_valid,
                w=w, ratio=ratio, sel=sel, adv_tok=adv_tok,
                resp_of_tok=resp_of_tok, head_of_tok=head_of_tok)


# --------------------------------------------------------------------------------------
# S7 + S8: backward
# --------------------------------------------------------------------------------------
def logprob_coefficient(w, adv_tok, ratio, sel, head_of_tok, grad_loss=None):
    """g_t = d loss_m / d logp_t = - w_t * A_t * ratio_t * [unclipped branch] * grad_loss_m."""
    g = -w * adv_tok * ratio * sel.astype(np.float64)
    if grad_loss is not None:
        gl = np.asarray(grad_loss, dtype=np.float64)
        g = g * np.where(head_of_tok >= 0, gl[np.maximum(head_of_tok, 0)], 0.0)
    return g


def head_backward_single(hidden, W, token_id, g):
    """Gradients of sum_t g_t * logp_t w.r.t. hidden rows and W, for ONE head.

    dZ[t, v]      = g_t * (1[v = y_t] - softmax(z_t)[v])
    dHidden[t, :] = sum_v dZ[t, v] * W[v, :]
    dW[v, :]      = sum_t dZ[t, v] * hidden[t, :]
    """
    h = np.asarray(hidden, dtype=np.float64)
    w = np.asarray(W, dtype=np.float64)
    y = np.asarray(token_id, dtype=np.int64)
    z = h @ w.T
    mx = z.max(axis=1, keepdims=True)
    e = np.exp(z - mx)
    p = e / e.sum(axis=1, keepdims=True)
    dZ = -p
    dZ[np.arange(z.shape[0]), y] += 1.0
    dZ *= np.asarray(g, dtype=np.float64)[:, None]
    return dZ @ w, dZ.T @ h


def head_backward_dw_rows(hidden, W_rows, vocab_ids, token_id, g, lse):
    """Selected rows of dW for ONE head, from the definition, given the log-sum-exp of every token:

        dW[v, :] = sum_t g_t * (1[y_t = v] - exp(<hidden[t], W[v]> - lse_t)) * hidden[t, :]

    hidden [n, H] are the head's rows, W_rows [len(vocab_ids), H] the head's weight rows W[vocab_ids],
    g [n] the coefficients, lse [n] the log-sum-exp over the WHOLE vocabulary of each row (an input:
    a row of dW needs only that one column of the logits).  Costs O(n * H) per requested row, which
    is what makes single rows of a full-size gradient checkable.  Returns [len(vocab_ids), H] fp64.
    """
    h = np.asarray(hidden, dtype=np.float64)
    w = np.asarray(W_rows, dtype=np.float64)
    v = np.asarray(vocab_ids, dtype=np.int64)
    y = np.asarray(token_id, dtype=np.int64)
    gg = np.asarray(g, dtype=np.float64)
    ls = np.asarray(lse, dtype=np.float64)
    z = h @ w.T                                            # [n, len(v)]: the requested logit columns
    dZ = -np.exp(z - ls[:, None])
    dZ += (y[:, None] == v[None, :]).astype(np.float64)
    dZ *= gg[:, None]
    return dZ.T @ h


def policy_loss_bwd(hidden, W_list, token_id, mask, cu_seqlens, resp_agent, head_of_agent,
                    old_logp, adv, eps_low: float, eps_high: float, agg: str = "token_mean",
                    grad_loss=None):
    """S7 + S8.  Returns dict(d_hidden[n_tok, H], dW[list of [V, H]], g[n_tok])."""
    fwd = policy_loss_fwd(hidden, W_list, token_id, mask, cu_seqlens, resp_agent, head_of_agent,
                          old_logp, adv, eps_low, eps_high, agg)
    g = logprob_coefficient(fwd["w"], fwd["adv_tok"], fwd["ratio"], fwd["sel"],
                            fwd["head_of_tok"], grad_loss)
    hid = np.asarray(hidden)
    d_hidden = np.zeros(hid.shape, dtype=np.float64)
    dW = []
    y = np.asarray(token_id)
    for k, W in enumerate(W_list):
        rows = np.nonzero((fwd["w"] > 0) & (fwd["head_of_tok"] == k))[0]
        if rows.size == 0:
            dW.append(np.zeros(np.asarray(W).shape, dtype=np.float64))
            continue
        dh, dw = head_backward_single(hid[rows], W, y[rows], g[rows])
        d_hidden[rows] = dh
        dW.append(dw)
    out = dict(fwd)
    out.update(d_hidden=d_hidden, dW=dW, g=g)
    return out


# --------------------------------------------------------------------------------------
# After the path: the update of the head (Alg. 1 Phase 2 "update policy m"; App. C.1)
# --------------------------------------------------------------------------------------
def global_grad_norm(grads) -> float:
    """L2 norm over all the gradient arrays taken together (what "gradient clipping at 1.0"
    of App. C.1 measures)."""
    total = 0.0
    for g in grads:
        g = np.asarray(g, dtype=np.float64)
        total += float((g * g).sum())
    return float(np.sqrt(total))


def clip_coefficient(norm: float, max_norm: float) -> float:
    """Factor every gradient is multiplied by: max_norm / (norm + 1e-6), never above 1."""
    return min(1.0, max_norm / (norm + 1e-6))


def adam_step(w, g, m, v, step: int, lr: float = 1e-6, beta1: float = 0.9, beta2: float = 0.999,
              eps: float = 1e-8, weight_decay: float = 0.01, decoupled: bool = True):
    """One Adam step on fp64 arrays; returns (w, m, v) after the step.  step counts from 1.

    m <- beta1 m + (1 - beta1) g,  v <- beta2 v + (1 - beta2) g^2,
    w <- w - lr * (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps)
    Weight decay (App. C.1 gives the value, not the form):
      decoupled: w is first scaled by (1 - lr * weight_decay)            (default reading)
      coupled:   g <- g + weight_decay * w before the moments (L2 penalty)
    """
    w = np.asarray(w, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    m = np.asarray(m, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    if decoupled:
        w = w * (1.0 - lr * weight_decay)
    else:
        g = g + weight_decay * w
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** step)
    v_hat = v / (1.0 - beta2 ** step)
    w = w - lr * m_hat / (np.sqrt(v_hat) + eps)
    return w, m, v


def head_update(W_list, dW_list, m_list, v_list, step: int, max_grad_norm: float = 1.0, **adam):
    """Clip the gradients of all heads by their joint norm, then one Adam step per head.

    Returns dict(W=[...], m=[...], v=[...], grad_norm=float) in fp64 (the norm is the one before
    clipping)."""
    norm = global_grad_norm(dW_list)
    c = clip_coefficient(norm, max_grad_norm) if max_grad_norm > 0 else 1.0
    Ws, ms, vs = [], [], []
    for w, g, m, v in zip(W_list, dW_list, m_list, v_list):
        w2, m2, v2 = adam_step(w, np.asarray(g, dtype=np.float64) * c, m, v, step, **adam)
        Ws.append(w2)
        ms.append(m2)
        vs.append(v2)
    return dict(W=Ws, m=ms, v=vs, grad_norm=norm)
