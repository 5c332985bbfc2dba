"""Stand-in for the rollout engine at sizes the CPU oracle cannot cover.

In the paper's system the sampled tokens and the behaviour-policy log-probs (pi_theta_old in
Eq. 2) come from a separate inference engine, not from the training step.  For synthetic
workloads this module plays that engine with stock torch ops: it draws y_t from softmax(h_t W^T)
by inverse CDF and returns old_logp = log pi(y_t) + drift.  It is input generation only: the
library never calls it, and nothing here is used to check the library's results.
"""
from __future__ import annotations

import torch


def _logits_fp32(h, W):
    """h W^T with fp32 results (fp32 accumulation of the stored input values)."""
    if h.dtype == torch.float32:
        return h @ W.T
    try:
        return torch.mm(h, W.T, out_dtype=torch.float32)
    except (TypeError, RuntimeError):
        return h.float() @ W.float().T


@torch.no_grad()
def draw_tokens_and_old_logp(hidden, W_list, head_of_tok, valid, u, noise, rows_per_chunk: int = 4096,
                             want_lse: bool = False):
    """hidden [n, H]; W_list of [V, H]; head_of_tok int64 [n]; valid bool [n]; u float64 [n] in
    [0, 1); noise float32 [n].  Returns (token_id int32 [n], old_logp float32 [n]); rows that are
    not valid get token 0 and old_logp 0.  With want_lse also the engine's own log-sum-exp of every
    row's logits (float32 [n], 0 on rows that are not valid) as a third value."""
    n = hidden.shape[0]
    dev = hidden.device
    token_id = torch.zeros(n, dtype=torch.int32, device=dev)
    old_logp = torch.zeros(n, dtype=torch.float32, device=dev)
    lse = torch.zeros(n, dtype=torch.float32, device=dev) if want_lse else None
    for k, W in enumerate(W_list):
        rows = torch.nonzero(valid & (head_of_tok == k)).squeeze(1)
        for s in range(0, rows.numel(), rows_per_chunk):
            r = rows[s:s + rows_per_chunk]
            logits = _logits_fp32(hidden[r], W)
            logp = torch.log_softmax(logits, dim=1)
            cdf = torch.cumsum(torch.exp(logp), dim=1)
            y = torch.searchsorted(cdf, u[r].float().unsqueeze(1)).squeeze(1).clamp_(max=W.shape[0] - 1)
            token_id[r] = y.to(torch.int32)
            old_logp[r] = logp.gather(1, y.unsqueeze(1)).squeeze(1) + noise[r]
            if want_lse:
                lse[r] = torch.logsumexp(logits, dim=1)
    if want_lse:
        return token_id, old_logp, lse
    return token_id, old_logp
