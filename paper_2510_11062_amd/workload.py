"""Builds one synthetic rollout batch on the GPU: structure, tensors, rollout stand-in outputs and the
at_grpo_batch description.  Used by bench.py and by the full-size GPU tests (input plumbing only)."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

from . import api, rollout_standin, synth


@dataclass
class DeviceWorkload:
    cfg: synth.RolloutConfig
    st: synth.RolloutStructure
    batch: api.Batch
    env_id: torch.Tensor
    agent_id: torch.Tensor
    turn_id: torch.Tensor
    reward: torch.Tensor
    old_logp: torch.Tensor
    resp_of_tok: torch.Tensor     # int64 [n_tok]
    head_of_tok: torch.Tensor     # int64 [n_tok]
    valid: torch.Tensor           # bool [n_tok]
    noise: Optional[torch.Tensor] = None
    engine_lse: Optional[torch.Tensor] = None   # the stand-in's log-sum-exp per row (keep_noise only)


def build(cfg: synth.RolloutConfig, dev, keep_noise: bool = False) -> DeviceWorkload:
    st = synth.make_structure(cfg)
    hidden, W = synth.make_tensors(cfg, st.n_tok, device=dev)
    u, noise = synth.make_rollout_randoms(cfg, st.n_tok, device=dev)
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
    cu = torch.from_numpy(st.cu_seqlens).to(dev)
    resp_of_tok = torch.repeat_interleave(torch.arange(len(st.lengths), device=dev), cu[1:] - cu[:-1])
    mask = None if st.mask is None else torch.from_numpy(st.mask).to(dev)
    valid = torch.ones(st.n_tok, dtype=torch.bool, device=dev) if mask is None else mask.bool()
    head_of_resp = torch.from_numpy(st.head_of_agent[st.agent_id].astype(np.int64)).to(dev)
    head_of_tok = head_of_resp[resp_of_tok]
    drawn = rollout_standin.draw_tokens_and_old_logp(hidden, W, head_of_tok, valid, u, noise, want_lse=keep_noise)
    token_id, old_logp = drawn[0], drawn[1]
    engine_lse = drawn[2] if keep_noise else None
    multi = cfg.n_heads > 1
    batch = api.Batch(hidden, W, token_id, cu, mask, i32(st.agent_id) if multi else None,
                      i32(st.head_of_agent) if multi else None)
    return DeviceWorkload(cfg, st, batch, i32(st.env_id), i32(st.agent_id), i32(st.turn_id),
                          torch.from_numpy(st.reward).to(dev), old_logp, resp_of_tok, head_of_tok, valid,
                          noise if keep_noise else None, engine_lse)
