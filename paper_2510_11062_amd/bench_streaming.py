"""Achieved HBM bandwidth of the streaming (non-contraction) kernels of the path.

    python -m paper_2510_11062_amd.bench_streaming

Reports, per line of JSON: the grouping + advantage call at the real workload shapes (these are
latency-bound: at most 20480 responses) and on a scaled-up twin with the same group structure
(K = 8 candidates per (e, i, t), 2^24 responses); the surrogate stage (routing, compaction, ratio /
clip / masked reduction) and the backward coefficient at the C5 row count and on a 16x twin.
GB/s = algorithmic bytes / measured time, against the 8 TB/s HBM3E peak:
  grouping + advantages : 16 B read (3 ids + reward) + 12 B written (group id, perm, adv) per response
  surrogate stage       : 13 B read (logp, old_logp, token id for the range check, mask) + 1 B written
                          (clip mask) per row
  head update           : 4 B read per parameter for the norm; 16 B read (gradient, two moments, fp32
                          weight) + 14 B written (moments, fp32 weight, bf16 weight) for the step
"""
from __future__ import annotations

import json
import sys
import time

import numpy as np
import torch

from . import api

HBM_PEAK_GBS = 8000.0


def _time(fn, iters=5, warmup=2):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(iters):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / iters


def grouping(dev, E, N, T, K, label, shuffle=True):
    g = torch.Generator(device=dev)
    g.manual_seed(1234)
    R = E * N * T * K
    key = torch.arange(R, device=dev) // K
    if shuffle:
        key = key[torch.randperm(R, generator=g, device=dev)]
    env = (key // (N * T)).to(torch.int32)
    agent = ((key // T) % N).to(torch.int32)
    turn = (key % T).to(torch.int32)
    reward = torch.rand(R, generator=g, device=dev)
    fn = lambda: api.at_grpo_group_advantage(env, agent, turn, reward, E, N, T, want_stats=False)
    dt = _time(fn)
    api.at_grpo_profile_enable(True)
    iters = 10
    for _ in range(iters):
        fn()
    k_us = api.at_grpo_profile_read()["group_advantage"][1] / iters * 1e3
    api.at_grpo_profile_enable(False)
    nbytes = 28.0 * R
    return {"kernel": "group_advantage (S1+S2, whole call)", "workload": label, "responses": R,
            "groups": E * N * T, "us_per_call": dt * 1e6, "us_on_stream": k_us,
            "achieved": nbytes / dt / 1e9, "unit": "GB/s",
            "peak": HBM_PEAK_GBS, "frac": nbytes / dt / 1e9 / HBM_PEAK_GBS}


def surrogate(dev, n_resp, mean_len, label):
    g = torch.Generator(device=dev)
    g.manual_seed(99)
    lengths = torch.randint(max(1, mean_len // 2), mean_len * 3 // 2 + 1, (n_resp,), generator=g, device=dev)
    cu = torch.zeros(n_resp + 1, dtype=torch.int64, device=dev)
    cu[1:] = torch.cumsum(lengths, 0)
    n_tok = int(cu[-1])
    logp = -torch.rand(n_tok, generator=g, device=dev) * 12
    old = logp + 0.2 * torch.randn(n_tok, generator=g, device=dev)
    adv = torch.randn(n_resp, generator=g, device=dev)
    mask = torch.ones(n_tok, dtype=torch.uint8, device=dev)
    token_id = torch.zeros(n_tok, dtype=torch.int32, device=dev)
    batch = api.Batch(None, None, token_id, cu, mask, None, None, n_tok=n_tok, V=151936, n_heads=1)
    fn = lambda: api.at_grpo_surrogate_from_logp(batch, logp, old, adv, 0.2, 0.2)
    dt = _time(fn)
    api.at_grpo_profile_enable(True)
    iters = 5
    for _ in range(iters):
        fn()
    prof = api.at_grpo_profile_read()
    api.at_grpo_profile_enable(False)
    nbytes = 14.0 * n_tok      # logp 4 + old_logp 4 + token id 4 (range check) + mask 1 read, clip mask 1 written
    k_ms = prof["surrogate"][1] / iters
    p_ms = prof["token_prep"][1] / iters
    return {"kernel": "surrogate stage (S5+S6)", "workload": label, "rows": n_tok,
            "us_per_call": dt * 1e6, "achieved_whole_call": nbytes / dt / 1e9,
            "us_surrogate_kernels": k_ms * 1e3, "us_routing_compaction": p_ms * 1e3,
            "achieved": nbytes / (k_ms * 1e-3) / 1e9, "unit": "GB/s", "peak": HBM_PEAK_GBS,
            "frac": nbytes / (k_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}


def head_update(dev, n_heads, V, H, label):
    g = torch.Generator(device=dev)
    g.manual_seed(7)
    master = [torch.randn((V, H), generator=g, device=dev) * 0.02 for _ in range(n_heads)]
    low = [w.to(torch.bfloat16) for w in master]
    dW = [torch.randn((V, H), generator=g, device=dev) * 1e-4 for _ in range(n_heads)]
    m = [torch.zeros_like(w) for w in master]
    v = [torch.zeros_like(w) for w in master]
    step = [0]

    def fn():
        step[0] += 1
        api.at_grpo_head_update(low, dW, m, v, step[0], W_master=master)

    dt = _time(fn)
    api.at_grpo_profile_enable(True)
    iters = 5
    for _ in range(iters):
        fn()
    prof = api.at_grpo_profile_read()
    api.at_grpo_profile_enable(False)
    n = float(n_heads) * V * H
    norm_ms, adam_ms = prof["grad_norm"][1] / iters, prof["adam"][1] / iters
    return {"kernel": "head update (clip + Adam)", "workload": label, "parameters": int(n),
            "us_per_call": dt * 1e6, "us_grad_norm": norm_ms * 1e3, "us_adam": adam_ms * 1e3,
            "grad_norm_GBs": 4.0 * n / (norm_ms * 1e-3) / 1e9, "adam_GBs": 30.0 * n / (adam_ms * 1e-3) / 1e9,
            "achieved": 34.0 * n / dt / 1e9, "unit": "GB/s", "peak": HBM_PEAK_GBS,
            "frac": 34.0 * n / dt / 1e9 / HBM_PEAK_GBS}


def copy_ceiling(dev, n_bytes: int = 1 << 30):
    """What a plain device-to-device copy of 1 GiB reaches on this GPU (bytes read + written per second):
    the measured ceiling the streaming kernels are also reported against."""
    src = torch.empty(n_bytes // 4, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    dt = _time(lambda: dst.copy_(src), iters=10)
    return {"kernel": "torch device-to-device copy", "bytes": n_bytes, "us_per_call": dt * 1e6,
            "achieved": 2.0 * n_bytes / dt / 1e9, "unit": "GB/s", "frac": 2.0 * n_bytes / dt / 1e9 / HBM_PEAK_GBS}


def main():
    if not torch.cuda.is_available():
        print("needs a GPU", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    api.load_library()
    out = []
    out.append(grouping(dev, 16, 2, 4, 8, "C2 shape"))
    out.append(grouping(dev, 256, 2, 10, 4, "C4 shape"))
    out.append(grouping(dev, 64, 3, 4, 8, "C5 shape"))
    out.append(grouping(dev, 262144, 2, 4, 8, "scaled twin of C2: 2^24 responses, K = 8, shuffled order"))
    out.append(grouping(dev, 262144, 2, 4, 8, "scaled twin of C2: 2^24 responses, K = 8, rollout order",
                        shuffle=False))
    out.append(surrogate(dev, 6144, 290, "C5 row count (~1.8 M rows)"))
    out.append(surrogate(dev, 6144 * 16, 290, "16x twin of C5 (~28 M rows)"))
    out.append(head_update(dev, 1, 151936, 2048, "C2 head: V=151936 H=2048, bf16 weights + fp32 master"))
    out.append(head_update(dev, 2, 151936, 4096, "C3 heads: 2 x (V=151936 H=4096)"))
    out.append(copy_ceiling(dev))
    for o in out:
        print(json.dumps(o))


if __name__ == "__main__":
    main()
