#!/usr/bin/env python3
"""Throughput of the AT-GRPO policy-loss hot path on one MI355X.

One step = grouped advantages + policy-loss forward + backward over one synthetic rollout batch
(all inputs resident in HBM before the timed region).  Prints ONE JSON line:
tokens/s over the response tokens, the roofline fraction of the dominant kernel (measured with
HIP events recorded on the launch stream inside the library) and the CPU oracle timed on a small
sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2510_11062_amd import api, synth, workload  # noqa: E402

PEAK = {"bf16": 2500.0, "f32": 157.3}      # dense MFMA TFLOP/s, MI355X data sheet
CHUNK_TOKENS = 32768                       # list positions one head-kernel launch covers
KERNEL_SYMBOL = {"head_fwd": "k_head_fwd", "head_dz": "k_head_dz", "head_dh": "k_head_dh", "head_dw": "k_head_dw"}


HEAD_KERNEL_SOURCES = ("common.hpp", "gemm_core.hpp", "head_kernels.hpp", "head_kernels.hip")


def kernel_source_digest():
    """sha256 over the sources of the head kernels (the ones `traffic` is quoted for): HBM counter
    readings are only reported for the code they were taken on."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2510_11062_amd", "csrc")
    for name in HEAD_KERNEL_SOURCES:
        h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()


def recorded_traffic(workload_name, kern):
    """HBM bytes per working launch of `kern` from the committed rocprofv3 --pmc summary, or None when
    there is none for this workload/kernel or the kernels changed since it was taken."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload_name}.txt")
    if not os.path.exists(path):
        return None
    rec = json.load(open(path))
    if rec.get("source_digest") != kernel_source_digest():
        return None
    k = rec.get("kernels", {}).get(KERNEL_SYMBOL[kern])
    return None if k is None else k["hbm_bytes_per_launch"]



def cpu_baseline(cfg, st, batch, old_logp, n_sample):
    """The CPU oracle (fp64 numpy), timed as it stands on a packed sample of response tokens."""
    from oracle import at_grpo_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    valid = torch.ones(st.n_tok, dtype=torch.bool) if st.mask is None else torch.from_numpy(st.mask != 0)
    rows = torch.nonzero(valid).squeeze(1)[:n_sample]
    dev_rows = rows.to(batch.hidden.device)
    hidden = batch.hidden[dev_rows].float().cpu().numpy()
    W = [w.float().cpu().numpy() for w in batch.W[:1]]
    y = batch.token_id[dev_rows].cpu().numpy()
    old = old_logp[dev_rows].cpu().numpy()
    n = hidden.shape[0]
    cu = np.arange(n + 1, dtype=np.int64)
    adv = np.random.default_rng(0).standard_normal(n).astype(np.float32)
    t0 = time.perf_counter()
    orc.policy_loss_bwd(hidden, W, y, None, cu, None, None, old, adv, cfg.eps_clip, cfg.eps_clip)
    dt = time.perf_counter() - t0
    cpu = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                cpu = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    n_all = int(valid.sum().item())
    return {"value": n / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{n} response tokens of {cfg.name} on one head, fp64 numpy forward+backward "
                      f"(one-token responses), {dt:.1f} s",
            "host_cpu": cpu, "host_logical_cpus": os.cpu_count(),
            "extrapolated_full_workload_s": n_all / (n / dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="C2")
    ap.add_argument("--cpu-sample", type=int, default=6144, help="response tokens given to the CPU oracle (0 = skip)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after the timed steps, copy 1 GiB with torch (known traffic, to scale HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS[args.config]
    api.load_library()

    wl = workload.build(cfg, dev)
    st, batch, old_logp, resp_of_tok, valid = wl.st, wl.batch, wl.old_logp, wl.resp_of_tok, wl.valid
    env_id, agent_id, turn_id, reward = wl.env_id, wl.agent_id, wl.turn_id, wl.reward
    eps = cfg.eps_clip

    d_hidden = torch.empty_like(batch.hidden)
    dW = [torch.empty(w.shape, dtype=torch.float32, device=dev) for w in batch.W]
    state = {}

    def step():
        ga = api.at_grpo_group_advantage(env_id, agent_id, turn_id, reward, cfg.E, cfg.N, cfg.T, want_stats=False)
        fwd = api.at_grpo_policy_loss_fwd(batch, old_logp, ga["adv"], eps, eps, out=state.get("fwd"))
        api.at_grpo_policy_loss_bwd(batch, old_logp, ga["adv"], fwd["logp"], fwd["lse"], eps, eps,
                                    dW=dW, d_hidden=d_hidden)
        state["fwd"], state["ga"] = fwd, ga

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    api.at_grpo_profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = api.at_grpo_profile_read()
    api.at_grpo_profile_enable(False)

    n_valid = int(valid.sum().item())
    fwd, ga = state["fwd"], state["ga"]
    err = api.error_word(fwd["workspace"])
    # rows that carry gradient: participating, advantage != 0, not on the clipped branch
    A_tok = ga["adv"][resp_of_tok]
    n_grad = int((valid & (A_tok != 0) & ((fwd["clip_mask"] & 4) == 0)).sum().item())
    ms_per_step = elapsed / args.steps * 1e3
    tokens_per_s = n_valid / (elapsed / args.steps)

    if args.calibration_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    hv2 = 2.0 * cfg.H * cfg.V
    flops = {"head_fwd": hv2 * n_valid, "head_dz": hv2 * n_grad, "head_dh": hv2 * n_grad, "head_dw": hv2 * n_grad}
    kern = max(flops, key=lambda k: prof[k][1])
    kern_ms = prof[kern][1] / args.steps
    achieved = flops[kern] / (kern_ms * 1e-3) / 1e12
    # launches that had rows to process (the others return at once): per head, ceil(rows / chunk)
    head_of_tok = wl.head_of_tok
    live = valid if kern == "head_fwd" else (valid & (A_tok != 0) & ((fwd["clip_mask"] & 4) == 0))
    rows_per_head = torch.bincount(head_of_tok[live], minlength=cfg.n_heads).tolist()
    work_launches = sum(-(-r // CHUNK_TOKENS) for r in rows_per_head)
    peak = PEAK[cfg.dtype]
    all_gemm_ms = sum(prof[k][1] for k in flops) / args.steps
    all_gemm_tflops = sum(flops.values()) / (all_gemm_ms * 1e-3) / 1e12

    out = {
        "metric": "policy-loss fwd+bwd tokens/sec at V=151936; MFMA util % and HBM GB/s",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: H={cfg.H} V={cfg.V} heads={cfg.n_heads} "
                               f"E{cfg.E}xN{cfg.N}xT{cfg.T}xK{cfg.K}={st.cfg.n_resp} responses, "
                               f"{n_valid} response tokens in {st.n_tok} rows"
                               f"{' (padded + mask)' if cfg.padded else ' (packed)'}",
                   "rows_with_gradient": n_grad, "device_error_word": err},
        "roofline": {"bound": "mfma", "kernel": kern, "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": recorded_traffic(cfg.name, kern),
                     "flop_per_launch": flops[kern] / max(work_launches, 1),
                     "ms_per_launch": kern_ms / max(work_launches, 1),
                     "launches_with_rows_per_step": work_launches,
                     "kernel_ms_per_step": kern_ms, "launches_per_step": prof[kern][0] / args.steps,
                     "all_head_contractions_tflops": all_gemm_tflops,
                     "all_head_contractions_frac": all_gemm_tflops / peak},
        "kernel_ms_per_step": {k: v[1] / args.steps for k, v in prof.items()},
    }
    if args.cpu_sample > 0:
        out["cpu_baseline"] = cpu_baseline(cfg, st, batch, old_logp, args.cpu_sample)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
