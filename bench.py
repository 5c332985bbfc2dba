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
def chunk_tokens(kern, cfg):
    """List positions one launch of a head kernel class covers (the library's launch plan)."""
    if kern == "head_dw":
        return 32768
    if kern == "head_fwd":
        return 16384
    # head_fe, head_dz, head_dh: the part of a super-chunk whose hidden rows fill 64 MB
    row_bytes = cfg.H * (2 if cfg.dtype == "bf16" else 4)
    return min(16384, (64 << 20) // row_bytes // 256 * 256)


KERNEL_SYMBOL = {"head_fwd": "k_head_fwd", "head_fe": "k_head_fe", "head_dz": "k_head_dz", "head_dh": "k_head_dh",
                 "head_dw": "k_head_dw"}


# the kernels and the launch plan (rows per launch) that decides what one launch moves
HEAD_KERNEL_SOURCES = ("common.hpp", "gemm_core.hpp", "head_kernels.hpp", "head_kernels.hip", "api.hip")


def kernel_source_digest():
    """sha256 over the sources of the head kernels and of their launch plan (what `traffic` is quoted for): HBM counter
    readings are only reported for the code they were taken on."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2510_11062_amd", "csrc")
    for name in HEAD_KERNEL_SOURCES:
        h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()


def recorded_traffic(workload_name, kern):
    """HBM bytes per working launch of `kern` from the committed rocprofv3 --pmc summary.  None when there
    is no summary for this workload/kernel; the string "stale: ..." when the head kernel sources changed
    since the counters were taken (they are then not quoted)."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload_name}.txt")
    if not os.path.exists(path):
        return None
    rec = json.load(open(path))
    now = kernel_source_digest()
    if rec.get("source_digest") != now:
        return f"stale: counters taken on sources {str(rec.get('source_digest'))[:12]}, now {now[:12]}"
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


def run_config(cfg, dev, steps, warmup, path="one_pass"):
    """Times `steps` steps (grouped advantages + loss forward + backward) of one workload; returns the
    measurements and what the caller needs for the CPU leg.  path: "one_pass" = at_grpo_policy_loss_fwd_bwd
    (logits produced once), "two_calls" = at_grpo_policy_loss_fwd then at_grpo_policy_loss_bwd (logits
    recomputed by the backward)."""
    wl = workload.build(cfg, dev)
    st, batch, old_logp, resp_of_tok, valid = wl.st, wl.batch, wl.old_logp, wl.resp_of_tok, wl.valid
    env_id, agent_id, turn_id, reward = wl.env_id, wl.agent_id, wl.turn_id, wl.reward
    eps = cfg.eps_clip
    d_hidden = torch.empty_like(batch.hidden)
    dW = [torch.empty(w.shape, dtype=torch.float32, device=dev) for w in batch.W]
    state = {}

    def step():
        ga = api.at_grpo_group_advantage(env_id, agent_id, turn_id, reward, cfg.E, cfg.N, cfg.T, want_stats=False)
        if path == "one_pass":
            fwd = api.at_grpo_policy_loss_fwd_bwd(batch, old_logp, ga["adv"], eps, eps, dW=dW, d_hidden=d_hidden,
                                                  out=state.get("fwd"))
        else:
            fwd = api.at_grpo_policy_loss_fwd(batch, old_logp, ga["adv"], eps, eps, out=state.get("fwd"))
            api.at_grpo_policy_loss_bwd(batch, old_logp, ga["adv"], fwd["logp"], fwd["lse"], eps, eps,
                                        dW=dW, d_hidden=d_hidden)
        state["fwd"], state["ga"] = fwd, ga

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    api.at_grpo_profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
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
    grad_rows = valid & (A_tok != 0) & ((fwd["clip_mask"] & 4) == 0)
    n_grad = int(grad_rows.sum().item())
    hv2 = 2.0 * cfg.H * cfg.V
    if path == "one_pass":
        # rows of non-zero advantage get their logits once (head_fe), the others only their log-probability
        # (head_fwd); the two backward contractions run over the first class and are credited with the rows that
        # carry gradient (the clipped ones among them multiply by a zero factor)
        adv_rows = valid & (A_tok != 0)
        n_adv = int(adv_rows.sum().item())
        flops = {"head_fwd": hv2 * (n_valid - n_adv), "head_fe": hv2 * n_adv, "head_dh": hv2 * n_grad,
                 "head_dw": hv2 * n_grad}
        rows_of = {"head_fwd": valid & ~adv_rows, "head_fe": adv_rows, "head_dh": adv_rows, "head_dw": adv_rows}
    else:
        flops = {"head_fwd": hv2 * n_valid, "head_dz": hv2 * n_grad, "head_dh": hv2 * n_grad, "head_dw": hv2 * n_grad}
        rows_of = {"head_fwd": valid, "head_dz": grad_rows, "head_dh": grad_rows, "head_dw": grad_rows}
    kern = max(flops, key=lambda k: prof[k][1])
    kern_ms = prof[kern][1] / steps
    achieved = flops[kern] / (kern_ms * 1e-3) / 1e12
    # launches that had rows to process (the others return at once): per head, ceil(rows / chunk)
    live = rows_of[kern]
    rows_per_head = torch.bincount(wl.head_of_tok[live], minlength=cfg.n_heads).tolist()
    work_launches = sum(-(-r // chunk_tokens(kern, cfg)) for r in rows_per_head)
    peak = PEAK[cfg.dtype]
    all_gemm_ms = sum(prof[k][1] for k in flops) / steps
    all_gemm_tflops = sum(flops.values()) / (all_gemm_ms * 1e-3) / 1e12
    rec = {
        "workload": f"{cfg.name}: H={cfg.H} V={cfg.V} heads={cfg.n_heads} "
                    f"E{cfg.E}xN{cfg.N}xT{cfg.T}xK{cfg.K}={st.cfg.n_resp} responses, "
                    f"{n_valid} response tokens in {st.n_tok} rows"
                    f"{' (padded + mask)' if cfg.padded else ' (packed)'}",
        "tokens_per_s": n_valid / (elapsed / steps), "ms_per_step": elapsed / steps * 1e3, "steps": steps,
        "response_tokens": n_valid, "rows_with_gradient": n_grad, "device_error_word": err, "path": path,
        "executed_flop_per_step": sum(flops.values()),
        "flop_per_step_if_logits_were_recomputed": hv2 * (n_valid + 3 * n_grad),
        # whole-step rates (every kernel of the step in the denominator): the contractions this path executes, and
        # the 8 H V per gradient token a path that recomputes the logits in the backward would be credited with
        "step_tflops_executed": sum(flops.values()) / (elapsed / steps) / 1e12,
        "step_tflops_if_logits_were_recomputed": hv2 * (n_valid + 3 * n_grad) / (elapsed / steps) / 1e12,
        "roofline": {"bound": "mfma", "kernel": kern, "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": recorded_traffic(cfg.name, kern),
                     "flop_per_launch": flops[kern] / max(work_launches, 1),
                     "ms_per_launch": kern_ms / max(work_launches, 1),
                     "launches_with_rows_per_step": work_launches,
                     "kernel_ms_per_step": kern_ms, "launches_per_step": prof[kern][0] / steps,
                     "all_head_contractions_tflops": all_gemm_tflops,
                     "all_head_contractions_frac": all_gemm_tflops / peak},
        "head_kernel_tflops": {k: flops[k] / (prof[k][1] / steps * 1e-3) / 1e12 for k in flops if prof[k][1] > 0},
        "kernel_ms_per_step": {k: v[1] / steps for k, v in prof.items()},
    }
    return rec, (st, batch, old_logp)


def streaming_records(dev):
    """Achieved HBM GB/s of the grouping call, the surrogate stage and the head update (the bandwidth half
    of the metric), measured in this run: the grouping call and the surrogate stage at the largest real
    shapes (latency-bound there) and on scaled twins, the update on the C2 head."""
    from paper_2510_11062_amd import bench_streaming as bs
    out = [bs.grouping(dev, 256, 2, 10, 4, "C4 shape (20480 responses)"),
           bs.grouping(dev, 262144, 2, 4, 8, "scaled twin of C2: 2^24 responses, K = 8, shuffled order"),
           bs.grouping(dev, 262144, 2, 4, 8, "scaled twin of C2: 2^24 responses, K = 8, rollout order", shuffle=False),
           bs.surrogate(dev, 6144, 290, "C5 row count (~1.8 M rows)"),
           bs.surrogate(dev, 6144 * 16, 290, "16x twin of C5 (~28 M rows)"),
           bs.head_update(dev, 1, 151936, 2048, "C2 head: V=151936 H=2048, bf16 weights + fp32 master")]
    copy = bs.copy_ceiling(dev)
    for o in out:
        o["frac_of_measured_copy"] = o["achieved"] / copy["achieved"]
    return {"hbm_peak_GBs": bs.HBM_PEAK_GBS, "measured_copy_ceiling": copy, "kernels": out}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="C2", help="the workload `value` is quoted on")
    ap.add_argument("--more-configs", default="C3,C4,C5",
                    help="further workloads timed after it and reported under `configs` ('none' to skip)")
    ap.add_argument("--more-steps", type=int, default=3, help="timed steps of each further workload")
    ap.add_argument("--no-streaming", action="store_true", help="skip the bandwidth records of the streaming kernels")
    ap.add_argument("--path", default="one_pass", choices=["one_pass", "two_calls"],
                    help="one_pass: at_grpo_policy_loss_fwd_bwd; two_calls: forward call, then backward call")
    ap.add_argument("--cpu-sample", type=int, default=6144, help="response tokens given to the CPU oracle (0 = skip)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after the timed steps, copy 1 GiB with torch (known traffic, to scale HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: the library has no multi-GPU path (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS[args.config]
    api.load_library()

    rec, (st, batch, old_logp) = run_config(cfg, dev, args.steps, args.warmup, args.path)

    if args.calibration_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    out = {
        "metric": "policy-loss fwd+bwd tokens/sec at V=151936; MFMA util % and HBM GB/s",
        "value": rec["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": rec["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": rec["workload"], "rows_with_gradient": rec["rows_with_gradient"],
                   "device_error_word": rec["device_error_word"], "path": rec["path"]},
        "roofline": rec["roofline"],
        "step_tflops_executed": rec["step_tflops_executed"],
        "step_tflops_if_logits_were_recomputed": rec["step_tflops_if_logits_were_recomputed"],
        "head_kernel_tflops": rec["head_kernel_tflops"],
        "kernel_ms_per_step": rec["kernel_ms_per_step"],
    }
    if args.cpu_sample > 0:
        out["cpu_baseline"] = cpu_baseline(cfg, st, batch, old_logp, args.cpu_sample)
    del st, batch, old_logp
    api.release_workspace()
    torch.cuda.empty_cache()

    if args.more_configs.lower() != "none":
        out["configs"] = {}
        for name in [c for c in args.more_configs.split(",") if c and c != args.config]:
            more, keep = run_config(synth.CONFIGS[name], dev, args.more_steps, 1, args.path)
            more.pop("kernel_ms_per_step")
            out["configs"][name] = more
            del keep
            api.release_workspace()
            torch.cuda.empty_cache()
    if not args.no_streaming:
        out["streaming"] = streaming_records(dev)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
