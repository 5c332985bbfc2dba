"""The library enqueues on the caller's stream, never synchronises and never allocates: a whole step
can therefore run on a side stream, and can be captured once in a HIP graph and replayed.

Both properties are checked bit for bit against the plain eager run on the default stream (the kernels
use no floating-point atomics, so equal inputs give equal bits)."""
import sys

import pytest
import torch

from paper_2510_11062_amd import api
from tests import helpers
from tests.gpu_case import DeviceCase
from tests.test_gpu_parity import mini_cfg


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def one_step(dc, cfg, path="two_calls"):
    ga = api.at_grpo_group_advantage(dc.env_id, dc.agent_id, dc.turn_id, dc.reward, cfg.E, cfg.N, cfg.T)
    if path == "one_pass":
        fwd = bwd = api.at_grpo_policy_loss_fwd_bwd(dc.batch(), dc.old_logp, ga["adv"], cfg.eps_clip, cfg.eps_clip)
    else:
        fwd = api.at_grpo_policy_loss_fwd(dc.batch(), dc.old_logp, ga["adv"], cfg.eps_clip, cfg.eps_clip)
        bwd = api.at_grpo_policy_loss_bwd(dc.batch(), dc.old_logp, ga["adv"], fwd["logp"], fwd["lse"],
                                          cfg.eps_clip, cfg.eps_clip)
    return [ga["adv"], ga["perm"], ga["group_id"], fwd["loss"], fwd["logp"], fwd["lse"], fwd["clip_mask"],
            fwd["n_valid"], bwd["d_hidden"]] + list(bwd["dW"])


@pytest.mark.gpu
@pytest.mark.parametrize("path", ["two_calls", "one_pass"])
def test_calls_follow_the_current_stream(gpu_device, path):
    cfg = mini_cfg("C5")
    c = helpers.build_case(cfg, device=gpu_device)
    dc = DeviceCase(c, gpu_device)
    say("[streams] eager on the default stream")
    ref = [t.clone() for t in one_step(dc, cfg, path)]
    torch.cuda.synchronize()
    side = torch.cuda.Stream(device=gpu_device)          # default priority
    side.wait_stream(torch.cuda.current_stream())
    say("[streams] the same step on a side stream")
    with torch.cuda.stream(side):
        out = one_step(dc, cfg, path)
        got = [t.clone() for t in out]
    side.synchronize()
    for a, b in zip(ref, got):
        assert torch.equal(a, b)


@pytest.mark.gpu
@pytest.mark.parametrize("path", ["two_calls", "one_pass"])
def test_step_captured_in_a_graph_replays_bit_identically(gpu_device, path):
    cfg = mini_cfg("C3")
    c = helpers.build_case(cfg, device=gpu_device)
    dc = DeviceCase(c, gpu_device)
    say("[graph] eager reference (also sizes the cached workspace)")
    ref = [t.clone() for t in one_step(dc, cfg, path)]
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    say("[graph] capture")
    with torch.cuda.graph(graph):
        static_out = one_step(dc, cfg, path)
    torch.cuda.synchronize()

    for rep in range(3):
        # eager work and a synchronisation between the replays; outputs poisoned so that a replay
        # that did nothing cannot pass
        for t in static_out:
            if t.dtype in (torch.float32, torch.bfloat16):
                t.fill_(float("nan"))
            else:
                t.fill_(-7 if t.dtype != torch.uint8 else 255)
        eager_again = one_step(dc, cfg, path)
        torch.cuda.synchronize()
        for a, b in zip(ref, eager_again):
            assert torch.equal(a, b)
        say(f"[graph] replay {rep}")
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(ref, static_out):
            assert torch.equal(a, b), f"replay {rep}"
    assert api.error_word(api._workspace(1, gpu_device)) == 0
