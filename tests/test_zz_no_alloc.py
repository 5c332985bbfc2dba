"""The grouping call that allocates nothing (fixed scratch array inside the library) against the call
that takes a workspace: same integers bit for bit, same floats bit for bit (same kernels, same order),
on two calls in a row of which the second is smaller, so whatever the first call left in the shared
array must not leak into the second."""
import sys
from dataclasses import replace

import numpy as np
import pytest
import torch

from paper_2510_11062_amd import api, synth

KEYS = ("group_id", "n_groups", "seg_offsets", "perm", "adv", "group_mean", "group_std")


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def device_inputs(cfg, dev):
    st = synth.make_structure(cfg)
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
    return st, (i32(st.env_id), i32(st.agent_id), i32(st.turn_id), torch.from_numpy(st.reward).to(dev))


def both_ways(cfg, dev, **kw):
    st, (e, i, t, r) = device_inputs(cfg, dev)
    ref = api.at_grpo_group_advantage(e, i, t, r, cfg.E, cfg.N, cfg.T, **kw)
    out = api.group_advantage_outputs(cfg.n_resp if st.reward.size == cfg.n_resp else st.reward.size,
                                      cfg.E * cfg.N * cfg.T, dev)
    for v in out.values():
        if v is not None:
            v.fill_(-7 if v.dtype == torch.int32 else float("nan"))     # outputs must be written, not inherited
    got = api.at_grpo_group_advantage_static(e, i, t, r, cfg.E, cfg.N, cfg.T, out=out, **kw)
    torch.cuda.synchronize()
    G = int(ref["n_groups"])
    assert int(got["n_groups"]) == G
    assert int(got["data_error"]) == api.error_word(ref["workspace"]) == 0
    for k in ("group_id", "perm", "adv"):
        assert torch.equal(got[k], ref[k]), k
    assert torch.equal(got["seg_offsets"][:G + 1], ref["seg_offsets"][:G + 1])
    for k in ("group_mean", "group_std"):
        assert torch.equal(got[k][:G], ref[k][:G]), k
    assert float(ref["adv"].abs().max()) > 0
    return G


@pytest.mark.gpu
def test_static_scratch_call_equals_workspace_call_twice_in_a_row(gpu_device):
    assert api.at_grpo_static_scratch_bytes() == 2 << 20
    big = synth.CONFIGS["C4"]                                      # 20480 responses, 5120 groups: multi-launch path
    small = replace(synth.CONFIGS["C2"], E=5, drop_tail_frac=0.3)    # a few hundred responses: one-workgroup path
    say(f"[no-alloc] first call: R={big.n_resp}")
    g1 = both_ways(big, gpu_device)
    say(f"[no-alloc] second call, smaller: R<={small.n_resp}")
    g2 = both_ways(small, gpu_device)
    assert g2 < g1
    say("[no-alloc] third call, medium, ddof 1")
    both_ways(replace(synth.CONFIGS["C5"], E=40), gpu_device, ddof=1)


@pytest.mark.gpu
def test_static_scratch_call_rejects_what_does_not_fit_and_flags_bad_ids(gpu_device):
    lib = api.load_library()
    # 64 responses over 2^22 keys need 32 MiB of scratch: refused on the host, nothing is launched.  Real
    # device buffers are passed all the same, and the refusal is established from the size query first.
    n_env = 1 << 22
    assert lib.at_grpo_workspace_bytes(api.CALL_GROUP_ADVANTAGE, None, 64, n_env, 1, 1) > api.at_grpo_static_scratch_bytes()
    ids = torch.zeros(64, dtype=torch.int32, device=gpu_device)
    rew = torch.zeros(64, dtype=torch.float32, device=gpu_device)
    out = api.group_advantage_outputs(64, n_env, gpu_device)
    with pytest.raises(api.AtGrpoError, match="scratch"):
        api.at_grpo_group_advantage_static(ids, ids, ids, rew, n_env, 1, 1, out=out)
    assert lib.at_grpo_status_string(5).startswith(b"input exceeds")
    cfg = synth.CONFIGS["C1"]
    st_, (e, i, t, r) = device_inputs(cfg, gpu_device)
    e[3] = cfg.E + 2
    got = api.at_grpo_group_advantage_static(e, i, t, r, cfg.E, cfg.N, cfg.T)
    torch.cuda.synchronize()
    assert int(got["data_error"]) & 1
    assert int(got["group_id"][3]) == -1 and float(got["adv"][3]) == 0.0
