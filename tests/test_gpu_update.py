"""The head update (gradient clipping + Adam, App. C.1) through the C ABI against the fp64 oracle.

fp32 arithmetic on the device against fp64 in the oracle: the moments agree to a few fp32 roundings,
the stepped weight to one unit in its last place (the step itself is ~1e-6 of a weight of ~1e-2, i.e.
a few hundred units in the last place, so one unit is a real check of the step).  The bf16 copy is an
integer decision (round to nearest even of the fp32 weight): it is checked exactly against the
device's own fp32 weight, and against the oracle's within one bf16 unit on a small fraction.
"""
import sys

import numpy as np
import pytest
import torch

from oracle import at_grpo_oracle as orc
from paper_2510_11062_amd import api
from tests.gpu_case import host

PAPER = dict(lr=1e-6, weight_decay=0.01, max_grad_norm=1.0)      # App. C.1


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def make_state(seed, n_heads, V, H, g_scale, bf16):
    """Seeded weights, gradients and moments (inputs only; no arithmetic of the method)."""
    rng = np.random.default_rng(seed)
    st = dict(W=[], g=[], m=[], v=[])
    for _ in range(n_heads):
        w = (rng.standard_normal((V, H)) * 0.02).astype(np.float32)
        st["W"].append(w)
        st["g"].append((rng.standard_normal((V, H)) * g_scale).astype(np.float32))
        st["m"].append((rng.standard_normal((V, H)) * g_scale * 0.1).astype(np.float32))
        st["v"].append(((rng.standard_normal((V, H)) * g_scale) ** 2 * 0.01).astype(np.float32))
    return st


def run_device(dev, st, step, bf16, **kw):
    t = lambda a: torch.from_numpy(a.copy()).to(dev)
    master = [t(w) for w in st["W"]]
    g, m, v = [t(x) for x in st["g"]], [t(x) for x in st["m"]], [t(x) for x in st["v"]]
    if bf16:
        low = [w.to(torch.bfloat16) for w in master]
        out = api.at_grpo_head_update(low, g, m, v, step, W_master=master, **kw)
    else:
        low = None
        out = api.at_grpo_head_update(master, g, m, v, step, **kw)
    torch.cuda.synchronize()
    return dict(master=master, low=low, m=m, v=v, grad_norm=host(out["grad_norm"]))


def as_passed(kw):
    """Hyper-parameters as the device receives them: the C struct holds floats, so both sides get the
    fp32 value of every one (1 - beta2 differs by 1e-5 relative between 0.999 and float(0.999))."""
    full = dict(lr=1e-6, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, max_grad_norm=1.0, decoupled=True)
    full.update(kw)
    return {k: (v if k == "decoupled" else float(np.float32(v))) for k, v in full.items()}


def ulp32(x):
    return np.spacing(np.abs(x).astype(np.float32)).astype(np.float64)


def check_against_oracle(got, st, step, bf16, **kw):
    kw = as_passed(kw)
    ref = orc.head_update(st["W"], st["g"], st["m"], st["v"], step, **kw)
    assert np.isclose(got["grad_norm"][0], ref["grad_norm"], rtol=2e-6)
    mg = kw.get("max_grad_norm", 1.0)
    coef = orc.clip_coefficient(ref["grad_norm"], mg) if mg > 0 else 1.0
    assert np.isclose(got["grad_norm"][1], coef, rtol=2e-6)
    for k in range(len(st["W"])):
        m, v, w = host(got["m"][k]).astype(np.float64), host(got["v"][k]).astype(np.float64), host(got["master"][k])
        # the two terms of m may cancel: bound the error by their magnitudes, not by the result's
        scale = 0.9 * np.abs(st["m"][k]) + 0.1 * np.abs(st["g"][k])
        assert np.all(np.abs(m - ref["m"][k]) <= 1e-6 * scale + 1e-30), f"m head {k}"
        assert np.allclose(v, ref["v"][k], rtol=1e-5, atol=1e-20), f"v head {k}"
        # weight: one rounding of the result, plus the fp32 error of the step propagated to first order
        # (the first moment's error is relative to its two terms, see above)
        err = np.abs(w.astype(np.float64) - ref["W"][k])
        denom = np.sqrt(ref["v"][k] / (1.0 - kw["beta2"] ** step)) + kw["eps"]
        step_err = 4e-6 * kw["lr"] / (1.0 - kw["beta1"] ** step) * (scale + np.abs(ref["m"][k])) / denom
        assert np.all(err <= 1.01 * ulp32(ref["W"][k]) + step_err + 1e-30), f"W head {k}: {err.max()}"
        # the step must actually have happened
        assert np.abs(ref["W"][k] - st["W"][k]).max() > 0
        if bf16:
            low = got["low"][k]
            assert torch.equal(low, got["master"][k].to(torch.bfloat16))          # nearest-even, exactly
            ref_low = torch.from_numpy(ref["W"][k].astype(np.float32)).to(torch.bfloat16).float().numpy()
            diff = np.abs(host(low.float()) - ref_low)
            assert np.mean(diff > 0) < 2e-3
            assert np.all(diff <= np.abs(ref_low) * 2.0 ** -7 + 1e-30)


@pytest.mark.gpu
@pytest.mark.parametrize("case", ["f32_one_head", "bf16_two_heads_paper", "bf16_coupled", "f32_no_clip",
                                  "bf16_step_one_zero_moments"])
def test_head_update_matches_oracle(gpu_device, case):
    if case == "f32_one_head":
        st, bf16, step, kw = make_state(1, 1, 96, 64, 5e-2, False), False, 3, dict(lr=1e-3, weight_decay=0.01)
    elif case == "bf16_two_heads_paper":
        st, bf16, step, kw = make_state(2, 2, 4736, 256, 2e-3, True), True, 7, dict(PAPER)
    elif case == "bf16_coupled":
        st, bf16, step, kw = make_state(3, 1, 1000, 128, 1e-2, True), True, 2, dict(PAPER, decoupled=False, lr=1e-4)
    elif case == "f32_no_clip":
        st, bf16, step, kw = make_state(4, 3, 130, 36, 1e-1, False), False, 11, dict(lr=1e-5, weight_decay=0.0, max_grad_norm=0.0)
    else:
        st, bf16, step, kw = make_state(5, 1, 777, 64, 1e-3, True), True, 1, dict(PAPER)
        st["m"] = [np.zeros_like(x) for x in st["m"]]
        st["v"] = [np.zeros_like(x) for x in st["v"]]
    say(f"[head_update] {case}: heads={len(st['W'])} shape={st['W'][0].shape} step={step}")
    got = run_device(gpu_device, st, step, bf16, **kw)
    check_against_oracle(got, st, step, bf16, **kw)


@pytest.mark.gpu
def test_head_update_several_steps_in_a_row(gpu_device):
    """Three updates with fresh gradients each; the device carries its own state forward."""
    dev = gpu_device
    st = make_state(6, 2, 600, 64, 3e-3, True)
    t = lambda a: torch.from_numpy(a.copy()).to(dev)
    master = [t(w) for w in st["W"]]
    low = [w.to(torch.bfloat16) for w in master]
    m = [torch.zeros_like(w) for w in master]
    v = [torch.zeros_like(w) for w in master]
    rW, rm, rv = [w.astype(np.float64) for w in st["W"]], [np.zeros_like(w, np.float64) for w in st["W"]], \
        [np.zeros_like(w, np.float64) for w in st["W"]]
    say("[head_update] three steps")
    for step in (1, 2, 3):
        gs = make_state(60 + step, 2, 600, 64, 3e-3, True)["g"]
        api.at_grpo_head_update(low, [t(g) for g in gs], m, v, step, W_master=master, **PAPER)
        ref = orc.head_update(rW, gs, rm, rv, step, **as_passed(PAPER))
        rW, rm, rv = ref["W"], ref["m"], ref["v"]
    torch.cuda.synchronize()
    for k in range(2):
        assert np.allclose(host(m[k]), rm[k], rtol=2e-5, atol=1e-9)
        assert np.allclose(host(v[k]), rv[k], rtol=2e-5, atol=1e-20)
        err = np.abs(host(master[k]).astype(np.float64) - rW[k])
        # one unit in the last place per step (of the larger of the start and end values: a weight
        # may cross a binade on the way), plus the propagated error of three steps of ~1e-6
        assert np.all(err <= 3.03 * ulp32(np.maximum(np.abs(rW[k]), np.abs(st["W"][k]))) + 2e-10)
        assert torch.equal(low[k], master[k].to(torch.bfloat16))


@pytest.mark.gpu
def test_head_update_full_size_head(gpu_device):
    """V = 151936, H = 2048 (the C2 head): sampled elements against the oracle, the norm in full,
    run-to-run reproducibility."""
    dev = gpu_device
    V, H = 151936, 2048
    say(f"[head_update] full size V={V} H={H}")
    gen = torch.Generator(device=dev)
    gen.manual_seed(251011062 + 77)
    master0 = torch.randn((V, H), generator=gen, device=dev, dtype=torch.float32) * 0.02
    g = torch.randn((V, H), generator=gen, device=dev, dtype=torch.float32) * 1e-4      # norm ~1.76: clipped
    m0 = torch.randn((V, H), generator=gen, device=dev, dtype=torch.float32) * 1e-5
    v0 = (torch.randn((V, H), generator=gen, device=dev, dtype=torch.float32) * 1e-5) ** 2

    def once():
        master, m, v = master0.clone(), m0.clone(), v0.clone()
        low = master.to(torch.bfloat16)
        out = api.at_grpo_head_update([low], [g], [m], [v], 5, W_master=[master], **PAPER)
        torch.cuda.synchronize()
        return master, low, m, v, out["grad_norm"].clone()

    master, low, m, v, gn = once()
    # norm: the oracle's definition on the full gradient (fp64 on the host, in slabs to bound memory)
    norm = orc.global_grad_norm(g[r0:r0 + 16384].cpu().numpy() for r0 in range(0, V, 16384))
    assert norm > 1.0
    assert np.isclose(float(gn[0]), norm, rtol=2e-6)
    coef = orc.clip_coefficient(norm, 1.0)
    assert np.isclose(float(gn[1]), coef, rtol=2e-6)
    # sampled rows, element by element
    rows = np.random.default_rng(9).choice(V, size=24, replace=False)
    rows_t = torch.from_numpy(rows).to(dev)
    w_ref, m_ref, v_ref = orc.adam_step(master0[rows_t].cpu().numpy(), g[rows_t].cpu().numpy().astype(np.float64) * coef,
                                        m0[rows_t].cpu().numpy(), v0[rows_t].cpu().numpy(), 5,
                                        **{k: v for k, v in as_passed(PAPER).items() if k != "max_grad_norm"})
    scale = 0.9 * np.abs(m0[rows_t].cpu().numpy()) + 0.1 * np.abs(g[rows_t].cpu().numpy())
    assert np.all(np.abs(m[rows_t].cpu().numpy() - m_ref) <= 1e-6 * scale + 1e-30)
    assert np.allclose(v[rows_t].cpu().numpy(), v_ref, rtol=1e-5, atol=1e-22)
    err = np.abs(master[rows_t].cpu().numpy().astype(np.float64) - w_ref)
    assert np.all(err <= 1.01 * ulp32(w_ref))
    assert torch.equal(low, master.to(torch.bfloat16))
    assert not torch.equal(master, master0)
    again = once()
    for a, b in zip((master, low, m, v, gn), again):
        assert torch.equal(a, b)
