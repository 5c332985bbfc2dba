"""The boundary from plain C: the header compiles as C99 and as C++, and a gcc-built client that
fills at_grpo_batch itself, owns its buffers through the HIP C API and never touches Python gets the
oracle's results (and, bit for bit, the results the Python binding gets)."""
import os
import subprocess
import sys

import numpy as np
import pytest
import torch

from oracle import at_grpo_oracle as orc
from paper_2510_11062_amd import api, synth
from tests import helpers
from tests.gpu_case import DeviceCase, host

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLIENT = os.path.join(ROOT, "paper_2510_11062_amd", "abi_client")
HEADER = os.path.join(ROOT, "include", "at_grpo.h")


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("compiler,std", [("gcc", "-std=c99"), ("gcc", "-std=c11"), ("g++", "-std=c++17")])
def test_header_is_valid_c_and_cxx(tmp_path, compiler, std):
    src = tmp_path / ("t.c" if compiler == "gcc" else "t.cpp")
    src.write_text('#include "at_grpo.h"\nint main(void) { at_grpo_batch b; at_grpo_adam a; (void)b; (void)a; '
                   'return (int)sizeof(at_grpo_batch) == 0; }\n')
    subprocess.run([compiler, std, "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only",
                    "-I", os.path.dirname(HEADER), str(src)], check=True)


def test_struct_layout_of_the_binding_matches_the_c_compiler(tmp_path):
    """sizeof and every field offset of at_grpo_batch / at_grpo_adam as gcc lays them out against the
    ctypes mirrors the Python binding passes."""
    fields_b = [f[0] for f in api._Batch._fields_]
    fields_a = [f[0] for f in api._Adam._fields_]
    lines = ['#include <stddef.h>', '#include <stdio.h>', '#include "at_grpo.h"', 'int main(void) {',
             '  printf("%zu\\n", sizeof(at_grpo_batch));']
    lines += [f'  printf("%zu\\n", offsetof(at_grpo_batch, {f}));' for f in fields_b]
    lines += ['  printf("%zu\\n", sizeof(at_grpo_adam));']
    lines += [f'  printf("%zu\\n", offsetof(at_grpo_adam, {f}));' for f in fields_a]
    lines += ['  return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines) + "\n")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-I", os.path.dirname(HEADER), str(src), "-o", str(exe)], check=True)
    got = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    want = [api.C.sizeof(api._Batch)] + [getattr(api._Batch, f).offset for f in fields_b]
    want += [api.C.sizeof(api._Adam)] + [getattr(api._Adam, f).offset for f in fields_a]
    assert got == want


def read_sections(path):
    scalars, arrays, cur = {}, {}, None
    for line in open(path):
        parts = line.split()
        if len(parts) == 2:
            scalars[parts[0]] = parts[1]
            cur = None
        elif len(parts) == 1 and not (parts[0][0].isdigit() or parts[0][0] in "-+" or parts[0].startswith("0x")
                                      or parts[0] in ("inf", "nan")):
            cur = parts[0]
            arrays[cur] = []
        elif len(parts) == 1:
            arrays[cur].append(parts[0])
    return scalars, arrays


def hexf(x):
    return float(np.float32(x)).hex()


@pytest.mark.gpu
def test_c_client_group_advantage(gpu_device, tmp_path):
    assert os.path.exists(CLIENT), "run python -m paper_2510_11062_amd.build first"
    cfg = synth.CONFIGS["C2"]
    st = synth.make_structure(cfg)
    inp, outp = tmp_path / "ga_in.txt", tmp_path / "ga_out.txt"
    with open(inp, "w") as f:
        f.write(f"group_advantage {cfg.n_resp} {cfg.E} {cfg.N} {cfg.T} {hexf(1e-6)} 0 0\n")
        for r in range(cfg.n_resp):
            f.write(f"{st.env_id[r]} {st.agent_id[r]} {st.turn_id[r]} {hexf(st.reward[r])}\n")
    say("[c client] group_advantage")
    subprocess.run([CLIENT, str(inp), str(outp)], check=True, timeout=120)
    sc, ar = read_sections(outp)
    assert int(sc["error_word"]) == 0 and int(sc["version"]) == api.at_grpo_version()
    key = orc.group_key(st.env_id, st.agent_id, st.turn_id, cfg.N, cfg.T)
    gid, G, offs, perm = orc.group_segments(key)
    adv, mean, std = orc.group_advantage(st.reward, gid, G)
    assert int(sc["n_groups"]) == G
    assert np.array_equal(np.array(ar["group_id"], dtype=np.int64), gid)
    assert np.array_equal(np.array(ar["perm"], dtype=np.int64), perm)
    assert np.array_equal(np.array(ar["seg_offsets"], dtype=np.int64), offs)
    got = np.array([float.fromhex(x) for x in ar["adv"]])
    assert np.allclose(got, adv, rtol=1e-4, atol=1e-6)
    assert np.allclose([float.fromhex(x) for x in ar["group_mean"]], mean, rtol=1e-4, atol=1e-7)
    assert np.allclose([float.fromhex(x) for x in ar["group_std"]], std, rtol=1e-4, atol=1e-7)
    # the Python binding drives the same library: identical bits
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(gpu_device)
    py = api.at_grpo_group_advantage(i32(st.env_id), i32(st.agent_id), i32(st.turn_id),
                                     torch.from_numpy(st.reward).to(gpu_device), cfg.E, cfg.N, cfg.T)
    torch.cuda.synchronize()
    assert np.array_equal(got.astype(np.float32).view(np.uint32), host(py["adv"]).view(np.uint32))


@pytest.mark.gpu
def test_c_client_policy_loss_fwd(gpu_device, tmp_path):
    assert os.path.exists(CLIENT), "run python -m paper_2510_11062_amd.build first"
    cfg = synth.CONFIGS["C1"]
    c = helpers.build_case(cfg)
    st = c.st
    ref = helpers.oracle_fwd(c)
    inp, outp = tmp_path / "fwd_in.txt", tmp_path / "fwd_out.txt"
    with open(inp, "w") as f:
        f.write(f"policy_loss_fwd {cfg.H} {cfg.V} {st.n_tok} {cfg.n_resp} {hexf(cfg.eps_clip)} {hexf(cfg.eps_clip)} 0\n")
        f.write(" ".join(str(int(x)) for x in st.cu_seqlens) + "\n")
        f.write(" ".join(hexf(x) for x in c.adv) + "\n")
        for t in range(st.n_tok):
            f.write(f"{int(c.token_id[t])} {hexf(c.old_logp[t])}\n")
        f.write("\n".join(" ".join(hexf(x) for x in row) for row in c.hidden) + "\n")
        f.write("\n".join(" ".join(hexf(x) for x in row) for row in c.W[0]) + "\n")
    say(f"[c client] policy_loss_fwd n_tok={st.n_tok}")
    subprocess.run([CLIENT, str(inp), str(outp)], check=True, timeout=120)
    sc, ar = read_sections(outp)
    assert int(sc["error_word"]) == 0
    assert int(sc["n_valid"]) == int(ref["n_valid"][0])
    loss = float.fromhex(sc["loss"])
    assert abs(loss - ref["loss"][0]) <= 1e-4 * abs(ref["loss"][0]) + 1e-6
    logp = np.array([float.fromhex(x) for x in ar["logp"]])
    assert (np.abs(logp - ref["logp"]) / np.maximum(np.abs(ref["logp"]), 1.0)).max() <= 1e-4
    dc = DeviceCase(c, gpu_device)
    py = api.at_grpo_policy_loss_fwd(dc.batch(), dc.old_logp, dc.adv, cfg.eps_clip, cfg.eps_clip)
    torch.cuda.synchronize()
    assert np.array_equal(logp.astype(np.float32).view(np.uint32), host(py["logp"]).view(np.uint32))
    assert np.array_equal(np.array(ar["clip_mask"], dtype=np.uint8), host(py["clip_mask"]))
    assert np.float32(loss).view(np.uint32) == host(py["loss"]).view(np.uint32)[0]
