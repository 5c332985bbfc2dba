"""Thin Python binding of libat_grpo.so: argument marshalling only.

Every function has the name of the C entry point it calls (see include/at_grpo.h) and takes
torch tensors that already live on the GPU; outputs and the workspace are allocated here with
torch (device memory plumbing) and everything is enqueued on torch's current stream.  There is
no fallback: if the HIP library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libat_grpo.so")
_lib = None

AGG = {"token_mean": 0, "seq_mean_token_mean": 1}
NORM = {"std": 0, "none": 1}
GROUP_BY = {"agent_turn": 0, "trajectory": 1, "parallel": 2}
CALL_GROUP_ADVANTAGE, CALL_TOKEN_LOGPROB, CALL_POLICY_LOSS_FWD, CALL_POLICY_LOSS_BWD, CALL_SURROGATE, \
    CALL_HEAD_UPDATE, CALL_DIAGNOSTICS, CALL_TOKEN_ENTROPY, CALL_POLICY_LOSS_FWD_BWD = range(9)
DTYPE = {torch.float32: 0, torch.bfloat16: 1}

EXPORTS = [
    "at_grpo_group_advantage", "at_grpo_group_advantage_mixed", "at_grpo_group_advantage_static",
    "at_grpo_group_advantage_keyed", "at_grpo_group_advantage_keyed_workspace_bytes",
    "at_grpo_static_scratch_bytes", "at_grpo_token_logprob", "at_grpo_surrogate_from_logp",
    "at_grpo_surrogate_diagnostics", "at_grpo_token_entropy",
    "at_grpo_policy_loss_fwd", "at_grpo_policy_loss_bwd", "at_grpo_policy_loss_fwd_bwd", "at_grpo_head_update", "at_grpo_workspace_bytes",
    "at_grpo_status_string", "at_grpo_version", "at_grpo_profile_enable", "at_grpo_profile_classes",
    "at_grpo_profile_read",
]


class AtGrpoError(RuntimeError):
    pass


class _Adam(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("max_grad_norm", C.c_float), ("step", C.c_int32),
                ("decoupled", C.c_int32)]


class _Batch(C.Structure):
    _fields_ = [
        ("dtype", C.c_int32), ("H", C.c_int32), ("V", C.c_int32), ("n_heads", C.c_int32),
        ("n_tok", C.c_int64), ("n_resp", C.c_int32), ("n_agent", C.c_int32),
        ("cu_seqlens", C.c_void_p), ("hidden", C.c_void_p), ("W", C.POINTER(C.c_void_p)),
        ("token_id", C.c_void_p), ("mask", C.c_void_p), ("resp_agent", C.c_void_p),
        ("head_of_agent", C.c_void_p),
    ]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libat_grpo.so (built in-tree by paper_2510_11062_amd.build); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise AtGrpoError(f"{_LIB_PATH} is missing: run `python -m paper_2510_11062_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, f32, sz = C.c_void_p, C.c_int32, C.c_float, C.c_size_t
    lib.at_grpo_group_advantage.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, f32, i32, i32,
                                            vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.at_grpo_group_advantage.restype = C.c_int
    lib.at_grpo_group_advantage_mixed.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, vp, f32, f32, i32, i32,
                                                  vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.at_grpo_group_advantage_mixed.restype = C.c_int
    lib.at_grpo_group_advantage_keyed.argtypes = [i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, f32, i32, i32,
                                                  vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.at_grpo_group_advantage_keyed.restype = C.c_int
    lib.at_grpo_group_advantage_keyed_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, i32]
    lib.at_grpo_group_advantage_keyed_workspace_bytes.restype = sz
    lib.at_grpo_group_advantage_static.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, f32, i32, i32,
                                                   vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.at_grpo_group_advantage_static.restype = C.c_int
    lib.at_grpo_static_scratch_bytes.argtypes = []
    lib.at_grpo_static_scratch_bytes.restype = sz
    lib.at_grpo_token_logprob.argtypes = [C.POINTER(_Batch), vp, vp, vp, sz, vp]
    lib.at_grpo_token_logprob.restype = C.c_int
    lib.at_grpo_surrogate_from_logp.argtypes = [C.POINTER(_Batch), vp, vp, vp, f32, f32, i32, vp, vp, vp,
                                                vp, sz, vp]
    lib.at_grpo_surrogate_from_logp.restype = C.c_int
    lib.at_grpo_token_entropy.argtypes = [C.POINTER(_Batch), vp, vp, vp, vp, sz, vp]
    lib.at_grpo_token_entropy.restype = C.c_int
    lib.at_grpo_surrogate_diagnostics.argtypes = [C.POINTER(_Batch), vp, vp, vp, f32, f32, vp, vp, vp, sz, vp]
    lib.at_grpo_surrogate_diagnostics.restype = C.c_int
    lib.at_grpo_policy_loss_fwd.argtypes = [C.POINTER(_Batch), vp, vp, f32, f32, i32, vp, vp, vp, vp, vp,
                                            vp, sz, vp]
    lib.at_grpo_policy_loss_fwd.restype = C.c_int
    lib.at_grpo_head_update.argtypes = [i32, i32, i32, i32, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                        C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                        C.POINTER(_Adam), vp, vp, sz, vp]
    lib.at_grpo_head_update.restype = C.c_int
    lib.at_grpo_policy_loss_bwd.argtypes = [C.POINTER(_Batch), vp, vp, vp, vp, f32, f32, i32, vp, vp,
                                            C.POINTER(C.c_void_p), i32, vp, sz, vp]
    lib.at_grpo_policy_loss_bwd.restype = C.c_int
    lib.at_grpo_policy_loss_fwd_bwd.argtypes = [C.POINTER(_Batch), vp, vp, f32, f32, i32, vp, vp, vp, vp, vp, vp,
                                                vp, C.POINTER(C.c_void_p), i32, vp, sz, vp]
    lib.at_grpo_policy_loss_fwd_bwd.restype = C.c_int
    lib.at_grpo_workspace_bytes.argtypes = [i32, C.POINTER(_Batch), i32, i32, i32, i32]
    lib.at_grpo_workspace_bytes.restype = sz
    lib.at_grpo_status_string.argtypes = [i32]
    lib.at_grpo_status_string.restype = C.c_char_p
    lib.at_grpo_version.restype = i32
    lib.at_grpo_profile_enable.argtypes = [i32]
    lib.at_grpo_profile_classes.restype = i32
    lib.at_grpo_profile_read.argtypes = [i32, C.POINTER(C.c_char_p), C.POINTER(C.c_int64),
                                         C.POINTER(C.c_double)]
    _lib = lib
    return lib


def _check(status: int, what: str):
    if status != 0:
        msg = load_library().at_grpo_status_string(status).decode()
        raise AtGrpoError(f"{what} failed: {msg} (status {status})")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev_check(*tensors):
    for t in tensors:
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise AtGrpoError("tensors must be contiguous CUDA/HIP tensors")


_workspace_cache = {}
_workspace_retired = []


def _workspace(nbytes: int, device) -> torch.Tensor:
    """A cached scratch tensor per (device, stream), grown on demand.

    Calls on different streams never share scratch (nothing orders them).  A workspace that is outgrown
    is kept alive until release_workspace(): a HIP graph captured earlier holds its raw pointer, and a
    replay must not find that memory handed to somebody else."""
    key = (str(device), int(torch.cuda.current_stream(device).cuda_stream))
    ws = _workspace_cache.get(key)
    if ws is None or ws.numel() < nbytes:
        if ws is not None:
            _workspace_retired.append(ws)
        ws = torch.empty(int(nbytes), dtype=torch.uint8, device=device)
        _workspace_cache[key] = ws
    return ws


def release_workspace():
    """Drops every cached workspace (only when no captured graph that used the binding will be replayed)."""
    _workspace_cache.clear()
    _workspace_retired.clear()


def _i32_check(**tensors):
    for name, t in tensors.items():
        if t is not None and t.dtype != torch.int32:
            raise AtGrpoError(f"{name} must be int32, got {t.dtype}")


def _f32_check(**tensors):
    for name, t in tensors.items():
        if t is not None and t.dtype != torch.float32:
            raise AtGrpoError(f"{name} must be float32, got {t.dtype}")


@dataclass
class Batch:
    """Python-side mirror of at_grpo_batch; keeps the tensors alive."""
    hidden: Optional[torch.Tensor]
    W: Optional[Sequence[torch.Tensor]]
    token_id: Optional[torch.Tensor]
    cu_seqlens: torch.Tensor
    mask: Optional[torch.Tensor] = None
    resp_agent: Optional[torch.Tensor] = None
    head_of_agent: Optional[torch.Tensor] = None
    n_tok: Optional[int] = None
    V: Optional[int] = None
    n_heads: Optional[int] = None

    def to_c(self):
        _dev_check(self.hidden, self.token_id, self.cu_seqlens, self.mask, self.resp_agent, self.head_of_agent)
        b = _Batch()
        if self.hidden is not None:
            if self.hidden.dtype == torch.float32:
                b.dtype = 0
            elif self.hidden.dtype == torch.bfloat16:
                b.dtype = 1
            else:
                raise AtGrpoError("hidden must be float32 or bfloat16")
            b.H = self.hidden.shape[1]
            n_tok = self.hidden.shape[0]
        else:
            b.dtype, b.H = 0, 0
            n_tok = self.n_tok
        heads = list(self.W) if self.W is not None else []
        for w in heads:
            _dev_check(w)
            if w.dtype != self.hidden.dtype or w.shape[1] != b.H:
                raise AtGrpoError("every head must have hidden's dtype and H columns")
        b.V = heads[0].shape[0] if heads else int(self.V)
        b.n_heads = len(heads) if heads else int(self.n_heads or 1)
        b.n_tok = int(n_tok)
        if self.cu_seqlens.dtype != torch.int64:
            raise AtGrpoError("cu_seqlens must be int64")
        b.n_resp = self.cu_seqlens.numel() - 1
        b.n_agent = 0 if self.head_of_agent is None else self.head_of_agent.numel()
        b.cu_seqlens = self.cu_seqlens.data_ptr()
        b.hidden = 0 if self.hidden is None else self.hidden.data_ptr()
        self._w_array = (C.c_void_p * max(len(heads), 1))(*[w.data_ptr() for w in heads])
        b.W = C.cast(self._w_array, C.POINTER(C.c_void_p)) if heads else None
        for name, dt in (("token_id", torch.int32), ("mask", torch.uint8), ("resp_agent", torch.int32),
                         ("head_of_agent", torch.int32)):
            t = getattr(self, name)
            if t is not None and t.dtype != dt:
                raise AtGrpoError(f"{name} must be {dt}")
            setattr(b, name, 0 if t is None else t.data_ptr())
        return b


def at_grpo_workspace_bytes(call: int, batch: Optional[Batch] = None, n_resp=0, n_env=0, n_agent=0, n_turn=0) -> int:
    lib = load_library()
    cb = batch.to_c() if batch is not None else None
    return int(lib.at_grpo_workspace_bytes(call, C.byref(cb) if cb is not None else None,
                                           n_resp, n_env, n_agent, n_turn))


def at_grpo_group_advantage(env_id, agent_id, turn_id, reward, n_env: int, n_agent: int, n_turn: int,
                            eps_std: float = 1e-6, ddof: int = 0, norm: str = "std", want_stats: bool = True):
    """Returns dict(group_id, n_groups, seg_offsets, perm, adv, group_mean, group_std, workspace)."""
    lib = load_library()
    _dev_check(env_id, agent_id, turn_id, reward)
    _f32_check(reward=reward)
    _i32_check(env_id=env_id, agent_id=agent_id, turn_id=turn_id)
    dev = reward.device
    R = reward.numel()
    n_keys = n_env * n_agent * n_turn
    gmax = min(R, n_keys)
    out = dict(
        group_id=torch.empty(R, dtype=torch.int32, device=dev),
        n_groups=torch.zeros(1, dtype=torch.int32, device=dev),
        seg_offsets=torch.zeros(gmax + 1, dtype=torch.int32, device=dev),
        perm=torch.zeros(R, dtype=torch.int32, device=dev),
        adv=torch.empty(R, dtype=torch.float32, device=dev),
        group_mean=torch.zeros(gmax, dtype=torch.float32, device=dev) if want_stats else None,
        group_std=torch.zeros(gmax, dtype=torch.float32, device=dev) if want_stats else None,
    )
    nbytes = lib.at_grpo_workspace_bytes(CALL_GROUP_ADVANTAGE, None, R, n_env, n_agent, n_turn)
    if nbytes == 0:
        raise AtGrpoError("at_grpo_workspace_bytes rejected the id extents")
    ws = _workspace(nbytes, dev)
    st = lib.at_grpo_group_advantage(R, n_env, n_agent, n_turn, _ptr(env_id), _ptr(agent_id), _ptr(turn_id),
                                     _ptr(reward), eps_std, ddof, NORM[norm], _ptr(out["group_id"]),
                                     _ptr(out["n_groups"]), _ptr(out["seg_offsets"]), _ptr(out["perm"]),
                                     _ptr(out["adv"]), _ptr(out["group_mean"]), _ptr(out["group_std"]),
                                     _ptr(ws), ws.numel(), _stream())
    _check(st, "at_grpo_group_advantage")
    out["workspace"] = ws
    return out


def group_advantage_outputs(R: int, n_keys: int, dev, want_stats: bool = True):
    """Output tensors of a grouping call (allocated by the caller, never by the library)."""
    gmax = min(R, n_keys)
    return dict(
        group_id=torch.empty(R, dtype=torch.int32, device=dev),
        n_groups=torch.zeros(1, dtype=torch.int32, device=dev),
        seg_offsets=torch.zeros(gmax + 1, dtype=torch.int32, device=dev),
        perm=torch.zeros(R, dtype=torch.int32, device=dev),
        adv=torch.empty(R, dtype=torch.float32, device=dev),
        group_mean=torch.zeros(gmax, dtype=torch.float32, device=dev) if want_stats else None,
        group_std=torch.zeros(gmax, dtype=torch.float32, device=dev) if want_stats else None,
        data_error=torch.zeros(1, dtype=torch.int32, device=dev),
    )


def at_grpo_group_advantage_keyed(group_by: str, env_id, agent_id, turn_id, reward, n_env: int, n_agent: int,
                                  n_turn: int, sample_id=None, n_sample: int = 1, eps_std: float = 1e-6,
                                  ddof: int = 0, norm: str = "std"):
    """at_grpo_group_advantage under the grouping `group_by` ("agent_turn", "trajectory", "parallel")."""
    lib = load_library()
    _dev_check(env_id, agent_id, turn_id, reward, sample_id)
    _f32_check(reward=reward)
    _i32_check(env_id=env_id, agent_id=agent_id, turn_id=turn_id, sample_id=sample_id)
    R = reward.numel()
    mode = GROUP_BY[group_by]
    n_keys = n_env if mode == 1 else n_env * n_agent * n_turn * (n_sample if mode == 2 else 1)
    out = group_advantage_outputs(R, n_keys, reward.device)
    nbytes = lib.at_grpo_group_advantage_keyed_workspace_bytes(mode, R, n_env, n_agent, n_turn, n_sample)
    if nbytes == 0:
        raise AtGrpoError("at_grpo_group_advantage_keyed_workspace_bytes rejected the extents")
    ws = _workspace(nbytes, reward.device)
    st = lib.at_grpo_group_advantage_keyed(mode, R, n_env, n_agent, n_turn, n_sample, _ptr(env_id), _ptr(agent_id),
                                           _ptr(turn_id), _ptr(sample_id), _ptr(reward), eps_std, ddof, NORM[norm],
                                           _ptr(out["group_id"]), _ptr(out["n_groups"]), _ptr(out["seg_offsets"]),
                                           _ptr(out["perm"]), _ptr(out["adv"]), _ptr(out["group_mean"]),
                                           _ptr(out["group_std"]), _ptr(ws), ws.numel(), _stream())
    _check(st, "at_grpo_group_advantage_keyed")
    out["workspace"] = ws
    return out


def at_grpo_static_scratch_bytes() -> int:
    return int(load_library().at_grpo_static_scratch_bytes())


def at_grpo_group_advantage_static(env_id, agent_id, turn_id, reward, n_env: int, n_agent: int, n_turn: int,
                                   eps_std: float = 1e-6, ddof: int = 0, norm: str = "std",
                                   out: Optional[dict] = None):
    """at_grpo_group_advantage on the library's own fixed scratch array: no workspace is passed and the
    call allocates nothing (pass `out` from group_advantage_outputs to keep the binding from allocating
    either).  Returns the dict of outputs, data_error[1] holding the call's error word."""
    lib = load_library()
    _dev_check(env_id, agent_id, turn_id, reward)
    _f32_check(reward=reward)
    _i32_check(env_id=env_id, agent_id=agent_id, turn_id=turn_id)
    R = reward.numel()
    if out is None:
        out = group_advantage_outputs(R, n_env * n_agent * n_turn, reward.device)
    st = lib.at_grpo_group_advantage_static(R, n_env, n_agent, n_turn, _ptr(env_id), _ptr(agent_id), _ptr(turn_id),
                                            _ptr(reward), eps_std, ddof, NORM[norm], _ptr(out["group_id"]),
                                            _ptr(out["n_groups"]), _ptr(out["seg_offsets"]), _ptr(out["perm"]),
                                            _ptr(out["adv"]), _ptr(out.get("group_mean")), _ptr(out.get("group_std")),
                                            _ptr(out.get("data_error")), _stream())
    _check(st, "at_grpo_group_advantage_static")
    return out


def at_grpo_group_advantage_mixed(env_id, agent_id, turn_id, r_team, r_loc, alpha: float, n_env: int,
                                  n_agent: int, n_turn: int, eps_std: float = 1e-6, ddof: int = 0,
                                  norm: str = "std", want_stats: bool = True, want_best: bool = True):
    """Eq. (3) mixing in front of at_grpo_group_advantage, plus the per-group arg max.

    Returns the dict of at_grpo_group_advantage extended by reward[R] and best[min(R, keys)]."""
    lib = load_library()
    _dev_check(env_id, agent_id, turn_id, r_team, r_loc)
    _f32_check(r_team=r_team, r_loc=r_loc)
    _i32_check(env_id=env_id, agent_id=agent_id, turn_id=turn_id)
    dev = r_team.device
    R = r_team.numel()
    n_keys = n_env * n_agent * n_turn
    gmax = min(R, n_keys)
    out = dict(
        reward=torch.empty(R, dtype=torch.float32, device=dev),
        group_id=torch.empty(R, dtype=torch.int32, device=dev),
        n_groups=torch.zeros(1, dtype=torch.int32, device=dev),
        seg_offsets=torch.zeros(gmax + 1, dtype=torch.int32, device=dev),
        perm=torch.zeros(R, dtype=torch.int32, device=dev),
        adv=torch.empty(R, dtype=torch.float32, device=dev),
        group_mean=torch.zeros(gmax, dtype=torch.float32, device=dev) if want_stats else None,
        group_std=torch.zeros(gmax, dtype=torch.float32, device=dev) if want_stats else None,
        best=torch.full((gmax,), -1, dtype=torch.int32, device=dev) if want_best else None,
    )
    nbytes = lib.at_grpo_workspace_bytes(CALL_GROUP_ADVANTAGE, None, R, n_env, n_agent, n_turn)
    if nbytes == 0:
        raise AtGrpoError("at_grpo_workspace_bytes rejected the id extents")
    ws = _workspace(nbytes, dev)
    st = lib.at_grpo_group_advantage_mixed(R, n_env, n_agent, n_turn, _ptr(env_id), _ptr(agent_id),
                                           _ptr(turn_id), _ptr(r_team), _ptr(r_loc), alpha, eps_std, ddof,
                                           NORM[norm], _ptr(out["reward"]), _ptr(out["group_id"]),
                                           _ptr(out["n_groups"]), _ptr(out["seg_offsets"]), _ptr(out["perm"]),
                                           _ptr(out["adv"]), _ptr(out["group_mean"]), _ptr(out["group_std"]),
                                           _ptr(out["best"]), _ptr(ws), ws.numel(), _stream())
    _check(st, "at_grpo_group_advantage_mixed")
    out["workspace"] = ws
    return out


def at_grpo_head_update(W, dW, m, v, step: int, W_master=None, lr: float = 1e-6, beta1: float = 0.9,
                        beta2: float = 0.999, eps: float = 1e-8, weight_decay: float = 0.01,
                        max_grad_norm: float = 1.0, decoupled: bool = True):
    """Clip by the joint gradient norm, then one Adam step per head, in place on W / W_master / m / v.

    W, dW, m, v (and W_master for bf16 heads) are lists of [V, H] tensors.  Returns
    dict(grad_norm=tensor[2] (norm, factor), workspace)."""
    lib = load_library()
    n_heads = len(W)
    _dev_check(*W, *dW, *m, *v, *(W_master or []))
    V, H = W[0].shape
    dtype = DTYPE[W[0].dtype]
    dev = W[0].device

    def arr(ts):
        return (C.c_void_p * n_heads)(*[t.data_ptr() for t in ts])

    masters = arr(W_master) if W_master is not None else None
    opt = _Adam(lr, beta1, beta2, eps, weight_decay, max_grad_norm, step, 1 if decoupled else 0)
    grad_norm = torch.zeros(2, dtype=torch.float32, device=dev)
    ws = _workspace(lib.at_grpo_workspace_bytes(CALL_HEAD_UPDATE, None, 0, 0, 0, 0), dev)
    st = lib.at_grpo_head_update(dtype, H, V, n_heads, arr(W), masters, arr(dW), arr(m), arr(v), C.byref(opt),
                                 _ptr(grad_norm), _ptr(ws), ws.numel(), _stream())
    _check(st, "at_grpo_head_update")
    return dict(grad_norm=grad_norm, workspace=ws)


def at_grpo_token_logprob(batch: Batch, want_lse: bool = True):
    lib = load_library()
    cb = batch.to_c()
    dev = batch.hidden.device
    logp = torch.empty(cb.n_tok, dtype=torch.float32, device=dev)
    lse = torch.empty(cb.n_tok, dtype=torch.float32, device=dev) if want_lse else None
    ws = _workspace(lib.at_grpo_workspace_bytes(CALL_TOKEN_LOGPROB, C.byref(cb), 0, 0, 0, 0), dev)
    st = lib.at_grpo_token_logprob(C.byref(cb), _ptr(logp), _ptr(lse), _ptr(ws), ws.numel(), _stream())
    _check(st, "at_grpo_token_logprob")
    return dict(logp=logp, lse=lse, workspace=ws)


def at_grpo_token_entropy(batch: Batch):
    """logp, lse and the entropy of the next-token distribution at every participating row."""
    lib = load_library()
    cb = batch.to_c()
    dev = batch.hidden.device
    logp = torch.empty(cb.n_tok, dtype=torch.float32, device=dev)
    lse = torch.empty(cb.n_tok, dtype=torch.float32, device=dev)
    entropy = torch.empty(cb.n_tok, dtype=torch.float32, device=dev)
    ws = _workspace(lib.at_grpo_workspace_bytes(CALL_TOKEN_ENTROPY, C.byref(cb), 0, 0, 0, 0), dev)
    st = lib.at_grpo_token_entropy(C.byref(cb), _ptr(logp), _ptr(lse), _ptr(entropy), _ptr(ws), ws.numel(), _stream())
    _check(st, "at_grpo_token_entropy")
    return dict(logp=logp, lse=lse, entropy=entropy, workspace=ws)


def at_grpo_surrogate_from_logp(batch: Batch, logp, old_logp, adv, eps_low: float, eps_high: float,
                                agg: str = "token_mean"):
    lib = load_library()
    cb = batch.to_c()
    _dev_check(logp, old_logp, adv)
    _f32_check(logp=logp, old_logp=old_logp, adv=adv)
    dev = logp.device
    loss = torch.empty(cb.n_heads, dtype=torch.float32, device=dev)
    clip_mask = torch.empty(cb.n_tok, dtype=torch.uint8, device=dev)
    n_valid = torch.empty(cb.n_heads, dtype=torch.int32, device=dev)
    ws = _workspace(lib.at_grpo_workspace_bytes(CALL_SURROGATE, C.byref(cb), 0, 0, 0, 0), dev)
    st = lib.at_grpo_surrogate_from_logp(C.byref(cb), _ptr(logp), _ptr(old_logp), _ptr(adv), eps_low, eps_high,
                                         AGG[agg], _ptr(loss), _ptr(clip_mask), _ptr(n_valid), _ptr(ws),
                                         ws.numel(), _stream())
    _check(st, "at_grpo_surrogate_from_logp")
    return dict(loss=loss, clip_mask=clip_mask, n_valid=n_valid, workspace=ws)


def at_grpo_surrogate_diagnostics(batch: Batch, logp, old_logp, adv, eps_low: float, eps_high: float):
    """Returns dict(counts int32[n_heads, 4] (rows, below, above, zero-gradient),
    stats float32[n_heads, 2] (KL estimate, mean ratio), workspace)."""
    lib = load_library()
    cb = batch.to_c()
    _dev_check(logp, old_logp, adv)
    _f32_check(logp=logp, old_logp=old_logp, adv=adv)
    dev = logp.device
    counts = torch.empty((cb.n_heads, 4), dtype=torch.int32, device=dev)
    stats = torch.empty((cb.n_heads, 2), dtype=torch.float32, device=dev)
    ws = _workspace(lib.at_grpo_workspace_bytes(CALL_DIAGNOSTICS, C.byref(cb), 0, 0, 0, 0), dev)
    st = lib.at_grpo_surrogate_diagnostics(C.byref(cb), _ptr(logp), _ptr(old_logp), _ptr(adv), eps_low, eps_high,
                                           _ptr(counts), _ptr(stats), _ptr(ws), ws.numel(), _stream())
    _check(st, "at_grpo_surrogate_diagnostics")
    return dict(counts=counts, stats=stats, workspace=ws)


def at_grpo_policy_loss_fwd(batch: Batch, old_logp, adv, eps_low: float, eps_high: float,
                            agg: str = "token_mean", out: Optional[dict] = None):
    lib = load_library()
    cb = batch.to_c()
    _dev_check(old_logp, adv)
    _f32_check(old_logp=old_logp, adv=adv)
    dev = batch.hidden.device
    if out is None:
        out = dict(
            loss=torch.empty(cb.n_heads, dtype=torch.float32, device=dev),
            logp=torch.empty(cb.n_tok, dtype=torch.float32, device=dev),
            lse=torch.empty(cb.n_tok, dtype=torch.float32, device=dev),
            clip_mask=torch.empty(cb.n_tok, dtype=torch.uint8, device=dev),
            n_valid=torch.empty(cb.n_heads, dtype=torch.int32, device=dev),
        )
    ws = _workspace(lib.at_grpo_workspace_bytes(CALL_POLICY_LOSS_FWD, C.byref(cb), 0, 0, 0, 0), dev)
    st = lib.at_grpo_policy_loss_fwd(C.byref(cb), _ptr(old_logp), _ptr(adv), eps_low, eps_high, AGG[agg],
                                     _ptr(out["loss"]), _ptr(out["logp"]), _ptr(out["lse"]),
                                     _ptr(out["clip_mask"]), _ptr(out["n_valid"]), _ptr(ws), ws.numel(),
                                     _stream())
    _check(st, "at_grpo_policy_loss_fwd")
    out["workspace"] = ws
    return out


def at_grpo_policy_loss_bwd(batch: Batch, old_logp, adv, logp, lse, eps_low: float, eps_high: float,
                            agg: str = "token_mean", grad_loss=None, dW: Optional[List[torch.Tensor]] = None,
                            accumulate_dW: bool = False, d_hidden: Optional[torch.Tensor] = None):
    lib = load_library()
    cb = batch.to_c()
    _dev_check(old_logp, adv, logp, lse, grad_loss, d_hidden)
    _f32_check(old_logp=old_logp, adv=adv, logp=logp, lse=lse, grad_loss=grad_loss)
    if d_hidden is not None and (d_hidden.dtype != batch.hidden.dtype or d_hidden.shape != batch.hidden.shape):
        raise AtGrpoError("d_hidden must have hidden's dtype and shape")
    dev = batch.hidden.device
    if d_hidden is None:
        d_hidden = torch.empty_like(batch.hidden)
    if dW is None:
        if accumulate_dW:
            raise AtGrpoError("accumulate_dW needs dW tensors")
        dW = [torch.empty(w.shape, dtype=torch.float32, device=dev) for w in batch.W]
    for g in dW:
        _dev_check(g)
        if g.dtype != torch.float32:
            raise AtGrpoError("dW must be float32")
    dw_array = (C.c_void_p * len(dW))(*[g.data_ptr() for g in dW])
    ws = _workspace(lib.at_grpo_workspace_bytes(CALL_POLICY_LOSS_BWD, C.byref(cb), 0, 0, 0, 0), dev)
    st = lib.at_grpo_policy_loss_bwd(C.byref(cb), _ptr(old_logp), _ptr(adv), _ptr(logp), _ptr(lse), eps_low,
                                     eps_high, AGG[agg], _ptr(grad_loss), _ptr(d_hidden),
                                     C.cast(dw_array, C.POINTER(C.c_void_p)), 1 if accumulate_dW else 0,
                                     _ptr(ws), ws.numel(), _stream())
    _check(st, "at_grpo_policy_loss_bwd")
    return dict(d_hidden=d_hidden, dW=dW, workspace=ws)


def at_grpo_policy_loss_fwd_bwd(batch: Batch, old_logp, adv, eps_low: float, eps_high: float,
                                agg: str = "token_mean", grad_loss=None, dW: Optional[List[torch.Tensor]] = None,
                                accumulate_dW: bool = False, d_hidden: Optional[torch.Tensor] = None,
                                out: Optional[dict] = None):
    """Forward and backward of the policy loss from one pass over the logits; returns the outputs of both."""
    lib = load_library()
    cb = batch.to_c()
    _dev_check(old_logp, adv, grad_loss, d_hidden)
    _f32_check(old_logp=old_logp, adv=adv, grad_loss=grad_loss)
    if d_hidden is not None and (d_hidden.dtype != batch.hidden.dtype or d_hidden.shape != batch.hidden.shape):
        raise AtGrpoError("d_hidden must have hidden's dtype and shape")
    dev = batch.hidden.device
    if out is None:
        out = dict(
            loss=torch.empty(cb.n_heads, dtype=torch.float32, device=dev),
            logp=torch.empty(cb.n_tok, dtype=torch.float32, device=dev),
            lse=torch.empty(cb.n_tok, dtype=torch.float32, device=dev),
            clip_mask=torch.empty(cb.n_tok, dtype=torch.uint8, device=dev),
            n_valid=torch.empty(cb.n_heads, dtype=torch.int32, device=dev),
        )
    if d_hidden is None:
        d_hidden = torch.empty_like(batch.hidden)
    if dW is None:
        if accumulate_dW:
            raise AtGrpoError("accumulate_dW needs dW tensors")
        dW = [torch.empty(w.shape, dtype=torch.float32, device=dev) for w in batch.W]
    for g in dW:
        _dev_check(g)
        if g.dtype != torch.float32:
            raise AtGrpoError("dW must be float32")
    dw_array = (C.c_void_p * len(dW))(*[g.data_ptr() for g in dW])
    ws = _workspace(lib.at_grpo_workspace_bytes(CALL_POLICY_LOSS_FWD_BWD, C.byref(cb), 0, 0, 0, 0), dev)
    st = lib.at_grpo_policy_loss_fwd_bwd(C.byref(cb), _ptr(old_logp), _ptr(adv), eps_low, eps_high, AGG[agg],
                                         _ptr(grad_loss), _ptr(out["loss"]), _ptr(out["logp"]), _ptr(out["lse"]),
                                         _ptr(out["clip_mask"]), _ptr(out["n_valid"]), _ptr(d_hidden),
                                         C.cast(dw_array, C.POINTER(C.c_void_p)), 1 if accumulate_dW else 0,
                                         _ptr(ws), ws.numel(), _stream())
    _check(st, "at_grpo_policy_loss_fwd_bwd")
    out.update(d_hidden=d_hidden, dW=dW, workspace=ws)
    return out


def error_word(workspace: torch.Tensor) -> int:
    """Device error word of the last call that used this workspace (synchronises)."""
    return int(workspace[:4].view(torch.int32).item())


def at_grpo_profile_enable(on: bool):
    _check(load_library().at_grpo_profile_enable(1 if on else 0), "at_grpo_profile_enable")


def at_grpo_profile_read():
    """{kernel class: (launches, total_ms)} since profiling was enabled (synchronises)."""
    lib = load_library()
    out = {}
    for k in range(lib.at_grpo_profile_classes()):
        name = C.c_char_p()
        n = C.c_int64()
        ms = C.c_double()
        _check(lib.at_grpo_profile_read(k, C.byref(name), C.byref(n), C.byref(ms)), "at_grpo_profile_read")
        out[name.value.decode()] = (int(n.value), float(ms.value))
    return out


def at_grpo_version() -> int:
    return int(load_library().at_grpo_version())
