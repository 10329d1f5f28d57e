"""ctypes binding of libpg_head.so: same names as the C ABI, argument marshalling only.

Every computation happens in the HIP kernels behind the C entry points.  torch is used
for device memory, data pointers and the current stream.  There is no fallback: if the
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libpg_head.so")

PG_OK = 0
CALL_LOGPROB_FWD = 0
CALL_LOSS_FWD_BWD = 1
CALL_LOSS_FWD_BWD_NORMED = 2
COUNTER_NAMES = ("active", "clip_hi", "clip_lo", "seg_geo", "seg_veto", "truncated", "loss_tokens", "seg_dropped")

EXPORTS = ("pg_last_error", "pg_init", "pg_workspace_bytes", "pg_backward_chunk_rows", "pg_w_transposed_bytes", "trloo_advantage", "pg_logprob_fwd", "pg_loss_fwd_bwd", "pg_loss_fwd_bwd_normed",
           "pg_sft_fwd_bwd", "pg_head_shard_fwd", "pg_head_partials_merge", "pg_head_partials_finish", "pg_loss_shard_bwd", "grpo_advantage",
           "turn_reward", "prs_retain", "pg_monitors_workspace_bytes", "pg_monitors", "pg_monitors_static", "pg_rmsnorm_fwd", "pg_rmsnorm_bwd_workspace_bytes", "pg_rmsnorm_bwd",
           "pg_profile_enable", "pg_profile_read")
MONITOR_NAMES = ("entropy_mean", "ppl_train", "ppl_rollout", "dH_norm", "dW_norm", "n")
KERNEL_CLASSES = ("fwd", "dlogits", "dw", "dh")


class PgParams(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("temperature", C.c_float), ("clip_eps_lo", C.c_float),
                ("clip_eps_hi", C.c_float), ("mismatch_mode", C.c_int32), ("geo_lo", C.c_float),
                ("geo_hi", C.c_float), ("veto_ratio", C.c_float), ("trunc_c", C.c_float),
                ("norm_override", C.c_float), ("accumulate_dW", C.c_int32), ("dW_dtype", C.c_int32),
                ("n_samples", C.c_int32), ("w_transposed", C.c_void_p), ("w_transposed_valid", C.c_int32)]


@dataclass
class Params:
    """Host-side mirror of pg_params (defaults: the paper's thresholds, Sec. 5.1)."""
    dtype: int = 0
    temperature: float = 1.0
    clip_eps_lo: float = 0.2
    clip_eps_hi: float = 0.2
    mismatch_mode: int = 0
    geo_lo: float = 0.999
    geo_hi: float = 1.001
    veto_ratio: float = 1e-4
    trunc_c: float = 2.0
    norm_override: float = 0.0
    accumulate_dW: int = 0
    dW_dtype: int = 0
    n_samples: int = 0       # length of the adv / sample_keep tables; the loss wrappers fill it in
    w_transposed: Optional[torch.Tensor] = None      # optional W^T cache (alloc_w_transposed), loss calls only
    w_transposed_valid: int = 0                      # 1: the cache already holds the transpose of this W

    def c_struct(self) -> PgParams:
        return PgParams(self.dtype, self.temperature, self.clip_eps_lo, self.clip_eps_hi, self.mismatch_mode,
                        self.geo_lo, self.geo_hi, self.veto_ratio, self.trunc_c, self.norm_override,
                        self.accumulate_dW, self.dW_dtype, self.n_samples,
                        None if self.w_transposed is None else C.c_void_p(self.w_transposed.data_ptr()),
                        self.w_transposed_valid)


class PgError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"pg_head error {code}: {msg}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """Loads the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2602_05885_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.pg_last_error.restype = C.c_char_p
        L.pg_last_error.argtypes = []
        L.pg_workspace_bytes.restype = C.c_size_t
        L.pg_workspace_bytes.argtypes = [C.c_int64, C.c_int64, C.c_int64, C.c_int32, C.POINTER(PgParams), C.c_int32]
        L.pg_w_transposed_bytes.restype = C.c_size_t
        L.pg_w_transposed_bytes.argtypes = [C.c_int64, C.c_int64]
        L.pg_backward_chunk_rows.restype = C.c_int64
        L.pg_backward_chunk_rows.argtypes = [C.c_int64, C.c_int64, C.c_int64, C.c_int32, C.POINTER(PgParams)]
        L.trloo_advantage.restype = C.c_int32
        L.trloo_advantage.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_float,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.pg_logprob_fwd.restype = C.c_int32
        L.pg_logprob_fwd.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64,
                                     C.POINTER(PgParams), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_size_t, C.c_void_p]
        L.pg_loss_fwd_bwd.restype = C.c_int32
        L.pg_loss_fwd_bwd.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                                      C.c_int64, C.POINTER(PgParams), C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.pg_loss_fwd_bwd_normed.restype = C.c_int32
        L.pg_loss_fwd_bwd_normed.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                             C.c_int64, C.c_int64, C.POINTER(PgParams), C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.pg_sft_fwd_bwd.restype = C.c_int32
        L.pg_sft_fwd_bwd.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64,
                                     C.POINTER(PgParams), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.pg_head_shard_fwd.restype = C.c_int32
        L.pg_head_shard_fwd.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64,
                                        C.c_int64, C.POINTER(PgParams), C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.pg_head_partials_merge.restype = C.c_int32
        L.pg_head_partials_merge.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.pg_head_partials_finish.restype = C.c_int32
        L.pg_head_partials_finish.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.pg_loss_shard_bwd.restype = C.c_int32
        L.pg_loss_shard_bwd.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                        C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                        C.c_int64, C.c_int64, C.c_int64, C.POINTER(PgParams), C.c_void_p, C.c_void_p,
                                        C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_size_t, C.c_void_p]
        L.grpo_advantage.restype = C.c_int32
        L.grpo_advantage.argtypes = L.trloo_advantage.argtypes
        L.turn_reward.restype = C.c_int32
        L.turn_reward.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_float,
                                  C.c_void_p, C.c_void_p, C.c_void_p]
        L.prs_retain.restype = C.c_int32
        L.prs_retain.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_float, C.c_float, C.c_int32, C.c_uint64,
                                 C.c_void_p, C.c_void_p, C.c_void_p]
        L.pg_monitors_workspace_bytes.restype = C.c_size_t
        L.pg_monitors_workspace_bytes.argtypes = []
        L.pg_monitors.restype = C.c_int32
        L.pg_monitors.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int32,
                                  C.c_int64, C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_size_t,
                                  C.c_void_p]
        L.pg_monitors_static.restype = C.c_int32
        L.pg_monitors_static.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int32,
                                         C.c_int64, C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p]
        L.pg_init.restype = C.c_int32
        L.pg_init.argtypes = []
        L.pg_rmsnorm_fwd.restype = C.c_int32
        L.pg_rmsnorm_fwd.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_float, C.c_int32, C.c_void_p,
                                     C.c_void_p, C.c_void_p]
        L.pg_rmsnorm_bwd_workspace_bytes.restype = C.c_size_t
        L.pg_rmsnorm_bwd_workspace_bytes.argtypes = [C.c_int64]
        L.pg_rmsnorm_bwd.restype = C.c_int32
        L.pg_rmsnorm_bwd.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_float, C.c_int32,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.pg_profile_enable.restype = C.c_int32
        L.pg_profile_enable.argtypes = [C.c_int32, C.c_int32]
        L.pg_profile_read.restype = C.c_int32
        L.pg_profile_read.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        _lib = L
    return _lib


_HEAD_DTYPES = {0: torch.bfloat16, 1: torch.float32}


def _want(name: str, t: Optional[torch.Tensor], dtype, shape=None, device=None, optional=False):
    """Raises ValueError unless `t` is a contiguous tensor of the dtype, shape and device the C ABI will
    assume (the library sees raw pointers and cannot check any of this).  bool counts as uint8."""
    if t is None:
        if optional:
            return
        raise ValueError(f"{name} must not be None")
    if not isinstance(t, torch.Tensor):
        raise ValueError(f"{name} must be a torch.Tensor")
    dtypes = dtype if isinstance(dtype, (tuple, list)) else (dtype,)
    if torch.uint8 in dtypes:
        dtypes = tuple(dtypes) + (torch.bool,)
    if t.dtype not in dtypes:
        raise ValueError(f"{name} has dtype {t.dtype}, the C ABI reads it as {' or '.join(str(x) for x in dtypes)}")
    if shape is not None:
        if tuple(t.shape) != tuple(shape):
            raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    if device is not None and t.device != device:
        raise ValueError(f"{name} is on {t.device}, expected {device}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")


def _want_head(H, W, y, params: "Params", w_name="W"):
    """Checks of the operands every head call takes; returns (T, d, V, device)."""
    if not isinstance(H, torch.Tensor) or H.dim() != 2:
        raise ValueError("H must be a [T, d] tensor")
    if not isinstance(W, torch.Tensor) or W.dim() != 2:
        raise ValueError(f"{w_name} must be a [V, d] tensor")
    if params.dtype not in _HEAD_DTYPES:
        raise ValueError(f"params.dtype must be 0 (bf16) or 1 (fp32), got {params.dtype}")
    if not H.is_cuda:
        raise ValueError(f"H is on {H.device}: the library takes device pointers only")
    T, d = H.shape
    V = W.shape[0]
    dt = _HEAD_DTYPES[params.dtype]
    _want("H", H, dt, (T, d))
    _want(w_name, W, dt, (V, d), H.device)
    _want("y", y, torch.int32, (T,), H.device)
    return T, d, V, H.device


def _want_loss_args(T, dev, loss_mask, cu_seqlens, adv, seg_sample, sample_keep, old_logp, rollout_logp):
    _want("loss_mask", loss_mask, torch.uint8, (T,), dev)
    _want("cu_seqlens", cu_seqlens, torch.int32, None, dev)
    if cu_seqlens.dim() != 1 or cu_seqlens.numel() < 1:
        raise ValueError("cu_seqlens must be a 1-d tensor of S + 1 offsets")
    S = cu_seqlens.numel() - 1
    _want("adv", adv, torch.float64, None, dev)
    if adv.dim() != 1:
        raise ValueError("adv must be a 1-d table (flatten the [P, K, Tmax] advantages)")
    _want("seg_sample", seg_sample, torch.int32, (S,), dev, optional=True)
    if seg_sample is None and adv.numel() < S:
        raise ValueError(f"adv has {adv.numel()} entries for {S} segments and no seg_sample")
    _want("sample_keep", sample_keep, torch.uint8, (adv.numel(),), dev, optional=True)
    _want("old_logp", old_logp, torch.float32, (T,), dev, optional=True)
    _want("rollout_logp", rollout_logp, torch.float32, (T,), dev, optional=True)
    return S


def _want_loss_out(out, T, d, V, dev, dH_dtype, dW, params: "Params"):
    if out is not None:
        loss, dH, logp, ent, counters = out
        _want("out loss", loss, torch.float32, (1,), dev)
        _want("out dH", dH, dH_dtype, (T, d), dev)
        _want("out logp", logp, torch.float32, (T,), dev)
        _want("out entropy", ent, torch.float32, (T,), dev)
        _want("out counters", counters, torch.int64, (8,), dev)
    if params.dW_dtype not in (0, 1):
        raise ValueError("params.dW_dtype must be 0 (fp32) or 1 (bf16)")
    _want("dW", dW, torch.bfloat16 if params.dW_dtype else torch.float32, (V, d), dev, optional=True)


def _want_workspace(ws, dev):
    _want("workspace", ws, torch.uint8, None, dev)


def _want_wt_cache(params: "Params", d, V, dev):
    if params.w_transposed is None:
        return
    _want("params.w_transposed", params.w_transposed, torch.uint8, None, dev)
    need = int(lib().pg_w_transposed_bytes(d, V))
    if need == 0 or params.w_transposed.numel() < need:
        raise ValueError(f"params.w_transposed has {params.w_transposed.numel()} bytes, {need} needed for d={d}, V={V}")


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensors passed to the C ABI must be contiguous")
    return C.c_void_p(t.data_ptr())


def _stream(stream=None):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _check(rc: int):
    if rc != PG_OK:
        raise PgError(rc, lib().pg_last_error().decode())


def pg_last_error() -> str:
    return lib().pg_last_error().decode()


def pg_profile_enable(on: bool, max_launches: int = 0) -> None:
    _check(lib().pg_profile_enable(1 if on else 0, max_launches))


def pg_profile_read():
    """Returns {class: (total_ms, launches)} for the launches recorded since the last read."""
    ms = (C.c_double * len(KERNEL_CLASSES))()
    n = (C.c_int64 * len(KERNEL_CLASSES))()
    _check(lib().pg_profile_read(ms, n))
    return {k: (float(ms[i]), int(n[i])) for i, k in enumerate(KERNEL_CLASSES)}


def pg_workspace_bytes(T: int, d: int, V: int, S: int, params: Params, which_call: int) -> int:
    p = params.c_struct()
    return int(lib().pg_workspace_bytes(T, d, V, S, C.byref(p), which_call))


def pg_backward_chunk_rows(T: int, d: int, V: int, S: int, params: Params) -> int:
    """Vocabulary rows per chunk of the backward pass for these sizes (inspection hook)."""
    p = params.c_struct()
    return int(lib().pg_backward_chunk_rows(T, d, V, S, C.byref(p)))


def alloc_w_transposed(d: int, V: int, device="cuda") -> torch.Tensor:
    """Buffer for Params.w_transposed (the W^T cache of the loss calls)."""
    n = int(lib().pg_w_transposed_bytes(d, V))
    if n == 0:
        raise PgError(-2, f"no W^T cache for d={d}, V={V}")
    return torch.empty(n, dtype=torch.uint8, device=device)


def alloc_workspace(T: int, d: int, V: int, S: int, params: Params, which_call: int, device="cuda") -> torch.Tensor:
    n = pg_workspace_bytes(T, d, V, S, params, which_call)
    if n == 0:
        raise PgError(-1, pg_last_error())
    return torch.empty(n, dtype=torch.uint8, device=device)


def trloo_advantage(rewards: torch.Tensor, valid: torch.Tensor, gamma: float = 1.0, want_returns=True,
                    want_group_n=True, stream=None):
    """rewards float32 [P,K,Tmax], valid uint8 [P,K,Tmax] (device).  Returns (adv f64, returns f64|None, N i32|None)."""
    P, K, Tm = rewards.shape
    assert rewards.dtype == torch.float32 and valid.dtype == torch.uint8 and valid.shape == rewards.shape
    adv = torch.empty((P, K, Tm), dtype=torch.float64, device=rewards.device)
    ret = torch.empty_like(adv) if want_returns else None
    gn = torch.empty((P, Tm), dtype=torch.int32, device=rewards.device) if want_group_n else None
    _check(lib().trloo_advantage(_ptr(rewards), _ptr(valid), P, K, Tm, gamma, _ptr(ret), _ptr(adv), _ptr(gn),
                                 _stream(stream)))
    return adv, ret, gn


def grpo_advantage(rewards: torch.Tensor, valid: torch.Tensor, gamma: float = 1.0, want_returns=True,
                   want_group_n=True, stream=None):
    """As trloo_advantage, with the group-mean baseline of Eq. (3)."""
    P, K, Tm = rewards.shape
    assert rewards.dtype == torch.float32 and valid.dtype == torch.uint8 and valid.shape == rewards.shape
    adv = torch.empty((P, K, Tm), dtype=torch.float64, device=rewards.device)
    ret = torch.empty_like(adv) if want_returns else None
    gn = torch.empty((P, Tm), dtype=torch.int32, device=rewards.device) if want_group_n else None
    _check(lib().grpo_advantage(_ptr(rewards), _ptr(valid), P, K, Tm, gamma, _ptr(ret), _ptr(adv), _ptr(gn),
                                _stream(stream)))
    return adv, ret, gn


def turn_reward(correct, t_reference, t_kernel, t_generated=None, t_total=None, speedup_cap: float = 3.0,
                want_pr=True, stream=None):
    """correct uint8 [n], times float32 [n] (device).  Returns (rewards f32 [n], C*PR f32 [n] | None)."""
    n = correct.numel()
    assert correct.dtype == torch.uint8
    for t in (t_reference, t_kernel, t_generated, t_total):
        assert t is None or (t.dtype == torch.float32 and t.numel() == n)
    R = torch.empty(n, dtype=torch.float32, device=correct.device)
    pr = torch.empty(n, dtype=torch.float32, device=correct.device) if want_pr else None
    _check(lib().turn_reward(_ptr(correct), _ptr(t_reference), _ptr(t_kernel), _ptr(t_generated), _ptr(t_total), n,
                             speedup_cap, _ptr(R), _ptr(pr), _stream(stream)))
    return R, pr


def prs_retain(pr, valid, seed: int, tau: float = 0.3, s: float = 0.1, hard: bool = False, want_p=True, stream=None):
    """pr float32 [n], valid uint8 [n] | None (device).  Returns (keep u8 [n], p f32 [n] | None)."""
    n = pr.numel()
    assert pr.dtype == torch.float32 and (valid is None or (valid.dtype == torch.uint8 and valid.numel() == n))
    keep = torch.empty(n, dtype=torch.uint8, device=pr.device)
    p = torch.empty(n, dtype=torch.float32, device=pr.device) if want_p else None
    _check(lib().prs_retain(_ptr(pr), _ptr(valid), n, tau, s, 1 if hard else 0, seed & 0xFFFFFFFFFFFFFFFF, _ptr(keep),
                            _ptr(p), _stream(stream)))
    return keep, p


def pg_monitors(logp_train, logp_rollout, entropy, loss_mask, dH=None, dW=None, stream=None):
    """Returns a float64 [8] device tensor; entries named by MONITOR_NAMES."""
    T, dev, dt = _monitor_args(logp_train, logp_rollout, entropy, loss_mask, dH, dW)
    out = torch.empty(8, dtype=torch.float64, device=dev)
    ws = torch.empty(int(lib().pg_monitors_workspace_bytes()), dtype=torch.uint8, device=dev)
    _check(lib().pg_monitors(_ptr(logp_train), _ptr(logp_rollout), _ptr(entropy), _ptr(loss_mask), T, _ptr(dH), dt(dH),
                             0 if dH is None else dH.numel(), _ptr(dW), dt(dW), 0 if dW is None else dW.numel(),
                             _ptr(out), _ptr(ws), ws.numel(), _stream(stream)))
    return out


def _monitor_args(logp_train, logp_rollout, entropy, loss_mask, dH, dW):
    _want("loss_mask", loss_mask, torch.uint8)
    if not loss_mask.is_cuda:
        raise ValueError("loss_mask must be a device tensor")
    T, dev = loss_mask.numel(), loss_mask.device
    _want("logp_train", logp_train, torch.float32, (T,), dev)
    _want("logp_rollout", logp_rollout, torch.float32, (T,), dev, optional=True)
    _want("entropy", entropy, torch.float32, (T,), dev, optional=True)
    _want("dH", dH, (torch.bfloat16, torch.float32), None, dev, optional=True)
    _want("dW", dW, (torch.bfloat16, torch.float32), None, dev, optional=True)
    return T, dev, (lambda t: 0 if t is None else (1 if t.dtype == torch.float32 else 0))


def pg_init() -> None:
    """Per-device set-up (kernel attributes, address of the static scratch) for the current device."""
    _check(lib().pg_init())


def pg_monitors_static(logp_train, logp_rollout, entropy, loss_mask, dH=None, dW=None, out=None, stream=None):
    """pg_monitors without a workspace (the library's static scratch); `out` float64 [8] may be passed in, so
    that the call itself allocates nothing.  Calls that overlap on one GPU race."""
    T, dev, dt = _monitor_args(logp_train, logp_rollout, entropy, loss_mask, dH, dW)
    if out is None:
        out = torch.empty(8, dtype=torch.float64, device=dev)
    _want("out", out, torch.float64, (8,), dev)
    _check(lib().pg_monitors_static(_ptr(logp_train), _ptr(logp_rollout), _ptr(entropy), _ptr(loss_mask), T, _ptr(dH),
                                    dt(dH), 0 if dH is None else dH.numel(), _ptr(dW), dt(dW),
                                    0 if dW is None else dW.numel(), _ptr(out), _stream(stream)))
    return out


def pg_logprob_fwd(H, W, y, row_mask, params: Params, workspace: torch.Tensor, want_entropy=True, want_lse=True,
                   out=None, stream=None):
    """Returns (logp, entropy|None, lse|None), float32 [T] on the device of H."""
    T, d, V, dev = _want_head(H, W, y, params)
    _want("row_mask", row_mask, torch.uint8, (T,), dev, optional=True)
    _want_workspace(workspace, dev)
    if out is None:
        logp = torch.empty(T, dtype=torch.float32, device=H.device)
        ent = torch.empty_like(logp) if want_entropy else None
        lse = torch.empty_like(logp) if want_lse else None
    else:
        logp, ent, lse = out
        _want("out logp", logp, torch.float32, (T,), dev)
        _want("out entropy", ent, torch.float32, (T,), dev, optional=True)
        _want("out lse", lse, torch.float32, (T,), dev, optional=True)
    p = params.c_struct()
    _check(lib().pg_logprob_fwd(_ptr(H), _ptr(W), _ptr(y), _ptr(row_mask), T, d, V, C.byref(p), _ptr(logp),
                                _ptr(ent), _ptr(lse), _ptr(workspace), workspace.numel(), _stream(stream)))
    return logp, ent, lse


def pg_loss_fwd_bwd(H, W, y, loss_mask, cu_seqlens, adv, seg_sample, old_logp, rollout_logp, params: Params,
                    workspace: torch.Tensor, dW: Optional[torch.Tensor] = None, out=None, stream=None,
                    sample_keep: Optional[torch.Tensor] = None):
    """Returns dict(loss [1] f32, dH, dW, logp, entropy, counters [8] i64), all on the device of H.

    sample_keep: uint8 keep flags indexed like adv (e.g. from prs_retain); None keeps every sample."""
    T, d, V, dev = _want_head(H, W, y, params)
    S = _want_loss_args(T, dev, loss_mask, cu_seqlens, adv, seg_sample, sample_keep, old_logp, rollout_logp)
    _want_loss_out(out, T, d, V, dev, H.dtype, dW, params)
    _want_workspace(workspace, dev)
    _want_wt_cache(params, d, V, dev)
    if out is None:
        loss = torch.empty(1, dtype=torch.float32, device=dev)
        dH = torch.empty_like(H)
        logp = torch.empty(T, dtype=torch.float32, device=dev)
        ent = torch.empty(T, dtype=torch.float32, device=dev)
        counters = torch.empty(8, dtype=torch.int64, device=dev)
    else:
        loss, dH, logp, ent, counters = out
    if dW is None:
        if params.accumulate_dW:
            raise ValueError("accumulate_dW needs an existing dW")
        dW = torch.empty((V, d), dtype=torch.bfloat16 if params.dW_dtype else torch.float32, device=dev)
    p = params.c_struct()
    p.n_samples = adv.numel()
    _check(lib().pg_loss_fwd_bwd(_ptr(H), _ptr(W), _ptr(y), _ptr(loss_mask), _ptr(cu_seqlens), S, _ptr(adv),
                                 _ptr(seg_sample), _ptr(sample_keep), _ptr(old_logp), _ptr(rollout_logp), T, d, V,
                                 C.byref(p),
                                 _ptr(loss), _ptr(dH), _ptr(dW), _ptr(logp), _ptr(ent), _ptr(counters),
                                 _ptr(workspace), workspace.numel(), _stream(stream)))
    return dict(loss=loss, dH=dH, dW=dW, logp=logp, entropy=ent, counters=counters)


def pg_loss_fwd_bwd_normed(X, gamma, eps: float, W, y, loss_mask, cu_seqlens, adv, seg_sample, old_logp, rollout_logp,
                           params: Params, workspace: torch.Tensor, dW: Optional[torch.Tensor] = None, out=None, stream=None,
                           sample_keep: Optional[torch.Tensor] = None):
    """pg_loss_fwd_bwd with the RMS normalisation h = x rstd gamma fused in front of the head and its backward
    behind dH.  Returns dict(loss, dX, dgamma f32 [d], dW, logp, entropy, counters)."""
    T, d, V, dev = _want_head(X, W, y, params)
    _want("gamma", gamma, X.dtype, (d,), dev)
    S = _want_loss_args(T, dev, loss_mask, cu_seqlens, adv, seg_sample, sample_keep, old_logp, rollout_logp)
    _want_loss_out(out, T, d, V, dev, X.dtype, dW, params)
    _want_workspace(workspace, dev)
    _want_wt_cache(params, d, V, dev)
    if out is None:
        loss = torch.empty(1, dtype=torch.float32, device=dev)
        dX = torch.empty_like(X)
        logp = torch.empty(T, dtype=torch.float32, device=dev)
        ent = torch.empty(T, dtype=torch.float32, device=dev)
        counters = torch.empty(8, dtype=torch.int64, device=dev)
    else:
        loss, dX, logp, ent, counters = out
    if dW is None:
        if params.accumulate_dW:
            raise ValueError("accumulate_dW needs an existing dW")
        dW = torch.empty((V, d), dtype=torch.bfloat16 if params.dW_dtype else torch.float32, device=dev)
    dgamma = torch.empty(d, dtype=torch.float32, device=dev)
    p = params.c_struct()
    p.n_samples = adv.numel()
    _check(lib().pg_loss_fwd_bwd_normed(_ptr(X), _ptr(gamma), eps, _ptr(W), _ptr(y), _ptr(loss_mask), _ptr(cu_seqlens), S,
                                        _ptr(adv), _ptr(seg_sample), _ptr(sample_keep), _ptr(old_logp), _ptr(rollout_logp),
                                        T, d, V, C.byref(p), _ptr(loss), _ptr(dX), _ptr(dgamma), _ptr(dW), _ptr(logp),
                                        _ptr(ent), _ptr(counters), _ptr(workspace), workspace.numel(), _stream(stream)))
    return dict(loss=loss, dX=dX, dgamma=dgamma, dW=dW, logp=logp, entropy=ent, counters=counters)


def pg_sft_fwd_bwd(H, W, y, loss_mask, params: Params, workspace: torch.Tensor, dW: Optional[torch.Tensor] = None,
                   out=None, stream=None):
    """Token-mean cross-entropy of the head, forward and backward.  Returns the same dict as pg_loss_fwd_bwd."""
    T, d, V, dev = _want_head(H, W, y, params)
    _want("loss_mask", loss_mask, torch.uint8, (T,), dev)
    _want_loss_out(out, T, d, V, dev, H.dtype, dW, params)
    _want_workspace(workspace, dev)
    _want_wt_cache(params, d, V, dev)
    if out is None:
        loss = torch.empty(1, dtype=torch.float32, device=dev)
        dH = torch.empty_like(H)
        logp = torch.empty(T, dtype=torch.float32, device=dev)
        ent = torch.empty(T, dtype=torch.float32, device=dev)
        counters = torch.empty(8, dtype=torch.int64, device=dev)
    else:
        loss, dH, logp, ent, counters = out
    if dW is None:
        if params.accumulate_dW:
            raise ValueError("accumulate_dW needs an existing dW")
        dW = torch.empty((V, d), dtype=torch.bfloat16 if params.dW_dtype else torch.float32, device=dev)
    p = params.c_struct()
    _check(lib().pg_sft_fwd_bwd(_ptr(H), _ptr(W), _ptr(y), _ptr(loss_mask), T, d, V, C.byref(p), _ptr(loss), _ptr(dH),
                                _ptr(dW), _ptr(logp), _ptr(ent), _ptr(counters), _ptr(workspace), workspace.numel(),
                                _stream(stream)))
    return dict(loss=loss, dH=dH, dW=dW, logp=logp, entropy=ent, counters=counters)


def pg_head_shard_fwd(H, W_shard, y, row_mask, v_offset: int, params: Params, workspace: torch.Tensor, out=None,
                      stream=None):
    """Softmax state (m, s, u, z_y) of every row over one vocab shard.  Returns partials [T, 4] f32."""
    T, d, Vs, dev = _want_head(H, W_shard, y, params, "W_shard")
    _want("row_mask", row_mask, torch.uint8, (T,), dev, optional=True)
    _want_workspace(workspace, dev)
    parts = torch.empty((T, 4), dtype=torch.float32, device=W_shard.device) if out is None else out
    _want("partials out", parts, torch.float32, (T, 4), dev)
    p = params.c_struct()
    _check(lib().pg_head_shard_fwd(_ptr(H), _ptr(W_shard), _ptr(y), _ptr(row_mask), T, d, Vs, int(v_offset), C.byref(p),
                                   _ptr(parts), _ptr(workspace), workspace.numel(), _stream(stream)))
    return parts


def pg_head_partials_merge(a, b, out=None, stream=None):
    """Row-wise merge of two [T, 4] softmax states of disjoint vocab ranges (out may be a or b)."""
    _want("a", a, torch.float32)
    if a.dim() != 2 or a.shape[1] != 4 or not a.is_cuda:
        raise ValueError("a must be a [T, 4] device tensor")
    _want("b", b, torch.float32, a.shape, a.device)
    out = torch.empty_like(a) if out is None else out
    _want("out", out, torch.float32, a.shape, a.device)
    _check(lib().pg_head_partials_merge(_ptr(a), _ptr(b), _ptr(out), a.shape[0], _stream(stream)))
    return out


def pg_head_partials_finish(partials, want_entropy=True, want_lse=True, stream=None):
    """(logp, entropy | None, lse | None), each [T] f32, from states merged over the whole vocabulary."""
    _want("partials", partials, torch.float32)
    if partials.dim() != 2 or partials.shape[1] != 4 or not partials.is_cuda:
        raise ValueError("partials must be a [T, 4] device tensor")
    T = partials.shape[0]
    mk = lambda: torch.empty(T, dtype=torch.float32, device=partials.device)
    logp, ent, lse = mk(), (mk() if want_entropy else None), (mk() if want_lse else None)
    _check(lib().pg_head_partials_finish(_ptr(partials), T, _ptr(logp), _ptr(ent), _ptr(lse), _stream(stream)))
    return logp, ent, lse


def pg_loss_shard_bwd(H, W_shard, y, loss_mask, cu_seqlens, adv, seg_sample, old_logp, rollout_logp, partials,
                      v_offset: int, params: Params, workspace: torch.Tensor, dH_f32: bool = True,
                      dW: Optional[torch.Tensor] = None, out=None, stream=None,
                      sample_keep: Optional[torch.Tensor] = None):
    """One vocab shard's loss + backward from the states merged over all shards.

    Returns dict(loss, dH (this shard's partial sum), dW (the shard's rows), logp, entropy, counters)."""
    T, d, Vs, dev = _want_head(H, W_shard, y, params, "W_shard")
    S = _want_loss_args(T, dev, loss_mask, cu_seqlens, adv, seg_sample, sample_keep, old_logp, rollout_logp)
    _want("partials", partials, torch.float32, (T, 4), dev)
    _want_loss_out(out, T, d, Vs, dev, torch.float32 if dH_f32 else H.dtype, dW, params)
    _want_workspace(workspace, dev)
    _want_wt_cache(params, d, Vs, dev)
    if out is None:
        loss = torch.empty(1, dtype=torch.float32, device=dev)
        dH = torch.empty((T, d), dtype=torch.float32 if dH_f32 else H.dtype, device=dev)
        logp = torch.empty(T, dtype=torch.float32, device=dev)
        ent = torch.empty(T, dtype=torch.float32, device=dev)
        counters = torch.empty(8, dtype=torch.int64, device=dev)
    else:
        loss, dH, logp, ent, counters = out
    if dW is None:
        if params.accumulate_dW:
            raise ValueError("accumulate_dW needs an existing dW")
        dW = torch.empty((Vs, d), dtype=torch.bfloat16 if params.dW_dtype else torch.float32, device=dev)
    p = params.c_struct()
    p.n_samples = adv.numel()
    _check(lib().pg_loss_shard_bwd(_ptr(H), _ptr(W_shard), _ptr(y), _ptr(loss_mask), _ptr(cu_seqlens), S, _ptr(adv),
                                   _ptr(seg_sample), _ptr(sample_keep), _ptr(old_logp), _ptr(rollout_logp),
                                   _ptr(partials), T, d, Vs,
                                   int(v_offset), C.byref(p), _ptr(loss), _ptr(dH), 1 if dH_f32 else 0, _ptr(dW),
                                   _ptr(logp), _ptr(ent), _ptr(counters), _ptr(workspace), workspace.numel(),
                                   _stream(stream)))
    return dict(loss=loss, dH=dH, dW=dW, logp=logp, entropy=ent, counters=counters)


def _norm_dtype(t: torch.Tensor) -> int:
    assert t.dtype in (torch.bfloat16, torch.float32)
    return 1 if t.dtype == torch.float32 else 0


def pg_rmsnorm_fwd(X, gamma, eps: float, want_rstd=True, out=None, stream=None):
    """h = x * rstd * gamma per row.  Returns (H in the dtype of X, rstd f32 [T] | None)."""
    _want("X", X, (torch.bfloat16, torch.float32))
    if X.dim() != 2 or not X.is_cuda:
        raise ValueError("X must be a [T, d] device tensor")
    T, d = X.shape
    _want("gamma", gamma, X.dtype, (d,), X.device)
    H = torch.empty_like(X) if out is None else out
    _want("out", H, X.dtype, (T, d), X.device)
    rstd = torch.empty(T, dtype=torch.float32, device=X.device) if want_rstd else None
    _check(lib().pg_rmsnorm_fwd(_ptr(X), _ptr(gamma), T, d, eps, _norm_dtype(X), _ptr(H), _ptr(rstd), _stream(stream)))
    return H, rstd


def pg_rmsnorm_bwd(X, gamma, dH, eps: float, out=None, stream=None):
    """Returns (dX in the dtype of X, dgamma f32 [d])."""
    _want("X", X, (torch.bfloat16, torch.float32))
    if X.dim() != 2 or not X.is_cuda:
        raise ValueError("X must be a [T, d] device tensor")
    T, d = X.shape
    _want("gamma", gamma, X.dtype, (d,), X.device)
    _want("dH", dH, X.dtype, (T, d), X.device)
    dX = torch.empty_like(X) if out is None else out
    _want("out", dX, X.dtype, (T, d), X.device)
    dg = torch.empty(d, dtype=torch.float32, device=X.device)
    n = int(lib().pg_rmsnorm_bwd_workspace_bytes(d))
    if n == 0:
        raise PgError(-2, f"d={d} is not supported by pg_rmsnorm_bwd")
    ws = torch.empty(n, dtype=torch.uint8, device=X.device)
    _check(lib().pg_rmsnorm_bwd(_ptr(X), _ptr(gamma), _ptr(dH), T, d, eps, _norm_dtype(X), _ptr(dX), _ptr(dg), _ptr(ws),
                                ws.numel(), _stream(stream)))
    return dX, dg
