"""ctypes binding of the C ABI: argument marshalling only, same names as the C entry points.

Tensors must live on the GPU; pointers are taken with ``data_ptr()`` and work is enqueued
on torch's current stream for that device.  Nothing here computes anything.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

AERO_F32, AERO_BF16, AERO_F16, AERO_F8E4M3 = 0, 1, 2, 3
AERO_ROW_PADDING, AERO_ROW_UNTOUCHED = -1, -2
AERO_DW_ACCUMULATE = 0x100
OP_GROUP_ADVANTAGE, OP_LOGPROB_FWD, OP_GRPO_LOSS_BWD, OP_LMHEAD_FUSED = 0, 1, 2, 3

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libaero_hip.so")


class AeroError(RuntimeError):
    pass


class _AdvParamsC(C.Structure):
    _fields_ = [("k_ratio", C.c_int32), ("s_rescue", C.c_int32), ("tau_num", C.c_int32),
                ("tau_den", C.c_int32), ("zero_keep", C.c_int32), ("reject_enable", C.c_int32),
                ("posterior_mode", C.c_int32), ("alpha0", C.c_float), ("beta0", C.c_float)]


@dataclass
class AdvParams:
    k_ratio: int = 1
    s_rescue: int = 0
    tau_num: int = 1
    tau_den: int = 2
    zero_keep: int = 4
    reject_enable: int = 0
    posterior_mode: int = 0
    alpha0: float = 1.0
    beta0: float = 1.0

    def to_c(self) -> _AdvParamsC:
        return _AdvParamsC(self.k_ratio, self.s_rescue, self.tau_num, self.tau_den, self.zero_keep,
                           self.reject_enable, self.posterior_mode, self.alpha0, self.beta0)


def library_path() -> str:
    return _LIB_PATH


def _load() -> C.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise AeroError(f"{_LIB_PATH} is missing: build it with `python -m paper_2602_14338_amd.build` "
                        "(there is no fallback path)")
    lib = C.CDLL(_LIB_PATH)
    p, i32, i64, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t
    lib.aero_status_string.restype = C.c_char_p
    lib.aero_status_string.argtypes = [i32]
    lib.aero_workspace_bytes.restype = sz
    lib.aero_workspace_bytes.argtypes = [i32, i64, i32, i32, i32, i32]
    lib.aero_group_advantage.restype = i32
    lib.aero_group_advantage.argtypes = [p, p, p, p, i32, i32, C.POINTER(_AdvParamsC)] + [p] * 7 + [p, p]
    lib.aero_logprob_fwd.restype = i32
    lib.aero_logprob_fwd.argtypes = [p, i32, i64, i32, i64, p, p, p, p, p, p, p]
    lib.aero_grpo_loss_bwd.restype = i32
    lib.aero_grpo_loss_bwd.argtypes = [p, i32, i64, i32, i64, p, p, p, p, p, p, p, i32, f32, f32, f32, f32, f32, p,
                                       p, p, p, p, p, p, p, p, sz, p]
    lib.aero_grpo_loss_bwd_noalloc.restype = i32
    lib.aero_grpo_loss_bwd_noalloc.argtypes = lib.aero_grpo_loss_bwd.argtypes[:-3] + [p]
    lib.aero_lmhead_logprob_fused.restype = i32
    lib.aero_lmhead_logprob_fused.argtypes = [p, p, i64, i32, i32, p, p, p, p, p, p, p, p, i32, f32, f32, f32, f32,
                                              f32, p, p, p, p, p, i32, p, p, sz, p]
    return lib


class _Lazy:
    """Loads the library on first use so that the package can be imported to build it."""
    _cdll = None

    def __getattr__(self, name):
        if _Lazy._cdll is None:
            _Lazy._cdll = _load()
        return getattr(_Lazy._cdll, name)


_lib = _Lazy()


def _check(status: int, what: str) -> None:
    if status != 0:
        raise AeroError(f"{what}: {_lib.aero_status_string(status).decode()} (status {status})")


def _ptr(t: Optional[torch.Tensor], dtype=None, name: str = "") -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise AeroError(f"{name}: expected a GPU tensor")
    if dtype is not None and t.dtype != dtype:
        raise AeroError(f"{name}: expected dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise AeroError(f"{name}: expected a contiguous tensor")
    return t.data_ptr()


def _stream(t: torch.Tensor) -> int:
    return torch.cuda.current_stream(t.device).cuda_stream


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return AERO_BF16
    if t.dtype == torch.float32:
        return AERO_F32
    if t.dtype == torch.float16:
        return AERO_F16
    if t.dtype == torch.float8_e4m3fn:
        return AERO_F8E4M3
    raise AeroError(f"unsupported dtype {t.dtype}")


def aero_workspace_bytes(op: int, T: int = 0, V: int = 0, H: int = 0, R: int = 0, Q: int = 0) -> int:
    return int(_lib.aero_workspace_bytes(op, T, V, H, R, Q))


def aero_group_advantage(rewards, lengths, group_offsets, keep_priority, Q: int, R: int, params: AdvParams,
                         adv, weight, keep_mask, kept_index, kept_offsets, group_zero_var, group_category,
                         err_flag=None) -> None:
    pc = params.to_c()
    st = _lib.aero_group_advantage(
        _ptr(rewards, torch.float32, "rewards"), _ptr(lengths, torch.int32, "lengths"),
        _ptr(group_offsets, torch.int32, "group_offsets"), _ptr(keep_priority, None, "keep_priority"),
        Q, R, C.byref(pc), _ptr(adv, torch.float32, "adv"), _ptr(weight, torch.float32, "weight"),
        _ptr(keep_mask, torch.uint8, "keep_mask"), _ptr(kept_index, torch.int32, "kept_index"),
        _ptr(kept_offsets, torch.int32, "kept_offsets"), _ptr(group_zero_var, torch.uint8, "group_zero_var"),
        _ptr(group_category, torch.uint8, "group_category"), _ptr(err_flag, torch.int32, "err_flag"),
        _stream(group_offsets))
    _check(st, "aero_group_advantage")


def aero_logprob_fwd(logits, T: int, V: int, ld: int, targets, row_active, logprob, entropy, lse,
                     err_flag=None) -> None:
    st = _lib.aero_logprob_fwd(
        _ptr(logits, None, "logits"), _dtype_code(logits), T, V, ld, _ptr(targets, torch.int32, "targets"),
        _ptr(row_active, torch.uint8, "row_active"), _ptr(logprob, torch.float32, "logprob"),
        _ptr(entropy, torch.float32, "entropy"), _ptr(lse, torch.float32, "lse"),
        _ptr(err_flag, torch.int32, "err_flag"), _stream(logits))
    _check(st, "aero_logprob_fwd")


def aero_grpo_loss_bwd(logits, T: int, V: int, ld: int, targets, lse, old_logprob, token_rollout, adv, weight,
                       R: int, eps_lo: float, eps_hi: float, grad_scale: float, loss, clip_frac, logprob_out,
                       dlogits, workspace, err_flag=None, entropy_out=None, lse_out=None,
                       entropy_coef: float = 0.0, entropy=None, kl_coef: float = 0.0, ref_logprob=None) -> None:
    if dlogits is not None and dlogits.dtype != logits.dtype:
        raise AeroError("dlogits must have the dtype of logits")
    st = _lib.aero_grpo_loss_bwd(
        _ptr(logits, None, "logits"), _dtype_code(logits), T, V, ld, _ptr(targets, torch.int32, "targets"),
        _ptr(lse, torch.float32, "lse"), _ptr(entropy, torch.float32, "entropy"),
        _ptr(old_logprob, torch.float32, "old_logprob"),
        _ptr(token_rollout, torch.int32, "token_rollout"), _ptr(adv, torch.float32, "adv"),
        _ptr(weight, torch.float32, "weight"), R, eps_lo, eps_hi, grad_scale, entropy_coef,
        kl_coef, _ptr(ref_logprob, torch.float32, "ref_logprob"),
        _ptr(loss, torch.float32, "loss"), _ptr(clip_frac, torch.float32, "clip_frac"),
        _ptr(logprob_out, torch.float32, "logprob_out"), _ptr(entropy_out, torch.float32, "entropy_out"),
        _ptr(lse_out, torch.float32, "lse_out"), _ptr(dlogits, None, "dlogits"),
        _ptr(err_flag, torch.int32, "err_flag"), _ptr(workspace, None, "workspace"),
        workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream(logits))
    _check(st, "aero_grpo_loss_bwd")


def aero_grpo_loss_bwd_noalloc(logits, T: int, V: int, ld: int, targets, lse, old_logprob, token_rollout, adv, weight,
                               R: int, eps_lo: float, eps_hi: float, grad_scale: float, loss, clip_frac,
                               logprob_out, dlogits, err_flag=None, entropy_out=None, lse_out=None,
                               entropy_coef: float = 0.0, entropy=None, kl_coef: float = 0.0,
                               ref_logprob=None) -> None:
    """aero_grpo_loss_bwd without a workspace argument: the library's own fixed scratch is used."""
    if dlogits is not None and dlogits.dtype != logits.dtype:
        raise AeroError("dlogits must have the dtype of logits")
    st = _lib.aero_grpo_loss_bwd_noalloc(
        _ptr(logits, None, "logits"), _dtype_code(logits), T, V, ld, _ptr(targets, torch.int32, "targets"),
        _ptr(lse, torch.float32, "lse"), _ptr(entropy, torch.float32, "entropy"),
        _ptr(old_logprob, torch.float32, "old_logprob"),
        _ptr(token_rollout, torch.int32, "token_rollout"), _ptr(adv, torch.float32, "adv"),
        _ptr(weight, torch.float32, "weight"), R, eps_lo, eps_hi, grad_scale, entropy_coef,
        kl_coef, _ptr(ref_logprob, torch.float32, "ref_logprob"),
        _ptr(loss, torch.float32, "loss"), _ptr(clip_frac, torch.float32, "clip_frac"),
        _ptr(logprob_out, torch.float32, "logprob_out"), _ptr(entropy_out, torch.float32, "entropy_out"),
        _ptr(lse_out, torch.float32, "lse_out"), _ptr(dlogits, None, "dlogits"),
        _ptr(err_flag, torch.int32, "err_flag"), _stream(logits))
    _check(st, "aero_grpo_loss_bwd_noalloc")


def aero_lmhead_logprob_fused(hidden, weight, T: int, H: int, V: int, targets, logprob, entropy, lse,
                              old_logprob=None, token_rollout=None, adv=None, weight_rollout=None, R: int = 0,
                              eps_lo: float = 0.2, eps_hi: float = 0.2, grad_scale: float = 1.0,
                              loss=None, clip_frac=None, dhidden=None, dweight=None, workspace=None,
                              err_flag=None, entropy_coef: float = 0.0, kl_coef: float = 0.0,
                              ref_logprob=None, dweight_accumulate: bool = False) -> None:
    st = _lib.aero_lmhead_logprob_fused(
        _ptr(hidden, torch.bfloat16, "hidden"), _ptr(weight, torch.bfloat16, "weight"), T, H, V,
        _ptr(targets, torch.int32, "targets"), _ptr(logprob, torch.float32, "logprob"),
        _ptr(entropy, torch.float32, "entropy"), _ptr(lse, torch.float32, "lse"),
        _ptr(old_logprob, torch.float32, "old_logprob"), _ptr(token_rollout, torch.int32, "token_rollout"),
        _ptr(adv, torch.float32, "adv"), _ptr(weight_rollout, torch.float32, "weight_rollout"), R,
        eps_lo, eps_hi, grad_scale, entropy_coef, kl_coef, _ptr(ref_logprob, torch.float32, "ref_logprob"),
        _ptr(loss, torch.float32, "loss"),
        _ptr(clip_frac, torch.float32, "clip_frac"),
        _ptr(dhidden, torch.bfloat16, "dhidden"), _ptr(dweight, None, "dweight"),
        (_dtype_code(dweight) if dweight is not None else AERO_F32) | (AERO_DW_ACCUMULATE if dweight_accumulate else 0),
        _ptr(err_flag, torch.int32, "err_flag"),
        _ptr(workspace, None, "workspace"),
        workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream(hidden))
    _check(st, "aero_lmhead_logprob_fused")
