"""Thin binding of the C-ABI library ``libjp_obrs.so`` (see ``include/jp_obrs.h``).

Argument marshalling only: torch supplies device memory and the stream handle, every step of
the path runs in the HIP kernels.  There is no CPU or PyTorch fallback: if the built library is
missing, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("JP_OBRS_LIB", os.path.join(_PKG, "libjp_obrs.so"))   # override: another build of the same ABI

JP_K_MAX = 256
JP_F32, JP_BF16 = 0, 1
JP_FLAG_EXACT_Z, JP_FLAG_TOPK_LOGPROBS, JP_FLAG_ALPHA_EXPECTED, JP_FLAG_DISTILL_KL = 1, 2, 4, 8
JP_FLAG_W_VOCAB_MAJOR = 16
JP_FLAG_ONE_WAVE_PER_ROW = 32
JP_DATA_ERR_ID_RANGE, JP_DATA_ERR_NONFINITE, JP_DATA_ERR_EMPTY = 1, 2, 4
JP_TAIL_DROP, JP_TAIL_KTH, JP_TAIL_REST = 0, 1, 2
JP_F_TRUNCATE, JP_F_IDENTITY, JP_F_BAND = 0, 1, 2
(JP_OK, JP_ERR_NULL, JP_ERR_SHAPE, JP_ERR_PARAM, JP_ERR_ALIGN, JP_ERR_WORKSPACE,
 JP_ERR_UNSUPPORTED, JP_ERR_HIP, JP_ERR_TOO_LARGE) = range(9)
JP_STATIC_MAX_T = 131072

EXPORTS = ("jp_obrs_workspace_bytes", "jp_obrs_forward", "jp_obrs_rows", "jp_obrs_finalize",
           "jp_obrs_lmhead_workspace_bytes", "jp_obrs_forward_lmhead", "jp_obrs_distill_grad",
           "jp_obrs_forward_stored", "jp_obrs_token_logprob", "jp_obrs_forward3",
           "jp_obrs_forward3_workspace_bytes", "jp_obrs_lambda_for_budget",
           "jp_obrs_lambda_for_budget_batch", "jp_obrs_budget_scratch_bytes",
           "jp_obrs_lmhead_stored_workspace_bytes", "jp_obrs_forward_lmhead_stored",
           "jp_obrs_forward_static", "jp_status_string", "jp_obrs_abi_version")


class Params(C.Structure):
    _fields_ = [("lambda_", C.c_float), ("k", C.c_int32), ("c1", C.c_float), ("c2", C.c_float),
                ("flags", C.c_uint32), ("f_mode", C.c_uint32), ("f_lo", C.c_float), ("f_hi", C.c_float)]


class Stats(C.Structure):
    _fields_ = [("n_valid", C.c_int64), ("n_accept", C.c_int64), ("alpha_hat", C.c_double),
                ("mean_z_approx", C.c_double), ("kappa", C.c_double), ("mean_z_exact", C.c_double),
                ("mean_accept", C.c_double), ("error_flags", C.c_uint32), ("reserved", C.c_uint32),
                ("mean_distill_kl", C.c_double)]


_OUT_FIELDS = ("accept_prob", "mask", "logq", "logp", "logratio", "z_approx", "z_exact", "w_obrs",
               "rho", "union_size", "topk_actor", "topk_policy", "topk_actor_logq",
               "topk_policy_logp", "stats", "distill_kl")


class Outputs(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _OUT_FIELDS]


if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build the HIP library first "
        "(python -c 'import __graft_entry__ as g; g.build()').  There is no fallback path.")

_lib = C.CDLL(LIB_PATH)
_lib.jp_obrs_workspace_bytes.restype = C.c_size_t
_lib.jp_obrs_workspace_bytes.argtypes = [C.c_int64, C.c_int64, C.c_int32, C.c_int, C.c_uint32]
_lib.jp_obrs_forward.restype = C.c_int
_lib.jp_obrs_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int,
                                 C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(Params),
                                 C.POINTER(Outputs), C.c_void_p, C.c_size_t, C.c_void_p]
_lib.jp_obrs_forward_static.restype = C.c_int
_lib.jp_obrs_forward_static.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int,
                                        C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(Params),
                                        C.POINTER(Outputs), C.c_void_p]
_lib.jp_obrs_rows.restype = C.c_int
_lib.jp_obrs_rows.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int,
                              C.c_void_p, C.c_void_p, C.POINTER(Params), C.POINTER(Outputs),
                              C.c_void_p, C.c_size_t, C.c_void_p]
_lib.jp_obrs_finalize.restype = C.c_int
_lib.jp_obrs_finalize.argtypes = [C.c_int64, C.c_void_p, C.c_void_p, C.POINTER(Params),
                                  C.POINTER(Outputs), C.c_void_p, C.c_size_t, C.c_void_p]
_lib.jp_obrs_lmhead_workspace_bytes.restype = C.c_size_t
_lib.jp_obrs_lmhead_workspace_bytes.argtypes = [C.c_int64, C.c_int64, C.c_int64, C.c_int64, C.c_int32, C.c_int64]
_lib.jp_obrs_forward_lmhead.restype = C.c_int
_lib.jp_obrs_forward_lmhead.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p,
                                        C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.POINTER(Params), C.POINTER(Outputs), C.c_void_p, C.c_size_t,
                                        C.c_void_p]
_lib.jp_obrs_distill_grad.restype = C.c_int
_lib.jp_obrs_distill_grad.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int,
                                      C.c_void_p, C.c_float, C.c_void_p, C.c_int64, C.c_int,
                                      C.c_void_p, C.c_size_t, C.c_void_p]
_lib.jp_obrs_forward_stored.restype = C.c_int
_lib.jp_obrs_forward_stored.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int, C.c_void_p,
                                        C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.POINTER(Params), C.c_int, C.POINTER(Outputs), C.c_void_p,
                                        C.c_size_t, C.c_void_p]
_lib.jp_obrs_token_logprob.restype = C.c_int
_lib.jp_obrs_token_logprob.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int, C.c_void_p,
                                       C.c_void_p, C.c_void_p]
_lib.jp_obrs_forward3_workspace_bytes.restype = C.c_size_t
_lib.jp_obrs_forward3_workspace_bytes.argtypes = [C.c_int64, C.c_int64, C.c_int32, C.c_int, C.c_uint32]
_lib.jp_obrs_forward3.restype = C.c_int
_lib.jp_obrs_forward3.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int64,
                                  C.c_int64, C.c_int, C.c_void_p, C.c_void_p, C.POINTER(Params),
                                  C.POINTER(Outputs), C.c_void_p, C.c_size_t, C.c_void_p]
_lib.jp_obrs_lambda_for_budget.restype = C.c_int
_lib.jp_obrs_lambda_for_budget.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int,
                                           C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_size_t,
                                           C.c_void_p]
_lib.jp_obrs_budget_scratch_bytes.restype = C.c_size_t
_lib.jp_obrs_budget_scratch_bytes.argtypes = []
_lib.jp_obrs_lambda_for_budget_batch.restype = C.c_int
_lib.jp_obrs_lambda_for_budget_batch.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64,
                                                 C.c_int, C.c_float, C.c_void_p, C.c_void_p, C.c_size_t,
                                                 C.c_void_p, C.c_size_t, C.c_void_p]
_lib.jp_obrs_lmhead_stored_workspace_bytes.restype = C.c_size_t
_lib.jp_obrs_lmhead_stored_workspace_bytes.argtypes = [C.c_int64, C.c_int64, C.c_int64, C.c_int32, C.c_int64]
_lib.jp_obrs_forward_lmhead_stored.restype = C.c_int
_lib.jp_obrs_forward_lmhead_stored.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int64, C.c_int64,
                                               C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                               C.c_void_p, C.POINTER(Params), C.c_int, C.POINTER(Outputs),
                                               C.c_void_p, C.c_size_t, C.c_void_p]
_lib.jp_status_string.restype = C.c_char_p
_lib.jp_status_string.argtypes = [C.c_int]
_lib.jp_obrs_abi_version.restype = C.c_int


class JpError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"jp_obrs status {status}: {jp_status_string(status)}")


def jp_status_string(status: int) -> str:
    return _lib.jp_status_string(int(status)).decode()


def jp_obrs_abi_version() -> int:
    return _lib.jp_obrs_abi_version()


def jp_obrs_workspace_bytes(T: int, V: int, k: int, dt: int, flags: int = 0) -> int:
    return _lib.jp_obrs_workspace_bytes(T, V, k, dt, flags)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return JP_BF16
    if t.dtype == torch.float32:
        return JP_F32
    raise TypeError(f"logits must be bfloat16 or float32, got {t.dtype}")


def _p(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream_handle(stream) -> C.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


@dataclass
class Buffers:
    """Device buffers of one call: the output struct, its tensors and the workspace."""
    out: Outputs
    tensors: dict
    workspace: torch.Tensor

    def __getattr__(self, name):
        t = self.__dict__.get("tensors", {})
        if name in t:
            return t[name]
        raise AttributeError(name)

    def stats(self) -> Stats:
        """Copy the device stats struct to the host (synchronises)."""
        raw = self.tensors["stats"].cpu().numpy().tobytes()
        return Stats.from_buffer_copy(raw)


def jp_obrs_lmhead_workspace_bytes(T: int, V: int, d_actor: int, d_policy: int, k: int,
                                   vocab_chunk: int = 0) -> int:
    return _lib.jp_obrs_lmhead_workspace_bytes(T, V, d_actor, d_policy, k, vocab_chunk)


def alloc_buffers(T: int, V: int, k: int, dt: int, flags: int, device, want=None,
                  workspace_bytes: Optional[int] = None) -> Buffers:
    """Allocate outputs + workspace with torch.  ``want``: iterable of output names (default all)."""
    names = set(_OUT_FIELDS if want is None else want)
    f32 = dict(dtype=torch.float32, device=device)
    t = {}
    for n in ("accept_prob", "logq", "logp", "logratio", "z_approx", "w_obrs", "rho"):
        if n in names:
            t[n] = torch.empty(T, **f32)
    if "z_exact" in names and (flags & JP_FLAG_EXACT_Z):
        t["z_exact"] = torch.empty(T, **f32)
    if "distill_kl" in names and (flags & JP_FLAG_DISTILL_KL):
        t["distill_kl"] = torch.empty(T, **f32)
    if "mask" in names:
        t["mask"] = torch.empty(T, dtype=torch.uint8, device=device)
    if "union_size" in names:
        t["union_size"] = torch.empty(T, dtype=torch.int32, device=device)
    for n in ("topk_actor", "topk_policy"):
        if n in names:
            t[n] = torch.empty((T, k), dtype=torch.int32, device=device)
    if flags & JP_FLAG_TOPK_LOGPROBS:
        for n in ("topk_actor_logq", "topk_policy_logp"):
            if n in names:
                t[n] = torch.empty((T, k), **f32)
    if "stats" in names:
        t["stats"] = torch.zeros(C.sizeof(Stats), dtype=torch.uint8, device=device)
    out = Outputs(**{n: (t[n].data_ptr() if n in t else None) for n in _OUT_FIELDS})
    nbytes = jp_obrs_workspace_bytes(T, V, k, dt, flags) if workspace_bytes is None else workspace_bytes
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
    return Buffers(out, t, ws)


def _logit_args(actor: torch.Tensor, policy: torch.Tensor):
    if actor.dim() != 2 or actor.shape != policy.shape or actor.dtype != policy.dtype:
        raise ValueError("actor/policy logits must be two [T, V] tensors of one dtype")
    if actor.stride(1) != 1 or policy.stride(1) != 1 or actor.stride(0) != policy.stride(0):
        raise ValueError("logit rows must be contiguous and both tensors must share one row stride")
    T, V = actor.shape
    return T, V, actor.stride(0) if T > 1 else max(actor.stride(0), V), _dtype_code(actor)


def _params(lam, k, c1, c2, flags, adjust=None) -> Params:
    """``adjust``: None (the paper's truncation min(w, c1)) or (JP_F_* mode, lo, hi)."""
    mode, lo, hi = (JP_F_TRUNCATE, 0.0, 0.0) if adjust is None else adjust
    return Params(float(lam), int(k), float(c1), float(c2), int(flags), int(mode), float(lo), float(hi))


def jp_obrs_forward(actor, policy, sampled_ids, uniforms, ref_logprob, lam, k, c1, c2, flags,
                    buf: Buffers, stream=None, adjust=None) -> None:
    """Whole hot path on ``stream`` (default: torch's current stream).  Raises JpError on failure."""
    T, V, stride, dt = _logit_args(actor, policy)
    prm = _params(lam, k, c1, c2, flags, adjust)
    st = _lib.jp_obrs_forward(_p(actor), _p(policy), T, V, stride, dt, _p(sampled_ids), _p(uniforms),
                              _p(ref_logprob), C.byref(prm), C.byref(buf.out), _p(buf.workspace),
                              buf.workspace.numel(), _stream_handle(stream))
    if st != JP_OK:
        raise JpError(st)


def jp_obrs_forward_static(actor, policy, sampled_ids, uniforms, ref_logprob, lam, k, c1, c2, flags,
                           buf: Buffers, stream=None, adjust=None) -> None:
    """jp_obrs_forward on the library's static scratch: ``buf.workspace`` is not used or passed."""
    T, V, stride, dt = _logit_args(actor, policy)
    prm = _params(lam, k, c1, c2, flags, adjust)
    st = _lib.jp_obrs_forward_static(_p(actor), _p(policy), T, V, stride, dt, _p(sampled_ids), _p(uniforms),
                                     _p(ref_logprob), C.byref(prm), C.byref(buf.out), _stream_handle(stream))
    if st != JP_OK:
        raise JpError(st)


def jp_obrs_lambda_for_budget(actor, policy, target, buf: Buffers, row_target=None, out=None, stream=None):
    """Per-row lambda whose OBRS rule accepts the fraction ``target`` (or ``row_target[t]``); needs the
    log-sum-exps a preceding jp_obrs_rows / jp_obrs_forward call left in ``buf.workspace``."""
    T, V, stride, dt = _logit_args(actor, policy)
    if out is None:
        out = torch.empty(T, dtype=torch.float32, device=actor.device)
    st = _lib.jp_obrs_lambda_for_budget(_p(actor), _p(policy), T, V, stride, dt, _p(row_target), float(target),
                                        _p(out), _p(buf.workspace), buf.workspace.numel(),
                                        _stream_handle(stream))
    if st != JP_OK:
        raise JpError(st)
    return out


def jp_obrs_lambda_for_budget_batch(actor, policy, target, buf: Buffers, out=None, scratch=None, stream=None):
    """One lambda with mean_t Z_t(lambda) = ``target`` over the batch -> device float32 [1]."""
    T, V, stride, dt = _logit_args(actor, policy)
    if out is None:
        out = torch.empty(1, dtype=torch.float32, device=actor.device)
    if scratch is None:
        scratch = torch.empty(_lib.jp_obrs_budget_scratch_bytes(), dtype=torch.uint8, device=actor.device)
    st = _lib.jp_obrs_lambda_for_budget_batch(_p(actor), _p(policy), T, V, stride, dt, float(target), _p(out),
                                              _p(buf.workspace), buf.workspace.numel(), _p(scratch),
                                              scratch.numel(), _stream_handle(stream))
    if st != JP_OK:
        raise JpError(st)
    return out


def jp_obrs_token_logprob(logits, sampled_ids, out=None, stream=None):
    """log softmax(logits[t])[sampled_ids[t]] per row -> float32 [T] (allocated with torch if not given)."""
    if logits.dim() != 2 or logits.stride(1) != 1:
        raise ValueError("logits must be a [T, V] tensor with contiguous rows")
    T, V = logits.shape
    stride = logits.stride(0) if T > 1 else max(logits.stride(0), V)
    if out is None:
        out = torch.empty(T, dtype=torch.float32, device=logits.device)
    st = _lib.jp_obrs_token_logprob(_p(logits), T, V, stride, _dtype_code(logits), _p(sampled_ids), _p(out),
                                    _stream_handle(stream))
    if st != JP_OK:
        raise JpError(st)
    return out


def jp_obrs_forward3_workspace_bytes(T: int, V: int, k: int, dt: int, flags: int = 0) -> int:
    return _lib.jp_obrs_forward3_workspace_bytes(T, V, k, dt, flags)


def jp_obrs_forward3(actor, policy_new, policy_ref, target_is_ref, sampled_ids, uniforms, lam, k, c1, c2,
                     flags, buf: Buffers, stream=None, adjust=None) -> None:
    """Three-distribution form: p_inf, p_new, p_ref as separate tensors, target selectable."""
    T, V, stride, dt = _logit_args(actor, policy_ref)
    if policy_new is not None:
        _logit_args(actor, policy_new)
    prm = _params(lam, k, c1, c2, flags, adjust)
    st = _lib.jp_obrs_forward3(_p(actor), _p(policy_new), _p(policy_ref), int(bool(target_is_ref)), T, V,
                               stride, dt, _p(sampled_ids), _p(uniforms), C.byref(prm), C.byref(buf.out),
                               _p(buf.workspace), buf.workspace.numel(), _stream_handle(stream))
    if st != JP_OK:
        raise JpError(st)


def jp_obrs_forward_stored(policy, actor_topk_ids, actor_topk_logprob, actor_logprob_x, sampled_ids,
                           uniforms, ref_logprob, lam, k, c1, c2, flags, tail_rule, buf: Buffers,
                           stream=None) -> None:
    """Whole hot path with the actor side as stored by the rollout phase (ids + log-probabilities)."""
    if policy.dim() != 2 or policy.stride(1) != 1:
        raise ValueError("policy logits must be a [T, V] tensor with contiguous rows")
    T, V = policy.shape
    stride = policy.stride(0) if T > 1 else max(policy.stride(0), V)
    for t_, shape, dtype in ((actor_topk_ids, (T, k), torch.int32), (actor_topk_logprob, (T, k), torch.float32),
                             (actor_logprob_x, (T,), torch.float32)):
        if tuple(t_.shape) != shape or t_.dtype != dtype or not t_.is_contiguous():
            raise ValueError("stored actor side: contiguous int32 [T, k], float32 [T, k], float32 [T]")
    prm = Params(float(lam), int(k), float(c1), float(c2), int(flags))
    st = _lib.jp_obrs_forward_stored(_p(policy), T, V, stride, _dtype_code(policy), _p(actor_topk_ids),
                                     _p(actor_topk_logprob), _p(actor_logprob_x), _p(sampled_ids),
                                     _p(uniforms), _p(ref_logprob), C.byref(prm), int(tail_rule),
                                     C.byref(buf.out), _p(buf.workspace), buf.workspace.numel(),
                                     _stream_handle(stream))
    if st != JP_OK:
        raise JpError(st)


def jp_obrs_distill_grad(actor, policy, row_scale, scale, grad, buf: Buffers, stream=None) -> None:
    """grad[t, v] = scale * row_scale[t] * (q_t(v) - p_t(v)) from the log-sum-exps that a preceding
    jp_obrs_rows / jp_obrs_forward call left in ``buf.workspace``."""
    T, V, stride, dt = _logit_args(actor, policy)
    if grad.dim() != 2 or tuple(grad.shape) != (T, V) or grad.stride(1) != 1:
        raise ValueError("grad must be a [T, V] tensor with contiguous rows")
    gstride = grad.stride(0) if T > 1 else max(grad.stride(0), V)
    st = _lib.jp_obrs_distill_grad(_p(actor), _p(policy), T, V, stride, dt, _p(row_scale), float(scale),
                                   _p(grad), gstride, _dtype_code(grad), _p(buf.workspace),
                                   buf.workspace.numel(), _stream_handle(stream))
    if st != JP_OK:
        raise JpError(st)


def jp_obrs_rows(actor, policy, sampled_ids, uniforms, lam, k, flags, buf: Buffers, stream=None) -> None:
    T, V, stride, dt = _logit_args(actor, policy)
    prm = Params(float(lam), int(k), 1.0, 1.0, int(flags))
    st = _lib.jp_obrs_rows(_p(actor), _p(policy), T, V, stride, dt, _p(sampled_ids), _p(uniforms),
                           C.byref(prm), C.byref(buf.out), _p(buf.workspace), buf.workspace.numel(),
                           _stream_handle(stream))
    if st != JP_OK:
        raise JpError(st)


def jp_obrs_finalize(T, sampled_ids, ref_logprob, lam, k, c1, c2, flags, buf: Buffers, stream=None,
                     adjust=None) -> None:
    prm = _params(lam, k, c1, c2, flags, adjust)
    st = _lib.jp_obrs_finalize(int(T), _p(sampled_ids), _p(ref_logprob), C.byref(prm), C.byref(buf.out),
                               _p(buf.workspace), buf.workspace.numel(), _stream_handle(stream))
    if st != JP_OK:
        raise JpError(st)


def jp_obrs_forward_lmhead(H_actor, W_actor, H_policy, W_policy, sampled_ids, uniforms, ref_logprob,
                           lam, k, c1, c2, flags, buf: Buffers, vocab_chunk: int = 0, stream=None) -> None:
    """Fused lm_head form: logits = H x W on the matrix cores, chunk by chunk over the vocabulary."""
    for t in (H_actor, W_actor, H_policy, W_policy):
        if t.dtype != torch.bfloat16 or t.dim() != 2 or not t.is_contiguous():
            raise ValueError("hidden states and weights must be contiguous 2-D bfloat16 tensors")
    T, d_a = H_actor.shape
    d_p = H_policy.shape[1]
    if flags & JP_FLAG_W_VOCAB_MAJOR:                        # weights as [V, d]
        V = W_actor.shape[0]
        ok = W_actor.shape[1] == d_a and tuple(W_policy.shape) == (V, d_p)
    else:                                                    # weights as [d, V]
        V = W_actor.shape[1]
        ok = W_actor.shape[0] == d_a and tuple(W_policy.shape) == (d_p, V)
    if H_policy.shape[0] != T or not ok:
        raise ValueError("shape mismatch between hidden states and weights")
    prm = Params(float(lam), int(k), float(c1), float(c2), int(flags))
    st = _lib.jp_obrs_forward_lmhead(_p(H_actor), d_a, _p(W_actor), _p(H_policy), d_p, _p(W_policy), T, V,
                                     int(vocab_chunk), _p(sampled_ids), _p(uniforms), _p(ref_logprob),
                                     C.byref(prm), C.byref(buf.out), _p(buf.workspace),
                                     buf.workspace.numel(), _stream_handle(stream))
    if st != JP_OK:
        raise JpError(st)


def jp_obrs_lmhead_stored_workspace_bytes(T, V, d_policy, k, vocab_chunk=0) -> int:
    return int(_lib.jp_obrs_lmhead_stored_workspace_bytes(T, V, d_policy, k, vocab_chunk))


def jp_obrs_forward_lmhead_stored(H_policy, W_policy, actor_topk_ids, actor_topk_logprob, actor_logprob_x,
                                  sampled_ids, uniforms, ref_logprob, lam, k, c1, c2, flags, tail_rule,
                                  buf: Buffers, vocab_chunk: int = 0, stream=None) -> None:
    """Target logits = H_policy x W_policy on the matrix cores chunk by chunk; actor side as stored."""
    for t in (H_policy, W_policy):
        if t.dtype != torch.bfloat16 or t.dim() != 2 or not t.is_contiguous():
            raise ValueError("hidden states and weights must be contiguous 2-D bfloat16 tensors")
    T, d_p = H_policy.shape
    if flags & JP_FLAG_W_VOCAB_MAJOR:                        # weights as [V, d]
        V, ok = W_policy.shape[0], W_policy.shape[1] == d_p
    else:                                                    # weights as [d, V]
        V, ok = W_policy.shape[1], W_policy.shape[0] == d_p
    if not ok:
        raise ValueError("shape mismatch between hidden states and weights")
    for t_, shape, dtype in ((actor_topk_ids, (T, k), torch.int32), (actor_topk_logprob, (T, k), torch.float32),
                             (actor_logprob_x, (T,), torch.float32)):
        if tuple(t_.shape) != shape or t_.dtype != dtype or not t_.is_contiguous():
            raise ValueError("stored actor side: contiguous int32 [T, k], float32 [T, k], float32 [T]")
    prm = Params(float(lam), int(k), float(c1), float(c2), int(flags))
    st = _lib.jp_obrs_forward_lmhead_stored(_p(H_policy), d_p, _p(W_policy), T, V, int(vocab_chunk),
                                            _p(actor_topk_ids), _p(actor_topk_logprob), _p(actor_logprob_x),
                                            _p(sampled_ids), _p(uniforms), _p(ref_logprob), C.byref(prm),
                                            int(tail_rule), C.byref(buf.out), _p(buf.workspace),
                                            buf.workspace.numel(), _stream_handle(stream))
    if st != JP_OK:
        raise JpError(st)


def raw():
    """The ctypes library handle, for tests of the C ABI itself."""
    return _lib


def run_workload(w, flags: int = 0, want=None, stream=None) -> Buffers:
    """Allocate buffers for a ``workloads.Workload`` and run the whole hot path on it."""
    T, V, _, dt = _logit_args(w.actor, w.policy)
    buf = alloc_buffers(T, V, w.k, dt, flags, w.actor.device, want)
    jp_obrs_forward(w.actor, w.policy, w.sampled_ids, w.uniforms, w.ref_logprob, w.lam, w.k, w.c1,
                    w.c2, flags, buf, stream)
    return buf
