"""ctypes access to the float64 C oracle (``obrs_oracle.c``) -- test infrastructure only.

The arithmetic lives in the C file; this module only builds it with gcc,
marshals numpy arrays, and unpacks the result structs.  It imports nothing
from the HIP library or its Python binding.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "obrs_oracle.c")
_LIB = os.path.join(_HERE, "libobrs_oracle.so")

F32, BF16, F64 = 0, 1, 2


class RowOut(C.Structure):
    _fields_ = [
        ("lse_q", C.c_double), ("lse_p", C.c_double),
        ("logq_x", C.c_double), ("logp_x", C.c_double),
        ("logratio", C.c_double), ("accept", C.c_double),
        ("z_approx", C.c_double), ("z_exact", C.c_double),
        ("kl_p_q", C.c_double), ("kl_p_qtilde", C.c_double),
        ("mask", C.c_int32), ("union_size", C.c_int32),
        ("valid", C.c_int32), ("pad_", C.c_int32),
    ]


class BatchOut(C.Structure):
    _fields_ = [
        ("n_valid", C.c_int64), ("n_accept", C.c_int64),
        ("alpha_hat", C.c_double), ("mean_z_approx", C.c_double),
        ("kappa", C.c_double), ("mean_z_exact", C.c_double),
        ("mean_accept", C.c_double), ("mean_kl_p_q", C.c_double),
    ]


ROW_DTYPE = np.dtype([
    ("lse_q", "f8"), ("lse_p", "f8"), ("logq_x", "f8"), ("logp_x", "f8"),
    ("logratio", "f8"), ("accept", "f8"), ("z_approx", "f8"), ("z_exact", "f8"),
    ("kl_p_q", "f8"), ("kl_p_qtilde", "f8"),
    ("mask", "i4"), ("union_size", "i4"), ("valid", "i4"), ("pad_", "i4"),
])
assert ROW_DTYPE.itemsize == C.sizeof(RowOut)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over independent rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
               "-fno-fast-math", "-ffp-contract=off", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        # JPO_ORACLE_LIB: a test may point this wrapper at a deliberately broken build of the
        # oracle to show that the pin tests catch the planted mistake.
        l = C.CDLL(os.environ.get("JPO_ORACLE_LIB") or build())
        l.jpo_logsumexp.restype = C.c_double
        l.jpo_logsumexp.argtypes = [C.c_void_p, C.c_int64]
        l.jpo_topk.restype = None
        l.jpo_topk.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p]
        l.jpo_row.restype = None
        l.jpo_row.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_double,
                              C.c_double, C.c_int32, C.POINTER(RowOut), C.c_void_p, C.c_void_p]
        l.jpo_post_rejection.restype = C.c_double
        l.jpo_post_rejection.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_double, C.c_void_p]
        l.jpo_rows.restype = C.c_int
        l.jpo_rows.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64,
                               C.c_void_p, C.c_void_p, C.c_double, C.c_int32,
                               C.c_void_p, C.c_void_p, C.c_void_p, C.c_int]
        l.jpo_batch.restype = None
        l.jpo_batch.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_double, C.c_double,
                                C.c_double, C.c_void_p, C.c_int, C.POINTER(BatchOut),
                                C.c_void_p, C.c_void_p]
        l.jpo_distill_grad_row.restype = None
        l.jpo_distill_grad_row.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_double, C.c_void_p]
        l.jpo_distill_grad.restype = None
        l.jpo_distill_grad.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64,
                                       C.c_void_p, C.c_void_p, C.c_double, C.c_void_p]
        l.jpo_row_stored.restype = None
        l.jpo_row_stored.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_int32, C.c_double,
                                     C.c_int32, C.c_double, C.c_double, C.c_int32, C.c_int,
                                     C.POINTER(RowOut), C.c_void_p]
        l.jpo_rows_stored.restype = C.c_int
        l.jpo_rows_stored.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_double,
                                      C.c_int32, C.c_int, C.c_void_p, C.c_void_p, C.c_int]
        l.jpo_adjust.restype = C.c_double
        l.jpo_adjust.argtypes = [C.c_double, C.c_int, C.c_double, C.c_double, C.c_double]
        l.jpo_batch_f.restype = None
        l.jpo_batch_f.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_double, C.c_int, C.c_double,
                                  C.c_double, C.c_double, C.c_double, C.c_void_p, C.c_int,
                                  C.POINTER(BatchOut), C.c_void_p, C.c_void_p]
        l.jpo_token_logprob.restype = None
        l.jpo_token_logprob.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_void_p,
                                        C.c_void_p]
        l.jpo_lambda_for_budget.restype = C.c_double
        l.jpo_lambda_for_budget.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_double]
        l.jpo_lambda_for_budget_rows.restype = None
        l.jpo_lambda_for_budget_rows.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int64,
                                                 C.c_int64, C.c_void_p, C.c_void_p, C.c_double, C.c_void_p]
        l.jpo_lambda_for_budget_batch.restype = C.c_double
        l.jpo_lambda_for_budget_batch.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int64,
                                                  C.c_int64, C.c_void_p, C.c_double]
        l.jpo_max_threads.restype = C.c_int
        l.jpo_widen_row.restype = None
        l.jpo_widen_row.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_void_p]
        _lib = l
    return _lib


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def logsumexp(l) -> float:
    l = _f64(l)
    return lib().jpo_logsumexp(_ptr(l), l.size)


def topk(l, k: int) -> np.ndarray:
    l = _f64(l)
    ids = np.empty(k, dtype=np.int32)
    lib().jpo_topk(_ptr(l), l.size, k, _ptr(ids))
    return ids


def row(lq, lp, x: int, u: float, lam: float, k: int):
    """One token position from float64 logit rows -> (RowOut, topk_q ids, topk_p ids)."""
    lq, lp = _f64(lq), _f64(lp)
    assert lq.shape == lp.shape and lq.ndim == 1
    out = RowOut()
    kq = np.empty(k, dtype=np.int32)
    kp = np.empty(k, dtype=np.int32)
    lib().jpo_row(_ptr(lq), _ptr(lp), lq.size, int(x), float(u), float(lam), int(k),
                  C.byref(out), _ptr(kq), _ptr(kp))
    return out, kq, kp


def post_rejection(lq, lp, lam: float):
    """q~ (Eq. obrs_dist) and Z for one row."""
    lq, lp = _f64(lq), _f64(lp)
    qt = np.empty_like(lq)
    z = lib().jpo_post_rejection(_ptr(lq), _ptr(lp), lq.size, float(lam), _ptr(qt))
    return qt, z


def storage_view(a: np.ndarray):
    """(raw array, dtype code) for logits stored as float32, float64, or bf16 bits in uint16."""
    if a.dtype == np.float32:
        return a, F32
    if a.dtype == np.float64:
        return a, F64
    if a.dtype == np.uint16:
        return a, BF16
    raise TypeError(f"unsupported logits storage {a.dtype}")


@dataclass
class Rows:
    out: np.ndarray          # structured array, ROW_DTYPE, [T]
    topk_q: np.ndarray       # int32 [T, k]
    topk_p: np.ndarray       # int32 [T, k]
    threads: int


def rows(actor: np.ndarray, policy: np.ndarray, x: np.ndarray, u, lam: float, k: int,
         n_threads: int = 0) -> Rows:
    """All rows of a batch.  ``actor``/``policy``: [T, V] float32 / float64 / uint16 (bf16 bits)."""
    assert actor.shape == policy.shape and actor.ndim == 2 and actor.dtype == policy.dtype
    assert actor.strides[1] == actor.itemsize and policy.strides == actor.strides
    a, code = storage_view(actor)
    T, V = a.shape
    stride = a.strides[0] // a.itemsize
    x = np.ascontiguousarray(x, dtype=np.int32)
    uu = None if u is None else np.ascontiguousarray(u, dtype=np.float32)
    out = np.zeros(T, dtype=ROW_DTYPE)
    kq = np.empty((T, k), dtype=np.int32)
    kp = np.empty((T, k), dtype=np.int32)
    used = lib().jpo_rows(_ptr(a), _ptr(policy), code, T, V, stride, _ptr(x), _ptr(uu),
                          float(lam), int(k), _ptr(out), _ptr(kq), _ptr(kp), int(n_threads))
    return Rows(out, kq, kp, used)


def batch(rows_out: np.ndarray, mask, lam: float, c1: float, c2: float, ref_logprob=None,
          use_expected_alpha: bool = False):
    """Bias correction + weights (Sec. 4.4.2, Alg. 1 steps 2-3) -> (BatchOut, w[T], rho[T])."""
    rows_out = np.ascontiguousarray(rows_out, dtype=ROW_DTYPE)
    T = rows_out.size
    mask = np.ascontiguousarray(mask, dtype=np.int32)
    ref = None if ref_logprob is None else _f64(ref_logprob)
    b = BatchOut()
    w = np.empty(T, dtype=np.float64)
    rho = np.empty(T, dtype=np.float64)
    lib().jpo_batch(_ptr(rows_out), _ptr(mask), T, float(lam), float(c1), float(c2), _ptr(ref),
                    int(use_expected_alpha), C.byref(b), _ptr(w), _ptr(rho))
    return b, w, rho


def lambda_for_budget(lq, lp, abar: float) -> float:
    """The lambda whose OBRS rule accepts exactly the fraction ``abar`` (Sec. 3.3, Theorem 2)."""
    lq, lp = _f64(lq), _f64(lp)
    return lib().jpo_lambda_for_budget(_ptr(lq), _ptr(lp), lq.size, float(abar))


def lambda_for_budget_rows(actor: np.ndarray, policy: np.ndarray, x, target: float, row_target=None):
    """Per-row lambdas for a batch stored as float32 / float64 / bf16 bits -> float64 [T]."""
    assert actor.shape == policy.shape and actor.ndim == 2 and actor.dtype == policy.dtype
    a, code = storage_view(actor)
    T, V = a.shape
    x = np.ascontiguousarray(x, dtype=np.int32)
    rt = None if row_target is None else np.ascontiguousarray(row_target, dtype=np.float32)
    out = np.empty(T, dtype=np.float64)
    lib().jpo_lambda_for_budget_rows(_ptr(a), _ptr(policy), code, T, V, a.strides[0] // a.itemsize,
                                     _ptr(x), _ptr(rt), float(target), _ptr(out))
    return out


def lambda_for_budget_batch(actor: np.ndarray, policy: np.ndarray, x, target: float) -> float:
    """One lambda with mean_t Z_t(lambda) = target over the valid rows of the batch."""
    assert actor.shape == policy.shape and actor.ndim == 2 and actor.dtype == policy.dtype
    a, code = storage_view(actor)
    T, V = a.shape
    x = np.ascontiguousarray(x, dtype=np.int32)
    return lib().jpo_lambda_for_budget_batch(_ptr(a), _ptr(policy), code, T, V, a.strides[0] // a.itemsize,
                                             _ptr(x), float(target))


F_TRUNCATE, F_IDENTITY, F_BAND = 0, 1, 2


def adjust(w: float, f_mode: int, c1: float, lo: float = 0.0, hi: float = 0.0) -> float:
    """F(w): truncation min(w, c1), identity, or two-sided truncation (Sec. 2)."""
    return lib().jpo_adjust(float(w), int(f_mode), float(c1), float(lo), float(hi))


def batch_f(rows_out: np.ndarray, mask, lam: float, f_mode: int, c1: float, f_lo: float, f_hi: float,
            c2: float, ref_logprob=None, use_expected_alpha: bool = False):
    """``batch`` with a selectable adjustment function F -> (BatchOut, w[T], rho[T])."""
    rows_out = np.ascontiguousarray(rows_out, dtype=ROW_DTYPE)
    T = rows_out.size
    mask = np.ascontiguousarray(mask, dtype=np.int32)
    ref = None if ref_logprob is None else _f64(ref_logprob)
    b = BatchOut()
    w = np.empty(T, dtype=np.float64)
    rho = np.empty(T, dtype=np.float64)
    lib().jpo_batch_f(_ptr(rows_out), _ptr(mask), T, float(lam), int(f_mode), float(c1), float(f_lo),
                      float(f_hi), float(c2), _ptr(ref), int(use_expected_alpha), C.byref(b), _ptr(w),
                      _ptr(rho))
    return b, w, rho


def token_logprob(logits: np.ndarray, x) -> np.ndarray:
    """log softmax(logits[t])[x[t]] per row (float32 / float64 / bf16 bits storage) -> float64 [T]."""
    assert logits.ndim == 2 and logits.strides[1] == logits.itemsize
    a, code = storage_view(logits)
    T, V = a.shape
    x = np.ascontiguousarray(x, dtype=np.int32)
    out = np.empty(T, dtype=np.float64)
    lib().jpo_token_logprob(_ptr(a), code, T, V, a.strides[0] // a.itemsize, _ptr(x), _ptr(out))
    return out


def distill_grad_row(lq, lp, weight: float = 1.0) -> np.ndarray:
    """d KL(SG(p) || q) / d lq for one row (Sec. 4.2 (3)): weight * (q - p)."""
    lq, lp = _f64(lq), _f64(lp)
    out = np.empty_like(lq)
    lib().jpo_distill_grad_row(_ptr(lq), _ptr(lp), lq.size, float(weight), _ptr(out))
    return out


def distill_grad(actor: np.ndarray, policy: np.ndarray, x, row_scale=None, scale: float = 1.0) -> np.ndarray:
    """The same for a batch stored as float32 / float64 / bf16 bits; float64 [T, V]."""
    assert actor.shape == policy.shape and actor.ndim == 2 and actor.dtype == policy.dtype
    assert actor.strides[1] == actor.itemsize and policy.strides == actor.strides
    a, code = storage_view(actor)
    T, V = a.shape
    x = np.ascontiguousarray(x, dtype=np.int32)
    rs = None if row_scale is None else np.ascontiguousarray(row_scale, dtype=np.float32)
    out = np.empty((T, V), dtype=np.float64)
    lib().jpo_distill_grad(_ptr(a), _ptr(policy), code, T, V, a.strides[0] // a.itemsize, _ptr(x),
                           _ptr(rs), float(scale), _ptr(out))
    return out


TAIL_DROP, TAIL_KTH, TAIL_REST = 0, 1, 2


def row_stored(lp, ids_q, logq_ids, logq_x: float, x: int, u: float, lam: float, k: int, tail_rule: int):
    """One token position with the actor side as stored by the rollout phase (Alg. 1, Phase 1):
    -> (RowOut, topk_p ids)."""
    lp = _f64(lp)
    ids = np.ascontiguousarray(ids_q, dtype=np.int32)
    lq = _f64(logq_ids)
    assert ids.shape == lq.shape and ids.ndim == 1
    out = RowOut()
    kp = np.empty(k, dtype=np.int32)
    lib().jpo_row_stored(_ptr(lp), lp.size, _ptr(ids), _ptr(lq), ids.size, float(logq_x), int(x),
                         float(u), float(lam), int(k), int(tail_rule), C.byref(out), _ptr(kp))
    return out, kp


def rows_stored(policy: np.ndarray, ids_q, logq_ids, logq_x, x, u, lam: float, k: int, tail_rule: int,
                n_threads: int = 0) -> Rows:
    """All rows of a batch in the stored-actor form; ``topk_q`` of the result is the stored id list."""
    assert policy.ndim == 2 and policy.strides[1] == policy.itemsize
    a, code = storage_view(policy)
    T, V = a.shape
    ids = np.ascontiguousarray(ids_q, dtype=np.int32)
    lq = np.ascontiguousarray(logq_ids, dtype=np.float32)
    assert ids.shape == (T, k) and lq.shape == (T, k)
    lqx = np.ascontiguousarray(logq_x, dtype=np.float32)
    x = np.ascontiguousarray(x, dtype=np.int32)
    uu = None if u is None else np.ascontiguousarray(u, dtype=np.float32)
    out = np.zeros(T, dtype=ROW_DTYPE)
    kp = np.empty((T, k), dtype=np.int32)
    used = lib().jpo_rows_stored(_ptr(a), code, T, V, a.strides[0] // a.itemsize, _ptr(ids), _ptr(lq),
                                 _ptr(lqx), _ptr(x), _ptr(uu), float(lam), int(k), int(tail_rule),
                                 _ptr(out), _ptr(kp), int(n_threads))
    return Rows(out, ids, kp, used)


def lm_head_logits(H: np.ndarray, W: np.ndarray) -> np.ndarray:
    """Logits of the fused lm_head form as the oracle defines them: the exact float64 product of the
    stored bf16 values, H [n, d] x W [d, V] (both given as bf16 bits in uint16, or as floats); nothing is
    rounded before the OBRS computation."""
    def wide(a):
        a = np.asarray(a)
        if a.dtype == np.uint16:
            return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        return a.astype(np.float64)
    return wide(H) @ wide(W)


def max_threads() -> int:
    return lib().jpo_max_threads()
