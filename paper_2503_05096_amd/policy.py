"""Thin binding of the host-side speculative-length policy (include/adaspec_policy.h).

Marshals numpy HOST arrays into the C ABI; all decisions are taken in the
library's C++ code.  No torch, no device memory.
"""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

from . import binding

EXPORTS = (
    "adaspec_policy_estimate_time", "adaspec_policy_goodput", "adaspec_policy_adaptive_draft",
    "adaspec_policy_eliminate", "adaspec_policy_fit_time_model", "adaspec_policy_count_tokens",
)


class TimeModel(C.Structure):
    """Coefficients of T = alpha * N_c + gamma * N_b + delta for the draft (d) and target (v) models."""
    _fields_ = [("alpha_d", C.c_double), ("gamma_d", C.c_double), ("delta_d", C.c_double),
                ("alpha_v", C.c_double), ("gamma_v", C.c_double), ("delta_v", C.c_double),
                ("verify_ctx_once", C.c_int32), ("reserved", C.c_int32)]


_ready = False


def _lib():
    global _ready
    L = binding.lib()
    if not _ready:
        vp, i32, dbl = C.c_void_p, C.c_int32, C.c_double
        L.adaspec_policy_estimate_time.restype = dbl
        L.adaspec_policy_estimate_time.argtypes = [C.POINTER(TimeModel), i32, vp, i32, vp]
        L.adaspec_policy_goodput.restype = dbl
        L.adaspec_policy_goodput.argtypes = [C.POINTER(TimeModel), i32, vp, i32, vp, vp, dbl]
        L.adaspec_policy_adaptive_draft.restype = C.c_int
        L.adaspec_policy_adaptive_draft.argtypes = [C.POINTER(TimeModel), i32, vp, vp, i32, dbl, dbl, vp, vp, vp]
        L.adaspec_policy_eliminate.restype = C.c_int
        L.adaspec_policy_eliminate.argtypes = [C.POINTER(TimeModel), i32, vp, i32, vp, dbl, vp, vp]
        L.adaspec_policy_count_tokens.restype = C.c_int
        L.adaspec_policy_count_tokens.argtypes = [i32, vp, vp, i32, vp, vp]
        L.adaspec_policy_fit_time_model.restype = C.c_int
        L.adaspec_policy_fit_time_model.argtypes = [i32, vp, vp, vp, vp, vp, vp]
        _ready = True
    return L


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def estimate_time(m: TimeModel, ctx_committed, draft_steps: int, spec_lens=None) -> float:
    c = _i32(ctx_committed)
    k = None if spec_lens is None else _i32(spec_lens)
    return float(_lib().adaspec_policy_estimate_time(C.byref(m), len(c), _p(c), int(draft_steps), _p(k)))


def goodput(m: TimeModel, ctx_committed, draft_steps: int, spec_lens, ar, tpot: float = float("inf")) -> float:
    c = _i32(ctx_committed)
    k = None if spec_lens is None else _i32(spec_lens)
    a = _f64(ar)
    return float(_lib().adaspec_policy_goodput(C.byref(m), len(c), _p(c), int(draft_steps), _p(k), _p(a), tpot))


def adaptive_draft(m: TimeModel, ctx_committed, conf, prev_conf: float, tpot: float = float("inf")
                   ) -> Tuple[int, np.ndarray, float]:
    """Returns (draft steps executed, ar[steps][B], goodput estimate after the last step)."""
    c = _i32(ctx_committed)
    cf = _f64(conf)
    max_steps, B = cf.shape
    assert B == len(c)
    ar = np.zeros((max_steps, B), np.float64)
    steps, g = C.c_int32(0), C.c_double(0.0)
    rc = _lib().adaspec_policy_adaptive_draft(C.byref(m), B, _p(c), _p(cf), max_steps, float(prev_conf), tpot,
                                              C.addressof(steps), _p(ar), C.addressof(g))
    if rc != 0:
        raise binding.AdaspecError(rc, "adaspec_policy_adaptive_draft")
    return int(steps.value), ar[:steps.value], float(g.value)


def eliminate(m: TimeModel, ctx_committed, draft_steps: int, ar, tpot: float = float("inf")
              ) -> Tuple[np.ndarray, float]:
    """Returns (spec_lens[B] int32, goodput estimate of the final token set)."""
    c = _i32(ctx_committed)
    a = _f64(ar)
    k = np.zeros(len(c), np.int32)
    g = C.c_double(0.0)
    rc = _lib().adaspec_policy_eliminate(C.byref(m), len(c), _p(c), int(draft_steps), _p(a), tpot, _p(k),
                                         C.addressof(g))
    if rc != 0:
        raise binding.AdaspecError(rc, "adaspec_policy_eliminate")
    return k, float(g.value)


def count_tokens(ctx_committed, spec_lens, verify_ctx_once: bool = False) -> Tuple[float, float]:
    """(N_c, N_b) of Eq. 4 for one target pass (adaspec_policy_count_tokens)."""
    c, k = _i32(ctx_committed), _i32(spec_lens)
    assert len(c) == len(k)
    n_c, n_b = C.c_double(0.0), C.c_double(0.0)
    rc = _lib().adaspec_policy_count_tokens(len(c), _p(c), _p(k), int(bool(verify_ctx_once)), C.addressof(n_c),
                                            C.addressof(n_b))
    if rc != 0:
        raise binding.AdaspecError(rc, "adaspec_policy_count_tokens")
    return float(n_c.value), float(n_b.value)


def fit_time_model(n_c, n_b, t) -> Tuple[float, float, float]:
    nc, nb, tt = _f64(n_c), _f64(n_b), _f64(t)
    out = [C.c_double(0.0) for _ in range(3)]
    rc = _lib().adaspec_policy_fit_time_model(len(tt), _p(nc), _p(nb), _p(tt), *[C.addressof(o) for o in out])
    if rc != 0:
        raise binding.AdaspecError(rc, "adaspec_policy_fit_time_model")
    return tuple(float(o.value) for o in out)
