"""ctypes front-end of the CPU oracle (``adaspec_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke``
and by ``bench.py``'s cpu-baseline leg.  The GPU library and its Python binding
never import this package, and this package never imports them.

All arguments are host numpy arrays; bfloat16 tensors are ``uint16`` bit
patterns.  ``build()`` compiles the C file with gcc into ``liboracle.so`` next
to it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "adaspec_oracle.c")
_SRC_TREE = os.path.join(_HERE, "adaspec_tree_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_DT = {"f32": 0, "f16": 1, "bf16": 2}
_lib = None


def build(force: bool = True) -> str:
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_TREE))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11",
                               "-ffp-contract=off", "-o", _LIB, _SRC, _SRC_TREE, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        L = C.CDLL(_LIB)
        L.oracle_round_to_dtype.restype = C.c_double
        L.oracle_round_to_dtype.argtypes = [C.c_double, C.c_int]
        L.oracle_widen_u16.restype = C.c_double
        L.oracle_widen_u16.argtypes = [C.c_uint16, C.c_int]
        L.oracle_verify_attn.restype = C.c_int
        L.oracle_verify_attn.argtypes = [C.c_void_p] * 8 + [C.c_int] * 8 + [C.c_double]
        L.oracle_accept_row.restype = None
        L.oracle_accept_row.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                        C.c_double, C.c_int, C.c_double, C.c_double, C.c_void_p]
        L.oracle_cdf_interval.restype = None
        L.oracle_cdf_interval.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                          C.c_double, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        L.oracle_accept.restype = C.c_int
        L.oracle_accept.argtypes = [C.c_void_p] * 9 + [C.c_int] * 4 + [C.c_int64, C.c_int64, C.c_int]
        L.oracle_draft_sample.restype = C.c_int
        L.oracle_draft_sample.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int, C.c_int, C.c_void_p,
                                          C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.oracle_verify_attn_tree.restype = C.c_int
        L.oracle_verify_attn_tree.argtypes = [C.c_void_p] * 9 + [C.c_int] * 8 + [C.c_double]
        L.oracle_accept_tree.restype = C.c_int
        L.oracle_accept_tree.argtypes = [C.c_void_p] * 12 + [C.c_int] * 4 + [C.c_int64, C.c_int64, C.c_int]
        L.oracle_tree_cdf_interval.restype = None
        L.oracle_tree_cdf_interval.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                               C.c_double, C.c_int, C.c_int,
                                               C.c_void_p, C.c_void_p, C.c_void_p]
        L.oracle_num_threads.restype = C.c_int
        _lib = L
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a: np.ndarray, dt=None) -> np.ndarray:
    return np.ascontiguousarray(a) if dt is None else np.ascontiguousarray(a, dtype=dt)


def round_to_dtype(x: float, dtype: str) -> float:
    return float(_load().oracle_round_to_dtype(float(x), _DT[dtype]))


def widen_u16(bits: int, dtype: str) -> float:
    return float(_load().oracle_widen_u16(int(bits), _DT[dtype]))


def verify_attn(q, k_pages, v_pages, block_table, ctx_lens, spec_lens, *, dtype: str,
                scale: float = 0.0, want_rounded: bool = True
                ) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """Ragged multi-query causal attention over the paged cache, in float64.

    Returns (out_f64, out_rounded) each [TQ][Hq][d]; out_rounded holds the
    values after one nearest-even rounding to `dtype` (as float64)."""
    q, k_pages, v_pages = _c(q), _c(k_pages), _c(v_pages)
    block_table, ctx_lens, spec_lens = (_c(block_table, np.int32), _c(ctx_lens, np.int32),
                                        _c(spec_lens, np.int32))
    TQ, Hq, d = q.shape
    num_pages, Hkv, P, d2 = k_pages.shape
    assert d2 == d and v_pages.shape == k_pages.shape
    B = spec_lens.shape[0]
    assert TQ == int(spec_lens.sum()) + B
    out = np.empty((TQ, Hq, d), dtype=np.float64)
    out_r = np.empty_like(out) if want_rounded else None
    rc = _load().oracle_verify_attn(_p(q), _p(k_pages), _p(v_pages), _p(block_table), _p(ctx_lens),
                                    _p(spec_lens), _p(out), _p(out_r), B, Hq, Hkv, d, P, num_pages,
                                    block_table.shape[1], _DT[dtype], float(scale))
    if rc != 0:
        raise ValueError(f"oracle_verify_attn rejected its inputs (code {rc})")
    return out, out_r


def accept_row(logits_row, q_row, *, logits_dtype: str, probs_dtype: str, T: float, x: int,
               u0: float, u1: float) -> dict:
    logits_row = _c(logits_row)
    q_row = None if q_row is None else _c(q_row)
    res = np.empty(6, dtype=np.float64)
    _load().oracle_accept_row(_p(logits_row), _DT[logits_dtype], _p(q_row), _DT[probs_dtype],
                              logits_row.shape[0], float(T), int(x), float(u0), float(u1), _p(res))
    return dict(accept=bool(res[0]), ratio=res[1], cand=int(res[2]), R=res[3],
                cdf_before=res[4], cdf_incl=res[5])


def cdf_interval(logits_row, q_row, *, logits_dtype: str, probs_dtype: str, T: float, t: int):
    logits_row = _c(logits_row)
    q_row = None if q_row is None else _c(q_row)
    lo, hi, R = C.c_double(), C.c_double(), C.c_double()
    _load().oracle_cdf_interval(_p(logits_row), _DT[logits_dtype], _p(q_row), _DT[probs_dtype],
                                logits_row.shape[0], float(T), int(t),
                                C.byref(lo), C.byref(hi), C.byref(R))
    return lo.value, hi.value, R.value


def accept(target_logits, draft_probs, draft_tokens, uniforms, spec_lens, temperature, *,
           logits_dtype: str, probs_dtype: str, out_stride: Optional[int] = None,
           want_row_info: bool = True):
    """Sequential accept / resample / bonus over the ragged batch.

    Returns (out_tokens [B][out_stride] int32, out_accept_len [B] int32,
    row_info [TQ][6] float64 or None)."""
    target_logits = _c(target_logits)
    spec_lens = _c(spec_lens, np.int32)
    B = spec_lens.shape[0]
    TQ, V = target_logits.shape
    TD = int(spec_lens.sum())
    assert TQ == TD + B
    draft_probs = _c(draft_probs) if TD else np.zeros((1, V), dtype=target_logits.dtype)
    draft_tokens = _c(draft_tokens, np.int32) if TD else np.zeros(1, dtype=np.int32)
    uniforms = _c(uniforms, np.float32)
    temperature = _c(temperature, np.float32)
    assert uniforms.shape == (TQ, 2) and temperature.shape == (B,)
    kmax = int(spec_lens.max()) if B else 0
    out_stride = kmax + 1 if out_stride is None else out_stride
    toks = np.empty((B, out_stride), dtype=np.int32)
    alen = np.empty(B, dtype=np.int32)
    info = np.empty((TQ, 6), dtype=np.float64) if want_row_info else None
    rc = _load().oracle_accept(_p(target_logits), _p(draft_probs), _p(draft_tokens), _p(uniforms),
                               _p(spec_lens), _p(temperature), _p(toks), _p(alen), _p(info),
                               B, V, _DT[logits_dtype], _DT[probs_dtype], V, V, out_stride)
    if rc != 0:
        raise ValueError(f"oracle_accept rejected its inputs (code {rc})")
    return toks, alen, info


def draft_sample(draft_logits, temperature, uniforms, *, logits_dtype: str, probs_dtype: str):
    """Draft-side sampling of every row.  Returns (q [R][V] float64: the rounded draft-probability
    rows, tokens [R] int32, confidence [R] float64, info [R][5] = token, confidence, Q = sum q,
    prefix sum before the token, prefix sum including it)."""
    L = _load()
    lg = _c(draft_logits)
    R, V = lg.shape
    temp = _c(np.asarray(temperature, dtype=np.float32))
    uni = _c(np.asarray(uniforms, dtype=np.float32))
    q = np.zeros((R, V), np.float64)
    tok = np.zeros(R, np.int32)
    conf = np.zeros(R, np.float64)
    info = np.zeros((R, 5), np.float64)
    rc = L.oracle_draft_sample(_p(lg), _DT[logits_dtype], V, R, V, _p(temp), _p(uni), _DT[probs_dtype],
                               _p(q), _p(tok), _p(conf), _p(info))
    assert rc == 0
    return q, tok, conf, info


# --------------------------------------------------------------------------
# tree verification (adaspec_tree_oracle.c)
# --------------------------------------------------------------------------
def verify_attn_tree(q, k_pages, v_pages, block_table, ctx_lens, spec_lens, parents, *, dtype: str,
                     scale: float = 0.0, want_rounded: bool = True
                     ) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """Attention of every tree node over the committed context plus its own ancestors, float64.
    `parents` [TQ] int32: parent index inside the request, -1 for each request's root."""
    q, k_pages, v_pages = _c(q), _c(k_pages), _c(v_pages)
    block_table, ctx_lens, spec_lens, parents = (_c(block_table, np.int32), _c(ctx_lens, np.int32),
                                                 _c(spec_lens, np.int32), _c(parents, np.int32))
    TQ, Hq, d = q.shape
    num_pages, Hkv, P, d2 = k_pages.shape
    assert d2 == d and v_pages.shape == k_pages.shape
    B = spec_lens.shape[0]
    assert TQ == int(spec_lens.sum()) + B and parents.shape == (TQ,)
    out = np.empty((TQ, Hq, d), dtype=np.float64)
    out_r = np.empty_like(out) if want_rounded else None
    rc = _load().oracle_verify_attn_tree(_p(q), _p(k_pages), _p(v_pages), _p(block_table), _p(ctx_lens),
                                         _p(spec_lens), _p(parents), _p(out), _p(out_r), B, Hq, Hkv, d, P,
                                         num_pages, block_table.shape[1], _DT[dtype], float(scale))
    if rc != 0:
        raise ValueError(f"oracle_verify_attn_tree rejected its inputs (code {rc})")
    return out, out_r


def accept_tree(target_logits, draft_probs, draft_tokens, parents, uniforms, spec_lens, temperature, *,
                logits_dtype: str, probs_dtype: str, out_stride: Optional[int] = None):
    """Tree acceptance walk of every request.

    Returns (out_tokens [B][out_stride], out_accept_len [B], out_path [B][out_stride],
    test_info [TQ][2] float64, stop_info [B][5] float64)."""
    target_logits = _c(target_logits)
    spec_lens = _c(spec_lens, np.int32)
    parents = _c(parents, np.int32)
    B = spec_lens.shape[0]
    TQ, V = target_logits.shape
    TD = int(spec_lens.sum())
    assert TQ == TD + B and parents.shape == (TQ,)
    draft_probs = _c(draft_probs) if TD else np.zeros((1, V), dtype=target_logits.dtype)
    draft_tokens = _c(draft_tokens, np.int32) if TD else np.zeros(1, dtype=np.int32)
    uniforms = _c(uniforms, np.float32)
    temperature = _c(temperature, np.float32)
    assert uniforms.shape == (TQ, 2) and temperature.shape == (B,)
    kmax = int(spec_lens.max()) if B else 0
    out_stride = kmax + 1 if out_stride is None else out_stride
    toks = np.empty((B, out_stride), dtype=np.int32)
    alen = np.empty(B, dtype=np.int32)
    path = np.empty((B, out_stride), dtype=np.int32)
    test_info = np.empty((TQ, 2), dtype=np.float64)
    stop_info = np.full((B, 5), np.nan, dtype=np.float64)
    rc = _load().oracle_accept_tree(_p(target_logits), _p(draft_probs), _p(draft_tokens), _p(parents),
                                    _p(uniforms), _p(spec_lens), _p(temperature), _p(toks), _p(alen),
                                    _p(path), _p(test_info), _p(stop_info),
                                    B, V, _DT[logits_dtype], _DT[probs_dtype], V, V, out_stride)
    if rc != 0:
        raise ValueError(f"oracle_accept_tree rejected its inputs (code {rc})")
    return toks, alen, path, test_info, stop_info


def tree_cdf_interval(logits_row, q_row, *, logits_dtype: str, probs_dtype: str, T: float,
                      rejections: int, t: int):
    """[lo, hi) of token t in the mass a node draws from after `rejections` rejected children, and
    that mass's total."""
    logits_row = _c(logits_row)
    q_row = None if q_row is None else _c(q_row)
    assert q_row is not None or rejections == 0
    lo, hi, R = C.c_double(), C.c_double(), C.c_double()
    _load().oracle_tree_cdf_interval(_p(logits_row), _DT[logits_dtype], _p(q_row), _DT[probs_dtype],
                                     logits_row.shape[0], float(T), int(rejections), int(t),
                                     C.byref(lo), C.byref(hi), C.byref(R))
    return lo.value, hi.value, R.value
