"""Thin Python binding of libadaspec.so (see include/adaspec.h).

Argument marshalling only: every step of the verification path runs inside the
library's HIP kernels.  PyTorch supplies device memory and streams.  There is
no CPU fallback: if the library has not been built, importing it fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libadaspec.so")

F32, F16, BF16 = 0, 1, 2
PATH_AUTO, PATH_VECTOR, PATH_FAST = 0, 1, 2
PLAN_BUILD_AND_RUN, PLAN_BUILD_ONLY, PLAN_REUSE = 0, 1, 2
_PLAN = {"run": PLAN_BUILD_AND_RUN, "build": PLAN_BUILD_ONLY, "reuse": PLAN_REUSE}
PATH_STREAM, PATH_TWO_PASS = 3, 4
_PATHS = {"auto": PATH_AUTO, "vector": PATH_VECTOR, "fast": PATH_FAST, "stream": PATH_STREAM,
          "two_pass": PATH_TWO_PASS}

EXPORTS = (
    "adaspec_verify_attn_workspace_bytes", "adaspec_verify_attn",
    "adaspec_accept_workspace_bytes", "adaspec_accept", "adaspec_accept_noalloc", "adaspec_accept_resolved_path",
    "adaspec_verify_attn_tree", "adaspec_accept_tree", "adaspec_kv_compact_path", "adaspec_check_tree_parents", "adaspec_check_accept_inputs",
    "adaspec_check_ragged_inputs", "adaspec_kv_append", "adaspec_commit",
    "adaspec_draft_sample_workspace_bytes", "adaspec_draft_sample",
    "adaspec_status_string", "adaspec_version",
)


class AttnDims(C.Structure):
    _fields_ = [("batch", C.c_int32), ("total_q", C.c_int32), ("max_spec_len", C.c_int32),
                ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("page_size", C.c_int32), ("num_pages", C.c_int32), ("max_pages_per_req", C.c_int32),
                ("dtype", C.c_int32), ("out_dtype", C.c_int32), ("path", C.c_int32),
                ("scale", C.c_float), ("plan_mode", C.c_int32),
                ("timing_start", C.c_void_p), ("timing_stop", C.c_void_p)]


class AcceptDims(C.Structure):
    _fields_ = [("batch", C.c_int32), ("total_q", C.c_int32), ("total_draft", C.c_int32),
                ("max_spec_len", C.c_int32), ("vocab", C.c_int32), ("logits_dtype", C.c_int32),
                ("probs_dtype", C.c_int32), ("out_stride", C.c_int32),
                ("logits_row_stride", C.c_int64), ("probs_row_stride", C.c_int64),
                ("path", C.c_int32), ("reserved", C.c_int32),
                ("timing_start", C.c_void_p), ("timing_stop", C.c_void_p)]


class CommitDims(C.Structure):
    _fields_ = [("batch", C.c_int32), ("max_spec_len", C.c_int32), ("out_stride", C.c_int32),
                ("seq_stride", C.c_int32)]


class DraftDims(C.Structure):
    _fields_ = [("rows", C.c_int32), ("vocab", C.c_int32), ("logits_dtype", C.c_int32),
                ("probs_dtype", C.c_int32), ("logits_row_stride", C.c_int64), ("probs_row_stride", C.c_int64),
                ("path", C.c_int32), ("reserved", C.c_int32),
                ("timing_start", C.c_void_p), ("timing_stop", C.c_void_p)]


class AdaspecError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def lib() -> C.CDLL:
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; "
                "g.build()' or python paper_2503_05096_amd/build.py). There is no fallback path.")
        # The process must hold ONE HIP runtime.  PyTorch ships its own copy and loads it by path;
        # the loader shares it with this library only if it is already mapped when the library is
        # opened (same SONAME).  Opened the other way round, the library would bind to the system
        # copy and launch kernels through a runtime that knows nothing of torch's streams and memory.
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp = C.c_void_p
        L.adaspec_verify_attn_workspace_bytes.restype = C.c_size_t
        L.adaspec_verify_attn_workspace_bytes.argtypes = [C.POINTER(AttnDims)]
        L.adaspec_verify_attn.restype = C.c_int
        L.adaspec_verify_attn.argtypes = [vp] * 7 + [C.POINTER(AttnDims), vp, C.c_size_t, vp]
        L.adaspec_accept_workspace_bytes.restype = C.c_size_t
        L.adaspec_accept_workspace_bytes.argtypes = [C.POINTER(AcceptDims)]
        L.adaspec_accept.restype = C.c_int
        L.adaspec_accept.argtypes = [vp] * 8 + [C.POINTER(AcceptDims), vp, C.c_size_t, vp]
        L.adaspec_accept_noalloc.restype = C.c_int
        L.adaspec_accept_noalloc.argtypes = [vp] * 8 + [C.POINTER(AcceptDims), vp]
        L.adaspec_accept_resolved_path.restype = C.c_int
        L.adaspec_accept_resolved_path.argtypes = [vp, vp, C.POINTER(AcceptDims)]
        L.adaspec_verify_attn_tree.restype = C.c_int
        L.adaspec_verify_attn_tree.argtypes = [vp] * 8 + [C.POINTER(AttnDims), vp, C.c_size_t, vp]
        L.adaspec_accept_tree.restype = C.c_int
        L.adaspec_accept_tree.argtypes = [vp] * 10 + [C.POINTER(AcceptDims), vp, C.c_size_t, vp]
        L.adaspec_kv_compact_path.restype = C.c_int
        L.adaspec_kv_compact_path.argtypes = [vp] * 7 + [C.POINTER(AttnDims), C.c_int32, vp]
        L.adaspec_check_accept_inputs.restype = C.c_int
        L.adaspec_check_accept_inputs.argtypes = [vp, vp, vp, C.POINTER(AcceptDims), vp, vp]
        L.adaspec_check_tree_parents.restype = C.c_int
        L.adaspec_check_tree_parents.argtypes = [vp, vp, C.c_int32, C.c_int32, C.c_int32, vp, vp]
        L.adaspec_check_ragged_inputs.restype = C.c_int
        L.adaspec_check_ragged_inputs.argtypes = [vp, vp, vp, C.POINTER(AttnDims), vp, vp]
        L.adaspec_kv_append.restype = C.c_int
        L.adaspec_kv_append.argtypes = [vp] * 7 + [C.POINTER(AttnDims), vp]
        L.adaspec_commit.restype = C.c_int
        L.adaspec_commit.argtypes = [vp] * 10 + [C.POINTER(CommitDims), vp]
        L.adaspec_draft_sample.restype = C.c_int
        L.adaspec_draft_sample.argtypes = [vp] * 7 + [C.POINTER(DraftDims), vp, C.c_size_t, vp]
        L.adaspec_draft_sample_workspace_bytes.restype = C.c_size_t
        L.adaspec_draft_sample_workspace_bytes.argtypes = [C.POINTER(DraftDims)]
        L.adaspec_status_string.restype = C.c_char_p
        L.adaspec_status_string.argtypes = [C.c_int]
        L.adaspec_version.restype = C.c_int
        _lib = L
    return _lib


def hip_runtime() -> C.CDLL:
    """The HIP runtime this process already uses (the copy torch loaded), for callers that need
    raw HIP calls such as hipEventCreate: opening "libamdhip64.so" by name could map a second copy."""
    lib()
    with open("/proc/self/maps") as f:
        paths = {line.split()[-1] for line in f if "libamdhip64" in line}
    if len(paths) != 1:
        raise RuntimeError(f"expected exactly one HIP runtime in the process, found {sorted(paths)}")
    return C.CDLL(paths.pop())


def status_string(status: int) -> str:
    return lib().adaspec_status_string(int(status)).decode()


def version() -> int:
    return int(lib().adaspec_version())


# --------------------------------------------------------------------------
# torch-facing wrappers
# --------------------------------------------------------------------------
def _dtype_code(t) -> int:
    import torch
    return {torch.float32: F32, torch.float16: F16, torch.bfloat16: BF16}[t.dtype]


def _torch_dtype(code: int):
    import torch
    return {F32: torch.float32, F16: torch.float16, BF16: torch.bfloat16}[code]


def _stream_ptr(stream) -> int:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


# Default workspaces: one per (device, call family), grown on demand.  Attention, acceptance and draft
# sampling never share one (a planned attention pass keeps its metadata in its workspace across calls).
# A buffer that is outgrown stays referenced until the process ends: a kernel on a caller-supplied,
# non-current stream may still be using it, and torch's allocator would hand a freed block to the next
# tensor at once.  Callers that issue calls on several streams must pass their own `workspace` per
# stream: calls that share a workspace have to be ordered on one stream.
_ws_cache = {}
_ws_retired = []


def _workspace(nbytes: int, device, workspace, family: str):
    import torch
    if workspace is not None:
        return workspace
    key = (str(device), family)
    ws = _ws_cache.get(key)
    if ws is None or ws.numel() < nbytes:
        if ws is not None:
            _ws_retired.append(ws)
        ws = torch.empty(max(nbytes, 1 << 20), dtype=torch.uint8, device=device)
        _ws_cache[key] = ws
    return ws


def _with_timing(dims, timing):
    """timing = (start, stop): raw hipEvent_t handles (ints or c_void_p) the library records around the call's
    main kernel(s) on the call's stream; None = no events."""
    if timing is not None:
        start, stop = timing
        dims.timing_start = start.value if isinstance(start, C.c_void_p) else start
        dims.timing_stop = stop.value if isinstance(stop, C.c_void_p) else stop
    return dims


def attn_dims(q, k_pages, block_table, *, max_spec_len: int, scale: float = 0.0,
              out_dtype: Optional[int] = None, path: str = "auto", plan: str = "run") -> AttnDims:
    dt = _dtype_code(q)
    TQ, Hq, d = q.shape
    num_pages, Hkv, P, _ = k_pages.shape
    B, max_pages = block_table.shape
    return AttnDims(B, TQ, int(max_spec_len), Hq, Hkv, d, P, num_pages, max_pages, dt,
                    dt if out_dtype is None else int(out_dtype), _PATHS[path], float(scale), _PLAN[plan])


def verify_attn(q, k_pages, v_pages, block_table, ctx_lens, spec_lens, out=None, *,
                max_spec_len: int, scale: float = 0.0, out_dtype: Optional[int] = None,
                path: str = "auto", plan: str = "run", workspace=None, stream=None, parents=None, timing=None):
    """adaspec_verify_attn on device tensors; returns `out` [TQ][Hq][d].

    plan: "run" (build the ragged metadata, then run), "build" (metadata only; returns None) or
    "reuse" (run with the metadata a previous call left in the same workspace).  "build" and "reuse"
    require `workspace`: a tensor of at least adaspec_verify_attn_workspace_bytes that the caller owns
    and that no other call touches between the build and the last reuse.
    parents [TQ] int32 (a draft tree): adaspec_verify_attn_tree instead."""
    import torch
    dims = _with_timing(attn_dims(q, k_pages, block_table, max_spec_len=max_spec_len, scale=scale,
                                  out_dtype=out_dtype, path=path, plan=plan), timing)
    for t in (q, k_pages, v_pages, block_table, ctx_lens, spec_lens):
        assert t.is_cuda and t.is_contiguous()
    assert block_table.dtype == torch.int32 and ctx_lens.dtype == torch.int32 and spec_lens.dtype == torch.int32
    assert v_pages.shape == k_pages.shape and v_pages.dtype == k_pages.dtype == q.dtype
    if out is None and plan != "build":
        out = torch.empty(q.shape, dtype=_torch_dtype(dims.out_dtype), device=q.device)
    L = lib()
    need = L.adaspec_verify_attn_workspace_bytes(C.byref(dims))
    if need == 0 and dims.batch > 0:
        raise AdaspecError(L.adaspec_verify_attn(None, None, None, None, None, None, None, C.byref(dims),
                                                 None, 0, None) or -2, "adaspec_verify_attn (dims)")
    if plan != "run" and workspace is None:
        # the metadata of a planned pass lives in the workspace between the calls: it has to be the
        # caller's own buffer, one that nothing else writes to meanwhile
        raise ValueError("verify_attn(plan='build' / 'reuse') needs an explicit workspace= tensor that the "
                         "caller keeps for the whole pass")
    ws = _workspace(need, q.device, workspace, "attn")
    if parents is not None:
        assert parents.is_cuda and parents.is_contiguous() and parents.dtype == torch.int32
        assert parents.shape == (q.shape[0],)
        rc = L.adaspec_verify_attn_tree(q.data_ptr(), k_pages.data_ptr(), v_pages.data_ptr(),
                                        block_table.data_ptr(), ctx_lens.data_ptr(), spec_lens.data_ptr(),
                                        parents.data_ptr(), None if out is None else out.data_ptr(),
                                        C.byref(dims), ws.data_ptr(), ws.numel(), _stream_ptr(stream))
        if rc != 0:
            raise AdaspecError(rc, "adaspec_verify_attn_tree")
        return out
    rc = L.adaspec_verify_attn(q.data_ptr(), k_pages.data_ptr(), v_pages.data_ptr(),
                               block_table.data_ptr(), ctx_lens.data_ptr(), spec_lens.data_ptr(),
                               None if out is None else out.data_ptr(), C.byref(dims), ws.data_ptr(), ws.numel(),
                               _stream_ptr(stream))
    if rc != 0:
        raise AdaspecError(rc, "adaspec_verify_attn")
    return out


def accept_dims(target_logits, draft_probs, draft_tokens, spec_lens, max_spec_len, out_stride, path):
    """(dims, draft_probs pointer, draft_tokens pointer) of an acceptance call: marshalling only."""
    import torch
    TQ, V = target_logits.shape
    B = spec_lens.shape[0]
    TD = TQ - B
    out_stride = int(max_spec_len) + 1 if out_stride is None else int(out_stride)
    assert target_logits.is_cuda and spec_lens.is_cuda
    assert target_logits.stride(1) == 1 and spec_lens.dtype == torch.int32
    if TD > 0:
        assert draft_probs.shape == (TD, V) and draft_probs.stride(1) == 1
        assert draft_tokens.dtype == torch.int32 and draft_tokens.shape == (TD,)
        pdt, pstride = _dtype_code(draft_probs), draft_probs.stride(0)
        pp, tp = draft_probs.data_ptr(), draft_tokens.data_ptr()
    else:
        pdt, pstride, pp, tp = _dtype_code(target_logits), V, None, None
    dims = AcceptDims(B, TQ, TD, int(max_spec_len), V, _dtype_code(target_logits), pdt, out_stride,
                      target_logits.stride(0), pstride, _PATHS[path], 0)
    return dims, pp, tp


def accept_resolved_path(target_logits, draft_probs, draft_tokens, spec_lens, *, max_spec_len: int,
                         out_stride: Optional[int] = None, path: str = "auto") -> str:
    """adaspec_accept_resolved_path: the kernel path adaspec_accept takes for these tensors."""
    dims, pp, _ = accept_dims(target_logits, draft_probs, draft_tokens, spec_lens, max_spec_len, out_stride, path)
    rc = lib().adaspec_accept_resolved_path(target_logits.data_ptr(), pp, C.byref(dims))
    if rc < 0:
        raise AdaspecError(rc, "adaspec_accept_resolved_path")
    return {v: k for k, v in _PATHS.items()}[rc]


def accept(target_logits, draft_probs, draft_tokens, uniforms, spec_lens, temperature, *,
           max_spec_len: int, out_tokens=None, out_accept_len=None, out_stride: Optional[int] = None,
           path: str = "auto", workspace=None, stream=None, timing=None) -> Tuple[object, object]:
    """adaspec_accept on device tensors; returns (out_tokens [B][out_stride], out_accept_len [B])."""
    import torch
    for t in (uniforms, temperature):
        assert t.is_cuda
    assert uniforms.is_contiguous() and uniforms.dtype == torch.float32 and temperature.dtype == torch.float32
    dims, pp, tp = accept_dims(target_logits, draft_probs, draft_tokens, spec_lens, max_spec_len, out_stride, path)
    _with_timing(dims, timing)
    B, out_stride = dims.batch, dims.out_stride
    if out_tokens is None:
        out_tokens = torch.empty((B, out_stride), dtype=torch.int32, device=target_logits.device)
    if out_accept_len is None:
        out_accept_len = torch.empty((B,), dtype=torch.int32, device=target_logits.device)
    L = lib()
    need = L.adaspec_accept_workspace_bytes(C.byref(dims))
    ws = _workspace(max(need, 256), target_logits.device, workspace, "accept")
    rc = L.adaspec_accept(target_logits.data_ptr(), pp, tp, uniforms.data_ptr(), spec_lens.data_ptr(),
                          temperature.data_ptr(), out_tokens.data_ptr(), out_accept_len.data_ptr(),
                          C.byref(dims), ws.data_ptr(), ws.numel(), _stream_ptr(stream))
    if rc != 0:
        raise AdaspecError(rc, "adaspec_accept")
    return out_tokens, out_accept_len


NOALLOC_SCRATCH_BYTES = 8 << 20


def accept_noalloc(target_logits, draft_probs, draft_tokens, uniforms, spec_lens, temperature, out_tokens,
                   out_accept_len, *, max_spec_len: int, out_stride: Optional[int] = None, path: str = "auto",
                   stream=None) -> None:
    """adaspec_accept_noalloc: acceptance into the caller's output tensors, on the library's built-in
    scratch memory.  Nothing is allocated here either: the outputs are required arguments."""
    import torch
    assert uniforms.is_cuda and uniforms.is_contiguous() and uniforms.dtype == torch.float32
    assert temperature.is_cuda and temperature.dtype == torch.float32
    dims, pp, tp = accept_dims(target_logits, draft_probs, draft_tokens, spec_lens, max_spec_len, out_stride, path)
    assert out_tokens.is_cuda and out_tokens.dtype == torch.int32 and out_tokens.is_contiguous()
    assert tuple(out_tokens.shape) == (dims.batch, dims.out_stride)
    assert out_accept_len.is_cuda and out_accept_len.dtype == torch.int32 and tuple(out_accept_len.shape) == (dims.batch,)
    rc = lib().adaspec_accept_noalloc(target_logits.data_ptr(), pp, tp, uniforms.data_ptr(), spec_lens.data_ptr(),
                                      temperature.data_ptr(), out_tokens.data_ptr(), out_accept_len.data_ptr(),
                                      C.byref(dims), _stream_ptr(stream))
    if rc != 0:
        raise AdaspecError(rc, "adaspec_accept_noalloc")


def accept_tree(target_logits, draft_probs, draft_tokens, parents, uniforms, spec_lens, temperature, *,
                max_spec_len: int, out_tokens=None, out_accept_len=None, out_path=None,
                out_stride: Optional[int] = None, path: str = "auto", workspace=None, stream=None, timing=None):
    """adaspec_accept_tree; returns (out_tokens [B][out_stride], out_accept_len [B], out_path [B][out_stride]).
    path: "auto", "vector" (portable per-node kernel) or "fast" (1024-thread per-node kernel)."""
    import torch
    for t in (uniforms, temperature, parents):
        assert t.is_cuda and t.is_contiguous()
    assert uniforms.dtype == torch.float32 and temperature.dtype == torch.float32 and parents.dtype == torch.int32
    assert parents.shape == (target_logits.shape[0],)
    dims, pp, tp = accept_dims(target_logits, draft_probs, draft_tokens, spec_lens, max_spec_len, out_stride, path)
    _with_timing(dims, timing)
    B, out_stride = dims.batch, dims.out_stride
    dev = target_logits.device
    if out_tokens is None:
        out_tokens = torch.empty((B, out_stride), dtype=torch.int32, device=dev)
    if out_accept_len is None:
        out_accept_len = torch.empty((B,), dtype=torch.int32, device=dev)
    if out_path is None:
        out_path = torch.empty((B, out_stride), dtype=torch.int32, device=dev)
    L = lib()
    need = L.adaspec_accept_workspace_bytes(C.byref(dims))
    ws = _workspace(max(need, 256), dev, workspace, "accept")
    rc = L.adaspec_accept_tree(target_logits.data_ptr(), pp, tp, parents.data_ptr(), uniforms.data_ptr(),
                               spec_lens.data_ptr(), temperature.data_ptr(), out_tokens.data_ptr(),
                               out_accept_len.data_ptr(), out_path.data_ptr(), C.byref(dims), ws.data_ptr(),
                               ws.numel(), _stream_ptr(stream))
    if rc != 0:
        raise AdaspecError(rc, "adaspec_accept_tree")
    return out_tokens, out_accept_len, out_path


def kv_compact_path(k_pages, v_pages, block_table, ctx_lens, spec_lens, out_path, out_accept_len, *,
                    max_spec_len: int, stream=None) -> None:
    """adaspec_kv_compact_path: moves the accepted nodes' K/V rows to chain positions, in place."""
    import torch
    num_pages, Hkv, P, d = k_pages.shape
    B, max_pages = block_table.shape
    for t in (k_pages, v_pages, block_table, ctx_lens, spec_lens, out_path, out_accept_len):
        assert t.is_cuda and t.is_contiguous()
    for t in (block_table, ctx_lens, spec_lens, out_path, out_accept_len):
        assert t.dtype == torch.int32
    assert v_pages.shape == k_pages.shape and v_pages.dtype == k_pages.dtype
    dt = _dtype_code(k_pages)
    dims = AttnDims(B, B, int(max_spec_len), Hkv, Hkv, d, P, num_pages, max_pages, dt, dt, PATH_AUTO, 0.0)
    rc = lib().adaspec_kv_compact_path(k_pages.data_ptr(), v_pages.data_ptr(), block_table.data_ptr(),
                                       ctx_lens.data_ptr(), spec_lens.data_ptr(), out_path.data_ptr(),
                                       out_accept_len.data_ptr(), C.byref(dims), out_path.shape[1],
                                       _stream_ptr(stream))
    if rc != 0:
        raise AdaspecError(rc, "adaspec_kv_compact_path")


def check_accept_inputs(draft_tokens, spec_lens, temperature, *, vocab: int, max_spec_len: int, stream=None) -> int:
    """Runs the device-side check of the acceptance inputs and returns the flag word (synchronises)."""
    import torch
    for t in (draft_tokens, spec_lens):
        assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()
    assert temperature.is_cuda and temperature.dtype == torch.float32
    B, TD = spec_lens.shape[0], draft_tokens.shape[0]
    dims = AcceptDims(B, TD + B, TD, int(max_spec_len), int(vocab), BF16, BF16, int(max_spec_len) + 1, int(vocab),
                      int(vocab), PATH_AUTO, 0)
    flags = torch.zeros(1, dtype=torch.int32, device=spec_lens.device)
    rc = lib().adaspec_check_accept_inputs(draft_tokens.data_ptr(), spec_lens.data_ptr(), temperature.data_ptr(),
                                           C.byref(dims), flags.data_ptr(), _stream_ptr(stream))
    if rc != 0:
        raise AdaspecError(rc, "adaspec_check_accept_inputs")
    return int(flags.item())


def check_tree_parents(parents, spec_lens, *, max_spec_len: int, stream=None) -> int:
    """Runs the device-side check of a parent array and returns the flag word (synchronises)."""
    import torch
    assert parents.is_cuda and parents.dtype == torch.int32 and spec_lens.dtype == torch.int32
    flags = torch.zeros(1, dtype=torch.int32, device=parents.device)
    rc = lib().adaspec_check_tree_parents(parents.data_ptr(), spec_lens.data_ptr(), spec_lens.shape[0],
                                          parents.shape[0], int(max_spec_len), flags.data_ptr(), _stream_ptr(stream))
    if rc != 0:
        raise AdaspecError(rc, "adaspec_check_tree_parents")
    return int(flags.item())


def check_ragged_inputs(block_table, ctx_lens, spec_lens, dims: AttnDims, stream=None) -> int:
    """Runs the device-side metadata check and returns the flag word (synchronises)."""
    import torch
    flags = torch.zeros(1, dtype=torch.int32, device=block_table.device)
    rc = lib().adaspec_check_ragged_inputs(block_table.data_ptr(), ctx_lens.data_ptr(),
                                           spec_lens.data_ptr(), C.byref(dims), flags.data_ptr(),
                                           _stream_ptr(stream))
    if rc != 0:
        raise AdaspecError(rc, "adaspec_check_ragged_inputs")
    return int(flags.item())


def kv_append(k_new, v_new, k_pages, v_pages, block_table, ctx_lens, spec_lens, *, max_spec_len: int,
              stream=None) -> None:
    """adaspec_kv_append: writes the new tokens' K/V rows [TQ][Hkv][d] into the pages, in place."""
    import torch
    TQ, Hkv, d = k_new.shape
    num_pages, Hkv2, P, d2 = k_pages.shape
    B, max_pages = block_table.shape
    assert (Hkv2, d2) == (Hkv, d) and v_new.shape == k_new.shape and v_pages.shape == k_pages.shape
    assert k_new.dtype == v_new.dtype == k_pages.dtype == v_pages.dtype
    for t in (k_new, v_new, k_pages, v_pages, block_table, ctx_lens, spec_lens):
        assert t.is_cuda and t.is_contiguous()
    assert block_table.dtype == torch.int32 and ctx_lens.dtype == torch.int32 and spec_lens.dtype == torch.int32
    dt = _dtype_code(k_new)
    dims = AttnDims(B, TQ, int(max_spec_len), Hkv, Hkv, d, P, num_pages, max_pages, dt, dt, PATH_AUTO, 0.0)
    rc = lib().adaspec_kv_append(k_new.data_ptr(), v_new.data_ptr(), k_pages.data_ptr(), v_pages.data_ptr(),
                                 block_table.data_ptr(), ctx_lens.data_ptr(), spec_lens.data_ptr(),
                                 C.byref(dims), _stream_ptr(stream))
    if rc != 0:
        raise AdaspecError(rc, "adaspec_kv_append")


def commit(out_tokens, out_accept_len, spec_lens, ctx_lens, *, max_spec_len: int, next_spec_lens=None,
           committed_lens=None, next_ctx_lens=None, last_token=None, seq_tokens=None, seq_lens=None,
           stream=None):
    """adaspec_commit; returns (committed_lens, next_ctx_lens or None, last_token)."""
    import torch
    B, out_stride = out_tokens.shape
    dev = out_tokens.device
    for t in (out_tokens, out_accept_len, spec_lens, ctx_lens):
        assert t.is_cuda and t.is_contiguous() and t.dtype == torch.int32
    if committed_lens is None:
        committed_lens = torch.empty((B,), dtype=torch.int32, device=dev)
    if last_token is None:
        last_token = torch.empty((B,), dtype=torch.int32, device=dev)
    if next_spec_lens is not None and next_ctx_lens is None:
        next_ctx_lens = torch.empty((B,), dtype=torch.int32, device=dev)
    seq_stride = 0
    if seq_tokens is not None:
        assert seq_lens is not None and seq_tokens.is_contiguous() and seq_tokens.dtype == torch.int32
        assert seq_lens.dtype == torch.int32
        seq_stride = seq_tokens.shape[1]
    dims = CommitDims(B, int(max_spec_len), out_stride, seq_stride)
    ptr = lambda t: None if t is None else t.data_ptr()
    rc = lib().adaspec_commit(out_tokens.data_ptr(), out_accept_len.data_ptr(), spec_lens.data_ptr(),
                              ctx_lens.data_ptr(), ptr(next_spec_lens), committed_lens.data_ptr(),
                              ptr(next_ctx_lens), last_token.data_ptr(), ptr(seq_tokens), ptr(seq_lens),
                              C.byref(dims), _stream_ptr(stream))
    if rc != 0:
        raise AdaspecError(rc, "adaspec_commit")
    return committed_lens, next_ctx_lens, last_token


def draft_sample(draft_logits, temperature, uniforms, *, probs_dtype=None, draft_probs=None, out_rows=None,
                 draft_tokens=None, confidence=None, path: str = "auto", workspace=None, stream=None, timing=None):
    """adaspec_draft_sample; returns (draft_probs, draft_tokens [R] int32, confidence [R] float32).
    path "split" (ADASPEC_PATH_TWO_PASS for this call) cuts every row into four parts."""
    import torch
    R, V = draft_logits.shape
    dev = draft_logits.device
    assert draft_logits.is_cuda and draft_logits.stride(1) == 1
    assert temperature.dtype == torch.float32 and uniforms.dtype == torch.float32
    if draft_probs is None:
        assert out_rows is None
        draft_probs = torch.empty((R, V), dtype=probs_dtype or draft_logits.dtype, device=dev)
    assert draft_probs.stride(1) == 1 and draft_probs.shape[1] == V
    if draft_tokens is None:
        draft_tokens = torch.empty((R,), dtype=torch.int32, device=dev)
    if confidence is None:
        confidence = torch.empty((R,), dtype=torch.float32, device=dev)
    dims = DraftDims(R, V, _dtype_code(draft_logits), _dtype_code(draft_probs), draft_logits.stride(0),
                     draft_probs.stride(0), PATH_TWO_PASS if path == "split" else _PATHS[path], 0)
    _with_timing(dims, timing)
    L = lib()
    need = L.adaspec_draft_sample_workspace_bytes(C.byref(dims))
    ws = _workspace(need, dev, workspace, "draft") if need else None
    rc = L.adaspec_draft_sample(draft_logits.data_ptr(), temperature.data_ptr(), uniforms.data_ptr(),
                                None if out_rows is None else out_rows.data_ptr(), draft_probs.data_ptr(),
                                draft_tokens.data_ptr(), confidence.data_ptr(), C.byref(dims),
                                None if ws is None else ws.data_ptr(), 0 if ws is None else ws.numel(),
                                _stream_ptr(stream))
    if rc != 0:
        raise AdaspecError(rc, "adaspec_draft_sample")
    return draft_probs, draft_tokens, confidence
