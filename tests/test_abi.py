"""Boundary checks that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments on the host before enqueuing anything.
Every call below fails validation, so no kernel is ever launched from this file."""
import ctypes as C
import os
import re

import pytest

import paper_2503_05096_amd as pkg
from paper_2503_05096_amd.binding import AttnDims, AcceptDims, EXPORTS, F32, BF16

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "adaspec.h")
PTR = 0x10000   # non-null, 256-byte aligned, never dereferenced: validation fails first


def test_header_symbols_are_exported():
    import glob
    from paper_2503_05096_amd import policy
    names = set()
    for h in glob.glob(os.path.join(os.path.dirname(HEADER), "*.h")):
        text = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names |= set(re.findall(r"\b(adaspec_[a-z_]+)\s*\(", text))
    assert names == set(EXPORTS) | set(policy.EXPORTS)
    L = pkg.lib()
    for n in names:
        assert hasattr(L, n), n
    assert pkg.version() >= 100
    assert pkg.status_string(0) == "ok" and "NULL" in pkg.status_string(-1)


def _attn_dims(**kw):
    base = dict(batch=2, total_q=5, max_spec_len=3, n_q_heads=8, n_kv_heads=2, head_dim=128, page_size=16,
                num_pages=64, max_pages_per_req=8, dtype=BF16, out_dtype=BF16, path=0, scale=0.0)
    base.update(kw)
    return AttnDims(**base)


def _accept_dims(**kw):
    base = dict(batch=2, total_q=5, total_draft=3, max_spec_len=3, vocab=1024, logits_dtype=BF16,
                probs_dtype=BF16, out_stride=4, logits_row_stride=1024, probs_row_stride=1024, path=0,
                reserved=0)
    base.update(kw)
    return AcceptDims(**base)


def _call_attn(dims, ptrs=None, ws=PTR, ws_bytes=1 << 40):
    p = [PTR] * 7 if ptrs is None else ptrs
    return pkg.lib().adaspec_verify_attn(*p, C.byref(dims), ws, ws_bytes, None)


def _call_accept(dims, ptrs=None, ws=PTR, ws_bytes=1 << 40):
    p = [PTR] * 8 if ptrs is None else ptrs
    return pkg.lib().adaspec_accept(*p, C.byref(dims), ws, ws_bytes, None)


@pytest.mark.parametrize("kw,code", [
    (dict(batch=-1), -2), (dict(total_q=1), -2), (dict(total_q=9), -2), (dict(n_kv_heads=3), -2),
    (dict(n_q_heads=0), -2), (dict(num_pages=0), -2), (dict(max_pages_per_req=0), -2),
    (dict(dtype=7), -3), (dict(out_dtype=1), -3), (dict(page_size=32), -6), (dict(head_dim=100), -6),
    (dict(head_dim=512), -6), (dict(path=5), -2), (dict(scale=-1.0), -2), (dict(max_spec_len=-1), -2),
    # work that does not fit the kernels' 32-bit counters: (request, split) pairs, then units
    (dict(batch=1 << 16, total_q=1 << 16, max_spec_len=0, max_pages_per_req=1 << 16), -6),
    (dict(batch=1 << 14, total_q=1 << 14, max_spec_len=0, max_pages_per_req=1 << 13, n_q_heads=1024,
          n_kv_heads=1024), -6),
])
def test_attn_rejects_bad_dims(kw, code):
    d = _attn_dims(**kw)
    assert _call_attn(d) == code
    assert pkg.lib().adaspec_verify_attn_workspace_bytes(C.byref(d)) == 0


def test_attn_rejects_null_misaligned_and_small_workspace():
    d = _attn_dims()
    need = pkg.lib().adaspec_verify_attn_workspace_bytes(C.byref(d))
    assert need > 0 and need % 256 == 0
    assert pkg.lib().adaspec_verify_attn(*[PTR] * 7, None, PTR, need, None) == -1
    for k in range(7):
        p = [PTR] * 7
        p[k] = None
        assert _call_attn(d, p) == -1
    assert _call_attn(d, ws=None) == -1
    for k in (0, 1, 2, 6):
        p = [PTR] * 7
        p[k] = PTR + 8
        assert _call_attn(d, p) == -4
    assert _call_attn(d, ws=PTR + 64) == -4
    assert _call_attn(d, ws_bytes=need - 1) == -5
    # out_dtype may be the input type or fp32, nothing else
    assert pkg.lib().adaspec_verify_attn_workspace_bytes(C.byref(_attn_dims(out_dtype=F32))) > 0


def test_attn_plan_mode_is_validated():
    assert _call_attn(_attn_dims(plan_mode=3)) == -2
    assert _call_attn(_attn_dims(plan_mode=-1)) == -2
    # metadata-only calls do not need the tensors, but they do need the metadata inputs and a workspace
    L = pkg.lib()
    d = _attn_dims(plan_mode=1)
    assert L.adaspec_verify_attn(None, None, None, None, PTR, PTR, None, C.byref(d), PTR, 1 << 30, None) == -1
    assert L.adaspec_verify_attn(None, None, None, PTR, PTR, PTR, None, C.byref(d), PTR, 16, None) == -5


def test_attn_workspace_grows_with_the_problem():
    f = lambda **kw: pkg.lib().adaspec_verify_attn_workspace_bytes(C.byref(_attn_dims(**kw)))
    assert f(batch=4, total_q=10) > f()
    assert f(max_pages_per_req=512) > f()
    assert f(max_spec_len=7) > f()


def test_empty_batch_is_a_no_op():
    assert _call_attn(_attn_dims(batch=0, total_q=0), [None] * 7, ws=None, ws_bytes=0) == 0
    assert _call_accept(_accept_dims(batch=0, total_q=0, total_draft=0), [None] * 8, ws=None, ws_bytes=0) == 0


@pytest.mark.parametrize("kw,code", [
    (dict(batch=-2), -2), (dict(total_draft=4), -2), (dict(vocab=0), -2), (dict(logits_dtype=9), -3),
    (dict(probs_dtype=-1), -3), (dict(logits_row_stride=1000), -2), (dict(probs_row_stride=8), -2),
    (dict(out_stride=3), -2), (dict(path=-1), -2), (dict(total_q=12, total_draft=10), -2),
])
def test_accept_rejects_bad_dims(kw, code):
    d = _accept_dims(**kw)
    assert _call_accept(d) == code
    assert pkg.lib().adaspec_accept_workspace_bytes(C.byref(d)) == 0


def test_accept_rejects_null_and_small_workspace():
    d = _accept_dims()
    need = pkg.lib().adaspec_accept_workspace_bytes(C.byref(d))
    assert need > 0
    for k in range(8):
        p = [PTR] * 8
        p[k] = None
        assert _call_accept(d, p) == -1
    assert _call_accept(d, ws=None) == -1
    assert _call_accept(d, ws=PTR + 16) == -4
    assert _call_accept(d, ws_bytes=need - 1) == -5
    # the register-resident path refuses shapes it cannot hold
    assert _call_accept(_accept_dims(path=2, logits_dtype=F32)) == -6
    assert _call_accept(_accept_dims(path=2, vocab=1001, logits_row_stride=1001, probs_row_stride=1001)) == -6


def test_accept_resolved_path_of_forced_paths():
    """The path query is host-only: forced paths come back as they are when the shape fits them, as
    ADASPEC_ERR_UNSUPPORTED when it does not, and invalid dims as their own status."""
    L = pkg.lib()
    q = lambda **kw: L.adaspec_accept_resolved_path(PTR, PTR, C.byref(_accept_dims(**kw)))
    for path in (1, 2, 3, 4):
        assert q(path=path) == path
    assert q(path=2, logits_dtype=F32) == -6 and q(path=4, logits_dtype=F32) == -6 and q(path=3, probs_dtype=F32) == -6
    big = dict(vocab=262144, logits_row_stride=262144, probs_row_stride=262144)
    assert q(path=3, **big) == 3 and q(path=2, **big) == -6 and q(path=4, **big) == -6
    assert L.adaspec_accept_resolved_path(PTR + 8, PTR, C.byref(_accept_dims(path=2))) == -6     # misaligned rows
    assert q(path=5) == -2 and q(vocab=0) == -2
    assert L.adaspec_accept_resolved_path(PTR, PTR, None) == -1


def test_misc_entry_points_validate():
    L = pkg.lib()
    assert L.adaspec_check_ragged_inputs(None, PTR, PTR, C.byref(_attn_dims()), PTR, None) == -1
    assert L.adaspec_check_ragged_inputs(PTR, PTR, PTR, C.byref(_attn_dims(batch=-1)), PTR, None) == -2
    assert "unknown" in pkg.status_string(-99)


def test_kv_append_and_commit_validate():
    from paper_2503_05096_amd.binding import CommitDims
    L = pkg.lib()
    d = _attn_dims()
    assert L.adaspec_kv_append(PTR, PTR, PTR, PTR, PTR, PTR, PTR, None, None) == -1
    assert L.adaspec_kv_append(None, PTR, PTR, PTR, PTR, PTR, PTR, C.byref(d), None) == -1
    assert L.adaspec_kv_append(PTR + 4, PTR, PTR, PTR, PTR, PTR, PTR, C.byref(d), None) == -4
    assert L.adaspec_kv_append(PTR, PTR, PTR, PTR, PTR, PTR, PTR, C.byref(_attn_dims(n_kv_heads=0)), None) == -2
    assert L.adaspec_kv_append(PTR, PTR, PTR, PTR, PTR, PTR, PTR, C.byref(_attn_dims(dtype=7)), None) == -3
    assert L.adaspec_kv_append(PTR, PTR, PTR, PTR, PTR, PTR, PTR, C.byref(_attn_dims(head_dim=4, dtype=BF16)), None) == -6
    assert L.adaspec_kv_append(None, None, None, None, None, None, None, C.byref(_attn_dims(batch=0, total_q=0)), None) == 0
    c = CommitDims(4, 3, 4, 0)
    args = [PTR] * 4 + [None] + [PTR, None, PTR, None, None]
    assert L.adaspec_commit(*args, None, None) == -1
    assert L.adaspec_commit(*args, C.byref(CommitDims(4, 3, 3, 0)), None) == -2      # out_stride < k_max + 1
    assert L.adaspec_commit(*args, C.byref(CommitDims(-1, 3, 4, 0)), None) == -2
    bad = list(args); bad[0] = None
    assert L.adaspec_commit(*bad, C.byref(c), None) == -1
    half = list(args); half[8] = PTR                                                  # seq_tokens without seq_lens
    assert L.adaspec_commit(*half, C.byref(c), None) == -1
    both = list(args); both[8] = PTR; both[9] = PTR
    assert L.adaspec_commit(*both, C.byref(c), None) == -2                            # seq_stride 0
    assert L.adaspec_commit(*[None] * 10, C.byref(CommitDims(0, 3, 4, 0)), None) == 0


def test_draft_sample_validates():
    from paper_2503_05096_amd.binding import DraftDims
    L = pkg.lib()
    ok = DraftDims(4, 1024, BF16, BF16, 1024, 1024, 0, 0)
    args = [PTR, PTR, PTR, None, PTR, PTR, PTR]
    call = lambda a, d, ws=None, nb=0: L.adaspec_draft_sample(*a, None if d is None else C.byref(d), ws, nb, None)
    assert call(args, None) == -1
    assert call(args, DraftDims(-1, 1024, BF16, BF16, 1024, 1024, 0, 0)) == -2
    assert call(args, DraftDims(4, 1024, BF16, BF16, 1000, 1024, 0, 0)) == -2
    assert call(args, DraftDims(4, 1024, 9, BF16, 1024, 1024, 0, 0)) == -3
    assert call(args, DraftDims(4, 1001, BF16, BF16, 1001, 1001, 0, 0)) == -6
    assert call(args, DraftDims(4, 1024, BF16, BF16, 1028, 1024, 0, 0)) == -6
    assert call(args, DraftDims(4, 1024, F32, BF16, 1024, 1024, 2, 0)) == -6   # fast path needs 16-bit logits
    assert call(args, DraftDims(4, 1024, BF16, BF16, 1024, 1024, 5, 0)) == -2
    assert call(args, DraftDims(4, 1024, BF16, BF16, 1024, 1024, 3, 0)) == -2  # the streaming path is the acceptance's
    bad = list(args); bad[0] = None
    assert call(bad, ok) == -1
    mis = list(args); mis[4] = PTR + 8
    assert call(mis, ok) == -4
    # the split form: needs its workspace, 256-byte aligned and large enough; not for fp32 logits
    split = DraftDims(4, 1024, BF16, BF16, 1024, 1024, 4, 0)
    need = L.adaspec_draft_sample_workspace_bytes(C.byref(split))
    assert need > 0 and L.adaspec_draft_sample_workspace_bytes(C.byref(ok)) == need
    assert L.adaspec_draft_sample_workspace_bytes(C.byref(DraftDims(4, 1024, BF16, BF16, 1024, 1024, 2, 0))) == 0
    assert L.adaspec_draft_sample_workspace_bytes(C.byref(DraftDims(4, 1024, F32, BF16, 1024, 1024, 0, 0))) == 0
    assert L.adaspec_draft_sample_workspace_bytes(None) == 0
    assert call(args, split) == -1 and call(args, split, PTR + 16, need) == -4 and call(args, split, PTR, need - 1) == -5
    assert call(args, DraftDims(4, 1024, F32, BF16, 1024, 1024, 4, 0), PTR, need) == -6
    assert call([None] * 7, DraftDims(0, 1024, BF16, BF16, 1024, 1024, 0, 0)) == 0


def test_one_hip_runtime_whatever_the_import_order():
    # torch ships its own HIP runtime; the library must bind to that copy even when it is the first
    # thing a fresh process touches (checked in a child process: this one has torch loaded already)
    import subprocess, sys
    code = ("import paper_2503_05096_amd as p; p.lib(); "
            "print(len({l.split()[-1] for l in open('/proc/self/maps') if 'libamdhip64' in l}))")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, cwd=root, check=True)
    assert out.stdout.strip() == "1", out.stdout + out.stderr
    assert pkg.binding.hip_runtime() is not None


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    from paper_2503_05096_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        binding.lib()


# ------------------------------------------------------------------ tree verification
def test_tree_calls_validate_on_the_host():
    L = pkg.lib()
    d = _attn_dims()
    tree_attn = lambda dims, ptrs, ws=PTR, nbytes=1 << 40: L.adaspec_verify_attn_tree(*ptrs, C.byref(dims), ws, nbytes, None)
    assert tree_attn(d, [PTR] * 6 + [None, PTR]) == -1                      # parents missing
    assert tree_attn(_attn_dims(batch=-1), [PTR] * 8) == -2
    assert tree_attn(_attn_dims(total_q=66, max_spec_len=64), [PTR] * 8) == -6   # more than 64 nodes per request
    assert tree_attn(d, [PTR] * 8, nbytes=16) == -5
    assert tree_attn(d, [PTR + 8] + [PTR] * 7) == -4
    assert tree_attn(_attn_dims(batch=0, total_q=0), [None] * 8, None, 0) == 0

    a = _accept_dims()
    tree_acc = lambda dims, ptrs, ws=PTR, nbytes=1 << 40: L.adaspec_accept_tree(*ptrs, C.byref(dims), ws, nbytes, None)
    for k in (0, 3, 4, 5, 6, 7, 8, 9):
        p = [PTR] * 10
        p[k] = None
        assert tree_acc(a, p) == -1, k
    assert tree_acc(_accept_dims(path=3), [PTR] * 10) == -6                 # no streaming / two-pass form for trees
    assert tree_acc(_accept_dims(path=2, vocab=1001, logits_row_stride=1001, probs_row_stride=1001),
                    [PTR] * 10) == -6                                       # the fast kernel needs V % 8 == 0
    assert tree_acc(_accept_dims(total_q=68, total_draft=66, max_spec_len=64, out_stride=65), [PTR] * 10) == -6
    assert tree_acc(_accept_dims(out_stride=3), [PTR] * 10) == -2
    assert tree_acc(a, [PTR] * 10, nbytes=16) == -5
    assert tree_acc(a, [PTR] * 10, ws=PTR + 64) == -4
    assert tree_acc(_accept_dims(batch=0, total_q=0, total_draft=0), [None] * 10, None, 0) == 0

    chka = L.adaspec_check_accept_inputs
    assert chka(PTR, None, PTR, C.byref(a), PTR, None) == -1 and chka(PTR, PTR, PTR, C.byref(a), None, None) == -1
    assert chka(None, PTR, PTR, C.byref(a), PTR, None) == -1 and chka(PTR, PTR, PTR, None, PTR, None) == -1
    assert chka(PTR, PTR, PTR, C.byref(_accept_dims(vocab=0)), PTR, None) == -2

    chk = L.adaspec_check_tree_parents
    assert chk(None, PTR, 2, 5, 3, PTR, None) == -1 and chk(PTR, PTR, 2, 5, 3, None, None) == -1
    assert chk(PTR, PTR, 2, 9, 3, PTR, None) == -2 and chk(PTR, PTR, 2, 66, 64, PTR, None) == -6

    compact = lambda dims, ptrs, stride=4: L.adaspec_kv_compact_path(*ptrs, C.byref(dims), stride, None)
    for k in range(7):
        p = [PTR] * 7
        p[k] = None
        assert compact(d, p) == -1, k
    assert compact(d, [PTR] * 7, stride=3) == -2                            # narrower than max_spec_len + 1
    assert compact(d, [PTR + 8] + [PTR] * 6) == -4
    assert compact(_attn_dims(head_dim=4), [PTR] * 7) == -6                 # rows are moved in 16-byte pieces
    assert compact(_attn_dims(batch=0, total_q=0), [None] * 7) == 0


# ------------------------------------------------------------------ the headers themselves
@pytest.mark.parametrize("header", ["adaspec.h", "adaspec_policy.h"])
def test_headers_are_plain_c(header, tmp_path):
    """The boundary is a C ABI: each header compiles on its own as C99 with warnings as errors."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    src = tmp_path / "t.c"
    src.write_text(f'#include "{header}"\nint main(void) {{ return 0; }}\n')
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", f"-I{inc}", str(src)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_accept_noalloc_rejects_on_the_host():
    """The entry point without a workspace validates like adaspec_accept, and refuses dims whose workspace
    would not fit its built-in scratch array, all before any HIP call."""
    from paper_2503_05096_amd.binding import NOALLOC_SCRATCH_BYTES
    L = pkg.lib()
    call = lambda d, ptrs=None: L.adaspec_accept_noalloc(*([PTR] * 8 if ptrs is None else ptrs), C.byref(d), None)
    assert call(_accept_dims(vocab=0)) == -2
    assert call(_accept_dims(logits_dtype=9)) == -3
    assert call(_accept_dims(), [None] + [PTR] * 7) == -1
    B = 200000
    big = _accept_dims(batch=B, total_q=2 * B, total_draft=B, max_spec_len=1, out_stride=2)
    assert L.adaspec_accept_workspace_bytes(C.byref(big)) > NOALLOC_SCRATCH_BYTES
    assert call(big) == -5
    header = open(HEADER).read()
    assert re.search(r"#define\s+ADASPEC_NOALLOC_SCRATCH_BYTES\s+\(\(size_t\)8\s*<<\s*20\)", header)
    assert NOALLOC_SCRATCH_BYTES == 8 << 20
