"""adaspec_accept_noalloc (acceptance on the library's built-in scratch array, for callers that cannot
allocate) against adaspec_accept on a caller workspace: same kernels, so the outputs must be equal bit
for bit; both are also held to the oracle's bar.  Two calls in a row, the second with a smaller input
(the scratch array keeps the first call's contents), then the first again."""
import sys

import numpy as np
import pytest

import workloads as W
from tests.harness import compare_accept, to_device

pytestmark = pytest.mark.gpu


def _steps():
    big = W.make_custom_step(4242, ctx_lens=[40] * 24, spec_lens=[3, 0, 5, 2, 4, 1, 6, 0, 2, 3, 1, 5] * 2,
                             vocab=32000, logits_dtype="bf16", attention=False, logits_sigma=3.0, noise_sigma=1.5,
                             draft_temp=1.2, temperature=[0.8, 1.0, 0.0, 0.7] * 6, name="noalloc-big")
    small = W.make_custom_step(4243, ctx_lens=[40] * 5, spec_lens=[2, 4, 0, 1, 3], vocab=8192, logits_dtype="bf16",
                               attention=False, logits_sigma=3.0, noise_sigma=1.5, draft_temp=1.2,
                               temperature=[1.0, 0.0, 0.9, 0.8, 1.0], name="noalloc-small")
    return big, small


@pytest.mark.parametrize("path", ["auto", "two_pass", "fast", "vector"])
def test_accept_noalloc_equals_accept(path, oracle_mod):
    import torch
    import paper_2503_05096_amd as pkg
    big, small = _steps()
    for st in (big, small, big):
        dev = to_device(st, attention=False)
        print(f"[case] accept_noalloc {st.name} path={path} B={st.batch} TQ={st.total_q} V={st.vocab}",
              file=sys.stderr, flush=True)
        args = (dev.target_logits, dev.draft_probs, dev.draft_tokens, dev.uniforms, dev.spec_lens, dev.temperature)
        ref_tok, ref_len = pkg.accept(*args, max_spec_len=st.max_spec_len, path=path)
        toks = torch.full_like(ref_tok, -7)
        alen = torch.full_like(ref_len, -7)
        pkg.accept_noalloc(*args, toks, alen, max_spec_len=st.max_spec_len, path=path)
        torch.cuda.synchronize()
        assert torch.equal(toks, ref_tok) and torch.equal(alen, ref_len)
        rep = compare_accept(st, toks.cpu().numpy(), alen.cpu().numpy(), oracle_mod)
        assert rep["hard_mismatches"] == 0, rep["details"][:5]
        assert rep["ratio_near_ties"] + rep["cdf_near_ties"] <= 2, rep


def test_accept_noalloc_rejects_what_does_not_fit():
    import torch
    import paper_2503_05096_amd as pkg
    from paper_2503_05096_amd.binding import NOALLOC_SCRATCH_BYTES, AcceptDims, BF16
    import ctypes as C
    B = 200000
    dims = AcceptDims(B, 2 * B, B, 1, 1024, BF16, BF16, 2, 1024, 1024, 0, 0)
    assert pkg.lib().adaspec_accept_workspace_bytes(C.byref(dims)) > NOALLOC_SCRATCH_BYTES
    p = torch.zeros(64, dtype=torch.int32, device="cuda:0").data_ptr()
    assert pkg.lib().adaspec_accept_noalloc(p, p, p, p, p, p, p, p, C.byref(dims), None) == -5
