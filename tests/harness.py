"""Shared test/bench plumbing: host workload -> device tensors, and the two
comparers (attention max-abs error; acceptance with near-tie accounting).

The comparers implement the parity bar: attention within a max-abs error of the
oracle; emitted tokens and accept lengths bit-exact, except at rows where the
decision sits within 1e-5 of its threshold in the oracle's own float64 numbers
(accept test: |u0 - p_x/q_x| < 1e-5; inverse-CDF draw: u1*R within 1e-5*R of the
interval the other token owns).  Such rows are counted and reported, never
silently dropped; a request is compared up to its first near-tie.
"""
from __future__ import annotations

from types import SimpleNamespace

import numpy as np

NEAR_TIE = 1e-5


def _torch_from(arr: np.ndarray, dtype: str, device):
    import torch
    if dtype == "bf16":
        return torch.from_numpy(arr.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(arr).to(device)


def to_device(st, device="cuda:0", attention=True, acceptance=True):
    import torch
    d = SimpleNamespace()
    d.spec_lens = torch.from_numpy(st.spec_lens).to(device)
    if attention and st.q is not None:
        d.ctx_lens = torch.from_numpy(st.ctx_lens).to(device)
        d.block_table = torch.from_numpy(st.block_table).to(device)
        d.q = _torch_from(st.q, st.dtype, device)
        d.k_pages = _torch_from(st.k_pages, st.dtype, device)
        d.v_pages = _torch_from(st.v_pages, st.dtype, device)
    if acceptance and st.target_logits is not None:
        d.target_logits = _torch_from(st.target_logits, st.logits_dtype, device)
        d.draft_probs = _torch_from(st.draft_probs, st.probs_dtype, device)
        d.draft_tokens = torch.from_numpy(st.draft_tokens).to(device)
        d.uniforms = torch.from_numpy(st.uniforms).to(device)
        d.temperature = torch.from_numpy(st.temperature).to(device)
    return d


def compare_attention(out_gpu, ref_f64: np.ndarray, ref_rounded, dtype: str) -> dict:
    import torch
    g = out_gpu.detach().to(torch.float64).cpu().numpy()
    rep = dict(nan=int(np.isnan(g).sum()),
               max_abs_vs_f64=float(np.nanmax(np.abs(g - ref_f64))) if g.size else 0.0)
    if ref_rounded is not None:
        rep["max_abs_vs_rounded"] = float(np.nanmax(np.abs(g - ref_rounded))) if g.size else 0.0
        rep["frac_bit_equal_rounded"] = float((g == ref_rounded).mean()) if g.size else 1.0
    if rep["nan"]:
        rep["max_abs_vs_f64"] = float("inf")
    return rep


def compare_accept(st, gpu_tokens: np.ndarray, gpu_alen: np.ndarray, oracle, out_stride=None) -> dict:
    """Element-by-element comparison of the acceptance outputs with the oracle's."""
    o_tok, o_alen, info = oracle.accept(st.target_logits, st.draft_probs, st.draft_tokens, st.uniforms,
                                        st.spec_lens, st.temperature, logits_dtype=st.logits_dtype,
                                        probs_dtype=st.probs_dtype, out_stride=out_stride)
    assert gpu_tokens.shape == o_tok.shape and gpu_alen.shape == o_alen.shape
    cu = st.cu_q
    rep = dict(requests=st.batch, exact=0, ratio_near_ties=0, cdf_near_ties=0, hard_mismatches=0,
               details=[], oracle_mean_accept_len=float(o_alen.mean()) if st.batch else 0.0)
    for i in range(st.batch):
        if gpu_alen[i] == o_alen[i] and np.array_equal(gpu_tokens[i], o_tok[i]):
            rep["exact"] += 1
            continue
        k, T = int(st.spec_lens[i]), float(st.temperature[i])
        ga, oa = int(gpu_alen[i]), int(o_alen[i])
        a = min(ga, oa)
        if not (0 <= ga <= k) or not np.array_equal(gpu_tokens[i, :a], o_tok[i, :a]):
            rep["hard_mismatches"] += 1
            rep["details"].append((i, "prefix", ga, oa))
            continue
        r = cu[i] + a
        if ga != oa:
            # the two sides disagree on the accept test of row a
            u0, ratio = float(st.uniforms[r, 0]), info[r, 1]
            if T != 0.0 and np.isfinite(ratio) and abs(u0 - ratio) < NEAR_TIE:
                rep["ratio_near_ties"] += 1
            else:
                rep["hard_mismatches"] += 1
                rep["details"].append((i, "accept-test", ga, oa, u0, float(ratio)))
            continue
        # same stop row, different emitted token; the -1 padding must still be right
        tg, to = int(gpu_tokens[i, a]), int(o_tok[i, a])
        pad_ok = np.all(gpu_tokens[i, a + 1:] == -1)
        if tg == to or T == 0.0 or not pad_ok or not (0 <= tg < st.vocab):
            rep["hard_mismatches"] += 1
            rep["details"].append((i, "token/padding", tg, to))
            continue
        bonus = a == k
        lo, hi, R = oracle.cdf_interval(st.target_logits[r], None if bonus else st.draft_probs[r - i],
                                        logits_dtype=st.logits_dtype, probs_dtype=st.probs_dtype,
                                        T=T, t=tg)
        tau = float(st.uniforms[r, 1]) * R
        if lo - NEAR_TIE * R <= tau < hi + NEAR_TIE * R:
            rep["cdf_near_ties"] += 1
        else:
            rep["hard_mismatches"] += 1
            rep["details"].append((i, "cdf", tg, to, tau, lo, hi, R))
    return rep
