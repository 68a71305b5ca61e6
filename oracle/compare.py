"""Comparers of the parity bar (TEST INFRASTRUCTURE, like everything under oracle/): attention max-abs
error; acceptance with near-tie accounting.

Attention within a max-abs error of the oracle; emitted tokens and accept lengths bit-exact, except at
rows where the decision sits within 1e-5 of its threshold in the oracle's own float64 numbers (accept
test: |u0 - p_x/q_x| < 1e-5; inverse-CDF draw: u1*R within 1e-5*R of the interval the other token owns).
Such rows are counted and reported, never silently dropped; a request is compared up to its first
near-tie.  The `oracle` argument is the oracle package itself (the functions are called through it).
"""
from __future__ import annotations

import numpy as np

NEAR_TIE = 1e-5


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


def compare_accept_tree(st, gpu_tokens, gpu_alen, gpu_path, oracle, out_stride=None) -> dict:
    """Tree acceptance against the oracle's walk, request by request.  Where the two walks part, the
    first decision they differ on is looked up in the oracle's own float64 numbers: an accept test
    within 1e-5 of its uniform, or a draw within 1e-5 of the mass of the boundary, is a counted
    near-tie; anything else is a hard mismatch."""
    o_tok, o_alen, o_path, test_info, stop_info = oracle.accept_tree(
        st.target_logits, st.draft_probs, st.draft_tokens, st.parents, st.uniforms, st.spec_lens,
        st.temperature, logits_dtype=st.logits_dtype, probs_dtype=st.probs_dtype, out_stride=out_stride)
    assert gpu_tokens.shape == o_tok.shape and gpu_alen.shape == o_alen.shape and gpu_path.shape == o_path.shape
    cu = st.cu_q
    rep = dict(requests=st.batch, exact=0, ratio_near_ties=0, cdf_near_ties=0, hard_mismatches=0,
               details=[], oracle_mean_accept_len=float(o_alen.mean()) if st.batch else 0.0)
    for i in range(st.batch):
        if (gpu_alen[i] == o_alen[i] and np.array_equal(gpu_tokens[i], o_tok[i])
                and np.array_equal(gpu_path[i], o_path[i])):
            rep["exact"] += 1
            continue
        k, T = int(st.spec_lens[i]), float(st.temperature[i])
        par = st.parents[cu[i]:cu[i] + k + 1]
        ga, oa = int(gpu_alen[i]), int(o_alen[i])
        # common prefix of the two paths
        a = 0
        while a < min(ga, oa) and gpu_path[i, a] == o_path[i, a]:
            a += 1
        u = int(o_path[i, a - 1]) if a else 0                      # node both walks stand on
        g_next = int(gpu_path[i, a]) if a < ga else -1
        o_next = int(o_path[i, a]) if a < oa else -1
        ok_shape = (0 <= ga <= k and np.array_equal(gpu_tokens[i, :a], o_tok[i, :a])
                    and (g_next < 0 or (u < g_next <= k and par[g_next] == u)))
        if not ok_shape or T == 0.0:
            rep["hard_mismatches"] += 1
            rep["details"].append((i, "shape/greedy", ga, oa, list(gpu_path[i]), list(o_path[i])))
            continue
        if g_next != o_next:
            # the first child the two sides judge differently is the smaller of the two (none = after all)
            c = min(x for x in (g_next, o_next) if x >= 0)
            u0, ratio = float(st.uniforms[cu[i] + c - 1, 0]), test_info[cu[i] + c, 0]
            if np.isfinite(ratio) and abs(u0 - ratio) < NEAR_TIE:
                rep["ratio_near_ties"] += 1
            else:
                rep["hard_mismatches"] += 1
                rep["details"].append((i, "accept-test", u, c, g_next, o_next, u0, float(ratio)))
            continue
        # both stop at u (g_next == o_next == -1) but emit different tokens
        tg, to = int(gpu_tokens[i, a]), int(o_tok[i, a])
        pad_ok = np.all(gpu_tokens[i, a + 1:] == -1) and np.all(gpu_path[i, a:] == -1)
        if g_next >= 0 or tg == to or not pad_ok or not (0 <= tg < st.vocab):
            rep["hard_mismatches"] += 1
            rep["details"].append((i, "token/padding", u, tg, to))
            continue
        rej = int(stop_info[i, 1])
        assert int(stop_info[i, 0]) == u
        lo, hi, R = oracle.tree_cdf_interval(st.target_logits[cu[i] + u],
                                             st.draft_probs[cu[i] - i + u] if rej else None,
                                             logits_dtype=st.logits_dtype, probs_dtype=st.probs_dtype,
                                             T=T, rejections=rej, t=tg)
        tau = float(st.uniforms[cu[i] + u, 1]) * R
        if lo - NEAR_TIE * R <= tau < hi + NEAR_TIE * R:
            rep["cdf_near_ties"] += 1
        else:
            rep["hard_mismatches"] += 1
            rep["details"].append((i, "cdf", u, tg, to, tau, lo, hi, R))
    return rep
