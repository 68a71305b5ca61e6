"""Pins for the tree-verification oracle (CPU only).

The paper fixes the chain case; the tree case is pinned by (i) its reduction to the chain oracle
(an independent, separately pinned function) when every node has at most one child, (ii) a dense
masked-softmax formulation of tree attention written differently, with the mask built by walking
the parent pointers in Python, (iii) the fact that makes tree verification lossless -- the emitted
tokens follow the target distribution -- by chi-square over 10^6 seeded trials, with the closed
forms for the per-child acceptance probabilities, (iv) the greedy walk as a direct integer check,
(v) a hand-worked residual chain (tests/golden/tree_residual_hand_example.txt), (vi) the closed
form of repeated residuals, max(0, p - c_s q) with c_{s+1} = c_s + its mass.
"""
import os

import numpy as np
import pytest
from scipy.stats import chi2

import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "tree_residual_hand_example.txt")


def _softmax64(l, T=1.0):
    z = (np.asarray(l, np.float64) - np.max(l)) / T
    e = np.exp(z)
    return e / e.sum()


def _chi2_ok(counts, probs, alpha=0.999):
    n = counts.sum()
    exp = n * probs
    keep = exp > 0
    assert counts[~keep].sum() == 0
    stat = float((((counts - exp) ** 2)[keep] / exp[keep]).sum())
    dof = max(int(keep.sum()) - 1, 1)
    return stat < float(chi2.ppf(alpha, dof)), stat, dof


# ------------------------------------------------------------------ attention
def _tree_step(seed, ctx, spec, width=3, **kw):
    st = W.make_custom_step(seed, ctx_lens=ctx, spec_lens=spec, acceptance=False, **kw)
    return W.attach_tree(st, max_width=width)


def _ancestors(par, j):
    out = []
    while j >= 0:
        out.append(j)
        j = int(par[j])
    return out


def _dense_tree_attention(st):
    """softmax(mask(Q K^T * scale)) V per request in matrix form; mask from the parent pointers."""
    G = st.n_q_heads // st.n_kv_heads
    out = np.empty((st.total_q, st.n_q_heads, st.head_dim))
    cu, P = st.cu_q, st.page_size
    scale = 1.0 / np.sqrt(st.head_dim)
    for i in range(st.batch):
        L, n = int(st.ctx_lens[i]), int(st.spec_lens[i]) + 1
        K = np.stack([W.to_f64(st.k_pages[st.block_table[i, t // P], :, t % P], st.dtype) for t in range(L)])
        V = np.stack([W.to_f64(st.v_pages[st.block_table[i, t // P], :, t % P], st.dtype) for t in range(L)])
        Q = W.to_f64(st.q[cu[i]:cu[i + 1]], st.dtype)
        par = st.parents[cu[i]:cu[i + 1]]
        mask = np.zeros((n, L), dtype=bool)
        mask[:, :L - n] = True
        for j in range(n):
            mask[j, [L - n + a for a in _ancestors(par, j)]] = True
        for h in range(st.n_q_heads):
            S = np.where(mask, (Q[:, h] @ K[:, h // G].T) * scale, -np.inf)
            E = np.exp(S - S.max(axis=1, keepdims=True))
            out[cu[i]:cu[i + 1], h] = (E / E.sum(axis=1, keepdims=True)) @ V[:, h // G]
    return out


def _run_tree(oracle_mod, st, **kw):
    return oracle_mod.verify_attn_tree(st.q, st.k_pages, st.v_pages, st.block_table, st.ctx_lens,
                                       st.spec_lens, st.parents, dtype=st.dtype, **kw)


@pytest.mark.parametrize("dtype,hq,hkv,d", [("f32", 4, 4, 16), ("bf16", 8, 2, 32)])
def test_tree_attention_dense_masked_form(oracle_mod, dtype, hq, hkv, d):
    st = _tree_step(21, [9, 16, 17, 40, 33, 12], [0, 3, 1, 7, 5, 11], n_q_heads=hq, n_kv_heads=hkv,
                    head_dim=d, dtype=dtype)
    cu = st.cu_q
    assert max(np.bincount(st.parents[cu[i] + 1:cu[i + 1]]).max() for i in (3, 4, 5)) > 1   # real branching
    out, _ = _run_tree(oracle_mod, st)
    assert not np.isnan(out).any()
    np.testing.assert_allclose(out, _dense_tree_attention(st), rtol=0, atol=1e-12)


def test_chain_parents_give_the_causal_oracle_bit_for_bit(oracle_mod):
    st = W.make_custom_step(5, ctx_lens=[20, 7, 48, 33], spec_lens=[4, 0, 6, 2], n_q_heads=4,
                            n_kv_heads=2, head_dim=32, dtype="bf16", acceptance=False)
    W.attach_tree(st, chain=True)
    a, ar = _run_tree(oracle_mod, st)
    b, br = oracle_mod.verify_attn(st.q, st.k_pages, st.v_pages, st.block_table, st.ctx_lens,
                                   st.spec_lens, dtype=st.dtype)
    assert np.array_equal(a, b) and np.array_equal(ar, br)


def test_a_node_sees_its_ancestors_and_nothing_else_of_the_tree(oracle_mod):
    st = _tree_step(8, [30], [6], n_q_heads=2, n_kv_heads=2, head_dim=16, dtype="f32", width=2)
    par = st.parents
    base, P = int(st.ctx_lens[0]) - 7, st.page_size
    ref, _ = _run_tree(oracle_mod, st)
    for b in range(7):
        k2 = st.k_pages.copy()
        t = base + b
        k2[st.block_table[0, t // P], :, t % P] += 1.0
        out = oracle_mod.verify_attn_tree(st.q, k2, st.v_pages, st.block_table, st.ctx_lens, st.spec_lens,
                                          par, dtype=st.dtype)[0]
        for j in range(7):
            changed = not np.array_equal(out[j], ref[j])
            assert changed == (b in _ancestors(par, j)), (b, j)


def test_tree_attention_rejects_a_parent_after_its_child(oracle_mod):
    st = _tree_step(3, [12], [3], n_q_heads=2, n_kv_heads=2, head_dim=16, dtype="f32")
    for bad in ([-1, 0, 2, 1], [0, 0, 1, 2], [-1, 1, 0, 0], [-1, 0, -1, 1]):
        with pytest.raises(ValueError):
            oracle_mod.verify_attn_tree(st.q, st.k_pages, st.v_pages, st.block_table, st.ctx_lens,
                                        st.spec_lens, np.array(bad, np.int32), dtype=st.dtype)


# ----------------------------------------------------------------- acceptance
def _accept_tree(oracle_mod, st, **kw):
    return oracle_mod.accept_tree(st.target_logits, st.draft_probs, st.draft_tokens, st.parents,
                                  st.uniforms, st.spec_lens, st.temperature,
                                  logits_dtype=st.logits_dtype, probs_dtype=st.probs_dtype, **kw)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_chain_tree_is_the_chain_oracle(oracle_mod, dtype):
    for seed in range(6):
        rng = np.random.default_rng(seed)
        B = 24
        spec = rng.integers(0, 7, size=B)
        T = rng.choice([0.0, 0.7, 1.0, 1.3], size=B)
        st = W.make_custom_step(400 + seed, ctx_lens=spec + 1, spec_lens=spec, vocab=64, logits_dtype=dtype,
                                temperature=T, attention=False, noise_sigma=0.6)
        W.attach_tree(st, chain=True)
        toks, alen, path, _, stop = _accept_tree(oracle_mod, st)
        o_tok, o_alen, info = oracle_mod.accept(st.target_logits, st.draft_probs, st.draft_tokens, st.uniforms,
                                                st.spec_lens, st.temperature, logits_dtype=st.logits_dtype,
                                                probs_dtype=st.probs_dtype)
        assert np.array_equal(toks, o_tok) and np.array_equal(alen, o_alen)
        assert 0 < alen.mean() < spec.mean()                      # both outcomes occur
        for i in range(B):
            assert list(path[i, :alen[i]]) == list(range(1, alen[i] + 1))
            assert stop[i, 0] == alen[i]
            if T[i] != 0.0:                                       # same mass and prefix sums, bit for bit
                r = st.cu_q[i] + alen[i]
                assert stop[i, 2] == info[r, 3] and stop[i, 3] == info[r, 4] and stop[i, 4] == info[r, 5]


def _star_trials(oracle_mod, logits_rows, q_root, w, n_trials, seed, T=1.0):
    """n_trials requests whose tree is a root with w children drawn independently from q_root."""
    rng = np.random.default_rng(seed)
    V = logits_rows.shape[1]
    assert logits_rows.shape[0] == w + 1
    tl = np.tile(logits_rows.astype(np.float32), (n_trials, 1))
    dp = np.zeros((n_trials, w, V), np.float32)
    dp[:, 0] = q_root.astype(np.float32)                           # only the root's row is ever read
    qn = q_root.astype(np.float32).astype(np.float64)
    toks = rng.choice(V, size=(n_trials, w), p=qn / qn.sum()).astype(np.int32)
    uni = rng.random((n_trials * (w + 1), 2), dtype=np.float32)
    par = np.tile(np.array([-1] + [0] * w, np.int32), n_trials)
    out = oracle_mod.accept_tree(tl, dp.reshape(-1, V), toks.reshape(-1), par, uni, np.full(n_trials, w, np.int32),
                                 np.full(n_trials, T, np.float32), logits_dtype="f32", probs_dtype="f32")
    return out, toks


@pytest.mark.parametrize("V,w,seed", [(3, 2, 1), (6, 2, 2), (6, 3, 3), (8, 4, 4)])
def test_first_token_of_a_star_tree_follows_the_target(oracle_mod, V, w, seed):
    rng = np.random.default_rng(50 + seed)
    logits = rng.normal(0, 1.5, size=(w + 1, V))
    q = _softmax64(logits[0] + rng.normal(0, 1.5, size=V))
    n = 1_000_000
    (out, alen, path, _, stop), toks = _star_trials(oracle_mod, logits, q, w, n, seed)
    p = _softmax64(logits[0].astype(np.float32))
    ok, stat, dof = _chi2_ok(np.bincount(out[:, 0], minlength=V), p)
    assert ok, (stat, dof)
    # closed forms: child m is reached after m-1 rejections and accepted with sum_x min(P_x, q_x)
    q32 = q.astype(np.float32).astype(np.float64)
    qn = q32 / q32.sum()
    P, reached = p.copy(), np.ones(n, dtype=bool)
    for m in range(1, w + 1):
        pacc = float(np.minimum(P / q32, 1.0) @ qn)
        acc = reached & (path[:, 0] == m)
        rate = acc.sum() / reached.sum()
        assert abs(rate - pacc) < 4.5 * np.sqrt(pacc * (1 - pacc) / reached.sum()), (m, rate, pacc)
        assert np.array_equal(out[acc, 0], toks[acc, m - 1])        # an accepted child emits its own token
        reached &= ~acc
        r = np.maximum(P - q32, 0)
        P = r / r.sum()
    # every child rejected: the token follows the last residual, and nothing comes after it
    assert np.array_equal(reached, alen == 0) and np.all(out[reached, 1] == -1)
    ok, stat, dof = _chi2_ok(np.bincount(out[reached, 0], minlength=V), P)
    assert ok, (stat, dof)
    assert np.all(stop[reached, 1] == w) and np.all(stop[~reached, 1] == 0)
    # after an accepted child c the next token is a plain draw from that child's row (it is a leaf)
    for c in range(1, w + 1):
        sel = path[:, 0] == c
        ok, stat, dof = _chi2_ok(np.bincount(out[sel, 1], minlength=V), _softmax64(logits[c].astype(np.float32)))
        assert ok, (c, stat, dof)


def test_two_level_tree_every_level_follows_its_nodes_target(oracle_mod):
    """root -> {1, 2}; 1 -> {3, 4}; 2 -> {5}.  Whatever node the walk stands on, the token it emits
    next (an accepted child's or a drawn one) follows that node's target row."""
    V, n = 5, 1_000_000
    par1 = np.array([-1, 0, 0, 1, 1, 2], np.int32)
    k = 5
    rng = np.random.default_rng(9)
    logits = rng.normal(0, 1.3, size=(k + 1, V))
    qs = np.stack([_softmax64(logits[j] + rng.normal(0, 1.0, size=V)) for j in range(k)]).astype(np.float32)
    toks = np.empty((n, k), np.int32)
    for c in range(1, k + 1):
        qn = qs[par1[c]].astype(np.float64)
        toks[:, c - 1] = rng.choice(V, size=n, p=qn / qn.sum())
    uni = rng.random((n * (k + 1), 2), dtype=np.float32)
    out, alen, path, _, stop = oracle_mod.accept_tree(
        np.tile(logits.astype(np.float32), (n, 1)), np.tile(qs, (n, 1)), toks.reshape(-1), np.tile(par1, n), uni,
        np.full(n, k, np.int32), np.ones(n, np.float32), logits_dtype="f32", probs_dtype="f32")
    assert set(np.unique(alen)) == {0, 1, 2}
    ok, stat, dof = _chi2_ok(np.bincount(out[:, 0], minlength=V), _softmax64(logits[0].astype(np.float32)))
    assert ok, (stat, dof)
    for c in (1, 2):
        sel = path[:, 0] == c
        ok, stat, dof = _chi2_ok(np.bincount(out[sel, 1], minlength=V), _softmax64(logits[c].astype(np.float32)))
        assert ok, (c, stat, dof)
        # ... and independently of the token that led there
        joint = np.bincount(out[sel, 0] * V + out[sel, 1], minlength=V * V).astype(float)
        first = np.bincount(out[sel, 0], minlength=V) / sel.sum()
        ok, stat, dof = _chi2_ok(joint, np.outer(first, _softmax64(logits[c].astype(np.float32))).reshape(-1))
        assert stat < float(chi2.ppf(0.999, V * V - V)), (c, stat)
    for c in (3, 4, 5):
        sel = path[:, 1] == c
        assert sel.sum() > 1000 and np.all(par1[c] == path[sel, 0])  # a path never jumps between branches
        ok, stat, dof = _chi2_ok(np.bincount(out[sel, 2], minlength=V), _softmax64(logits[c].astype(np.float32)))
        assert ok, (c, stat, dof)
    assert np.array_equal((out >= 0).sum(axis=1), alen + 1) and np.array_equal((path >= 0).sum(axis=1), alen)


def test_greedy_walk_follows_the_targets_argmax(oracle_mod):
    rng = np.random.default_rng(3)
    B = 64
    spec = rng.integers(0, 9, size=B)
    st = W.make_custom_step(77, ctx_lens=spec + 1, spec_lens=spec, vocab=12, temperature=0.0, attention=False,
                            noise_sigma=0.7, planted_ties=True)
    W.attach_tree(st, max_width=3)
    toks, alen, path, test_info, _ = _accept_tree(oracle_mod, st)
    assert np.isnan(test_info).all() and alen.max() >= 2 and (alen == 0).any()
    cu = st.cu_q
    for i in range(B):
        par = st.parents[cu[i]:cu[i + 1]]
        u, walked, emitted = 0, [], []
        while True:
            z = int(np.argmax(st.target_logits[cu[i] + u]))         # numpy: first maximum
            nxt = [c for c in range(u + 1, spec[i] + 1) if par[c] == u and st.draft_tokens[cu[i] - i + c - 1] == z]
            emitted.append(z)
            if not nxt:
                break
            u = nxt[0]
            walked.append(u)
        assert list(path[i, :alen[i]]) == walked and list(toks[i, :alen[i] + 1]) == emitted


def test_p_equals_q_accepts_the_first_child(oracle_mod):
    V, n, w = 16, 200, 3
    rng = np.random.default_rng(1)
    logits = rng.normal(0, 2, size=(n * (w + 1), V)).astype(np.float32)
    dp = np.zeros((n, w, V), np.float32)
    for i in range(n):
        dp[i, 0] = _softmax64(logits[i * (w + 1)])
    toks = rng.integers(0, V, size=(n, w)).astype(np.int32)
    uni = rng.random((n * (w + 1), 2), dtype=np.float32)
    # ratio is 1 up to the float32 rounding of q: keep the uniforms clear of it
    uni[:, 0] = np.minimum(uni[:, 0], 0.999)
    out, alen, path, test_info, _ = oracle_mod.accept_tree(
        logits, dp.reshape(-1, V), toks.reshape(-1), np.tile(np.array([-1, 0, 0, 0], np.int32), n), uni,
        np.full(n, w, np.int32), np.ones(n, np.float32), logits_dtype="f32", probs_dtype="f32")
    assert np.all(alen == 1) and np.all(path[:, 0] == 1) and np.array_equal(out[:, 0], toks[:, 0])
    ratios = test_info.reshape(n, w + 1, 2)[:, 1, 0]
    assert np.allclose(ratios, 1.0, atol=1e-6)


def test_hand_worked_residual_chain(oracle_mod):
    """p = (.1,.2,.3,.4), q = (.4,.3,.2,.1): one rejection leaves (0,0,.1,.3) (mass .4), a second one
    max(0, (0,0,.25,.75) - q) = (0,0,.05,.65) (mass .7); the file lists intervals and ratios."""
    logits = np.log(np.array([1, 2, 3, 4], dtype=np.float64)).astype(np.float32)
    q = np.array([0.4, 0.3, 0.2, 0.1], dtype=np.float32)
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    kinds = set()
    for kind, *vals in rows:
        kinds.add(kind)
        if kind == "interval":
            rej, t, lo, hi, R = int(vals[0]), int(vals[1]), *map(float, vals[2:])
            got = oracle_mod.tree_cdf_interval(logits, q, logits_dtype="f32", probs_dtype="f32", T=1.0,
                                               rejections=rej, t=t)
            assert np.allclose(got, (lo, hi, R), atol=2e-7), (vals, got)
        else:                                                       # walk: tokens u0s u1 -> path token
            toks = [int(x) for x in vals[0].split(",")]
            u0s = [float(x) for x in vals[1].split(",")]
            u1, want_child, want_tok = float(vals[2]), int(vals[3]), int(vals[4])
            w = len(toks)
            uni = np.zeros((w + 1, 2), np.float32)
            uni[:w, 0] = u0s
            uni[:, 1] = u1
            dp = np.zeros((w, 4), np.float32)
            dp[0] = q
            out, alen, path, _, _ = oracle_mod.accept_tree(
                np.tile(logits, (w + 1, 1)), dp, np.array(toks, np.int32), np.array([-1] + [0] * w, np.int32), uni,
                np.array([w], np.int32), np.ones(1, np.float32), logits_dtype="f32", probs_dtype="f32")
            assert (int(path[0, 0]), int(out[0, 0])) == (want_child, want_tok), (vals, path, out)
    assert kinds == {"interval", "walk"}


@pytest.mark.parametrize("seed,V,T", [(1, 50, 1.0), (2, 333, 0.7), (3, 1000, 1.6)])
def test_repeated_residuals_have_a_closed_form(oracle_mod, seed, V, T):
    """Unrolling P_s = norm(max(0, P_{s-1} - q)) gives P_s = max(0, p - c_s q) / G_s with
    G_s = sum_v max(0, p_v - c_s q_v), c_0 = 0 and c_{s+1} = c_s + G_s (substitute and pull the positive
    factor 1/G_s out of the max).  The oracle steps through the stages; this evaluates the closed form
    directly and compares every token's interval width and the mass the s-th stage leaves."""
    rng = np.random.default_rng(seed)
    logits = rng.normal(0, 2.0, V).astype(np.float32)
    q = _softmax64(logits.astype(np.float64) / T + rng.normal(0, 0.7, V)).astype(np.float32)
    p = _softmax64(logits, T)
    q64 = q.astype(np.float64)
    c, G_prev = 0.0, 1.0
    for s in range(0, 5):
        g = np.maximum(0.0, p - c * q64)
        G = g.sum()
        assert G > 1e-6                                            # the case this form covers
        # mass of the stage as the oracle reports it: R_s = G_s / G_{s-1} (R_0 = 1: the target distribution)
        for t in rng.choice(V, size=12, replace=False):
            lo, hi, R = oracle_mod.tree_cdf_interval(logits, q if s else None, logits_dtype="f32",
                                                     probs_dtype="f32", T=T, rejections=s, t=int(t))
            assert abs(R - G / G_prev) < 1e-12, (s, R, G / G_prev)
            assert abs((hi - lo) / R - g[t] / G) < 1e-12, (s, t)
            assert abs(lo / R - g[:t].sum() / G) < 1e-11, (s, t)
        c, G_prev = c + G, G


def test_zero_mass_residual_is_left_as_it_was(oracle_mod):
    """Once the distribution equals q the positive part of (P - q) is empty: the state stays, and a
    token of zero draft probability is accepted on sight."""
    logits = np.array([0.0, -np.inf, 0.0], np.float32)             # p = (.5, 0, .5) exactly
    q = np.array([0.5, 0.0, 0.5], np.float32)
    lo, hi, R = oracle_mod.tree_cdf_interval(logits, q, logits_dtype="f32", probs_dtype="f32", T=1.0,
                                             rejections=3, t=2)
    assert (lo, hi, R) == (0.5, 1.0, 1.0)
    q0 = np.array([0.0, 0.5, 0.5], np.float32)
    out, alen, path, info, _ = oracle_mod.accept_tree(
        np.tile(logits, (2, 1)), q0[None], np.array([0], np.int32), np.array([-1, 0], np.int32),
        np.array([[0.999, 0.1], [0.2, 0.3]], np.float32), np.array([1], np.int32), np.ones(1, np.float32),
        logits_dtype="f32", probs_dtype="f32")
    assert alen[0] == 1 and np.isinf(info[1, 0])


def test_accept_tree_rejects_bad_arguments(oracle_mod):
    logits = np.zeros((3, 4), np.float32)
    args = (np.full((2, 4), .25, np.float32), np.zeros(2, np.int32))
    uni, T = np.zeros((3, 2), np.float32), np.ones(1, np.float32)
    with pytest.raises(ValueError):
        oracle_mod.accept_tree(logits, *args, np.array([-1, 0, 2], np.int32), uni, np.array([2], np.int32), T,
                               logits_dtype="f32", probs_dtype="f32")
    with pytest.raises(ValueError):
        oracle_mod.accept_tree(logits, *args, np.array([-1, 0, 0], np.int32), uni, np.array([2], np.int32), T,
                               logits_dtype="f32", probs_dtype="f32", out_stride=2)
