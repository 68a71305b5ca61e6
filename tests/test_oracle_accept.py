"""Pins for the acceptance oracle (CPU only).

The rule is randomised, so it is pinned by (i) a hand-derived example, (ii) the
distributional facts that make speculative decoding lossless (Sec. 2.2: same
outputs as autoregressive decoding) checked by chi-square over 10^6 seeded
trials, (iii) closed forms that follow from the rule (acceptance probability
sum_x min(p_x, q_x); residual distribution), (iv) the greedy statement of
Sec. 2.2 / Fig. 1 as a direct integer check, (v) special cases that reduce to
textbook inverse-CDF sampling.
"""
import os

import numpy as np
import pytest
from scipy.stats import chi2

import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "accept_hand_example.txt")
# textbook chi-square critical values at alpha = 0.001 for 1..7 degrees of freedom
CHI2_CRIT_001 = [10.83, 13.82, 16.27, 18.47, 20.52, 22.46, 24.32]


def _softmax64(l, T=1.0):
    z = (np.asarray(l, np.float64) - np.max(l)) / T
    e = np.exp(z)
    return e / e.sum()


def _chi2_stat(counts, probs):
    n = counts.sum()
    exp = n * probs
    keep = exp > 0
    assert counts[~keep].sum() == 0
    return float((((counts - exp) ** 2)[keep] / exp[keep]).sum()), int(keep.sum()) - 1


def _crit(dof):
    return CHI2_CRIT_001[dof - 1] if dof <= 7 else float(chi2.ppf(0.999, dof))


def test_textbook_critical_values_agree_with_scipy():
    for dof, c in enumerate(CHI2_CRIT_001, start=1):
        assert abs(chi2.ppf(0.999, dof) - c) < 0.01


# ---------------------------------------------------------------- hand example
def test_hand_example(oracle_mod):
    logits = np.log(np.array([1, 2, 3, 4], dtype=np.float64)).astype(np.float32)
    q = np.array([0.4, 0.3, 0.2, 0.1], dtype=np.float32)
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 12
    for x, u0, u1, acc, cand in rows:
        x = int(x)
        r = oracle_mod.accept_row(logits, None if x < 0 else q, logits_dtype="f32", probs_dtype="f32",
                                  T=1.0, x=x, u0=float(u0), u1=float(u1))
        assert (r["accept"], r["cand"]) == (bool(int(acc)), int(cand)), (x, u0, u1, r)
    r = oracle_mod.accept_row(logits, q, logits_dtype="f32", probs_dtype="f32", T=1.0, x=1, u0=0.5, u1=0.5)
    assert abs(r["ratio"] - 2.0 / 3.0) < 1e-7 and abs(r["R"] - 0.4) < 1e-7


# ---------------------------------------------------- distributional invariants
def _trial_batch(oracle_mod, logits_rows, q_rows, k, n_trials, seed, T=1.0):
    """n_trials independent requests, all with the same k target rows (+ bonus
    row) and the same k draft distributions; x_j ~ q_j, fresh uniforms."""
    rng = np.random.default_rng(seed)
    V = logits_rows.shape[1]
    tl = np.tile(logits_rows.astype(np.float32), (n_trials, 1))             # [(k+1) n][V]
    dp = np.tile(q_rows.astype(np.float32), (n_trials, 1)) if k else np.zeros((0, V), np.float32)
    toks = np.empty((n_trials, k), dtype=np.int32)
    for j in range(k):
        qn = q_rows[j].astype(np.float32).astype(np.float64)
        toks[:, j] = rng.choice(V, size=n_trials, p=qn / qn.sum())
    uni = rng.random((n_trials * (k + 1), 2), dtype=np.float32)
    out, alen, _ = oracle_mod.accept(tl, dp, toks.reshape(-1), uni, np.full(n_trials, k, np.int32),
                                     np.full(n_trials, T, np.float32), logits_dtype="f32",
                                     probs_dtype="f32", want_row_info=False)
    return out, alen, toks


@pytest.mark.parametrize("V,seed", [(2, 1), (5, 2), (8, 3)])
def test_invariant1_output_distribution_is_target(oracle_mod, V, seed):
    """k = 1: the first emitted token (accepted draft or recovered token) ~ p."""
    rng = np.random.default_rng(100 + seed)
    logits = rng.normal(0, 1.5, size=(2, V))
    q = _softmax64(logits[0] + rng.normal(0, 1.5, size=V))[None]
    n = 1_000_000
    out, alen, toks = _trial_batch(oracle_mod, logits, q, 1, n, seed)
    p32 = _softmax64(logits[0].astype(np.float32))
    q32 = q[0].astype(np.float32).astype(np.float64)
    stat, dof = _chi2_stat(np.bincount(out[:, 0], minlength=V), p32)
    assert dof == V - 1 and stat < _crit(dof), (stat, dof)
    # acceptance probability = sum_x min(p_x, q_x) (q normalised exactly as sampled)
    qn = q32 / q32.sum()
    pacc = np.minimum(p32 / q32, 1.0) @ qn
    rate = (alen == 1).mean()
    assert abs(rate - pacc) < 4 * np.sqrt(pacc * (1 - pacc) / n)
    # conditional on rejection the token ~ max(0, p - q) normalised
    rej = alen == 0
    res = np.maximum(p32 - q32, 0)
    stat, dof = _chi2_stat(np.bincount(out[rej, 0], minlength=V), res / res.sum())
    assert stat < _crit(max(dof, 1)), (stat, dof)
    # accepted trials emitted the draft itself, then a bonus token ~ p(bonus row)
    acc = ~rej
    assert np.array_equal(out[acc, 0], toks[acc, 0]) and np.all(out[rej, 1] == -1)
    stat, dof = _chi2_stat(np.bincount(out[acc, 1], minlength=V), _softmax64(logits[1].astype(np.float32)))
    assert stat < _crit(dof), (stat, dof)


def test_invariant1_multi_draft_positions(oracle_mod):
    """k = 3: position 0 ~ p_0 over all trials; position j (given it was emitted)
    ~ p_j; the position after three accepted drafts is the bonus row's p_3."""
    V, k, n = 6, 3, 1_000_000
    rng = np.random.default_rng(7)
    logits = rng.normal(0, 1.2, size=(k + 1, V))
    q = np.stack([_softmax64(logits[j] + rng.normal(0, 0.8, size=V)) for j in range(k)])
    out, alen, _ = _trial_batch(oracle_mod, logits, q, k, n, 11)
    assert np.array_equal((out >= 0).sum(axis=1), alen + 1)        # a_i drafts + exactly one more
    for j in range(k + 1):
        emitted = out[:, j] >= 0
        assert np.array_equal(emitted, alen >= j)
        stat, dof = _chi2_stat(np.bincount(out[emitted, j], minlength=V),
                               _softmax64(logits[j].astype(np.float32)))
        assert stat < _crit(dof), (j, stat, dof)
    # independence of consecutive positions: joint of (pos 0, pos 1) given both emitted
    both = alen >= 1
    joint = np.bincount(out[both, 0] * V + out[both, 1], minlength=V * V).astype(float)
    p0c = np.bincount(out[both, 0], minlength=V) / both.sum()
    p1 = _softmax64(logits[1].astype(np.float32))
    stat, dof = _chi2_stat(joint, np.outer(p0c, p1).reshape(-1))
    assert stat < float(chi2.ppf(0.999, V * V - V)), stat


def test_temperature_scales_logits_not_draft(oracle_mod):
    V = 7
    rng = np.random.default_rng(3)
    logits = rng.normal(0, 2, size=(1, V))
    n = 400_000
    out, _, _ = _trial_batch(oracle_mod, logits, np.zeros((0, V)), 0, n, 5, T=0.5)
    stat, dof = _chi2_stat(np.bincount(out[:, 0], minlength=V), _softmax64(logits[0].astype(np.float32), 0.5))
    assert stat < _crit(dof)
    stat_wrong, _ = _chi2_stat(np.bincount(out[:, 0], minlength=V), _softmax64(logits[0].astype(np.float32), 1.0))
    assert stat_wrong > 100 * _crit(dof)


# --------------------------------------------------------------- invariant 2
def _greedy_expect(st):
    cu = st.cu_q
    toks, alens = [], []
    for i in range(st.batch):
        k = int(st.spec_lens[i])
        a, emitted = k, []
        for j in range(k):
            z = int(np.argmax(W.to_f64(st.target_logits[cu[i] + j], st.logits_dtype)))
            x = int(st.draft_tokens[cu[i] - i + j])
            if x != z:
                a = j
                emitted.append(z)
                break
            emitted.append(x)
        if a == k:
            emitted.append(int(np.argmax(W.to_f64(st.target_logits[cu[i] + k], st.logits_dtype))))
        toks.append(emitted)
        alens.append(a)
    return toks, alens


@pytest.mark.parametrize("ties", [False, True])
def test_invariant2_greedy_longest_matching_prefix(oracle_mod, ties):
    st = W.make_custom_step(31, ctx_lens=[64] * 40, spec_lens=list(np.arange(40) % 6), vocab=64,
                            logits_dtype="bf16", temperature=0.0, logits_sigma=3.0, noise_sigma=0.7,
                            attention=False, planted_ties=ties)
    # make some drafts certainly match the target argmax so long prefixes occur
    cu = st.cu_q
    rng = np.random.default_rng(0)
    for i in range(st.batch):
        for j in range(int(st.spec_lens[i])):
            if rng.random() < 0.6:
                st.draft_tokens[cu[i] - i + j] = np.argmax(W.to_f64(st.target_logits[cu[i] + j], "bf16"))
    out, alen, _ = oracle_mod.accept(st.target_logits, st.draft_probs, st.draft_tokens, st.uniforms,
                                     st.spec_lens, st.temperature, logits_dtype="bf16", probs_dtype="bf16")
    toks, alens = _greedy_expect(st)
    assert list(alen) == alens
    assert len(set(alens)) > 3
    for i in range(st.batch):
        assert list(out[i, :len(toks[i])]) == toks[i] and np.all(out[i, len(toks[i]):] == -1)
    if ties:   # np.argmax and the oracle must both take the lowest index of a tie
        row = W.to_f64(st.target_logits[0], "bf16")
        assert (row == row.max()).sum() >= 2


# --------------------------------------------------------------- invariant 3
def test_invariant3_p_equals_q_accepts_everything(oracle_mod):
    # (a) exactly equal: constant logits, V a power of two -> p = q = 1/V exactly
    V, B, k = 16, 50, 4
    rng = np.random.default_rng(2)
    tl = np.full((B * (k + 1), V), 0.375, dtype=np.float32)
    dp = np.full((B * k, V), 1.0 / V, dtype=np.float32)
    toks = rng.integers(0, V, size=B * k).astype(np.int32)
    uni = rng.random((B * (k + 1), 2), dtype=np.float32)
    uni[::3, 0] = np.float32(1.0 - 2.0 ** -24)            # the largest float32 below 1
    out, alen, info = oracle_mod.accept(tl, dp, toks, uni, np.full(B, k, np.int32),
                                        np.full(B, 0.7, np.float32), logits_dtype="f32", probs_dtype="f32")
    assert np.all(alen == k) and np.array_equal(out[:, :k].reshape(-1), toks)
    assert np.all(info[:, 1][~np.isnan(info[:, 1])] == 1.0)
    # (b) q = float32(softmax(logits / T)): ratio = 1 up to one float32 rounding
    tl = rng.normal(0, 2, size=(B * (k + 1), 200)).astype(np.float32)
    T = 0.8
    dp = np.stack([_softmax64(tl[r], np.float64(np.float32(T))) for r in range(tl.shape[0])
                   if (r % (k + 1)) != k]).astype(np.float32)
    toks = np.array([rng.choice(200, p=dp[d].astype(np.float64) / dp[d].astype(np.float64).sum())
                     for d in range(B * k)], dtype=np.int32)
    uni = np.minimum(rng.random((B * (k + 1), 2), dtype=np.float32), np.float32(0.999999))
    _, alen, _ = oracle_mod.accept(tl, dp, toks, uni, np.full(B, k, np.int32),
                                   np.full(B, T, np.float32), logits_dtype="f32", probs_dtype="f32")
    assert np.all(alen == k)


def test_residual_zero_falls_back_to_target(oracle_mod):
    V = 8
    tl = np.zeros(V, dtype=np.float32)
    q = np.full(V, 1.0 / V, dtype=np.float32)
    for u1, want in [(0.0, 0), (0.124, 0), (0.126, 1), (0.99, 7)]:
        r = oracle_mod.accept_row(tl, q, logits_dtype="f32", probs_dtype="f32", T=1.0, x=3, u0=0.5, u1=u1)
        assert r["accept"] and r["cand"] == want and abs(r["R"] - 1.0) < 1e-15


# ------------------------------------------------------------- special cases
def test_k0_is_plain_inverse_cdf_sampling(oracle_mod):
    st = W.make_custom_step(41, ctx_lens=[32] * 300, spec_lens=[0] * 300, vocab=500,
                            logits_dtype="bf16", temperature=0.9, attention=False)
    out, alen, _ = oracle_mod.accept(st.target_logits, st.draft_probs, st.draft_tokens, st.uniforms,
                                     st.spec_lens, st.temperature, logits_dtype="bf16", probs_dtype="bf16")
    assert np.all(alen == 0) and np.all(out[:, 1:] == -1) if out.shape[1] > 1 else True
    T = np.float64(np.float32(0.9))
    for i in range(300):
        p = _softmax64(W.to_f64(st.target_logits[i], "bf16"), T)
        c = np.cumsum(p)
        want = int(np.searchsorted(c, np.float64(st.uniforms[i, 1]) * c[-1], side="right"))
        assert out[i, 0] == want


def test_inverse_cdf_never_picks_zero_mass_and_is_strict(oracle_mod):
    logits = np.log(np.array([1, 2, 3, 4], dtype=np.float64)).astype(np.float32)
    q = np.array([0.4, 0.3, 0.2, 0.1], dtype=np.float32)
    r = oracle_mod.accept_row(logits, q, logits_dtype="f32", probs_dtype="f32", T=1.0, x=0, u0=0.9, u1=0.0)
    assert r["cand"] == 2                     # tokens 0, 1 carry no residual mass; u1 = 0 skips them
    lo, hi, R = oracle_mod.cdf_interval(logits, q, logits_dtype="f32", probs_dtype="f32", T=1.0, t=3)
    assert abs(lo - 0.1) < 1e-7 and abs(hi - 0.4) < 1e-7 and abs(R - 0.4) < 1e-7
    assert abs(r["cdf_before"]) < 1e-12 and abs(r["cdf_incl"] - 0.1) < 1e-7


def test_zero_draft_probability_counts_as_accept(oracle_mod):
    logits = np.zeros(4, dtype=np.float32)
    q = np.array([0.0, 0.5, 0.5, 0.0], dtype=np.float32)
    r = oracle_mod.accept_row(logits, q, logits_dtype="f32", probs_dtype="f32", T=1.0, x=0, u0=0.999, u1=0.5)
    assert r["accept"] and np.isinf(r["ratio"])


def test_tiny_temperature_agrees_with_greedy_branch(oracle_mod):
    st = W.make_custom_step(43, ctx_lens=[32] * 60, spec_lens=list(np.arange(60) % 4 + 1), vocab=128,
                            logits_dtype="f32", temperature=0.0, attention=False)
    cu = st.cu_q
    rng = np.random.default_rng(1)
    top = np.argmax(st.target_logits, axis=1)
    st.target_logits[np.arange(st.total_q), top] += np.float32(0.1)   # a clear winner per row
    for i in range(st.batch):                 # mix of matching and non-matching drafts
        for j in range(int(st.spec_lens[i])):
            if rng.random() < 0.7:
                st.draft_tokens[cu[i] - i + j] = np.argmax(st.target_logits[cu[i] + j])
    srt = np.sort(st.target_logits, axis=1)
    assert np.all(srt[:, -1] - srt[:, -2] > 0.02)     # no near-ties at the top
    uni = np.maximum(st.uniforms, np.float32(1e-6))
    args = (st.target_logits, st.draft_probs, st.draft_tokens, uni, st.spec_lens)
    g = oracle_mod.accept(*args, np.zeros(60, np.float32), logits_dtype="f32", probs_dtype="f32")
    s = oracle_mod.accept(*args, np.full(60, 1e-4, np.float32), logits_dtype="f32", probs_dtype="f32")
    assert np.array_equal(g[0], s[0]) and np.array_equal(g[1], s[1])


def test_mixed_temperatures_and_layout(oracle_mod):
    """Per-request temperature, row ownership (cu_q / cu_q - i), out_stride padding:
    the batched call equals row-by-row calls assembled by hand."""
    st = W.make_custom_step(47, ctx_lens=[32] * 9, spec_lens=[0, 2, 5, 1, 0, 3, 4, 2, 1], vocab=300,
                            logits_dtype="bf16", temperature=[0, 0.7, 1.0, 0, 1.0, 0.7, 0, 1.0, 0.7],
                            attention=False)
    out, alen, info = oracle_mod.accept(st.target_logits, st.draft_probs, st.draft_tokens, st.uniforms,
                                        st.spec_lens, st.temperature, logits_dtype="bf16",
                                        probs_dtype="bf16", out_stride=8)
    assert out.shape == (9, 8)
    cu = st.cu_q
    for i in range(9):
        k, T = int(st.spec_lens[i]), float(st.temperature[i])
        exp_tokens, a = [], k
        for j in range(k + 1):
            r = cu[i] + j
            bonus = j == k
            res = oracle_mod.accept_row(st.target_logits[r], None if bonus else st.draft_probs[r - i],
                                        logits_dtype="bf16", probs_dtype="bf16", T=T,
                                        x=-1 if bonus else int(st.draft_tokens[r - i]),
                                        u0=float(st.uniforms[r, 0]), u1=float(st.uniforms[r, 1]))
            assert info[r, 2] == res["cand"]
            if bonus or not res["accept"]:
                exp_tokens.append(res["cand"])
                a = j
                break
            exp_tokens.append(int(st.draft_tokens[r - i]))
        assert alen[i] == a and list(out[i, :a + 1]) == exp_tokens and np.all(out[i, a + 1:] == -1)
        assert np.all(np.isnan(info[cu[i] + a + 1:cu[i + 1], 0]))   # rows after the stop were not visited


def test_rejects_bad_arguments(oracle_mod):
    st = W.make_custom_step(49, ctx_lens=[32] * 2, spec_lens=[2, 1], vocab=32, attention=False)
    with pytest.raises(ValueError):
        oracle_mod.accept(st.target_logits, st.draft_probs, st.draft_tokens, st.uniforms, st.spec_lens,
                          st.temperature, logits_dtype="f32", probs_dtype="f32", out_stride=2)


def test_masked_tokens_are_never_emitted(oracle_mod):
    """-inf target logits (masked tokens) have p = 0: never accepted unless q is 0 there too (then the ratio
    test is skipped by the q == 0 rule only for tokens the draft can never propose), never recovered, never
    drawn as bonus."""
    rng = np.random.default_rng(5)
    B = 200
    spec = rng.integers(0, 5, size=B).astype(np.int32)
    st = W.make_custom_step(88, ctx_lens=spec + 1, spec_lens=spec, vocab=32, attention=False, masked_frac=0.5,
                            temperature=rng.choice([0.0, 0.6, 1.0], size=B), noise_sigma=0.5)
    toks, alen, _ = oracle_mod.accept(st.target_logits, st.draft_probs, st.draft_tokens, st.uniforms, st.spec_lens,
                                      st.temperature, logits_dtype="f32", probs_dtype="f32")
    cu = st.cu_q
    assert alen.max() >= 2
    for i in range(B):
        for j in range(alen[i] + 1):
            assert np.isfinite(st.target_logits[cu[i] + j, toks[i, j]]), (i, j)
