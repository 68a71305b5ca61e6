"""Pins for the oracle of the draft-side sampling step (probability row, token, confidence).

The softmax is checked against scipy's, the draw against numpy's searchsorted on the cumulative
sum and against the frequencies a regular grid of uniforms must produce, the greedy form against
planted ties, and the rule "a token of probability zero is never drawn" at its edge (u = 0).
"""
import numpy as np
import pytest
from scipy.special import softmax

import workloads as W


def test_hand_example(oracle_mod):
    l = np.log(np.array([[1, 2, 1, 4.0]], np.float32))               # p = 1/8, 1/4, 1/8, 1/2
    for u, tok in [(0.0, 0), (0.12, 0), (0.13, 1), (0.3, 1), (0.38, 2), (0.49, 2), (0.51, 3), (0.999, 3)]:
        q, t, c, info = oracle_mod.draft_sample(l, [1.0], [u], logits_dtype="f32", probs_dtype="f32")
        assert t[0] == tok, (u, t)
        assert abs(c[0] - [0.125, 0.25, 0.125, 0.5][tok]) < 1e-7
    # temperature sharpens: T = 0.5 squares the weights -> 1, 4, 1, 16 over 22
    q, t, c, _ = oracle_mod.draft_sample(l, [0.5], [0.25], logits_dtype="f32", probs_dtype="f32")
    assert np.allclose(q[0], np.array([1, 4, 1, 16]) / 22, rtol=1e-6) and t[0] == 2      # cum 1/22, 5/22, 6/22 > 5.5/22


@pytest.mark.parametrize("pdt", ["f32", "bf16", "f16"])
def test_probability_row_is_the_rounded_textbook_softmax(pdt, oracle_mod):
    rng = np.random.default_rng(4)
    R, V = 5, 4096
    l = (3 * rng.standard_normal((R, V))).astype(np.float32)
    T = np.array([1.0, 0.7, 1.3, 0.0, 2.0], np.float32)
    q, tok, conf, info = oracle_mod.draft_sample(l, T, rng.random(R).astype(np.float32), logits_dtype="f32",
                                                  probs_dtype=pdt)
    Teff = np.where(T == 0, 1.0, T).astype(np.float64)
    ref = softmax(l.astype(np.float64) / Teff[:, None], axis=1)
    ulp = {"f32": 2.0 ** -23, "bf16": 2.0 ** -7, "f16": 2.0 ** -10}[pdt]
    assert np.all(np.abs(q - ref) <= 0.5 * ulp * ref + 1e-300 + (6e-8 if pdt == "f16" else 0))   # one rounding (f16: subnormal quantum)
    ref_r = np.vectorize(lambda x: oracle_mod.round_to_dtype(float(x), pdt))(ref[:, :256])
    assert np.mean(ref_r == q[:, :256]) > 0.999                      # identical but for last-bit ties of exp
    assert np.allclose(info[:, 2], q.sum(axis=1), rtol=1e-12)
    assert np.all(conf == q[np.arange(R), tok])


def test_draw_is_the_strict_inverse_cdf_of_the_rounded_row(oracle_mod):
    rng = np.random.default_rng(8)
    R, V = 64, 2048
    l = W.f32_to_bf16_bits((3 * rng.standard_normal((R, V))).astype(np.float32))
    u = rng.random(R).astype(np.float32)
    T = np.full(R, 0.9, np.float32)
    q, tok, conf, info = oracle_mod.draft_sample(l, T, u, logits_dtype="bf16", probs_dtype="bf16")
    for r in range(R):
        cs = np.cumsum(q[r])                                          # same left-to-right order
        t = int(np.searchsorted(cs, float(u[r]) * cs[-1], side="right"))
        assert tok[r] == t
        assert q[r, tok[r]] > 0


def test_grid_of_uniforms_reproduces_the_row(oracle_mod):
    l = np.log(np.array([[3, 0.5, 2, 0.25, 1, 1.25]], np.float32))
    N = 4000
    u = ((np.arange(N) + 0.5) / N).astype(np.float32)
    L = np.repeat(l, N, axis=0)
    q, tok, _, _ = oracle_mod.draft_sample(L, np.ones(N, np.float32), u, logits_dtype="f32", probs_dtype="f32")
    freq = np.bincount(tok, minlength=6) / N
    assert np.all(np.abs(freq - q[0] / q[0].sum()) <= 1.5 / N)


def test_zero_probability_tokens_are_never_drawn(oracle_mod):
    l = np.array([[-np.inf, -np.inf, 0.0, -np.inf, 1.0, -np.inf]], np.float32)
    for u in (0.0, 0.2, 0.26, 0.27, 0.999999):
        q, tok, conf, _ = oracle_mod.draft_sample(l, [1.0], [u], logits_dtype="f32", probs_dtype="f32")
        assert tok[0] in (2, 4) and conf[0] > 0
    q, tok, _, _ = oracle_mod.draft_sample(l, [1.0], [0.0], logits_dtype="f32", probs_dtype="f32")
    assert tok[0] == 2                                                # first token with mass, not index 0
    # bf16 rounding flushes tiny probabilities to zero: such tokens cannot be drawn either
    l2 = np.array([[0.0, -200.0, 0.0]], np.float32)
    q, tok, _, _ = oracle_mod.draft_sample(l2, [1.0], [0.5], logits_dtype="f32", probs_dtype="bf16")
    assert q[0, 1] == 0.0 and tok[0] == 2                             # cum .5, .5, 1.0 ; .5 is not > .5


def test_greedy_takes_the_lowest_index_among_ties(oracle_mod):
    rng = np.random.default_rng(2)
    l = W.f32_to_bf16_bits(rng.standard_normal((3, 512)).astype(np.float32))
    top = W.f32_to_bf16_bits(np.array([9.0], np.float32))[0]
    l[0, [77, 300, 301]] = top
    l[1, [511]] = top
    l[2, [0, 5]] = top
    q, tok, conf, info = oracle_mod.draft_sample(l, np.zeros(3, np.float32), [0.9, 0.9, 0.9],
                                                  logits_dtype="bf16", probs_dtype="bf16")
    assert tok.tolist() == [77, 511, 0]
    assert np.all(conf == q.max(axis=1)) and np.all(np.isnan(info[:, 3]))
    # greedy rows still carry the temperature-1 distribution
    ref = softmax(W.bf16_bits_to_f32(l).astype(np.float64), axis=1)
    assert np.all(np.abs(q - ref) <= 2.0 ** -8 * ref + 1e-40)


def test_greedy_drafts_pair_with_greedy_verification_only(oracle_mod):
    """Which pairing of draft and verification temperatures keeps the output the target's (Sec. 2.2):
    a draft SAMPLED from its stored row q and verified at T > 0 does (chi-square over 200 000 trials); a
    GREEDY draft (T == 0: token = arg-max, stored row = softmax at temperature 1) is not a draw from the row
    it stores, so verifying it at T > 0 skews the output, while verifying it at T == 0, where q is not
    looked at, reproduces greedy decoding exactly.  The library guarantees the first and the third."""
    from tests.test_oracle_accept import _chi2_stat, _crit, _softmax64
    V, n = 6, 200_000
    rng = np.random.default_rng(21)
    tl = rng.normal(0, 1.0, (2, V)).astype(np.float32)                 # target rows: draft position, bonus
    dl = (tl[0] + rng.normal(0, 0.7, V)).astype(np.float32)            # the drafter's logits
    p = _softmax64(tl[0])
    spec, uni = np.ones(n, np.int32), rng.random((2 * n, 2), dtype=np.float32)
    logits = np.tile(tl, (n, 1))

    def first_tokens(draft_T, verify_T):
        q, tok, _, _ = oracle_mod.draft_sample(np.tile(dl, (n, 1)), np.full(n, draft_T, np.float32),
                                               rng.random(n, dtype=np.float32), logits_dtype="f32", probs_dtype="f32")
        out, _, _ = oracle_mod.accept(logits, q.astype(np.float32), tok, uni, spec, np.full(n, verify_T, np.float32),
                                      logits_dtype="f32", probs_dtype="f32", want_row_info=False)
        return out[:, 0]

    stat, dof = _chi2_stat(np.bincount(first_tokens(1.0, 1.0), minlength=V), p)
    assert stat < _crit(dof), (stat, dof)                              # sampled draft, sampled verification: ~ p
    stat, dof = _chi2_stat(np.bincount(first_tokens(0.0, 1.0), minlength=V), p)
    assert stat > 10 * _crit(dof), (stat, dof)                         # greedy draft, sampled verification: NOT ~ p
    assert np.all(first_tokens(0.0, 0.0) == int(np.argmax(tl[0])))     # greedy draft, greedy verification: arg-max
