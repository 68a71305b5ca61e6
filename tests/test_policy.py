"""The speculative-length policy: pins of the oracle (oracle/policy.py) against what
the paper and the mathematics fix, then the library's host code against the oracle.

Pins: Lemma 1's closed form of T_sd (Sec. 4.1), the three properties of the
accepted-token model (Lemma 2, Sec. 4.2), a hand-computed estimator value
(Alg. 3), a hand-traced run of the drafter loop (Alg. 1) and of the draft-token
elimination (Alg. 2), brute force over all request-level length vectors, and a
textbook least-squares fit (offline analyzer, Sec. 6).
"""
import itertools
import math

import numpy as np
import pytest

from oracle import policy as OP
from paper_2503_05096_amd import policy as PP

M = OP.TimeModel(alpha_d=2e-7, gamma_d=3e-5, delta_d=4e-3, alpha_v=9e-7, gamma_v=2e-4, delta_v=2.5e-2)


def _lib_model(m=None):
    m = M if m is None else m
    return PP.TimeModel(m.alpha_d, m.gamma_d, m.delta_d, m.alpha_v, m.gamma_v, m.delta_v, int(m.verify_ctx_once), 0)


# ------------------------------------------------------------------ oracle pins
@pytest.mark.parametrize("BS,SL,Nc", [(1, 0, 100), (8, 3, 512), (32, 7, 1777)])
def test_time_model_matches_lemma1_closed_form(BS, SL, Nc):
    # Lemma 1: T_sd as a quadratic in SL for a batch with average context Nc
    ad, gd, dd, av, gv, dv = M.alpha_d, M.gamma_d, M.delta_d, M.alpha_v, M.gamma_v, M.delta_v
    closed = BS * (SL * SL * (ad + av) / 2
                   + SL * (ad * Nc + av * Nc - ad / 2 + av / 2 + gd + gv + dd / BS)
                   + av * Nc + gv + dv / BS)
    got = OP.estimate_time(M, [Nc] * BS, SL, [SL] * BS)
    assert math.isclose(got, closed, rel_tol=1e-12)


def test_time_model_is_the_sum_of_single_passes():
    # Eq. 3 / Eq. 4 written out pass by pass for a ragged batch
    C, k, steps = [10, 200, 33], [2, 0, 1], 2
    td = sum(M.alpha_d * sum(c + s - 1 for c in C) + M.gamma_d * len(C) + M.delta_d for s in (1, 2))
    n_c = (10 + 11 + 12) + (200) + (33 + 34)
    tv = M.alpha_v * n_c + M.gamma_v * 6 + M.delta_v
    assert math.isclose(OP.estimate_time(M, C, steps, k), td + tv, rel_tol=1e-13)


def test_nat_properties_of_lemma2():
    rng = np.random.default_rng(0)
    B, SL = 16, 8
    conf = rng.uniform(0, 1, (SL, B))
    ars = np.cumprod(conf, axis=0)
    avg = [OP.nat(ars, [s] * B) / B for s in range(SL + 1)]
    assert avg[0] == 1.0                                             # initialization
    gains = np.diff(avg)
    assert np.all(gains >= 0) and np.all(gains <= 1)                 # marginal gain in [0, 1]
    assert np.all(np.diff(gains) <= 1e-15)                           # diminishing returns
    assert math.isclose(gains[2], ars[2].mean(), rel_tol=1e-12)      # the gain IS the mean AR of the new position


def test_goodput_hand_value_and_tpot():
    m = OP.TimeModel(0, 0, 1.0, 0, 0, 2.0)                           # every draft pass 1 s, the verify pass 2 s
    ars = [[0.5, 0.8], [0.25, 0.4]]
    # 2 draft steps, both requests keep 2 drafts: NAT = 2 + 0.5 + 0.8 + 0.25 + 0.4 = 3.95, T = 2*1 + 2 = 4
    assert math.isclose(OP.goodput(m, [5, 9], 2, [2, 2], ars, tpot=10.0), 3.95 / 4.0)
    assert math.isclose(OP.goodput(m, [5, 9], 2, [1, 0], ars, tpot=10.0), 2.5 / 4.0)
    assert OP.goodput(m, [5, 9], 2, [2, 2], ars, tpot=3.9) == -1.0   # over the TPOT constraint
    assert OP.goodput(m, [5, 9], 2, [2, 2], ars, tpot=4.0) > 0.98          # "exceeds", not "reaches"


def test_adaptive_drafter_hand_trace():
    # one request; draft pass costs 1, verify pass costs 4 + (positions): T(s) = s + 4 + (s + 1)
    m = OP.TimeModel(0, 0, 1.0, 0, 1.0, 4.0)
    conf = np.array([[0.9], [0.9], [0.2], [0.9]])
    # prev_conf = 0.8.  s=0: predict (1+.8)/7=.257 > -1 -> run: AR1=.9, best=1.9/7=.2714
    #   predict (1.9+.8)/9=.3 > .2714 -> run: AR2=.81, best=2.71/9=.3011
    #   predict (2.71+.8)/11=.3191 > .3011 -> run: AR3=.162, best=2.872/11=.2611
    #   predict (2.872+.8)/13=.2825 > .2611 -> run: AR4=.1458, best=3.0178/13=.2321 ; table exhausted -> stop
    steps, arss, hist = OP.adaptive_drafter(m, [50], conf, prev_conf=0.8, tpot=math.inf)
    assert steps == 4
    assert np.allclose([a[0] for a in arss], [0.9, 0.81, 0.162, 0.1458])
    assert np.allclose(hist, [1.9 / 7, 2.71 / 9, 2.872 / 11, 3.0178 / 13])
    # a pessimistic history stops it at once: predict (1 + 0.1)/7 = .157 > -1 runs step 1 (best .2714),
    # then predict (1.9 + .1)/9 = .222 < .2714 -> stop after one step
    steps, arss, _ = OP.adaptive_drafter(m, [50], conf, prev_conf=0.1, tpot=math.inf)
    assert steps == 1 and len(arss) == 1
    # TPOT below the cost of even one draft step: nothing is drafted
    steps, arss, _ = OP.adaptive_drafter(m, [50], conf, prev_conf=0.8, tpot=6.5)
    assert steps == 0 and arss == []


def test_elimination_hand_trace():
    # verify cost dominated by batch tokens: T = 2 (draft, sunk) + 1 + 0.5 * positions
    m = OP.TimeModel(0, 0, 1.0, 0, 0.5, 1.0)
    ars = np.array([[0.9, 0.3, 0.6], [0.8, 0.03, 0.5]])             # [step][request]
    # start k=(2,2,2): NAT = 3 + 1.8 + 1.33 = 6.13, T = 3 + 4.5 = 7.5 -> .8173
    # drop r1's 2nd (.03): 6.10 / 7.0 = .8714 better; drop r1's 1st (.3): 5.8/6.5 = .8923 better;
    # drop r2's 2nd (.5): 5.3/6.0 = .8833 worse -> stop
    k, g = OP.eliminate(m, [7, 7, 7], 2, ars, tpot=math.inf)
    assert k.tolist() == [2, 0, 2] and math.isclose(g, 5.8 / 6.5)


def test_elimination_result_is_a_local_optimum_and_brute_force_agrees_when_unimodal():
    rng = np.random.default_rng(5)
    for trial in range(20):
        B, SL = 3, 3
        C = rng.integers(10, 2000, B)
        ars = np.cumprod(rng.uniform(0.05, 1, (SL, B)), axis=0)
        k, g = OP.eliminate(M, C, SL, ars, tpot=math.inf)
        assert math.isclose(g, OP.goodput(M, C, SL, k, ars, math.inf), rel_tol=1e-12)
        assert g >= OP.goodput(M, C, SL, [SL] * B, ars, math.inf) - 1e-15
        # the greedy path visits prefixes of the ascending-AR order; its result is at least as good as
        # every token set on that path before it, and the next one is not better
        best_all = max(OP.goodput(M, C, SL, kk, ars, math.inf) for kk in itertools.product(range(SL + 1), repeat=B))
        assert g <= best_all + 1e-15                                  # brute force bounds it from above


def test_fit_recovers_exact_coefficients():
    rng = np.random.default_rng(1)
    n_c, n_b = rng.integers(1000, 500000, 40), rng.integers(1, 600, 40)
    t = 3e-7 * n_c + 2e-4 * n_b + 0.011
    a, g, d = OP.fit_time_model(n_c, n_b, t)
    assert math.isclose(a, 3e-7, rel_tol=1e-9) and math.isclose(g, 2e-4, rel_tol=1e-9) and math.isclose(d, 0.011, rel_tol=1e-9)


def test_context_counted_once_variant():
    import dataclasses
    m1 = dataclasses.replace(M, verify_ctx_once=True)
    C, k = [10, 200, 33], [2, 0, 1]
    tv = M.alpha_v * ((10 + 3) + (200 + 1) + (33 + 2)) + M.gamma_v * 6 + M.delta_v
    assert math.isclose(OP.t_verify(m1, C, k), tv, rel_tol=1e-13)
    # with no drafts the two counts differ only by the request's own new token (it is read from the cache too)
    assert math.isclose(OP.t_verify(m1, C, [0, 0, 0]) - OP.t_verify(M, C, [0, 0, 0]), 3 * M.alpha_v, rel_tol=1e-9)


# ------------------------------------------------------------------ library (host C++) against the oracle
def _random_case(rng, B, SL):
    C = rng.integers(1, 5000, B).astype(np.int32)
    conf = rng.uniform(0.02, 1.0, (SL, B))
    return C, conf


@pytest.mark.parametrize("seed", range(6))
def test_library_time_and_goodput_match_oracle(seed):
    rng = np.random.default_rng(seed)
    B, SL = int(rng.integers(1, 40)), int(rng.integers(0, 9))
    C, conf = _random_case(rng, B, max(SL, 1))
    ars = np.cumprod(conf, axis=0)[:max(SL, 1)]
    k = rng.integers(0, SL + 1, B).astype(np.int32)
    lm = _lib_model()
    assert math.isclose(PP.estimate_time(lm, C, SL, k), OP.estimate_time(M, C, SL, k), rel_tol=1e-12)
    assert math.isclose(PP.estimate_time(lm, C, SL), OP.estimate_time(M, C, SL, [SL] * B), rel_tol=1e-12)
    for tpot in (math.inf, OP.estimate_time(M, C, SL, k) * 0.999):
        assert math.isclose(PP.goodput(lm, C, SL, k, ars, tpot), OP.goodput(M, C, SL, k, ars, tpot), rel_tol=1e-12)


@pytest.mark.parametrize("seed", range(12))
def test_library_drafter_and_elimination_match_oracle(seed):
    import dataclasses
    global M
    rng = np.random.default_rng(100 + seed)
    M0 = M
    M = dataclasses.replace(M0, verify_ctx_once=bool(seed & 1))
    try:
        _drafter_and_elimination_case(rng)
    finally:
        M = M0


def _drafter_and_elimination_case(rng):
    B, SL = int(rng.integers(1, 64)), int(rng.integers(1, 9))
    C, conf = _random_case(rng, B, SL)
    prev = float(rng.uniform(0.3, 0.95))
    t_full = OP.estimate_time(M, C, SL, [SL] * B)
    for tpot in (math.inf, 0.7 * t_full):
        steps_o, arss_o, hist = OP.adaptive_drafter(M, C, conf, prev, tpot)
        steps_l, ar_l, g_l = PP.adaptive_draft(_lib_model(), C, conf, prev, tpot)
        assert steps_l == steps_o
        if steps_o:
            assert np.allclose(ar_l, np.stack(arss_o), rtol=1e-13, atol=0)
            assert math.isclose(g_l, hist[-1], rel_tol=1e-12)
            k_o, g_o = OP.eliminate(M, C, steps_o, np.stack(arss_o), tpot)
            k_l, g_l2 = PP.eliminate(_lib_model(), C, steps_o, ar_l, tpot)
            assert np.array_equal(k_l, k_o) and math.isclose(g_l2, g_o, rel_tol=1e-12)
        else:
            assert g_l == -1.0


def test_library_fit_matches_oracle_on_noisy_data():
    rng = np.random.default_rng(3)
    n_c, n_b = rng.integers(1000, 900000, 60), rng.integers(1, 700, 60)
    t = 4e-7 * n_c + 1.5e-4 * n_b + 0.02 + rng.normal(0, 1e-3, 60)
    o = OP.fit_time_model(n_c, n_b, t)
    l = PP.fit_time_model(n_c, n_b, t)
    assert np.allclose(l, o, rtol=1e-8)


def test_library_policy_argument_errors():
    lm = _lib_model()
    assert math.isnan(PP.estimate_time(lm, [5, 6], 2, [3, 0]))        # k_i > draft steps
    with pytest.raises(Exception):
        PP.fit_time_model([1, 2], [1, 2], [1, 2])                     # n < 3
    with pytest.raises(Exception):
        PP.fit_time_model([1, 2, 3], [2, 4, 6], [1, 2, 3])            # dependent columns


# ------------------------------------------------------------------ Eq. 4 token counts
def test_token_counts_of_eq4_by_hand_and_closed_form():
    # three requests with caches 10, 200, 33 and 2, 0, 1 drafts: positions see 10,11,12 | 200 | 33,34
    assert OP.count_tokens([10, 200, 33], [2, 0, 1]) == (33 + 200 + 67, 6)
    # every request's cache once for all its positions: (10+3) + (200+1) + (33+2)
    assert OP.count_tokens([10, 200, 33], [2, 0, 1], verify_ctx_once=True) == (249, 6)
    rng = np.random.default_rng(4)
    C, k = rng.integers(0, 5000, 40), rng.integers(0, 9, 40)
    n_c, n_b = OP.count_tokens(C, k)
    assert n_b == int((k + 1).sum())
    assert n_c == int(((k + 1) * C + k * (k + 1) // 2).sum())          # arithmetic series per request
    # the time model charges exactly these counts
    tv = OP.t_verify(M, C, k)
    assert math.isclose(tv, M.alpha_v * n_c + M.gamma_v * n_b + M.delta_v, rel_tol=1e-13)


def test_library_token_counts_equal_the_oracle():
    rng = np.random.default_rng(5)
    for once in (False, True):
        for B in (0, 1, 7, 300):
            C, k = rng.integers(0, 100000, B), rng.integers(0, 65, B)
            got = PP.count_tokens(C, k, verify_ctx_once=once)
            assert got == tuple(float(v) for v in OP.count_tokens(C, k, verify_ctx_once=once))
    with pytest.raises(Exception):
        PP.count_tokens([5], [-1])


def test_shipped_time_model_record_is_complete_and_feeds_the_policy():
    """The MI355X record the analyzer wrote (paper_2503_05096_amd/data): both verification fits and the
    draft fit are there, and the policy, library and oracle alike, runs on them to the same decisions."""
    import workloads as W
    from paper_2503_05096_amd import analyzer
    for once in (False, True):
        lm = analyzer.load_time_model(verify_ctx_once=once)
        assert lm.alpha_d > 0 and lm.delta_d > 0 and lm.alpha_v > 0 and lm.delta_v > 0 and lm.verify_ctx_once == int(once)
        om = OP.TimeModel(lm.alpha_d, lm.gamma_d, lm.delta_d, lm.alpha_v, lm.gamma_v, lm.delta_v, bool(once))
        pin = W.policy_inputs(3, batch=48)
        for tpot in (float("inf"), 2.5e-3):
            steps, ar, g = PP.adaptive_draft(lm, pin["ctx_committed"], pin["conf"], pin["prev_conf"], tpot)
            o_steps, o_ars, _ = OP.adaptive_drafter(om, pin["ctx_committed"], pin["conf"], pin["prev_conf"], tpot)
            assert steps == o_steps
            k, gk = PP.eliminate(lm, pin["ctx_committed"], steps, ar, tpot)
            o_k, o_g = OP.eliminate(om, pin["ctx_committed"], o_steps, o_ars, tpot)
            assert np.array_equal(k, o_k) and math.isclose(gk, o_g, rel_tol=1e-12)
