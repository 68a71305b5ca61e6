"""CPU oracle of the speculative-length policy (paper Sec. 4 and 5): the time
model (Eq. 2-4), the accepted-token model (Eq. 5-6), the SLO-aware efficiency
estimator (Alg. 3), the adaptive drafter's predict-execute-correct loop
(Alg. 1) and the confidence-prior verifier's draft-token elimination (Alg. 2).

TEST INFRASTRUCTURE ONLY (see the package docstring).  Plain Python/numpy in
float64, recomputing every estimate from scratch, in the paper's order and
notation.  The draft model is not part of this build: Alg. 1 is driven by a
table conf[s][i] that holds the confidence the draft model WOULD report for
request i at draft step s + 1.

Conventions
  C_i        cached context tokens of request i BEFORE the step (the tokens that
             precede the first new token), the paper's N_c of the first pass
  N_c(i, j)  context tokens of the j-th pass / position, j = 1, 2, ...:
             C_i + j - 1   (this is the count that reproduces Lemma 1)
  ars[s][i]  AR_{i, s+1} = prod_{k <= s+1} c_{i,k}  (Eq. 6); AR_{i,0} = 1 is
             the bonus token and is added by nat()
  k_i        draft tokens of request i that go to verification
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np


@dataclass
class TimeModel:
    """Performance coefficients of Eq. 2 for the draft (d) and target (v) models."""
    alpha_d: float
    gamma_d: float
    delta_d: float
    alpha_v: float
    gamma_v: float
    delta_v: float
    # False: Eq. 4 as printed (every verified position counts its own context).  True: the context of
    # a request counts once in the target pass (C_i + k_i + 1 tokens), the cost shape of a kernel
    # that reads the cache once for all positions of a request.
    verify_ctx_once: bool = False


def t_fwd(alpha: float, gamma: float, delta: float, n_c: float, n_b: float) -> float:
    """Eq. 2: forward time, linear in context tokens and batch tokens."""
    return alpha * n_c + gamma * n_b + delta


def t_draft(m: TimeModel, C: Sequence[int], draft_steps: int) -> float:
    """Eq. 3: `draft_steps` forward passes of the draft model over the whole batch."""
    t = 0.0
    for s in range(1, draft_steps + 1):
        n_c = sum(int(c) + s - 1 for c in C)
        n_b = len(C)
        t += t_fwd(m.alpha_d, m.gamma_d, m.delta_d, n_c, n_b)
    return t


def t_verify(m: TimeModel, C: Sequence[int], k: Sequence[int]) -> float:
    """Eq. 4: ONE target pass over the k_i + 1 positions of every request."""
    n_c = 0
    n_b = 0
    for c, ki in zip(C, k):
        if m.verify_ctx_once:
            n_c += int(c) + int(ki) + 1
        for j in range(1, int(ki) + 2):
            if not m.verify_ctx_once:
                n_c += int(c) + j - 1
            n_b += 1
    return t_fwd(m.alpha_v, m.gamma_v, m.delta_v, n_c, n_b)


def count_tokens(C: Sequence[int], k: Sequence[int], verify_ctx_once: bool = False) -> Tuple[int, int]:
    """(N_c, N_b) of Eq. 4, counted position by position: N_b = number of verified positions; N_c = context
    tokens before each position, summed over positions (as printed), or each request's C_i + k_i + 1 once."""
    n_c = n_b = 0
    for c, ki in zip(C, k):
        for j in range(1, int(ki) + 2):
            n_b += 1
            if not verify_ctx_once:
                n_c += int(c) + j - 1
        if verify_ctx_once:
            n_c += int(c) + int(ki) + 1
    return n_c, n_b


def estimate_time(m: TimeModel, C, draft_steps: int, k) -> float:
    """Eq. 1: T_sd = T_d + T_v."""
    return t_draft(m, C, draft_steps) + t_verify(m, C, k)


def nat(ars: Sequence[Sequence[float]], k: Sequence[int]) -> float:
    """Eq. 5: sum over requests of (bonus token + acceptance rates of its k_i drafts)."""
    total = 0.0
    for i, ki in enumerate(k):
        total += 1.0
        for s in range(int(ki)):
            total += float(ars[s][i])
    return total


def goodput(m: TimeModel, C, draft_steps: int, k, ars, tpot: float) -> float:
    """Alg. 3: NAT / T_sd, or -1 when the step would break the TPOT constraint."""
    t = estimate_time(m, C, draft_steps, k)
    if t > tpot:
        return -1.0
    return nat(ars, k) / t


def adaptive_drafter(m: TimeModel, C, conf: np.ndarray, prev_conf: float, tpot: float
                     ) -> Tuple[int, List[np.ndarray], List[float]]:
    """Alg. 1.  conf[s][i]: confidence of request i's draft token at step s + 1 (the draft model's
    answer, revealed only when that step is executed); at most conf.shape[0] steps can be run.
    Returns (number of draft steps executed, ars of the executed steps, goodput after each step)."""
    B = len(C)
    max_steps = conf.shape[0]
    best = -1.0
    dts = 0
    prev = np.full(B, float(prev_conf))
    arss: List[np.ndarray] = [prev.copy()]              # tentative entry: the step not yet executed
    history: List[float] = []
    while True:
        steps = len(arss)                                # executed steps + the tentative one
        thpt = goodput(m, C, steps, [steps] * B, arss, tpot)
        if thpt > best and dts < max_steps:
            confs = np.asarray(conf[dts], dtype=np.float64)      # execute the draft model
            dts += 1
            arss.pop()                                           # correct: drop the prediction ...
            if not arss:
                arss.append(confs.copy())
            else:
                arss.append(arss[-1] * confs)                    # ... and chain the real confidence (Eq. 6)
            best = goodput(m, C, dts, [dts] * B, arss, tpot)
            history.append(best)
            arss.append(prev.copy())                             # predict the next step
        else:
            arss.pop()
            break
    return dts, arss, history


def eliminate(m: TimeModel, C, draft_steps: int, ars, tpot: float) -> Tuple[np.ndarray, float]:
    """Alg. 2: drop draft tokens in ascending order of acceptance rate while the goodput improves.
    AR is non-increasing along a request, so the smallest remaining AR always belongs to the LAST
    remaining draft of some request; among equal values the lowest request index goes first.
    Returns (k_i per request, goodput of the final token set)."""
    B = len(C)
    k = np.full(B, int(draft_steps), dtype=np.int32)
    best = goodput(m, C, draft_steps, k, ars, tpot)
    while True:
        cand = -1
        for i in range(B):
            if k[i] > 0 and (cand < 0 or ars[k[i] - 1][i] < ars[k[cand] - 1][cand]):
                cand = i
        if cand < 0:
            break
        k[cand] -= 1
        thpt = goodput(m, C, draft_steps, k, ars, tpot)
        if thpt > best:
            best = thpt
        else:
            k[cand] += 1
            break
    return k, best


def fit_time_model(n_c, n_b, t) -> Tuple[float, float, float]:
    """Sec. 6, offline analyzer: least-squares (alpha, gamma, delta) of Eq. 2 from measured passes."""
    A = np.stack([np.asarray(n_c, np.float64), np.asarray(n_b, np.float64), np.ones(len(t))], axis=1)
    sol, *_ = np.linalg.lstsq(A, np.asarray(t, np.float64), rcond=None)
    return float(sol[0]), float(sol[1]), float(sol[2])
