#!/usr/bin/env python3
"""Offline analyzer (paper Sec. 6): measures this library's verification step on the GPU at hand
over a grid of batch sizes, context lengths and speculative lengths, and fits the performance
coefficients (alpha_v, gamma_v, delta_v) of the forward-time model of Eq. 2,

        T_v = alpha_v * N_c + gamma_v * N_b + delta_v,

with N_c = sum over requests and positions of the context tokens before the position and
N_b = number of verified positions (Eq. 4).  The step timed is one attention layer plus one
acceptance, as in bench.py; `--layers n` weights the attention call n times (a whole model has n
attention layers per acceptance).  The fit itself is done by adaspec_policy_fit_time_model.

    python -m paper_2503_05096_amd.analyzer [--layers 32] [--out time_model.txt]

Inputs are random device tensors of the Llama-3-8B shape (32 q heads, 8 kv heads, d = 128,
V = 128256, bf16): the kernels' running time does not depend on the values.
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np


def measure(B: int, ctx: int, k: int, *, iters: int, seed: int, layers: int):
    import torch
    from . import binding as bd
    Hq, Hkv, d, V, P = 32, 8, 128, 128256, 16
    g = torch.Generator(device="cuda:0").manual_seed(seed)
    spec = torch.full((B,), k, dtype=torch.int32)
    if k > 0:                                           # ragged: k_i in [max(0, k-2), k]
        spec = torch.randint(max(0, k - 2), k + 1, (B,), dtype=torch.int32)
    C = torch.randint(max(1, ctx // 2), ctx + ctx // 2 + 1, (B,), dtype=torch.int32)   # cached tokens before the step
    L = C + spec + 1
    TQ = int((spec + 1).sum())
    TD = TQ - B
    max_pages = int((L.max() + P - 1) // P)
    need = int(((L + P - 1) // P).sum())
    bt = torch.full((B, max_pages), -1, dtype=torch.int32)
    perm = torch.randperm(need, dtype=torch.int32)
    o = 0
    for i in range(B):
        n = int((L[i] + P - 1) // P)
        bt[i, :n] = perm[o:o + n]
        o += n
    dev = "cuda:0"
    rnd = lambda *s: torch.randn(*s, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    q, kp, vp = rnd(TQ, Hq, d), rnd(need, Hkv, P, d), rnd(need, Hkv, P, d)
    logits = (3.0 * torch.randn(TQ, V, generator=g, device=dev)).to(torch.bfloat16)
    probs = torch.softmax(torch.randn(max(TD, 1), V, generator=g, device=dev), dim=-1).to(torch.bfloat16)
    toks = torch.randint(0, V, (max(TD, 1),), generator=g, device=dev, dtype=torch.int32)
    uni = torch.rand(TQ, 2, generator=g, device=dev)
    temp = torch.full((B,), 0.8, device=dev)
    spec_d, L_d, bt_d = spec.to(dev), L.to(dev), bt.to(dev)
    out = torch.empty_like(q)
    kmax = max(k, 1)

    def step():
        for _ in range(layers):
            bd.verify_attn(q, kp, vp, bt_d, L_d, spec_d, out, max_spec_len=kmax)
        bd.accept(logits, probs if TD else None, toks if TD else None, uni, spec_d, temp, max_spec_len=kmax)

    for _ in range(3):
        step()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(iters):
        step()
    e1.record()
    torch.cuda.synchronize()
    t = e0.elapsed_time(e1) * 1e-3 / iters
    # context tokens per position (Eq. 4 as printed) and per request (each request's cache counted once)
    n_c = float(sum(int(c) * (int(s) + 1) + int(s) * (int(s) + 1) // 2 for c, s in zip(C.tolist(), spec.tolist())))
    n_c_once = float(L.sum())
    return n_c, n_c_once, float(TQ), t


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=1)
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--out", default=None)
    args = ap.parse_args()
    from . import policy
    grid = [(B, ctx, k) for B in (16, 64, 128) for ctx in (256, 1024, 4096) for k in (0, 3, 6)]
    rows = []
    for n, (B, ctx, k) in enumerate(grid):
        n_c, n_c_once, n_b, t = measure(B, ctx, k, iters=args.iters, seed=n, layers=args.layers)
        rows.append((B, ctx, k, n_c, n_c_once, n_b, t))
        print(f"B={B:4d} ctx~{ctx:5d} k<={k}  N_c={n_c:11.0f}  N_c(once)={n_c_once:9.0f}  N_b={n_b:5.0f}  "
              f"t={t * 1e6:9.1f} us", flush=True)
    a = np.array(rows, dtype=np.float64)

    def fit(col, once):
        alpha, gamma, delta = policy.fit_time_model(a[:, col], a[:, 5], a[:, 6])
        pred = alpha * a[:, col] + gamma * a[:, 5] + delta
        ss_res, ss_tot = float(((a[:, 6] - pred) ** 2).sum()), float(((a[:, 6] - a[:, 6].mean()) ** 2).sum())
        return {"verify_ctx_once": once, "alpha_v_s_per_context_token": alpha, "gamma_v_s_per_batch_token": gamma,
                "delta_v_s": delta, "r2": 1.0 - ss_res / ss_tot,
                "max_rel_err": float(np.max(np.abs(pred - a[:, 6]) / a[:, 6]))}

    rec = {"layers": args.layers, "points": len(rows), "fits": [fit(3, 0), fit(4, 1)]}
    print(json.dumps(rec))
    if args.out:
        with open(args.out, "w") as f:
            f.write("# python -m paper_2503_05096_amd.analyzer --layers %d --iters %d\n" % (args.layers, args.iters))
            f.write("# B ctx k N_c(per position) N_c(once per request) N_b t_seconds\n")
            for r in rows:
                f.write("%d %d %d %.0f %.0f %.0f %.6e\n" % r)
            f.write(json.dumps(rec, indent=1) + "\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())
