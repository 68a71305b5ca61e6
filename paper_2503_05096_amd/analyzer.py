#!/usr/bin/env python3
"""Offline analyzer (paper Sec. 6): measures this library's kernels on the GPU at hand over a grid of
batch sizes, context lengths and speculative lengths, and fits the performance coefficients of the
forward-time model of Eq. 2,

        T = alpha * N_c + gamma * N_b + delta,

once for the target's verification pass (alpha_v, gamma_v, delta_v; Eq. 4) and once for a draft pass
(alpha_d, gamma_d, delta_d; Eq. 3).  N_c and N_b are counted by adaspec_policy_count_tokens, the fit is
done by adaspec_policy_fit_time_model; nothing of either is computed here.

What a pass is, for this build (the models' dense layers are outside it):
  verification pass   `layers` calls of adaspec_verify_attn over the ragged batch + one adaspec_accept
  draft pass          `draft_layers` calls of adaspec_verify_attn with one query row per request
                      (a decode step of the drafter) + one adaspec_draft_sample

    python -m paper_2503_05096_amd.analyzer [--layers 32] [--draft-layers 2] [--json time_model.json]

Inputs are random device tensors of the Llama-3-8B shape (32 q heads, 8 kv heads, d = 128,
V = 128256, bf16): the kernels' running time does not depend on the values.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys

import numpy as np

DATA_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "data")
DEFAULT_MODEL_FILE = os.path.join(DATA_DIR, "time_model_mi355x.json")


def _ragged_batch(B: int, ctx: int, k: int, seed: int):
    """Host side of one grid point: committed context lengths C_i ~ U[ctx/2, 3 ctx/2], draft lengths
    k_i in [max(0, k-2), k], a shuffled block table."""
    import torch
    P = 16
    g = torch.Generator().manual_seed(seed)
    spec = torch.full((B,), k, dtype=torch.int32)
    if k > 0:
        spec = torch.randint(max(0, k - 2), k + 1, (B,), dtype=torch.int32, generator=g)
    C = torch.randint(max(1, ctx // 2), ctx + ctx // 2 + 1, (B,), dtype=torch.int32, generator=g)
    L = C + spec + 1
    max_pages = int((L.max() + P - 1) // P)
    need = int(((L + P - 1) // P).sum())
    bt = torch.full((B, max_pages), -1, dtype=torch.int32)
    perm = torch.randperm(need, dtype=torch.int32, generator=g)
    o = 0
    for i in range(B):
        n = int((L[i] + P - 1) // P)
        bt[i, :n] = perm[o:o + n]
        o += n
    return C, spec, L, bt, need


def _timed(fn, iters: int) -> float:
    import torch
    for _ in range(3):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / iters


def measure(B: int, ctx: int, k: int, *, iters: int, seed: int, layers: int, draft_layers: int = 0):
    """One grid point.  Returns a dict with the verification pass's (N_c per position, N_c once per request,
    N_b, seconds) and, if draft_layers > 0, the draft pass's (N_c, N_b, seconds)."""
    import torch
    from . import binding as bd
    from . import policy
    Hq, Hkv, d, V, P = 32, 8, 128, 128256, 16
    Cc, spec, L, bt, need = _ragged_batch(B, ctx, k, seed)
    TQ = int((spec + 1).sum())
    TD = TQ - B
    dev = "cuda:0"
    g = torch.Generator(device=dev).manual_seed(seed)
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

    a_dims = bd.attn_dims(q, kp, bt_d, max_spec_len=kmax)
    ws = torch.empty(max(bd.lib().adaspec_verify_attn_workspace_bytes(C.byref(a_dims)), 256), dtype=torch.uint8, device=dev)

    def verify_pass():
        # the ragged metadata once per pass, reused by every layer (as a model's forward pass would)
        bd.verify_attn(q, kp, vp, bt_d, L_d, spec_d, max_spec_len=kmax, plan="build", workspace=ws)
        for _ in range(layers):
            bd.verify_attn(q, kp, vp, bt_d, L_d, spec_d, out, max_spec_len=kmax, plan="reuse", workspace=ws)
        bd.accept(logits, probs if TD else None, toks if TD else None, uni, spec_d, temp, max_spec_len=kmax)

    rec = {"B": B, "ctx": ctx, "k": k, "t_verify": _timed(verify_pass, iters)}
    Cn, kn = Cc.numpy(), spec.numpy()
    rec["n_c"], rec["n_b"] = policy.count_tokens(Cn, kn, verify_ctx_once=False)
    rec["n_c_once"], _ = policy.count_tokens(Cn, kn, verify_ctx_once=True)
    if draft_layers > 0:
        # a draft pass: every request one new token over its committed context (the drafter's cache is
        # given the target's shape here: one kv-head group of the same width)
        zero = torch.zeros(B, dtype=torch.int32, device=dev)
        Ld = (Cc + 1).to(dev)
        q1, out1 = rnd(B, Hq, d), torch.empty(B, Hq, d, dtype=torch.bfloat16, device=dev)
        d_logits = logits[:B]
        d_probs = torch.empty_like(d_logits)
        d_tok = torch.empty(B, dtype=torch.int32, device=dev)
        d_conf = torch.empty(B, dtype=torch.float32, device=dev)
        d_uni = torch.rand(B, generator=g, device=dev)

        def draft_pass():
            bd.verify_attn(q1, kp, vp, bt_d, Ld, zero, max_spec_len=kmax, plan="build", workspace=ws)
            for _ in range(draft_layers):
                bd.verify_attn(q1, kp, vp, bt_d, Ld, zero, out1, max_spec_len=kmax, plan="reuse", workspace=ws)
            bd.draft_sample(d_logits, temp, d_uni, draft_probs=d_probs, draft_tokens=d_tok, confidence=d_conf)

        rec["t_draft"] = _timed(draft_pass, iters)
        rec["n_c_draft"], rec["n_b_draft"] = policy.count_tokens(Cn, np.zeros(B, np.int32), verify_ctx_once=False)
    return rec


def fit(points, xcol: str, bcol: str, tcol: str) -> dict:
    """Least squares of t on (n_c, n_b, 1) through the library's C ABI, with the fit's quality."""
    from . import policy
    x = np.array([p[xcol] for p in points], np.float64)
    b = np.array([p[bcol] for p in points], np.float64)
    t = np.array([p[tcol] for p in points], np.float64)
    alpha, gamma, delta = policy.fit_time_model(x, b, t)
    pred = alpha * x + gamma * b + delta
    ss_res, ss_tot = float(((t - pred) ** 2).sum()), float(((t - t.mean()) ** 2).sum())
    return {"alpha_s_per_context_token": alpha, "gamma_s_per_batch_token": gamma, "delta_s": delta,
            "r2": 1.0 - ss_res / ss_tot, "max_rel_err": float(np.max(np.abs(pred - t) / t))}


def run_grid(grid, *, iters: int, layers: int, draft_layers: int, log=print) -> dict:
    points = []
    for n, (B, ctx, k) in enumerate(grid):
        p = measure(B, ctx, k, iters=iters, seed=n, layers=layers, draft_layers=draft_layers)
        points.append(p)
        log(f"B={B:4d} ctx~{ctx:5d} k<={k}  N_c={p['n_c']:11.0f}  N_c(once)={p['n_c_once']:9.0f}  N_b={p['n_b']:5.0f}  "
            f"verify {p['t_verify'] * 1e6:9.1f} us" + (f"  draft {p['t_draft'] * 1e6:8.1f} us" if draft_layers else ""))
    rec = {"layers": layers, "draft_layers": draft_layers, "points": points,
           "verify": {"ctx_per_position": dict(fit(points, "n_c", "n_b", "t_verify"), verify_ctx_once=0),
                      "ctx_once_per_request": dict(fit(points, "n_c_once", "n_b", "t_verify"), verify_ctx_once=1)}}
    if draft_layers > 0:
        # (the draft grid does not depend on k: one point per (B, ctx) would do, the repeats are harmless)
        rec["draft"] = fit(points, "n_c_draft", "n_b_draft", "t_draft")
    return rec


def load_time_model(path: str = DEFAULT_MODEL_FILE, verify_ctx_once: bool = True):
    """The policy's TimeModel from an analyzer record (default: the MI355X record shipped with the
    package).  verify_ctx_once picks which of the two verification fits is used."""
    from . import policy
    with open(path) as f:
        rec = json.load(f)
    v = rec["verify"]["ctx_once_per_request" if verify_ctx_once else "ctx_per_position"]
    dft = rec["draft"]
    return policy.TimeModel(dft["alpha_s_per_context_token"], dft["gamma_s_per_batch_token"], dft["delta_s"],
                            v["alpha_s_per_context_token"], v["gamma_s_per_batch_token"], v["delta_s"],
                            int(bool(verify_ctx_once)), 0)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=32, help="attention calls per verification pass")
    ap.add_argument("--draft-layers", type=int, default=2, help="attention calls per draft pass (0: no draft fit)")
    ap.add_argument("--iters", type=int, default=5)
    ap.add_argument("--json", default=None, help="write the record (grid points and fits) here")
    args = ap.parse_args()
    grid = [(B, ctx, k) for B in (16, 64, 128) for ctx in (256, 1024, 4096) for k in (0, 3, 6)]
    rec = run_grid(grid, iters=args.iters, layers=args.layers, draft_layers=args.draft_layers,
                   log=lambda s: print(s, flush=True))
    rec["command"] = (f"python -m paper_2503_05096_amd.analyzer --layers {args.layers} "
                      f"--draft-layers {args.draft_layers} --iters {args.iters}")
    rec["shape"] = "32 q heads, 8 kv heads, d=128, V=128256, bf16"
    print(json.dumps({k: v for k, v in rec.items() if k != "points"}))
    if args.json:
        with open(args.json, "w") as f:
            json.dump(rec, f, indent=1)
            f.write("\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())
