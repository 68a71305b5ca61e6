"""Randomised GPU parity: seeded random shapes through every entry point, each held to the same bar
as the fixed cases (attention within 2e-3 of the oracle and its stored output the rounding of the
accumulator; acceptance, tree acceptance and draft sampling exact except counted near-ties; KV
append bit for bit).  A few dozen cases by default; ADASPEC_SOAK_CASES=<n> runs n cases of each kind
(several thousand cases take a few minutes)."""
import os
import sys

import numpy as np
import pytest

import workloads as W
from oracle import kv_cache as KV
from tests import test_gpu_draft as TD, test_gpu_kv_cache as TK, test_gpu_parity as TP, test_gpu_tree as TT
from tests.harness import compare_accept, to_device

pytestmark = pytest.mark.gpu

CASES = int(os.environ.get("ADASPEC_SOAK_CASES", "6"))
KINDS = ["chain-attention", "tree-attention", "chain-acceptance", "tree-acceptance", "draft-sampling",
         "attention-many-rows", "acceptance-masked-padded", "kv-append", "commit", "kv-compact-path"]


def _say(msg):
    print(f"[case] {msg}", file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def pkg():
    import paper_2503_05096_amd as p
    return p


@pytest.mark.parametrize("kind", range(len(KINDS)), ids=KINDS)
def test_random_shapes(kind, oracle_mod, pkg):
    import torch
    near = 0
    for case in range(CASES):
        seed = 300000 + 1000 * kind + case
        rng = np.random.default_rng(seed)
        _say(f"random {KINDS[kind]} seed {seed}")
        near += _one_case(kind, case, seed, rng, oracle_mod, pkg, torch)
    assert near <= max(3, CASES // 20), near          # near-ties are rare by construction (1e-5 windows)


def _one_case(kind, case, seed, rng, oracle_mod, pkg, torch):
    near = 0
    if kind == 0:      # chain attention
        B = int(rng.integers(1, 24))
        spec = rng.integers(0, 9, B).astype(np.int32)
        ctx = (spec + 1 + rng.integers(0, int(rng.choice([40, 600, 5000])), B)).astype(np.int32)
        hkv = int(rng.choice([1, 2, 4, 8])); G = int(rng.choice([1, 2, 4, 8]))
        dt = str(rng.choice(["bf16", "f16", "f32"]))
        d = int(rng.choice([64, 128])) if dt != "f32" else int(rng.choice([32, 64, 128]))
        st = W.make_custom_step(seed, ctx_lens=ctx, spec_lens=spec, n_q_heads=hkv * G, n_kv_heads=hkv, head_dim=d,
                                dtype=dt, acceptance=False, name=f"random-attn-{seed}")
        TP.check_attention(st, oracle_mod, pkg)
        if case % 8 == 0:
            TP.check_attention(st, oracle_mod, pkg, path="vector")
    elif kind == 1:    # tree attention
        B = int(rng.integers(1, 16))
        spec = rng.integers(0, 20, B).astype(np.int32)
        ctx = (spec + 1 + rng.integers(0, int(rng.choice([40, 600, 3000])), B)).astype(np.int32)
        hkv = int(rng.choice([1, 2, 8])); G = int(rng.choice([1, 4]))
        dt = str(rng.choice(["bf16", "f16"]))
        st = W.make_custom_step(seed, ctx_lens=ctx, spec_lens=spec, n_q_heads=hkv * G, n_kv_heads=hkv, head_dim=128,
                                dtype=dt, acceptance=False, name=f"random-tattn-{seed}")
        W.attach_tree(st, max_width=int(rng.integers(1, 5)))
        TT._check_tree_attention(st, oracle_mod, pkg)
    elif kind == 2:    # chain acceptance, every path the shape supports
        B = int(rng.integers(1, 48))
        spec = rng.integers(0, 9, B).astype(np.int32)
        V = int(rng.choice([8, 512, 4096, 8200, 32000, 50264, 65536, 128256, 151936]))
        T = rng.choice(np.array([0.0, 0.4, 1.0, 1.5], np.float32), B, p=[0.2, 0.2, 0.4, 0.2])
        dt = str(rng.choice(["bf16", "f16"]))
        st = W.make_custom_step(seed, ctx_lens=[48] * B, spec_lens=spec, vocab=V, logits_dtype=dt, temperature=T,
                                attention=False, logits_sigma=3.0, noise_sigma=float(rng.choice([0.2, 1.0, 2.0])),
                                draft_temp=1.1, name=f"random-acc-{seed}")
        paths = ["auto", "vector", "stream"] + (["fast", "two_pass"] if V <= 131072 else [])
        for p in paths:
            rep = TP.check_accept(st, oracle_mod, pkg, path=p, max_near_tie_frac=1.0)
            near += rep["ratio_near_ties"] + rep["cdf_near_ties"]
    elif kind == 3:    # tree acceptance, both kernels
        B = int(rng.integers(1, 20))
        spec = rng.integers(0, 24, B).astype(np.int32)
        V = int(rng.choice([8, 64, 4096, 8200, 32000, 128256]))
        T = rng.choice([0.0, 0.5, 1.0, 1.7], size=B)
        dt = str(rng.choice(["bf16", "f16"]))
        st = W.make_custom_step(seed, ctx_lens=spec + 1, spec_lens=spec, vocab=V, logits_dtype=dt, temperature=T,
                                attention=False, noise_sigma=float(rng.choice([0.2, 0.8, 2.5])), name=f"random-tacc-{seed}")
        W.attach_tree(st, max_width=int(rng.integers(1, 7)))
        for kp in ("fast", "vector"):
            rep, _ = TT._check_tree_accept(st, oracle_mod, pkg, kpath=kp, max_near_tie_frac=1.0)
            near += rep["ratio_near_ties"] + rep["cdf_near_ties"]
    elif kind == 4:     # draft sampling
        R = int(rng.integers(1, 40)); V = int(rng.choice([8, 1000, 4096, 8200, 32000, 40000, 128256, 151936]))
        ldt = str(rng.choice(["bf16", "f16", "f32"])); pdt = str(rng.choice(["bf16", "f16", "f32"]))
        base_l = (float(rng.choice([1.0, 2.5, 4.0])) * rng.standard_normal((R, V))).astype(np.float32)
        lg = base_l if ldt == "f32" else (W.f32_to_bf16_bits(base_l) if ldt == "bf16" else base_l.astype(np.float16))
        T = rng.choice(np.array([0.0, 0.5, 1.0, 1.8], np.float32), R).astype(np.float32)
        u = rng.random(R).astype(np.float32)
        for path in (["vector", "auto"] if ldt == "f32" or V % 8 else ["fast", "split", "vector", "auto"]):
            if path in ("fast", "split") and V > 131072:
                continue
            TD._check(lg, ldt, pdt, T, u, oracle_mod, pkg, path=path)
    elif kind == 5:   # attention with many query rows per kv head (several row groups) and long contexts
        B = int(rng.integers(1, 6))
        spec = rng.integers(0, 48, B).astype(np.int32)
        ctx = (spec + 1 + rng.integers(0, int(rng.choice([300, 9000, 30000])), B)).astype(np.int32)
        hkv = int(rng.choice([1, 2])); G = int(rng.choice([4, 8, 16]))
        dt = str(rng.choice(["bf16", "f16"]))
        st = W.make_custom_step(seed, ctx_lens=ctx, spec_lens=spec, n_q_heads=hkv * G, n_kv_heads=hkv, head_dim=128,
                                dtype=dt, acceptance=False, name=f"random-bigrow-{seed}")
        TP.check_attention(st, oracle_mod, pkg)
        W.attach_tree(st, max_width=int(rng.integers(1, 4)))
        TT._check_tree_attention(st, oracle_mod, pkg)
    elif kind == 6:   # acceptance over masked logits in padded buffers with a wider out_stride
        B = int(rng.integers(1, 30))
        spec = rng.integers(0, 7, B).astype(np.int32)
        spec[0] = max(int(spec[0]), 1)
        V = int(rng.choice([512, 5000, 8200, 32000, 65536, 128256]))
        T = rng.choice(np.array([0.0, 0.6, 1.0], np.float32), B)
        dt = str(rng.choice(["bf16", "f16"]))
        st = W.make_custom_step(seed, ctx_lens=[48] * B, spec_lens=spec, vocab=V, logits_dtype=dt, temperature=T,
                                attention=False, logits_sigma=3.0, noise_sigma=1.0, draft_temp=1.1,
                                masked_frac=float(rng.choice([0.0, 0.3, 0.9])), name=f"random-mask-{seed}")
        dev = to_device(st, attention=False)
        tdt = torch.bfloat16 if dt == "bf16" else torch.float16
        padl, padp = int(rng.choice([0, 8, 64])), int(rng.choice([0, 8, 24]))
        wl = torch.full((st.total_q, V + padl), float("nan"), dtype=tdt, device="cuda:0")
        wp = torch.full((max(st.total_draft, 1), V + padp), float("nan"), dtype=tdt, device="cuda:0")
        wl[:, :V] = dev.target_logits
        if st.total_draft:
            wp[:st.total_draft, :V] = dev.draft_probs
        ostr = st.max_spec_len + 1 + int(rng.integers(0, 4))
        for path in ("auto", "vector", "stream", "fast", "two_pass"):
            _say(f"masked/padded accept path={path} V={V} B={B}")
            toks, alen = pkg.accept(wl[:, :V], wp[:st.total_draft, :V], dev.draft_tokens, dev.uniforms, dev.spec_lens,
                                    dev.temperature, max_spec_len=st.max_spec_len, path=path, out_stride=ostr)
            torch.cuda.synchronize()
            rep = compare_accept(st, toks.cpu().numpy(), alen.cpu().numpy(), oracle_mod, out_stride=ostr)
            assert rep["hard_mismatches"] == 0, (path, rep["details"][:4])
            near += rep["ratio_near_ties"] + rep["cdf_near_ties"]
    elif kind == 7:   # KV append, bit for bit
        B = int(rng.integers(1, 40))
        spec = rng.integers(0, 12, B).astype(np.int32)
        ctx = (spec + 1 + rng.integers(0, 300, B)).astype(np.int32)
        dt = str(rng.choice(["bf16", "f16", "f32"])); hkv = int(rng.choice([1, 2, 8])); d = int(rng.choice([64, 128]))
        st = W.make_custom_step(seed, ctx_lens=ctx, spec_lens=spec, n_q_heads=hkv, n_kv_heads=hkv, head_dim=d,
                                dtype=dt, acceptance=False, name=f"random-kv-{seed}")
        shape = (st.total_q, hkv, d)
        k_new, v_new = TK._new_rows(rng, shape, dt), TK._new_rows(rng, shape, dt)
        k_ref, v_ref = KV.kv_append(k_new, v_new, st.k_pages, st.v_pages, st.block_table, st.ctx_lens, st.spec_lens)
        kp, vp = TK._torch_from(st.k_pages, dt, "cuda:0"), TK._torch_from(st.v_pages, dt, "cuda:0")
        _say(f"kv_append B={B} TQ={st.total_q} {dt} Hkv={hkv} d={d}")
        pkg.kv_append(TK._torch_from(k_new, dt, "cuda:0"), TK._torch_from(v_new, dt, "cuda:0"), kp, vp,
                      torch.from_numpy(st.block_table).to("cuda:0"), torch.from_numpy(st.ctx_lens).to("cuda:0"),
                      torch.from_numpy(st.spec_lens).to("cuda:0"), max_spec_len=st.max_spec_len)
        torch.cuda.synchronize()
        assert np.array_equal(TK._bits(kp), TK._host_bits(k_ref)) and np.array_equal(TK._bits(vp), TK._host_bits(v_ref))
    elif kind == 8:    # commit of random acceptance results (any valid lengths), token history with overflow
        B = int(rng.integers(1, 300))
        kmax = int(rng.integers(0, 12))
        spec = rng.integers(0, kmax + 1, B).astype(np.int32)
        alen = (rng.random(B) * (spec + 1)).astype(np.int32)
        ostr = kmax + 1 + int(rng.integers(0, 3))
        toks = -np.ones((B, ostr), np.int32)
        for i in range(B):
            toks[i, :alen[i] + 1] = rng.integers(0, 50000, alen[i] + 1)
        ctx = (spec + 1 + rng.integers(0, 4000, B)).astype(np.int32)
        nxt = rng.integers(0, 7, B).astype(np.int32)
        cap = int(rng.integers(1, 20))
        seq_lens = rng.integers(0, cap + 1, B).astype(np.int32)
        seq = rng.integers(0, 1000, (B, cap)).astype(np.int32)
        ref = KV.commit(toks, alen, spec, ctx, nxt, seq, seq_lens)
        d = lambda a: torch.from_numpy(a).to("cuda:0")
        seq_d, sl_d = d(seq), d(seq_lens)
        _say(f"commit B={B} kmax={kmax} out_stride={ostr} cap={cap}")
        com, nctx, last = pkg.commit(d(toks), d(alen), d(spec), d(ctx), max_spec_len=kmax, next_spec_lens=d(nxt),
                                     seq_tokens=seq_d, seq_lens=sl_d)
        torch.cuda.synchronize()
        assert np.array_equal(com.cpu().numpy(), ref["committed_lens"])
        assert np.array_equal(nctx.cpu().numpy(), ref["next_ctx_lens"])
        assert np.array_equal(last.cpu().numpy(), ref["last_token"])
        assert np.array_equal(seq_d.cpu().numpy(), ref["seq_tokens"])
        assert np.array_equal(sl_d.cpu().numpy(), ref["seq_lens"])
    elif kind == 9:    # compaction of a random root-to-node path of every request's tree, bit for bit
        B = int(rng.integers(1, 24))
        spec = rng.integers(0, int(rng.choice([4, 20, 64])), B).astype(np.int32)
        ctx = (spec + 1 + rng.integers(0, 200, B)).astype(np.int32)
        dt = str(rng.choice(["bf16", "f16", "f32"])); hkv = int(rng.choice([1, 2, 8])); dd = int(rng.choice([64, 128]))
        st = W.make_custom_step(seed, ctx_lens=ctx, spec_lens=spec, n_q_heads=hkv, n_kv_heads=hkv, head_dim=dd,
                                dtype=dt, acceptance=False, name=f"random-compact-{seed}")
        W.attach_tree(st, max_width=int(rng.integers(1, 5)))
        cu = st.cu_q
        pstr = st.max_spec_len + 1 + int(rng.integers(0, 3))
        path = -np.ones((B, pstr), np.int32)
        alen = np.zeros(B, np.int32)
        for i in range(B):
            par = st.parents[cu[i]:cu[i + 1]]
            u, walk = 0, []
            while True:
                kids = [c for c in range(u + 1, spec[i] + 1) if par[c] == u]
                if not kids or rng.random() < 0.15:
                    break
                u = int(rng.choice(kids))
                walk.append(u)
            path[i, :len(walk)] = walk
            alen[i] = len(walk)
        k2, v2 = KV.kv_compact_path(st.k_pages, st.v_pages, st.block_table, st.ctx_lens, spec, path, alen)
        dev = to_device(st, acceptance=False)
        _say(f"kv_compact_path B={B} {dt} Hkv={hkv} d={dd} max k={st.max_spec_len}")
        pkg.kv_compact_path(dev.k_pages, dev.v_pages, dev.block_table, dev.ctx_lens, dev.spec_lens,
                            torch.from_numpy(path).cuda(), torch.from_numpy(alen).cuda(), max_spec_len=st.max_spec_len)
        torch.cuda.synchronize()
        assert np.array_equal(TK._bits(dev.k_pages), TK._host_bits(k2)) and np.array_equal(TK._bits(dev.v_pages), TK._host_bits(v2))
    return near
