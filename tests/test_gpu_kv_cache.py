"""GPU parity of the steps around verification (adaspec_kv_append, adaspec_commit)
and of a multi-step loop  append -> verify attention -> accept -> commit  that
never goes back to the host between the four calls.  The page contents and all
integers must match the oracle bit for bit; attention keeps its 2e-3 bound.
"""
import os
import sys

import numpy as np
import pytest

import workloads as W
from oracle import kv_cache as KV
from tests.harness import _torch_from, compare_accept

pytestmark = pytest.mark.gpu
F32 = 0


def _say(msg):
    print(f"[case] {msg}", file=sys.stderr, flush=True)
    report = os.environ.get("ADASPEC_TEST_REPORT")      # optional file that keeps the measured figures of the run
    if report:
        with open(report, "a") as f:
            f.write(msg + "\n")


@pytest.fixture(scope="module")
def pkg():
    import paper_2503_05096_amd as p
    return p


def _new_rows(rng, shape, dtype):
    if dtype == "bf16":
        return W.f32_to_bf16_bits(rng.standard_normal(shape, np.float32))
    return rng.standard_normal(shape, np.float32).astype({"f32": np.float32, "f16": np.float16}[dtype])


def _bits(t):
    """Device tensor -> host integer view (NaN-safe, bit-exact comparison)."""
    import torch
    it = {2: torch.int16, 4: torch.int32}[t.element_size()]
    return t.view(it).cpu().numpy()


def _host_bits(a):
    return a.view({2: np.int16, 4: np.int32}[a.dtype.itemsize])


@pytest.mark.parametrize("cfg", [1, 2, 3, 5])
def test_kv_append_matches_oracle_bitwise(cfg, pkg):
    import torch
    st = W.make_verify_step(cfg, acceptance=False)       # unused pages / tail slots hold NaN
    rng = np.random.default_rng(100 + cfg)
    shape = (st.total_q, st.n_kv_heads, st.head_dim)
    k_new, v_new = _new_rows(rng, shape, st.dtype), _new_rows(rng, shape, st.dtype)
    k_ref, v_ref = KV.kv_append(k_new, v_new, st.k_pages, st.v_pages, st.block_table, st.ctx_lens, st.spec_lens)
    dev = "cuda:0"
    kp, vp = _torch_from(st.k_pages, st.dtype, dev), _torch_from(st.v_pages, st.dtype, dev)
    _say(f"kv_append {st.name} TQ={st.total_q} Hkv={st.n_kv_heads} d={st.head_dim} {st.dtype}")
    pkg.kv_append(_torch_from(k_new, st.dtype, dev), _torch_from(v_new, st.dtype, dev), kp, vp,
                  torch.from_numpy(st.block_table).to(dev), torch.from_numpy(st.ctx_lens).to(dev),
                  torch.from_numpy(st.spec_lens).to(dev), max_spec_len=st.max_spec_len)
    torch.cuda.synchronize()
    assert np.array_equal(_bits(kp), _host_bits(k_ref))
    assert np.array_equal(_bits(vp), _host_bits(v_ref))


def test_kv_append_edge_shapes(pkg):
    import torch
    dev = "cuda:0"
    # k = 0 everywhere; a request whose new tokens straddle a page boundary; L == n (empty history)
    for ctx, spec, hkv, d, dt in [([1, 16, 17], [0, 0, 0], 1, 8, "bf16"),
                                  ([18, 33, 7], [4, 6, 6], 3, 64, "f16"),
                                  ([5, 2], [4, 1], 2, 4, "f32")]:
        st = W.make_custom_step(5, ctx_lens=ctx, spec_lens=spec, n_q_heads=hkv, n_kv_heads=hkv, head_dim=d,
                                dtype=dt, acceptance=False)
        rng = np.random.default_rng(9)
        shape = (st.total_q, hkv, d)
        k_new, v_new = _new_rows(rng, shape, dt), _new_rows(rng, shape, dt)
        k_ref, v_ref = KV.kv_append(k_new, v_new, st.k_pages, st.v_pages, st.block_table, st.ctx_lens, st.spec_lens)
        kp, vp = _torch_from(st.k_pages, dt, dev), _torch_from(st.v_pages, dt, dev)
        _say(f"kv_append edge ctx={ctx} spec={spec} Hkv={hkv} d={d} {dt}")
        pkg.kv_append(_torch_from(k_new, dt, dev), _torch_from(v_new, dt, dev), kp, vp,
                      torch.from_numpy(st.block_table).to(dev), torch.from_numpy(st.ctx_lens).to(dev),
                      torch.from_numpy(st.spec_lens).to(dev), max_spec_len=max(spec) + 2)
        torch.cuda.synchronize()
        assert np.array_equal(_bits(kp), _host_bits(k_ref)) and np.array_equal(_bits(vp), _host_bits(v_ref))


@pytest.mark.parametrize("cfg", [2, 5])
def test_commit_matches_oracle(cfg, oracle_mod, pkg):
    import torch
    st = W.make_verify_step(cfg, attention=False)
    toks, alen, _ = oracle_mod.accept(st.target_logits, st.draft_probs, st.draft_tokens, st.uniforms,
                                      st.spec_lens, st.temperature, logits_dtype=st.logits_dtype,
                                      probs_dtype=st.probs_dtype)
    rng = np.random.default_rng(cfg)
    B = st.batch
    ctx = rng.integers(20, 4000, B).astype(np.int32)
    nxt = rng.integers(0, 7, B).astype(np.int32)
    cap = 6
    seq_lens = rng.integers(0, cap + 1, B).astype(np.int32)        # some already full, some overflow now
    seq = rng.integers(0, 1000, (B, cap)).astype(np.int32)
    ref = KV.commit(toks, alen, st.spec_lens, ctx, nxt, seq, seq_lens)
    dev = "cuda:0"
    d = lambda a: torch.from_numpy(a).to(dev)
    seq_d, sl_d = d(seq), d(seq_lens)
    _say(f"commit {st.name} B={B}")
    com, nctx, last = pkg.commit(d(toks), d(alen), d(st.spec_lens), d(ctx), max_spec_len=st.max_spec_len,
                                 next_spec_lens=d(nxt), seq_tokens=seq_d, seq_lens=sl_d)
    torch.cuda.synchronize()
    assert np.array_equal(com.cpu().numpy(), ref["committed_lens"])
    assert np.array_equal(nctx.cpu().numpy(), ref["next_ctx_lens"])
    assert np.array_equal(last.cpu().numpy(), ref["last_token"])
    assert np.array_equal(seq_d.cpu().numpy(), ref["seq_tokens"])
    assert np.array_equal(sl_d.cpu().numpy(), ref["seq_lens"])
    # in place: committed_lens aliases ctx_lens; optional outputs left out
    ctx_d = d(ctx)
    com2, nctx2, _ = pkg.commit(d(toks), d(alen), d(st.spec_lens), ctx_d, max_spec_len=st.max_spec_len,
                                committed_lens=ctx_d)
    torch.cuda.synchronize()
    assert nctx2 is None and np.array_equal(ctx_d.cpu().numpy(), ref["committed_lens"])


def test_multi_step_decode_loop(oracle_mod, pkg):
    """Three consecutive speculative steps; the GPU side chains the four calls on device data only."""
    import torch
    dev = "cuda:0"
    B, Hq, Hkv, d, V, kmax, P = 6, 8, 2, 128, 4096, 5, 16
    dt = "bf16"
    rng = np.random.default_rng(2503)
    hist = rng.integers(1, 300, B).astype(np.int32)                 # committed cache length before step 0
    hist[0] = 0                                                     # a request with an empty history
    max_pages = int((hist.max() + 3 * (kmax + 1) + P - 1) // P) + 1
    num_pages = B * max_pages + 3
    block_table = rng.permutation(num_pages)[:B * max_pages].reshape(B, max_pages).astype(np.int32)
    k_pages = W.f32_to_bf16_bits(rng.standard_normal((num_pages, Hkv, P, d), np.float32))
    v_pages = W.f32_to_bf16_bits(rng.standard_normal((num_pages, Hkv, P, d), np.float32))
    t = lambda a: torch.from_numpy(a).to(dev)
    kp_d, vp_d, bt_d = _torch_from(k_pages, dt, dev), _torch_from(v_pages, dt, dev), t(block_table)
    committed = hist.copy()
    committed_d = t(committed)
    spec = rng.integers(0, kmax + 1, B).astype(np.int32)
    ctx = (committed + spec + 1).astype(np.int32)
    ctx_d = t(ctx)
    seq = -np.ones((B, 12), np.int32)
    seq_lens = np.zeros(B, np.int32)
    seq_d, sl_d = t(seq), t(seq_lens)
    for step in range(3):
        st = W.make_custom_step(700 + step, ctx_lens=ctx, spec_lens=spec, n_q_heads=Hq, n_kv_heads=Hkv,
                                head_dim=d, dtype=dt, vocab=V, logits_dtype="bf16",
                                temperature=[0.8, 1.0, 0.0, 0.7, 1.0, 0.0], attention=True, poison=False)
        shape = (st.total_q, Hkv, d)
        k_new, v_new = _new_rows(rng, shape, dt), _new_rows(rng, shape, dt)
        nxt = rng.integers(0, kmax + 1, B).astype(np.int32)
        # ---- oracle
        k_pages, v_pages = KV.kv_append(k_new, v_new, k_pages, v_pages, block_table, ctx, spec)
        ref_out, _ = oracle_mod.verify_attn(st.q, k_pages, v_pages, block_table, ctx, spec, dtype=dt)
        # ---- GPU: four calls, device data only
        _say(f"loop step {step} ctx={ctx.tolist()} spec={spec.tolist()}")
        spec_d = t(spec)
        pkg.kv_append(_torch_from(k_new, dt, dev), _torch_from(v_new, dt, dev), kp_d, vp_d, bt_d, ctx_d, spec_d,
                      max_spec_len=kmax)
        out = pkg.verify_attn(_torch_from(st.q, dt, dev), kp_d, vp_d, bt_d, ctx_d, spec_d, max_spec_len=kmax,
                              out_dtype=F32)
        toks_d, alen_d = pkg.accept(_torch_from(st.target_logits, "bf16", dev),
                                    _torch_from(st.draft_probs, "bf16", dev) if st.total_draft else None,
                                    t(st.draft_tokens) if st.total_draft else None, t(st.uniforms), spec_d,
                                    t(st.temperature), max_spec_len=kmax)
        _, nctx_d, last_d = pkg.commit(toks_d, alen_d, spec_d, ctx_d, max_spec_len=kmax, next_spec_lens=t(nxt),
                                       committed_lens=committed_d, seq_tokens=seq_d, seq_lens=sl_d)
        torch.cuda.synchronize()
        # ---- compare
        assert np.array_equal(_bits(kp_d), _host_bits(k_pages)) and np.array_equal(_bits(vp_d), _host_bits(v_pages))
        err = float(np.abs(out.double().cpu().numpy() - ref_out).max())
        assert err <= 2e-3, err
        rep = compare_accept(st, toks_d.cpu().numpy(), alen_d.cpu().numpy(), oracle_mod, out_stride=kmax + 1)
        assert rep["hard_mismatches"] == 0 and rep["exact"] == B, rep     # (no near-tie expected at this size)
        ref = KV.commit(toks_d.cpu().numpy(), alen_d.cpu().numpy(), spec, ctx, nxt, seq, seq_lens)
        assert np.array_equal(committed_d.cpu().numpy(), ref["committed_lens"])
        assert np.array_equal(nctx_d.cpu().numpy(), ref["next_ctx_lens"])
        assert np.array_equal(last_d.cpu().numpy(), ref["last_token"])
        assert np.array_equal(seq_d.cpu().numpy(), ref["seq_tokens"]) and np.array_equal(sl_d.cpu().numpy(), ref["seq_lens"])
        # ---- next step's shape comes from the device results
        seq, seq_lens = ref["seq_tokens"], ref["seq_lens"]
        committed, ctx, spec = ref["committed_lens"], ref["next_ctx_lens"], nxt
        ctx_d = nctx_d
    assert seq_lens.sum() > 3 * B - 1                                   # every request emitted >= 1 token per step


def test_append_and_commit_with_many_requests(pkg):
    import torch
    dev = "cuda:0"
    rng = np.random.default_rng(15)
    B = 1500
    spec = rng.integers(0, 4, B).astype(np.int32)
    ctx = (rng.integers(0, 50, B) + spec + 1).astype(np.int32)
    st = W.make_custom_step(16, ctx_lens=ctx, spec_lens=spec, n_q_heads=2, n_kv_heads=2, head_dim=64, dtype="f16",
                            acceptance=False)
    shape = (st.total_q, 2, 64)
    k_new, v_new = _new_rows(rng, shape, "f16"), _new_rows(rng, shape, "f16")
    k_ref, v_ref = KV.kv_append(k_new, v_new, st.k_pages, st.v_pages, st.block_table, st.ctx_lens, st.spec_lens)
    kp, vp = _torch_from(st.k_pages, "f16", dev), _torch_from(st.v_pages, "f16", dev)
    _say(f"kv_append B={B} TQ={st.total_q}")
    t = lambda a: torch.from_numpy(a).to(dev)
    pkg.kv_append(_torch_from(k_new, "f16", dev), _torch_from(v_new, "f16", dev), kp, vp, t(st.block_table),
                  t(st.ctx_lens), t(st.spec_lens), max_spec_len=3)
    torch.cuda.synchronize()
    assert np.array_equal(_bits(kp), _host_bits(k_ref)) and np.array_equal(_bits(vp), _host_bits(v_ref))
    alen = np.minimum(rng.integers(0, 4, B), spec).astype(np.int32)
    toks = rng.integers(0, 1000, (B, 4)).astype(np.int32)
    ref = KV.commit(toks, alen, spec, ctx)
    com, _, last = pkg.commit(t(toks), t(alen), t(spec), t(ctx), max_spec_len=3)
    torch.cuda.synchronize()
    assert np.array_equal(com.cpu().numpy(), ref["committed_lens"]) and np.array_equal(last.cpu().numpy(), ref["last_token"])
