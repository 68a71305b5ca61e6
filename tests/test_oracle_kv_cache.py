"""Pins for the oracle of the steps around verification (KV append, commit).

Both are byte / integer work, so the pins are exact: a hand-written example,
reconstruction of the written rows through the paged-addressing definition,
equivalence of one multi-token append with token-by-token appends, and the
bookkeeping identities of the commit.
"""
import numpy as np
import pytest

import workloads as W
from oracle import kv_cache as KV


def _gather(pages, block_table, i, pos):
    P = pages.shape[2]
    return pages[block_table[i, pos // P], :, pos % P, :]


def _new_rows(rng, shape, dtype):
    if dtype == np.uint16:                               # bf16 bit patterns
        return W.f32_to_bf16_bits(rng.standard_normal(shape, np.float32))
    return rng.standard_normal(shape, np.float32).astype(dtype)


def test_append_hand_example():
    # 2 requests, P = 4, one kv head, d = 2; pages filled with -1
    P, d = 4, 2
    kp = -np.ones((5, 1, P, d), np.float32)
    vp = kp.copy()
    bt = np.array([[3, 0], [4, 1]], np.int32)           # request 0 -> pages 3,0 ; request 1 -> pages 4,1
    ctx = np.array([6, 3], np.int32)                     # lengths INCLUDING the new tokens
    spec = np.array([2, 0], np.int32)                    # n = 3, 1
    k_new = np.arange(4 * d, dtype=np.float32).reshape(4, 1, d)
    v_new = 100 + k_new
    k2, v2 = KV.kv_append(k_new, v_new, kp, vp, bt, ctx, spec)
    # request 0: positions 3,4,5 -> (page 3, slot 3), (page 0, slot 0), (page 0, slot 1)
    assert np.array_equal(k2[3, 0, 3], [0, 1]) and np.array_equal(k2[0, 0, 0], [2, 3])
    assert np.array_equal(k2[0, 0, 1], [4, 5])
    # request 1: position 2 -> (page 4, slot 2)
    assert np.array_equal(k2[4, 0, 2], [6, 7]) and np.array_equal(v2[4, 0, 2], [106, 107])
    # nothing else changed
    changed = (k2 != kp)
    assert changed.sum() == 4 * d and (v2 != vp).sum() == 4 * d
    assert np.array_equal(kp, -np.ones_like(kp))         # inputs untouched


@pytest.mark.parametrize("cfg", [1, 2])
def test_append_then_gather_returns_the_rows(cfg):
    st = W.make_verify_step(cfg, acceptance=False, poison=False)
    rng = np.random.default_rng(7)
    TQ = st.total_q
    shape = (TQ, st.n_kv_heads, st.head_dim)
    k_new, v_new = _new_rows(rng, shape, st.k_pages.dtype), _new_rows(rng, shape, st.k_pages.dtype)
    k2, v2 = KV.kv_append(k_new, v_new, st.k_pages, st.v_pages, st.block_table, st.ctx_lens, st.spec_lens)
    row = 0
    touched = np.zeros(st.k_pages.shape[:1] + st.k_pages.shape[2:3], bool)    # [page][slot]
    for i in range(st.batch):
        n, L = int(st.spec_lens[i]) + 1, int(st.ctx_lens[i])
        for j in range(n):
            pos = L - n + j
            assert np.array_equal(_gather(k2, st.block_table, i, pos), k_new[row])
            assert np.array_equal(_gather(v2, st.block_table, i, pos), v_new[row])
            touched[st.block_table[i, pos // st.page_size], pos % st.page_size] = True
            row += 1
    assert touched.sum() == TQ                            # distinct slots
    same = ~touched[:, None, :, None]
    assert np.array_equal(np.where(same, k2, 0), np.where(same, st.k_pages, 0))
    assert np.array_equal(np.where(same, v2, 0), np.where(same, st.v_pages, 0))


def test_one_append_equals_token_by_token_appends():
    st = W.make_custom_step(11, ctx_lens=[40, 17, 5], spec_lens=[4, 0, 2], acceptance=False, poison=False)
    rng = np.random.default_rng(3)
    shape = (st.total_q, st.n_kv_heads, st.head_dim)
    k_new, v_new = rng.standard_normal(shape, np.float32), rng.standard_normal(shape, np.float32)
    k_all, v_all = KV.kv_append(k_new, v_new, st.k_pages, st.v_pages, st.block_table, st.ctx_lens, st.spec_lens)
    kp, vp = st.k_pages, st.v_pages
    cu = st.cu_q
    for i in range(st.batch):
        n, L = int(st.spec_lens[i]) + 1, int(st.ctx_lens[i])
        for j in range(n):                                # one request, one token (k = 0) at a time
            kp, vp = KV.kv_append(k_new[cu[i] + j:cu[i] + j + 1], v_new[cu[i] + j:cu[i] + j + 1], kp, vp,
                                  st.block_table[i:i + 1], np.array([L - n + j + 1], np.int32),
                                  np.array([0], np.int32))
    assert np.array_equal(k_all, kp) and np.array_equal(v_all, vp)


def test_commit_hand_example():
    # request 0: k = 3, accepted 1 -> emits x0, recovered; request 1: k = 2, all accepted + bonus;
    # request 2: k = 0 -> bonus only
    out_tokens = np.array([[11, 99, -1, -1], [21, 22, 77, -1], [55, -1, -1, -1]], np.int32)
    alen = np.array([1, 2, 0], np.int32)
    spec = np.array([3, 2, 0], np.int32)
    ctx = np.array([104, 53, 9], np.int32)               # includes the n = 4, 3, 1 new tokens
    nxt = np.array([2, 5, 0], np.int32)
    seq = -np.ones((3, 4), np.int32)
    seq[0, :2] = [1, 2]
    seq[1, :3] = [3, 4, 5]
    sl = np.array([2, 3, 0], np.int32)
    r = KV.commit(out_tokens, alen, spec, ctx, nxt, seq, sl)
    assert r["committed_lens"].tolist() == [102, 53, 9]  # 100 old + x_n + 1 accepted; 50 + 1 + 2; 8 + 1
    assert r["last_token"].tolist() == [99, 77, 55]
    assert r["next_ctx_lens"].tolist() == [105, 59, 10]
    assert r["seq_lens"].tolist() == [4, 4, 1]
    assert r["seq_tokens"].tolist() == [[1, 2, 11, 99], [3, 4, 5, 21], [55, -1, -1, -1]]   # request 1 clipped


def test_commit_identities_on_a_config(oracle_mod):
    st = W.make_verify_step(2, attention=False)
    toks, alen, _ = oracle_mod.accept(st.target_logits, st.draft_probs, st.draft_tokens, st.uniforms,
                                      st.spec_lens, st.temperature, logits_dtype=st.logits_dtype,
                                      probs_dtype=st.probs_dtype)
    ctx = (1000 + np.arange(st.batch)).astype(np.int32)
    r = KV.commit(toks, alen, st.spec_lens, ctx)
    k = st.spec_lens
    # the cache shrinks by exactly the rejected drafts
    assert np.array_equal(ctx - r["committed_lens"], k - alen)
    # the old tokens (ctx - n) and the first new one are always kept
    assert np.all(r["committed_lens"] >= ctx - k) and np.all(r["committed_lens"] <= ctx)
    assert np.array_equal(r["last_token"], toks[np.arange(st.batch), alen])
    assert np.all(r["last_token"] >= 0)
    assert r["next_ctx_lens"] is None and r["seq_tokens"] is None


# ------------------------------------------------------------ tree: compaction of the accepted path
def test_compact_path_hand_example():
    # one request, P = 4, base = 2, nodes 0..4 at positions 2..6; accepted path = nodes 2, 4
    P, d = 4, 1
    kp = np.arange(3 * P, dtype=np.float32).reshape(3, 1, P, d)      # page p, slot s holds 4p + s
    vp = 100 + kp
    bt = np.array([[2, 0]], np.int32)                                 # positions 0..3 -> page 2, 4..7 -> page 0
    ctx, spec = np.array([7], np.int32), np.array([4], np.int32)
    path = np.array([[2, 4, -1, -1, -1]], np.int32)
    k2, v2 = KV.kv_compact_path(kp, vp, bt, ctx, spec, path, np.array([2], np.int32))
    # node 2 sat at position 4 (page 0, slot 0, value 0) -> position 3 (page 2, slot 3)
    # node 4 sat at position 6 (page 0, slot 2, value 2) -> position 4 (page 0, slot 0)
    assert k2[2, 0, 3, 0] == 0 and k2[0, 0, 0, 0] == 2 and v2[2, 0, 3, 0] == 100 and v2[0, 0, 0, 0] == 102
    changed = (k2 != kp)
    assert changed.sum() == 2                                         # nothing else moved


def test_compact_path_properties():
    rng = np.random.default_rng(4)
    spec = np.array([0, 5, 9, 3, 16], np.int32)
    st = W.make_custom_step(9, ctx_lens=[1, 20, 33, 4, 50], spec_lens=spec, n_q_heads=2, n_kv_heads=2,
                            head_dim=8, dtype="f32", acceptance=False, poison=False)
    W.attach_tree(st, max_width=3)
    cu = st.cu_q
    B = st.batch
    path = -np.ones((B, int(spec.max()) + 1), np.int32)
    alen = np.zeros(B, np.int32)
    for i in range(B):                                                # a random root-to-node path
        par = st.parents[cu[i]:cu[i + 1]]
        u, walk = 0, []
        while True:
            kids = [c for c in range(u + 1, spec[i] + 1) if par[c] == u]
            if not kids or rng.random() < 0.2:
                break
            u = int(rng.choice(kids))
            walk.append(u)
        path[i, :len(walk)] = walk
        alen[i] = len(walk)
    assert alen.max() >= 2
    k2, v2 = KV.kv_compact_path(st.k_pages, st.v_pages, st.block_table, st.ctx_lens, spec, path, alen)
    for i in range(B):
        base = int(st.ctx_lens[i]) - int(spec[i]) - 1
        for pos in range(base + 1):                                   # committed context and root untouched
            assert np.array_equal(_gather(k2, st.block_table, i, pos), _gather(st.k_pages, st.block_table, i, pos))
        for j in range(alen[i]):
            assert np.array_equal(_gather(k2, st.block_table, i, base + 1 + j),
                                  _gather(st.k_pages, st.block_table, i, base + path[i, j]))
            assert np.array_equal(_gather(v2, st.block_table, i, base + 1 + j),
                                  _gather(st.v_pages, st.block_table, i, base + path[i, j]))
    # a chain's path is 1, 2, ...: nothing moves
    W.attach_tree(st, chain=True)
    chain_path = np.where(np.arange(path.shape[1])[None] < alen[:, None], np.arange(1, path.shape[1] + 1)[None], -1)
    k3, v3 = KV.kv_compact_path(st.k_pages, st.v_pages, st.block_table, st.ctx_lens, spec,
                                chain_path.astype(np.int32), alen)
    assert np.array_equal(k3, st.k_pages) and np.array_equal(v3, st.v_pages)
