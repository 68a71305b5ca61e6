"""Pins for the attention oracle (CPU only).

The paper prints no numeric example of the verification pass, so the oracle is
pinned by what the mathematics fixes: a dense brute-force formulation written
differently (full L x L masked softmax in numpy matrix form), closed forms, and
invariances (causality, paging, GQA, decomposition into single-query decode).
A dropped term, a wrong mask offset, a transposed head/page index or a wrong
softmax axis fails at least one of them.
"""
import numpy as np
import pytest

import workloads as W


def _dense_kv(st, i):
    """Gather request i's K and V through the block table -> [L][Hkv][d] float64."""
    L, P = int(st.ctx_lens[i]), st.page_size
    K = np.empty((L, st.n_kv_heads, st.head_dim))
    V = np.empty_like(K)
    for t in range(L):
        page = st.block_table[i, t // P]
        K[t] = W.to_f64(st.k_pages[page, :, t % P], st.dtype)
        V[t] = W.to_f64(st.v_pages[page, :, t % P], st.dtype)
    return K, V


def _brute_force(st, seed=0):
    """softmax(Q K^T * scale + causal mask) V with ALL L positions as queries
    (random queries for the old positions); keep the last n_i rows."""
    rng = np.random.default_rng(seed)
    G = st.n_q_heads // st.n_kv_heads
    out = np.empty((st.total_q, st.n_q_heads, st.head_dim))
    cu = st.cu_q
    scale = 1.0 / np.sqrt(st.head_dim)
    for i in range(st.batch):
        L, n = int(st.ctx_lens[i]), int(st.spec_lens[i]) + 1
        K, V = _dense_kv(st, i)
        Qall = rng.standard_normal((L, st.n_q_heads, st.head_dim))
        Qall[L - n:] = W.to_f64(st.q[cu[i]:cu[i + 1]], st.dtype)
        mask = np.tril(np.ones((L, L), dtype=bool))
        for h in range(st.n_q_heads):
            S = (Qall[:, h] @ K[:, h // G].T) * scale
            S = np.where(mask, S, -np.inf)
            S -= S.max(axis=1, keepdims=True)
            E = np.exp(S)
            Wt = E / E.sum(axis=1, keepdims=True)
            out[cu[i]:cu[i + 1], h] = (Wt @ V[:, h // G])[L - n:]
    return out


def _run(oracle_mod, st, **kw):
    return oracle_mod.verify_attn(st.q, st.k_pages, st.v_pages, st.block_table, st.ctx_lens,
                                  st.spec_lens, dtype=st.dtype, **kw)


@pytest.mark.parametrize("dtype,hq,hkv,d", [("f32", 4, 4, 16), ("bf16", 8, 2, 32), ("f16", 6, 3, 64)])
def test_brute_force_dense(oracle_mod, dtype, hq, hkv, d):
    st = W.make_custom_step(11, ctx_lens=[5, 16, 17, 40, 33], spec_lens=[0, 3, 1, 7, 2],
                            n_q_heads=hq, n_kv_heads=hkv, head_dim=d, dtype=dtype,
                            acceptance=False)
    out, _ = _run(oracle_mod, st)
    ref = _brute_force(st)
    assert not np.isnan(out).any()
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)


def test_hand_example_closed_form(oracle_mod):
    """d = 1, scale forced to 1, q = 1, K = [0, ln 3], V = [1, 5], two query rows.
    Row 0 sees token 0 only -> 1.  Row 1: weights 1:3 -> (1 + 15) / 4 = 4."""
    q = np.ones((2, 1, 1), dtype=np.float32)
    k_pages = np.zeros((1, 1, 16, 1), dtype=np.float32)
    v_pages = np.zeros((1, 1, 16, 1), dtype=np.float32)
    k_pages[0, 0, :2, 0] = [0.0, np.log(3.0)]
    v_pages[0, 0, :2, 0] = [1.0, 5.0]
    k_pages[0, 0, 2:] = np.nan
    v_pages[0, 0, 2:] = np.nan
    out, _ = oracle_mod.verify_attn(q, k_pages, v_pages, np.array([[0]], np.int32),
                                    np.array([2], np.int32), np.array([1], np.int32),
                                    dtype="f32", scale=1.0)
    np.testing.assert_allclose(out[:, 0, 0], [1.0, 4.0], rtol=0, atol=1e-6)


def test_default_scale_is_rsqrt_head_dim(oracle_mod):
    st = W.make_custom_step(3, ctx_lens=[19], spec_lens=[2], n_q_heads=2, n_kv_heads=2, head_dim=16,
                            acceptance=False)
    a, _ = _run(oracle_mod, st)
    b, _ = _run(oracle_mod, st, scale=0.25)
    c, _ = _run(oracle_mod, st, scale=0.5)
    assert np.array_equal(a, b) and not np.allclose(a, c)


def test_decomposition_into_single_query_decodes(oracle_mod):
    """n query rows over L tokens == n independent one-row requests with
    contexts L-n+1 .. L sharing the same pages (textbook decode attention)."""
    st = W.make_custom_step(5, ctx_lens=[37, 64], spec_lens=[4, 2], n_q_heads=4, n_kv_heads=2,
                            head_dim=32, dtype="bf16", acceptance=False)
    out, _ = _run(oracle_mod, st)
    cu = st.cu_q
    for i in range(st.batch):
        n, L = int(st.spec_lens[i]) + 1, int(st.ctx_lens[i])
        for j in range(n):
            one, _ = oracle_mod.verify_attn(st.q[cu[i] + j:cu[i] + j + 1], st.k_pages, st.v_pages,
                                            st.block_table[i:i + 1], np.array([L - n + 1 + j], np.int32),
                                            np.array([0], np.int32), dtype=st.dtype)
            assert np.array_equal(one[0], out[cu[i] + j])


def test_softmax_normalisation_closed_forms(oracle_mod):
    st = W.make_custom_step(7, ctx_lens=[50, 23], spec_lens=[3, 0], n_q_heads=4, n_kv_heads=4,
                            head_dim=16, acceptance=False)
    v1 = np.ones_like(st.v_pages)
    out, _ = oracle_mod.verify_attn(st.q, st.k_pages, v1, st.block_table, st.ctx_lens, st.spec_lens,
                                    dtype="f32")
    np.testing.assert_allclose(out, 1.0, rtol=0, atol=1e-14)
    # identical keys -> uniform weights -> running mean of V
    kc = np.broadcast_to(st.k_pages[st.block_table[0, 0], 0, 0], st.k_pages.shape).copy()
    out, _ = oracle_mod.verify_attn(st.q, kc, st.v_pages, st.block_table, st.ctx_lens, st.spec_lens,
                                    dtype="f32")
    cu = st.cu_q
    for i in range(st.batch):
        _, V = _dense_kv(st, i)
        n, L = int(st.spec_lens[i]) + 1, int(st.ctx_lens[i])
        for j in range(n):
            pos = L - n + j
            np.testing.assert_allclose(out[cu[i] + j], V[:pos + 1].mean(axis=0), rtol=0, atol=1e-13)


def test_causality_and_poison(oracle_mod):
    st = W.make_custom_step(9, ctx_lens=[45], spec_lens=[5], n_q_heads=2, n_kv_heads=1, head_dim=16,
                            acceptance=False, poison=True)
    out, _ = _run(oracle_mod, st)
    assert not np.isnan(out).any()           # NaN beyond L_i and in unused pages never read
    L, n, P = 45, 6, st.page_size
    for j in range(n - 1):
        pos = L - n + j
        k2, v2 = st.k_pages.copy(), st.v_pages.copy()
        for t in range(pos + 1, L):           # perturb everything row j must not see
            page = st.block_table[0, t // P]
            k2[page, :, t % P] += 3.0
            v2[page, :, t % P] -= 2.0
        out2, _ = oracle_mod.verify_attn(st.q, k2, v2, st.block_table, st.ctx_lens, st.spec_lens,
                                         dtype="f32")
        assert np.array_equal(out2[:j + 1], out[:j + 1])
        assert not np.array_equal(out2[j + 1:], out[j + 1:])


def test_last_row_sees_whole_context(oracle_mod):
    st = W.make_custom_step(10, ctx_lens=[20], spec_lens=[2], n_q_heads=1, n_kv_heads=1, head_dim=8,
                            acceptance=False)
    out, _ = _run(oracle_mod, st)
    k2 = st.k_pages.copy()
    page = st.block_table[0, 19 // 16]
    k2[page, :, 19 % 16] += 1.0               # the newest token: only the last row sees it
    out2, _ = oracle_mod.verify_attn(st.q, k2, st.v_pages, st.block_table, st.ctx_lens, st.spec_lens,
                                     dtype="f32")
    assert np.array_equal(out2[:2], out[:2]) and not np.array_equal(out2[2], out[2])


def test_page_permutation_invariance(oracle_mod):
    st = W.make_custom_step(13, ctx_lens=[70, 33, 16], spec_lens=[1, 4, 0], n_q_heads=4, n_kv_heads=2,
                            head_dim=32, dtype="f16", acceptance=False)
    out, _ = _run(oracle_mod, st)
    perm = np.random.default_rng(1).permutation(st.num_pages)
    inv = np.empty_like(perm)
    inv[perm] = np.arange(st.num_pages)
    k2, v2 = st.k_pages[perm], st.v_pages[perm]          # new page p holds old page perm[p]
    bt2 = np.where(st.block_table >= 0, inv[np.maximum(st.block_table, 0)], -1).astype(np.int32)
    out2, _ = oracle_mod.verify_attn(st.q, k2, v2, bt2, st.ctx_lens, st.spec_lens, dtype="f16")
    assert np.array_equal(out, out2)


def test_gqa_equals_mha_with_repeated_kv_heads(oracle_mod):
    st = W.make_custom_step(17, ctx_lens=[29, 48], spec_lens=[2, 3], n_q_heads=8, n_kv_heads=2,
                            head_dim=16, dtype="bf16", acceptance=False)
    out, _ = _run(oracle_mod, st)
    k2 = np.repeat(st.k_pages, 4, axis=1)
    v2 = np.repeat(st.v_pages, 4, axis=1)
    out2, _ = oracle_mod.verify_attn(st.q, k2, v2, st.block_table, st.ctx_lens, st.spec_lens,
                                     dtype="bf16")
    assert np.array_equal(out, out2)


def test_chunked_merge_matches_one_shot(oracle_mod):
    """Split-KV identity used by the GPU path, checked on the oracle's numbers:
    merging per-chunk (m, l, O) states reproduces the one-shot result."""
    st = W.make_custom_step(19, ctx_lens=[100], spec_lens=[0], n_q_heads=1, n_kv_heads=1, head_dim=8,
                            acceptance=False)
    out, _ = _run(oracle_mod, st)
    K, V = _dense_kv(st, 0)
    qv = W.to_f64(st.q[0, 0], "f32")
    s = (K[:, 0] @ qv) / np.sqrt(8.0)
    parts = []
    for lo in range(0, 100, 32):
        sc = s[lo:lo + 32]
        m = sc.max()
        e = np.exp(sc - m)
        parts.append((m, e.sum(), e @ V[lo:lo + 32, 0]))
    mstar = max(p[0] for p in parts)
    num = sum(np.exp(p[0] - mstar) * p[2] for p in parts)
    den = sum(np.exp(p[0] - mstar) * p[1] for p in parts)
    np.testing.assert_allclose(out[0, 0], num / den, rtol=0, atol=1e-12)


def test_rejects_inconsistent_metadata(oracle_mod):
    st = W.make_custom_step(21, ctx_lens=[20], spec_lens=[2], n_q_heads=1, n_kv_heads=1, head_dim=8,
                            acceptance=False)
    with pytest.raises(ValueError):
        oracle_mod.verify_attn(st.q, st.k_pages, st.v_pages, st.block_table,
                               np.array([2], np.int32), st.spec_lens, dtype="f32")  # L < n
    bt = st.block_table.copy()
    bt[0, 0] = st.num_pages
    with pytest.raises(ValueError):
        oracle_mod.verify_attn(st.q, st.k_pages, st.v_pages, bt, st.ctx_lens, st.spec_lens, dtype="f32")


# ---- storage formats: widening and the single final rounding ---------------
def test_widening_matches_numpy(oracle_mod):
    rng = np.random.default_rng(0)
    for bits in list(rng.integers(0, 1 << 16, size=2000)) + [0, 0x8000, 1, 0x03FF, 0x0400, 0x7BFF]:
        h = np.array([bits], dtype=np.uint16).view(np.float16)[0]
        a = oracle_mod.widen_u16(int(bits), "f16")
        assert (np.isnan(a) and np.isnan(h)) or a == float(h)
        b = oracle_mod.widen_u16(int(bits), "bf16")
        f = W.bf16_bits_to_f32(np.array([bits], dtype=np.uint16))[0]
        assert (np.isnan(b) and np.isnan(f)) or b == float(f)


def test_final_rounding_is_nearest_even(oracle_mod):
    rng = np.random.default_rng(1)
    xs = np.concatenate([rng.standard_normal(3000), rng.standard_normal(500) * 1e-6,
                         rng.standard_normal(500) * 3e4, [0.0, 1.0, -1.0, 65504.0, 65520.0, 1e-8]])
    with np.errstate(over="ignore"):
        for x in xs:
            assert oracle_mod.round_to_dtype(x, "f16") == float(np.float64(x).astype(np.float16))
            assert oracle_mod.round_to_dtype(x, "f32") == float(np.float32(x))
    # bf16: ties to even checked on exactly representable midpoints, plus random float32 inputs
    assert oracle_mod.round_to_dtype(1.0 + 2.0 ** -8, "bf16") == 1.0               # tie -> even (down)
    assert oracle_mod.round_to_dtype(1.0 + 3 * 2.0 ** -8, "bf16") == 1.0 + 2.0 ** -6  # tie -> even (up)
    assert oracle_mod.round_to_dtype(1.0 + 2.0 ** -8 + 2.0 ** -40, "bf16") == 1.0 + 2.0 ** -7
    f = rng.standard_normal(3000).astype(np.float32)
    want = W.bf16_bits_to_f32(W.f32_to_bf16_bits(f))
    got = np.array([oracle_mod.round_to_dtype(float(v), "bf16") for v in f])
    assert np.array_equal(got, want.astype(np.float64))


def test_rounded_output_is_rounding_of_f64_output(oracle_mod):
    st = W.make_custom_step(23, ctx_lens=[33], spec_lens=[1], n_q_heads=2, n_kv_heads=1, head_dim=16,
                            dtype="f16", acceptance=False)
    out, out_r = _run(oracle_mod, st)
    assert np.array_equal(out_r, out.astype(np.float16).astype(np.float64))
