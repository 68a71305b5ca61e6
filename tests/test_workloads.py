"""Host-side checks of the seeded input generators (CPU only)."""
import numpy as np
import pytest

import workloads as W


def test_config1_matches_its_statement():
    st = W.make_verify_step(1)
    assert st.batch == 4 and list(st.ctx_lens) == [128, 256, 384, 512] and list(st.spec_lens) == [1, 2, 3, 4]
    assert st.total_q == 14 and st.total_draft == 10
    assert st.q.shape == (14, 8, 64) and st.q.dtype == np.float32
    assert st.k_pages.shape == (st.num_pages, 8, 16, 64)
    assert st.target_logits.shape == (14, 1024) and st.draft_probs.shape == (10, 1024)
    assert st.uniforms.shape == (14, 2) and st.uniforms.min() >= 0 and st.uniforms.max() < 1
    assert np.allclose(st.draft_probs.sum(axis=1), 1.0, atol=1e-5)
    assert 1.8 < st.target_logits.std() < 2.2


def test_determinism_and_seed_dependence():
    a, b = W.make_verify_step(1), W.make_verify_step(1)
    c = W.make_verify_step(1, seed=77)
    for f in ("q", "k_pages", "block_table", "target_logits", "draft_probs", "draft_tokens", "uniforms"):
        assert np.array_equal(getattr(a, f), getattr(b, f), equal_nan=True)
    assert not np.array_equal(a.q, c.q)


def test_block_table_is_a_shuffled_partition_with_poison():
    st = W.make_verify_step(2, batch=6, acceptance=False)
    P = st.page_size
    used = st.block_table[st.block_table >= 0]
    assert len(np.unique(used)) == len(used) and used.max() < st.num_pages
    assert st.num_pages >= int(np.ceil(1.25 * len(used))) - 1
    assert not np.all(np.diff(used) == 1)                      # shuffled, not the identity layout
    kv = st.k_pages.view(np.float16)
    for i in range(st.batch):
        n_pages = -(-int(st.ctx_lens[i]) // P)
        assert np.all(st.block_table[i, :n_pages] >= 0) and np.all(st.block_table[i, n_pages:] == -1)
        tail = int(st.ctx_lens[i]) % P
        last = st.block_table[i, n_pages - 1]
        assert not np.isnan(kv[last, :, :tail or P]).any()
        if tail:
            assert np.isnan(kv[last, :, tail:]).all()
    unused = np.setdiff1d(np.arange(st.num_pages), used)
    assert np.isnan(kv[unused]).all()


@pytest.mark.parametrize("cfg,lo,hi,kmax", [(2, 256, 2048, 8), (3, 128, 4096, 6), (4, 2048, 8192, 5),
                                            (5, 1024, 2048, 1)])
def test_ragged_structure_ranges(cfg, lo, hi, kmax):
    st = W.make_verify_step(cfg, attention=False, acceptance=False)
    assert st.batch == {2: 32, 3: 128, 4: 64, 5: 256}[cfg]
    assert st.ctx_lens.min() >= lo and st.ctx_lens.max() <= hi
    assert st.spec_lens.min() >= 0 and st.spec_lens.max() <= kmax
    assert np.all(st.ctx_lens >= st.spec_lens + 1)
    if cfg == 3:      # mean draft length in the range the paper's Table 2 reports for its policy
        assert 2.5 < st.spec_lens.mean() < 3.7
    if cfg == 5:
        assert set(np.unique(st.temperature)) <= {np.float32(0), np.float32(0.7), np.float32(1.0)}


def test_draft_tokens_have_positive_draft_probability_and_greedy_drafter():
    st = W.make_custom_step(3, ctx_lens=[32] * 6, spec_lens=[3, 2, 0, 4, 1, 2], vocab=2000,
                            logits_dtype="bf16", temperature=[1, 0, 1, 0.7, 0, 1], attention=False,
                            logits_sigma=3.0, noise_sigma=1.5, draft_temp=1.2)
    qd = W.to_f64(st.draft_probs, "bf16")
    assert np.all(qd[np.arange(st.total_draft), st.draft_tokens] > 0)
    cu = st.cu_q
    for i in (1, 4):
        for j in range(int(st.spec_lens[i])):
            d = cu[i] - i + j
            assert st.draft_tokens[d] == np.argmax(qd[d])


def test_bf16_storage_roundtrip():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -2.5, 1e-3, 3.0e38, np.inf], dtype=np.float32)
    b = W.f32_to_bf16_bits(x)
    back = W.bf16_bits_to_f32(b)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == np.float32(1.0 + 2.0 ** -6)
    assert back[3] == -2.5 and abs(back[4] - 1e-3) < 1e-5 and np.isinf(back[6])
    assert np.isnan(W.bf16_bits_to_f32(W.f32_to_bf16_bits(np.array([np.nan], np.float32))))[0]


def test_algorithmic_bytes_formula():
    st = W.make_custom_step(5, ctx_lens=[40, 17], spec_lens=[2, 0], n_q_heads=4, n_kv_heads=2, head_dim=32,
                            dtype="bf16", vocab=64, logits_dtype="bf16", temperature=[1.0, 0.0])
    b = W.algorithmic_bytes(st)
    assert b["kv"] == (40 + 17) * 2 * 2 * 32 * 2
    assert b["q_out"] == 4 * 4 * 32 * 2 * 2
    assert b["block_table"] == (3 + 2) * 4
    assert b["logits"] == 4 * 64 * 2 and b["probs"] == 2 * 64 * 2
    assert b["total"] == b["attn"] + b["accept"]


def test_accept_bytes_of_the_skipping_form():
    st = W.make_custom_step(6, ctx_lens=[40, 17, 30, 21], spec_lens=[2, 0, 3, 1], vocab=64, logits_dtype="bf16",
                            temperature=[1.0, 0.5, 0.0, 0.0], attention=False)
    row = 64 * 2
    # request 0 rejects its 2nd draft (sampled), 1 has only a bonus row, 2 (greedy) rejects at once, 3 (greedy) accepts
    b = W.accept_bytes_skipping_form(st, [1, 0, 0, 1])
    assert b["test_logits"] == 6 * row                     # every draft row once
    assert b["decide_logits"] == 3 * row                   # requests 0, 1, 3; the rejected greedy one re-reads nothing
    assert b["decide_probs"] == 1 * row                    # request 0 only
    assert b["accept"] == 10 * row
    full = W.algorithmic_bytes(st)["accept"]
    assert full == 10 * row + 2 * row and b["accept"] <= full


def test_bench_refuses_more_than_one_gpu():
    import subprocess, sys, os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_attach_tree_structure_and_determinism():
    st = W.make_custom_step(31, ctx_lens=[40, 9, 20, 64], spec_lens=[12, 0, 5, 30], vocab=32, attention=False,
                            temperature=[1.0, 1.0, 0.0, 0.8])
    chain_tokens = st.draft_tokens.copy()
    W.attach_tree(st, max_width=3)
    again = W.attach_tree(W.make_custom_step(31, ctx_lens=[40, 9, 20, 64], spec_lens=[12, 0, 5, 30], vocab=32,
                                             attention=False, temperature=[1.0, 1.0, 0.0, 0.8]), max_width=3)
    assert np.array_equal(st.parents, again.parents) and np.array_equal(st.draft_tokens, again.draft_tokens)
    assert st.parents.shape == (st.total_q,) and st.draft_tokens.shape == chain_tokens.shape
    cu = st.cu_q
    for i in range(st.batch):
        par = st.parents[cu[i]:cu[i + 1]]
        assert par[0] == -1 and all(0 <= par[c] < c for c in range(1, len(par)))     # parents come first
        if len(par) > 1:
            assert np.bincount(par[1:]).max() <= 3
        # a token handed out by the generator has mass in its parent's draft distribution
        for c in range(1, len(par)):
            q = W.to_f64(st.draft_probs[cu[i] - i + par[c]], st.probs_dtype)
            assert q[st.draft_tokens[cu[i] - i + c - 1]] > 0
    # greedy request: siblings are the distinct top tokens of the parent's row, best first
    i = 2
    par = st.parents[cu[i]:cu[i + 1]]
    for u in range(len(par)):
        kids = [c for c in range(1, len(par)) if par[c] == u]
        if kids:
            q = W.to_f64(st.draft_probs[cu[i] - i + u], st.probs_dtype)
            assert [st.draft_tokens[cu[i] - i + c - 1] for c in kids] == list(np.argsort(-q, kind="stable")[:len(kids)])
    assert max(np.bincount(st.parents[st.parents >= 0]).max(), 0) >= 2                # some node branches
    W.attach_tree(st, chain=True)
    for i in range(st.batch):
        assert list(st.parents[cu[i]:cu[i + 1]]) == list(range(-1, int(st.spec_lens[i])))


def test_tree_byte_accounting():
    st = W.make_custom_step(5, ctx_lens=[9, 3, 30], spec_lens=[4, 0, 6], vocab=64, logits_dtype="bf16",
                            attention=False, temperature=[1.0, 1.0, 0.0])
    W.attach_tree(st, max_width=2)
    has = W.tree_internal_nodes(st)
    cu = st.cu_q
    for i in range(st.batch):
        par = st.parents[cu[i]:cu[i + 1]]
        for u in range(len(par)):
            assert has[cu[i] + u] == (u in set(par[1:]))
        assert not has[cu[i + 1] - 1]                                   # the last node is a leaf
    b = W.algorithmic_bytes_tree(st)
    assert b["logits"] == st.total_q * 64 * 2
    assert b["probs"] == int(has[cu[0]:cu[1]].sum()) * 64 * 2           # only request 0 is sampled and has drafts
    assert b["accept"] == b["logits"] + b["probs"] == b["total"]
    # a chain: every node but the last of each request has a child -> the per-row chain figure
    W.attach_tree(st, chain=True)
    assert W.algorithmic_bytes_tree(st) == W.algorithmic_bytes(st)


def test_tree_walk_form_bytes():
    st = W.make_custom_step(6, ctx_lens=[9, 9, 9], spec_lens=[3, 3, 2], vocab=16, logits_dtype="bf16",
                            attention=False, temperature=[1.0, 1.0, 0.0])
    st.parents = np.array([-1, 0, 0, 1,   -1, 0, 1, 2,   -1, 0, 0], np.int32)
    # request 0: root has children 1, 2; walk accepts 2 (child 1 rejected: root rejects), node 2 is a leaf
    # request 1: a chain; walk accepts 1, then stops at node 1 (its child rejected)
    # request 2: greedy: nothing beyond the statistics
    path = np.array([[2, -1, -1, -1], [1, -1, -1, -1], [-1, -1, -1, -1]], np.int32)
    b = W.tree_accept_bytes_walk_form(st, path, np.array([1, 1, 0]))
    assert b["rejecting_nodes_on_walks"] == 2
    assert b["stats_logits"] == 11 * 16 * 2 and b["walk_rows"] == 2 * 16 * 4 and b["accept"] == b["stats_logits"] + b["walk_rows"]
    # first children accepted all the way down to a leaf: no rejecting node
    path = np.array([[1, 3, -1, -1], [1, 2, 3, -1], [-1, -1, -1, -1]], np.int32)
    assert W.tree_accept_bytes_walk_form(st, path, np.array([2, 3, 0]))["rejecting_nodes_on_walks"] == 0


def test_masked_logits_option():
    st = W.make_custom_step(3, ctx_lens=[5, 9, 4], spec_lens=[3, 5, 0], vocab=64, logits_dtype="bf16",
                            attention=False, masked_frac=0.4, temperature=[1.0, 0.7, 1.0])
    logits = W.to_f64(st.target_logits, "bf16")
    masked = np.isinf(logits)
    assert 0.25 < masked.mean() < 0.55 and (logits[masked] < 0).all()
    assert (~masked).any(axis=1).all()                                 # every row keeps a finite entry
    q = W.to_f64(st.draft_probs, "bf16")
    keep = np.ones(st.total_q, dtype=bool)
    keep[st.cu_q[1:] - 1] = False
    assert not np.isnan(q).any() and (q[masked[keep]] == 0).all()      # the draft puts no mass on masked tokens
    for d in range(st.total_draft):
        assert q[d, st.draft_tokens[d]] > 0


def test_policy_inputs_and_policy_shaped_step():
    """The synthetic inputs of the speculative-length policy are seeded and hold draws only; the step built
    from a vector of draft lengths has ctx_lens = committed + k + 1 and the config's tensor shapes."""
    a, b = W.policy_inputs(3, batch=12), W.policy_inputs(3, batch=12)
    assert np.array_equal(a["ctx_committed"], b["ctx_committed"]) and np.array_equal(a["conf"], b["conf"])
    assert a["conf"].shape == (8, 12) and a["conf"].dtype == np.float64
    assert np.all(a["conf"] > 0) and np.all(a["conf"] <= 1) and 0 < a["prev_conf"] < 1
    assert not np.array_equal(a["conf"], W.policy_inputs(3, batch=12, seed=7)["conf"])
    k = np.arange(12, dtype=np.int32) % 5
    st = W.make_policy_step(a, k, attention=False)
    assert np.array_equal(st.spec_lens, k) and np.array_equal(st.ctx_lens, a["ctx_committed"] + k + 1)
    assert st.vocab == W.CONFIGS[3]["vocab"] and st.total_q == int((k + 1).sum()) and st.name.endswith("-policy")
    assert np.array_equal(st.temperature, a["temperature"])
