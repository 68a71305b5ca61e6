"""GPU parity of tree verification (adaspec_verify_attn_tree, adaspec_accept_tree,
adaspec_kv_compact_path) against the CPU oracle, through the C ABI.  Same bars as the chain
calls: attention max-abs 2e-3 on the fp32 accumulator; tokens, accept lengths and paths bit-exact
except counted near-ties; page contents bit-exact.
"""
import os
import sys

import numpy as np
import pytest

import workloads as W
from oracle import kv_cache as KV
from tests.harness import _torch_from, compare_accept_tree, compare_attention, to_device

pytestmark = pytest.mark.gpu
ATTN_TOL = 2e-3                                             # the benchmark's bar
ATTN_GUARD = {"f32": 2e-5, "bf16": 2e-5, "f16": 1e-3}       # what the tests enforce (see test_gpu_parity.py)
NEAR_TIE_FRAC = 0.025
F32 = 0


def _say(msg):
    print(f"[case] {msg}", file=sys.stderr, flush=True)
    report = os.environ.get("ADASPEC_TEST_REPORT")
    if report:
        with open(report, "a") as f:
            f.write(msg + "\n")


@pytest.fixture(scope="module")
def pkg():
    import paper_2503_05096_amd as p
    return p


def _check_tree_attention(st, oracle, pkg, path="auto"):
    import torch
    dev = to_device(st, acceptance=False)
    ref, _ = oracle.verify_attn_tree(st.q, st.k_pages, st.v_pages, st.block_table, st.ctx_lens, st.spec_lens,
                                     st.parents, dtype=st.dtype, want_rounded=False)
    _say(f"tree attn {st.name} path={path} B={st.batch} TQ={st.total_q} dtype={st.dtype}")
    kw = dict(max_spec_len=st.max_spec_len, path=path, parents=dev.parents)
    acc = pkg.verify_attn(dev.q, dev.k_pages, dev.v_pages, dev.block_table, dev.ctx_lens, dev.spec_lens,
                          out_dtype=F32, **kw)
    torch.cuda.synchronize()
    rep = compare_attention(acc, ref, None, st.dtype)
    assert rep["nan"] == 0 and rep["max_abs_vs_f64"] <= ATTN_GUARD[st.dtype], rep
    out = pkg.verify_attn(dev.q, dev.k_pages, dev.v_pages, dev.block_table, dev.ctx_lens, dev.spec_lens, **kw)
    out2 = pkg.verify_attn(dev.q, dev.k_pages, dev.v_pages, dev.block_table, dev.ctx_lens, dev.spec_lens, **kw)
    torch.cuda.synchronize()
    want = acc.to(out.dtype)
    assert torch.equal(out, want) and torch.equal(out, out2)
    _say(f"tree attn {st.name} ok {rep}")
    return rep


def _check_tree_accept(st, oracle, pkg, out_stride=None, max_near_tie_frac=NEAR_TIE_FRAC, kpath="auto"):
    import torch
    dev = to_device(st, attention=False)
    _say(f"tree accept {st.name} path={kpath} B={st.batch} TQ={st.total_q} V={st.vocab}")
    toks, alen, path = pkg.accept_tree(dev.target_logits, dev.draft_probs, dev.draft_tokens, dev.parents,
                                       dev.uniforms, dev.spec_lens, dev.temperature,
                                       max_spec_len=st.max_spec_len, out_stride=out_stride, path=kpath)
    torch.cuda.synchronize()
    rep = compare_accept_tree(st, toks.cpu().numpy(), alen.cpu().numpy(), path.cpu().numpy(), oracle,
                              out_stride=out_stride)
    _say(f"tree accept {st.name} {({k: v for k, v in rep.items() if k != 'details'})}")
    assert rep["hard_mismatches"] == 0, rep["details"][:5]
    assert rep["ratio_near_ties"] + rep["cdf_near_ties"] <= max(2, max_near_tie_frac * st.batch), rep
    again = pkg.accept_tree(dev.target_logits, dev.draft_probs, dev.draft_tokens, dev.parents, dev.uniforms,
                            dev.spec_lens, dev.temperature, max_spec_len=st.max_spec_len, out_stride=out_stride,
                            path=kpath)
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip((toks, alen, path), again))
    return rep, (toks, alen, path)


# ------------------------------------------------------------------ attention
@pytest.mark.parametrize("cfg,width", [(1, 2), (2, 3), (3, 3), (4, 2), (5, 2)])
def test_config_tree_attention(cfg, width, oracle_mod, pkg):
    st = W.attach_tree(W.make_verify_step(cfg, acceptance=False), max_width=width)
    _check_tree_attention(st, oracle_mod, pkg)


@pytest.mark.parametrize("dtype,hq,hkv,d,path", [("f32", 4, 2, 64, "auto"), ("bf16", 8, 2, 128, "auto"),
                                                  ("f16", 8, 8, 128, "auto"), ("bf16", 8, 2, 128, "vector")])
def test_tree_attention_edges(dtype, hq, hkv, d, path, oracle_mod, pkg):
    """Trees of 1 to 64 nodes, new positions that straddle pages, 32-token blocks and KV splits,
    contexts with and without committed tokens in front of the tree."""
    ctx = [1, 64, 65, 40, 300, 2100, 33, 16, 700, 17]
    spec = [0, 63, 63, 39, 7, 30, 32, 15, 1, 5]
    st = W.make_custom_step(91, ctx_lens=ctx, spec_lens=spec, n_q_heads=hq, n_kv_heads=hkv, head_dim=d,
                            dtype=dtype, acceptance=False, name=f"tree-edges-{dtype}")
    W.attach_tree(st, max_width=4)
    _check_tree_attention(st, oracle_mod, pkg, path=path)


@pytest.mark.parametrize("B", [300, 2100])
def test_tree_attention_many_requests(B, oracle_mod, pkg):
    """More requests than one mask workgroup serves, and (2100) more than the metadata kernel builds masks
    for itself: the separate mask kernel takes over."""
    rng = np.random.default_rng(B)
    spec = rng.integers(0, 9, B).astype(np.int32)
    ctx = (spec + 1 + rng.integers(0, 70, B)).astype(np.int32)
    st = W.make_custom_step(B, ctx_lens=ctx, spec_lens=spec, n_q_heads=4, n_kv_heads=2, head_dim=128, dtype="bf16",
                            acceptance=False, name=f"tree-many-{B}")
    W.attach_tree(st, max_width=3)
    _check_tree_attention(st, oracle_mod, pkg)


def test_chain_parents_reproduce_the_chain_call(pkg):
    import torch
    st = W.attach_tree(W.make_verify_step(3, acceptance=False, batch=24), chain=True)
    dev = to_device(st, acceptance=False)
    kw = dict(max_spec_len=st.max_spec_len)
    a = pkg.verify_attn(dev.q, dev.k_pages, dev.v_pages, dev.block_table, dev.ctx_lens, dev.spec_lens, **kw)
    b = pkg.verify_attn(dev.q, dev.k_pages, dev.v_pages, dev.block_table, dev.ctx_lens, dev.spec_lens,
                        parents=dev.parents, **kw)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_tree_attention_metadata_reuse(oracle_mod, pkg):
    """The ancestor masks are part of the metadata a multi-layer pass builds once."""
    import torch
    st = W.attach_tree(W.make_verify_step(3, acceptance=False, batch=16), max_width=3)
    dev = to_device(st, acceptance=False)
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda:0")
    kw = dict(max_spec_len=st.max_spec_len, parents=dev.parents, workspace=ws)
    one = pkg.verify_attn(dev.q, dev.k_pages, dev.v_pages, dev.block_table, dev.ctx_lens, dev.spec_lens, **kw)
    pkg.verify_attn(dev.q, dev.k_pages, dev.v_pages, dev.block_table, dev.ctx_lens, dev.spec_lens,
                    plan="build", **kw)
    two = pkg.verify_attn(dev.q, dev.k_pages, dev.v_pages, dev.block_table, dev.ctx_lens, dev.spec_lens,
                          plan="reuse", **kw)
    torch.cuda.synchronize()
    assert torch.equal(one, two)


# ----------------------------------------------------------------- acceptance
@pytest.mark.parametrize("cfg,greedy,width", [(1, False, 2), (2, False, 3), (3, False, 3), (4, False, 2),
                                              (4, True, 3), (5, False, 2)])
def test_config_tree_accept(cfg, greedy, width, oracle_mod, pkg):
    """AUTO: the 1024-thread node kernel for the 16-bit configs, the portable one for config 1."""
    st = W.attach_tree(W.make_verify_step(cfg, greedy=greedy, attention=False), max_width=width)
    rep, _ = _check_tree_accept(st, oracle_mod, pkg)
    assert 0 < rep["oracle_mean_accept_len"]


@pytest.mark.parametrize("cfg,width", [(2, 3), (3, 2)])
def test_config_tree_accept_portable_kernel(cfg, width, oracle_mod, pkg):
    st = W.attach_tree(W.make_verify_step(cfg, attention=False, batch=24), max_width=width)
    _check_tree_accept(st, oracle_mod, pkg, kpath="vector")


@pytest.mark.parametrize("dtype,V,sigma", [("bf16", 4096, 0.3), ("f16", 32000, 0.5), ("bf16", 131072, 0.6),
                                           ("bf16", 8, 0.3), ("bf16", 200008, 0.6), ("f16", 524288, 0.8)])
def test_tree_accept_fast_kernel_shapes(dtype, V, sigma, oracle_mod, pkg):
    """The 1024-thread kernels on vocabularies from one partial step to the sixty-four steps they hold, with
    a draft close enough to the target that later children get tested and long paths occur."""
    rng = np.random.default_rng(8)
    spec = np.array([0, 1, 8, 8, 20, 63, 3, 5, 12, 2, 7, 7, 30, 4], np.int32)
    if V > 131072:
        spec = spec[[0, 1, 2, 6, 7, 9]]                              # (keeps the host tensors of the big rows small)
    T = rng.choice([0.0, 0.6, 1.0, 1.4], size=spec.shape[0])
    st = W.make_custom_step(321, ctx_lens=spec + 1, spec_lens=spec, vocab=V, logits_dtype=dtype, temperature=T,
                            attention=False, noise_sigma=sigma, name=f"tree-fast-{dtype}-{V}")
    W.attach_tree(st, max_width=4)
    cu = st.cu_q
    st.parents[cu[2] + 1:cu[3]] = 0                                  # request 2: a star of 8 children
    rep, (toks, alen, path) = _check_tree_accept(st, oracle_mod, pkg, kpath="fast", max_near_tie_frac=0.2)
    if 4096 <= V <= 131072:
        assert alen.max().item() >= 2


@pytest.mark.parametrize("dtype,V", [("f32", 1000), ("bf16", 4104), ("f16", 777)])
def test_tree_accept_edges(dtype, V, oracle_mod, pkg):
    """Stars (every draft a child of the root), chains, single nodes, wide and deep trees, mixed
    temperatures, a row stride wider than needed, vocabularies that are no multiple of the tile."""
    rng = np.random.default_rng(5)
    spec = np.array([0, 1, 8, 8, 20, 63, 3, 5, 12, 2, 7, 7], np.int32)
    T = rng.choice([0.0, 0.6, 1.0, 1.4], size=spec.shape[0])
    st = W.make_custom_step(123, ctx_lens=spec + 1, spec_lens=spec, vocab=V, logits_dtype=dtype, temperature=T,
                            attention=False, noise_sigma=0.8, name=f"tree-accept-edges-{dtype}")
    W.attach_tree(st, max_width=3)
    cu = st.cu_q
    st.parents[cu[2] + 1:cu[3]] = 0                                  # request 2: a star
    st.parents[cu[3]:cu[4]] = np.arange(-1, 8)                       # request 3: a chain
    # the tokens of the two rewired requests still come from a valid distribution (any token is legal input)
    _check_tree_accept(st, oracle_mod, pkg, out_stride=70, max_near_tie_frac=0.2)


@pytest.mark.parametrize("kpath", ["fast", "vector"])
def test_tree_accept_residual_without_mass(kpath, oracle_mod, pkg):
    """A draft distribution that lies above the target everywhere (each of 8 equal probabilities rounded up
    to the next bf16 value): a child can be rejected (p/q = 0.992 < u), but max(0, P - q) is empty, so the
    distribution stays as it was for every later child and for the draw.  Stars of 1..5 children, all
    rejected, plus a request whose second child is accepted from the unchanged distribution."""
    V, spec = 8, np.array([1, 3, 5, 3], np.int32)
    st = W.make_custom_step(9, ctx_lens=spec + 1, spec_lens=spec, vocab=V, logits_dtype="bf16", temperature=1.0,
                            attention=False, name="no-mass")
    W.attach_tree(st, max_width=3)
    cu = st.cu_q
    for i in range(st.batch):
        st.parents[cu[i] + 1:cu[i + 1]] = 0                          # stars
    st.target_logits[:] = 0                                          # p = 1/8 everywhere (bf16 zero bits)
    st.draft_probs[:] = W.f32_to_bf16_bits(np.full(st.draft_probs.shape, 0.1259765625, np.float32))
    st.uniforms[:, 0] = 0.999                                        # above p/q = 0.9922...: every child rejected
    st.uniforms[:, 1] = np.linspace(0.05, 0.95, st.total_q)
    st.uniforms[cu[3] + 1, 0] = 0.5                                  # request 3: its second child is accepted
    rep, (toks, alen, path) = _check_tree_accept(st, oracle_mod, pkg, kpath=kpath)
    assert rep["exact"] == st.batch
    assert alen.cpu().tolist() == [0, 0, 0, 1] and int(path[3, 0]) == 2
    # the draws come from the target itself: token = floor(u1 * 8)
    for i in range(3):
        assert int(toks[i, 0]) == int(st.uniforms[cu[i], 1] * 8)


def test_chain_tree_accept_equals_the_chain_call(pkg):
    import torch
    st = W.attach_tree(W.make_verify_step(2, attention=False), chain=True)
    dev = to_device(st, attention=False)
    t1, a1 = pkg.accept(dev.target_logits, dev.draft_probs, dev.draft_tokens, dev.uniforms, dev.spec_lens,
                        dev.temperature, max_spec_len=st.max_spec_len, path="vector")
    t2, a2, p2 = pkg.accept_tree(dev.target_logits, dev.draft_probs, dev.draft_tokens, dev.parents, dev.uniforms,
                                 dev.spec_lens, dev.temperature, max_spec_len=st.max_spec_len, path="vector")
    torch.cuda.synchronize()
    assert torch.equal(t1, t2) and torch.equal(a1, a2)
    p2, a2 = p2.cpu().numpy(), a2.cpu().numpy()
    for i in range(st.batch):
        assert list(p2[i, :a2[i]]) == list(range(1, a2[i] + 1)) and np.all(p2[i, a2[i]:] == -1)


# ------------------------------------------------ compaction and a whole tree step
def test_tree_step_end_to_end(oracle_mod, pkg):
    """append -> tree attention -> tree acceptance -> path compaction -> commit, device side only;
    afterwards the cache holds the accepted path where a chain would have put it."""
    import torch
    rng0 = np.random.default_rng(40)
    spec = rng0.integers(0, 13, size=48)
    # a draft close to the target (small noise), so that paths are long and leave the first branch
    st = W.make_custom_step(41, ctx_lens=rng0.integers(64, 1500, size=48) + spec + 1, spec_lens=spec,
                            n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16", vocab=4096,
                            logits_dtype="bf16", temperature=rng0.choice([0.0, 0.8, 1.0], size=48),
                            noise_sigma=0.35, name="tree-step")
    W.attach_tree(st, max_width=3)
    dev = to_device(st)
    rng = np.random.default_rng(17)
    shape = (st.total_q, st.n_kv_heads, st.head_dim)
    k_new = W.f32_to_bf16_bits(rng.standard_normal(shape, np.float32))
    v_new = W.f32_to_bf16_bits(rng.standard_normal(shape, np.float32))
    kw = dict(max_spec_len=st.max_spec_len)
    pkg.kv_append(_torch_from(k_new, "bf16", "cuda:0"), _torch_from(v_new, "bf16", "cuda:0"), dev.k_pages,
                  dev.v_pages, dev.block_table, dev.ctx_lens, dev.spec_lens, **kw)
    out = pkg.verify_attn(dev.q, dev.k_pages, dev.v_pages, dev.block_table, dev.ctx_lens, dev.spec_lens,
                          parents=dev.parents, out_dtype=F32, **kw)
    toks, alen, path = pkg.accept_tree(dev.target_logits, dev.draft_probs, dev.draft_tokens, dev.parents,
                                       dev.uniforms, dev.spec_lens, dev.temperature, **kw)
    pkg.kv_compact_path(dev.k_pages, dev.v_pages, dev.block_table, dev.ctx_lens, dev.spec_lens, path, alen, **kw)
    committed, _, last = pkg.commit(toks, alen, dev.spec_lens, dev.ctx_lens, **kw)
    torch.cuda.synchronize()
    # oracle side of the same step
    k1, v1 = KV.kv_append(k_new, v_new, st.k_pages, st.v_pages, st.block_table, st.ctx_lens, st.spec_lens)
    ref, _ = oracle_mod.verify_attn_tree(st.q, k1, v1, st.block_table, st.ctx_lens, st.spec_lens, st.parents,
                                         dtype=st.dtype, want_rounded=False)
    rep = compare_attention(out, ref, None, st.dtype)
    assert rep["nan"] == 0 and rep["max_abs_vs_f64"] <= ATTN_GUARD[st.dtype], rep
    arep = compare_accept_tree(st, toks.cpu().numpy(), alen.cpu().numpy(), path.cpu().numpy(), oracle_mod)
    assert arep["hard_mismatches"] == 0, arep["details"][:5]
    # compaction and commit are integer / byte work: exact, given the GPU's own path
    k2, v2 = KV.kv_compact_path(k1, v1, st.block_table, st.ctx_lens, st.spec_lens, path.cpu().numpy(),
                                alen.cpu().numpy())
    assert np.array_equal(dev.k_pages.view(torch.int16).cpu().numpy(), k2.view(np.int16))
    assert np.array_equal(dev.v_pages.view(torch.int16).cpu().numpy(), v2.view(np.int16))
    c = KV.commit(toks.cpu().numpy(), alen.cpu().numpy(), st.spec_lens, st.ctx_lens)
    assert np.array_equal(committed.cpu().numpy(), c["committed_lens"]) and np.array_equal(last.cpu().numpy(), c["last_token"])
    assert alen.cpu().numpy().max() >= 2 and (path.cpu().numpy()[:, 0] > 1).any()     # some path left the first branch
    _say(f"tree step ok: attention {rep}, acceptance { {k: v for k, v in arep.items() if k != 'details'} }")


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("f16", 128)])
def test_kv_compact_path_matches_oracle_bitwise(dtype, d, pkg):
    import torch
    rng = np.random.default_rng(2)
    spec = np.array([0, 5, 9, 3, 16, 63], np.int32)
    st = W.make_custom_step(19, ctx_lens=[1, 20, 33, 4, 50, 200], spec_lens=spec, n_q_heads=4, n_kv_heads=2,
                            head_dim=d, dtype=dtype, acceptance=False)
    W.attach_tree(st, max_width=3)
    cu, B = st.cu_q, st.batch
    path = -np.ones((B, 64), np.int32)
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
    pkg.kv_compact_path(dev.k_pages, dev.v_pages, dev.block_table, dev.ctx_lens, dev.spec_lens,
                        torch.from_numpy(path).cuda(), torch.from_numpy(alen).cuda(), max_spec_len=63)
    torch.cuda.synchronize()
    it = torch.int32 if dtype == "f32" else torch.int16
    nt = np.int32 if dtype == "f32" else np.int16
    assert np.array_equal(dev.k_pages.view(it).cpu().numpy(), k2.view(nt))
    assert np.array_equal(dev.v_pages.view(it).cpu().numpy(), v2.view(nt))


# ------------------------------------------------------------------ robustness
def test_tree_step_replayed_from_a_hip_graph(pkg):
    """The tree calls launch kernels only, so a captured tree step replays bit for bit with new inputs."""
    import torch
    steps = []
    for s in range(3):
        st = W.make_custom_step(700 + s, ctx_lens=[300, 77, 2500, 40, 1200, 640], spec_lens=[3, 0, 5, 2, 4, 1],
                                n_q_heads=16, n_kv_heads=4, head_dim=128, dtype="bf16", vocab=8192,
                                logits_dtype="bf16", temperature=[0.8, 1.0, 0.0, 0.7, 1.0, 0.9], poison=False,
                                noise_sigma=0.5)
        steps.append(W.attach_tree(st, max_width=2, seed=50 + s))
    devs = [to_device(st) for st in steps]
    kmax = steps[0].max_spec_len
    buf = to_device(steps[0])
    names = ("q", "k_pages", "v_pages", "block_table", "target_logits", "draft_probs", "draft_tokens", "uniforms",
             "parents")
    out = torch.empty_like(buf.q)
    B = steps[0].batch
    toks = torch.empty((B, kmax + 1), dtype=torch.int32, device="cuda:0")
    path = torch.empty((B, kmax + 1), dtype=torch.int32, device="cuda:0")
    alen = torch.empty((B,), dtype=torch.int32, device="cuda:0")
    ws_a = torch.empty(32 << 20, dtype=torch.uint8, device="cuda:0")
    ws_b = torch.empty(4 << 20, dtype=torch.uint8, device="cuda:0")

    def run(d, o, t, a, p):
        pkg.verify_attn(d.q, d.k_pages, d.v_pages, d.block_table, d.ctx_lens, d.spec_lens, o, max_spec_len=kmax,
                        workspace=ws_a, parents=d.parents)
        pkg.accept_tree(d.target_logits, d.draft_probs, d.draft_tokens, d.parents, d.uniforms, d.spec_lens,
                        d.temperature, max_spec_len=kmax, out_tokens=t, out_accept_len=a, out_path=p, workspace=ws_b)

    run(buf, out, toks, alen, path)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    _say("capturing tree attention + tree acceptance into a HIP graph")
    with torch.cuda.graph(g):
        run(buf, out, toks, alen, path)
    for rep in range(2):
        for s, d in enumerate(devs):
            ref = (torch.empty_like(out), torch.empty_like(toks), torch.empty_like(alen), torch.empty_like(path))
            run(d, *ref)
            torch.cuda.synchronize()
            for n in names:
                getattr(buf, n).copy_(getattr(d, n))
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(out.view(torch.int16), ref[0].view(torch.int16)), (rep, s)
            assert torch.equal(toks, ref[1]) and torch.equal(alen, ref[2]) and torch.equal(path, ref[3]), (rep, s)


@pytest.mark.parametrize("kpath", ["fast", "vector"])
def test_tree_accept_many_requests(kpath, oracle_mod, pkg):
    """More requests than a plan workgroup has threads (the metadata scan loops) and than the device has
    compute units (several walk workgroups per unit)."""
    rng = np.random.default_rng(12)
    B = 1500 if kpath == "vector" else 2500        # (above 2048 the fast form takes its row offsets from the metadata kernel)
    spec = rng.integers(0, 6, size=B).astype(np.int32)
    st = W.make_custom_step(55, ctx_lens=spec + 1, spec_lens=spec, vocab=512, logits_dtype="bf16",
                            temperature=rng.choice([0.0, 0.9], size=B), attention=False, noise_sigma=0.4,
                            name="tree-many")
    W.attach_tree(st, max_width=3)
    _check_tree_accept(st, oracle_mod, pkg, kpath=kpath)


def test_malformed_parents_are_forced_into_the_request(oracle_mod, pkg):
    """Parent indices outside [0, j) for node j are clamped into that range (a root keeps no parent):
    the outputs are those of the clamped tree, and nothing is read or written outside the request."""
    import torch
    st = W.make_custom_step(77, ctx_lens=[40, 300, 33, 700], spec_lens=[5, 9, 0, 12], n_q_heads=8, n_kv_heads=2,
                            head_dim=128, dtype="bf16", vocab=2048, logits_dtype="bf16", noise_sigma=0.4,
                            name="tree-malformed")
    W.attach_tree(st, max_width=3)
    good = st.parents.copy()
    bad = good.copy()
    cu = st.cu_q
    rng = np.random.default_rng(3)
    for i in range(st.batch):
        n = int(st.spec_lens[i]) + 1
        bad[cu[i]] = int(rng.integers(-5, 100))                      # the root's entry is ignored
        for j in range(1, n):
            r = rng.random()
            if r < 0.25:
                bad[cu[i] + j] = j + int(rng.integers(0, 1000))      # too large -> j - 1
                good[cu[i] + j] = j - 1
            elif r < 0.5:
                bad[cu[i] + j] = -int(rng.integers(1, 1000))         # negative -> 0
                good[cu[i] + j] = 0
    dev = to_device(st)
    bad_dev = torch.from_numpy(bad).cuda()
    kw = dict(max_spec_len=st.max_spec_len)
    # the optional device-side check tells the two arrays apart (the root's entry is never looked at)
    assert pkg.check_tree_parents(bad_dev, dev.spec_lens, **kw) == 16
    assert pkg.check_tree_parents(torch.from_numpy(good).cuda(), dev.spec_lens, **kw) == 0
    out = pkg.verify_attn(dev.q, dev.k_pages, dev.v_pages, dev.block_table, dev.ctx_lens, dev.spec_lens,
                          out_dtype=F32, parents=bad_dev, **kw)
    res = {p: pkg.accept_tree(dev.target_logits, dev.draft_probs, dev.draft_tokens, bad_dev, dev.uniforms,
                              dev.spec_lens, dev.temperature, path=p, **kw) for p in ("fast", "vector")}
    torch.cuda.synchronize()
    st.parents = good
    ref, _ = oracle_mod.verify_attn_tree(st.q, st.k_pages, st.v_pages, st.block_table, st.ctx_lens, st.spec_lens,
                                         good, dtype=st.dtype, want_rounded=False)
    rep = compare_attention(out, ref, None, st.dtype)
    assert rep["nan"] == 0 and rep["max_abs_vs_f64"] <= ATTN_GUARD[st.dtype], rep
    for p, (toks, alen, path) in res.items():
        arep = compare_accept_tree(st, toks.cpu().numpy(), alen.cpu().numpy(), path.cpu().numpy(), oracle_mod)
        assert arep["hard_mismatches"] == 0, (p, arep["details"][:3])


def test_tree_accept_random_shapes(oracle_mod, pkg):
    """Many small random cases through both kernels: vocabularies from one vector to several steps, stars wide
    enough that more stages are taken than the walk kernel keeps in registers, drafts far from and close to
    the target, mixed temperatures.  Every case is held to the usual bar against the oracle."""
    import torch
    rng = np.random.default_rng(2024)
    near = 0
    for case in range(24):
        B = int(rng.integers(1, 13))
        spec = rng.integers(0, 14, size=B).astype(np.int32)
        V = int(rng.choice([8, 64, 1000 // 8 * 8, 4096, 8200, 20000]))
        dtype = str(rng.choice(["bf16", "f16"]))
        T = rng.choice([0.0, 0.5, 1.0, 1.7], size=B)
        sigma = float(rng.choice([0.2, 0.8, 2.5]))
        st = W.make_custom_step(5000 + case, ctx_lens=spec + 1, spec_lens=spec, vocab=V, logits_dtype=dtype,
                                temperature=T, attention=False, noise_sigma=sigma, name=f"tree-rand-{case}")
        W.attach_tree(st, max_width=int(rng.integers(1, 6)))
        if case % 3 == 0:                                            # one request becomes a star
            i = int(np.argmax(spec))
            cu = st.cu_q
            st.parents[cu[i] + 1:cu[i + 1]] = 0
        for kpath in ("fast", "vector"):
            rep, _ = _check_tree_accept(st, oracle_mod, pkg, kpath=kpath, max_near_tie_frac=1.0)
            near += rep["ratio_near_ties"] + rep["cdf_near_ties"]
    assert near <= 6, near                                           # rare by construction (1e-5 windows)


@pytest.mark.parametrize("kpath", ["fast", "vector"])
def test_tree_accept_with_masked_logits(kpath, oracle_mod, pkg):
    """A share of every target row is -inf (and the draft distribution 0 there), whole 16-lane groups
    included: the group-relative sums of the statistics kernel must not produce NaN."""
    rng = np.random.default_rng(32)
    B = 30
    spec = rng.integers(0, 9, size=B).astype(np.int32)
    st = W.make_custom_step(641, ctx_lens=spec + 1, spec_lens=spec, vocab=16384, logits_dtype="bf16",
                            temperature=rng.choice([0.0, 0.8, 1.0], size=B), attention=False, noise_sigma=0.5,
                            masked_frac=0.35, name="tree-masked-logits")
    # mask a long aligned stretch of every row as well: whole steps without a finite logit
    st.target_logits[:, 2048:12288] = np.uint16(0xFF80)
    st.draft_probs[:, 2048:12288] = 0
    W.attach_tree(st, max_width=3)
    _check_tree_accept(st, oracle_mod, pkg, kpath=kpath, max_near_tie_frac=0.1)
