"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer: the CPU oracle's C files and the
policy's host C++ are built with -fsanitize=address,undefined into a small driver
(tests/native/sanitize_driver.c), which runs every entry point on seeded inputs.  The driver must end
without a report, and its results must equal those of the ordinary builds."""
import os
import subprocess
import sys

import numpy as np
import pytest

import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g"]


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    build = tmp_path_factory.mktemp("sanitize_build")
    objs = []
    for src in ("oracle/adaspec_oracle.c", "oracle/adaspec_tree_oracle.c", "tests/native/sanitize_driver.c"):
        obj = str(build / (os.path.basename(src) + ".o"))
        subprocess.check_call(["gcc", "-O1", "-std=c11", "-ffp-contract=off", "-fopenmp", *SAN, "-I",
                               os.path.join(ROOT, "include"), "-c", os.path.join(ROOT, src), "-o", obj])
        objs.append(obj)
    obj = str(build / "policy.o")
    subprocess.check_call(["g++", "-O1", "-std=c++17", *SAN, "-I", os.path.join(ROOT, "include"), "-c",
                           os.path.join(ROOT, "paper_2503_05096_amd", "csrc", "policy.cpp"), "-o", obj])
    objs.append(obj)
    exe = str(build / "sanitize_driver")
    subprocess.check_call(["g++", *SAN, "-fopenmp", "-static-libasan", "-static-libubsan", *objs, "-o", exe, "-lm"])
    return exe


def test_oracle_and_policy_host_code_under_asan_and_ubsan(driver, tmp_path, oracle_mod):
    from oracle import policy as OP
    from paper_2503_05096_amd import policy as PP
    st = W.make_custom_step(31337, ctx_lens=[70, 33, 130, 17, 48], spec_lens=[2, 0, 4, 3, 1], n_q_heads=4,
                            n_kv_heads=2, head_dim=32, dtype="bf16", vocab=200, logits_dtype="bf16",
                            temperature=[0.8, 1.0, 0.0, 0.7, 1.2], name="sanitize")
    chain_tokens = st.draft_tokens.copy()
    W.attach_tree(st, max_width=2)
    tree_tokens = st.draft_tokens.copy()
    B, max_steps = st.batch, 6
    rng = np.random.default_rng(9)
    C_committed = (st.ctx_lens - st.spec_lens - 1).astype(np.int32)
    conf = rng.uniform(0.2, 0.99, (max_steps, B))
    m = PP.TimeModel(2e-9, 3e-7, 5e-5, 2.2e-8, 6e-7, 1e-4, 1, 0)
    dt = {"f32": 0, "f16": 1, "bf16": 2}
    dims = np.array([B, st.total_q, st.n_q_heads, st.n_kv_heads, st.head_dim, st.page_size, st.k_pages.shape[0],
                     st.block_table.shape[1], dt[st.dtype], st.vocab, dt[st.logits_dtype], dt[st.probs_dtype],
                     st.max_spec_len + 1, max_steps], np.int32)
    files = dict(dims=dims, q=st.q, k_pages=st.k_pages, v_pages=st.v_pages, block_table=st.block_table,
                 ctx_lens=st.ctx_lens, spec_lens=st.spec_lens, parents=st.parents, tree_draft_tokens=tree_tokens,
                 target_logits=st.target_logits, draft_probs=st.draft_probs, draft_tokens=chain_tokens,
                 uniforms=st.uniforms, temperature=st.temperature, ctx_committed=C_committed, conf=conf)
    for name, arr in files.items():
        np.ascontiguousarray(arr).tofile(str(tmp_path / f"{name}.bin"))
    with open(tmp_path / "time_model.bin", "wb") as f:
        f.write(bytes(m))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="2")
    r = subprocess.run([driver, str(tmp_path)], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0 and "sanitizer driver: done" in r.stdout, (r.returncode, r.stdout[-500:], r.stderr[-3000:])
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-3000:]

    def out(name, dtype, shape=None):
        a = np.fromfile(str(tmp_path / f"{name}.bin"), dtype=dtype)
        return a if shape is None else a.reshape(shape)

    # the same calls through the ordinary builds
    ref, ref_r = oracle_mod.verify_attn(st.q, st.k_pages, st.v_pages, st.block_table, st.ctx_lens, st.spec_lens,
                                        dtype=st.dtype)
    assert np.array_equal(out("out_attn", np.float64, ref.shape), ref)
    assert np.array_equal(out("out_attn_rounded", np.float64, ref.shape), ref_r)
    ref_t, _ = oracle_mod.verify_attn_tree(st.q, st.k_pages, st.v_pages, st.block_table, st.ctx_lens, st.spec_lens,
                                           st.parents, dtype=st.dtype, want_rounded=False)
    assert np.array_equal(out("out_attn_tree", np.float64, ref_t.shape), ref_t)
    o_tok, o_len, _ = oracle_mod.accept(st.target_logits, st.draft_probs, chain_tokens, st.uniforms, st.spec_lens,
                                        st.temperature, logits_dtype=st.logits_dtype, probs_dtype=st.probs_dtype)
    assert np.array_equal(out("out_tokens", np.int32, o_tok.shape), o_tok)
    assert np.array_equal(out("out_accept_len", np.int32), o_len)
    t_tok, t_len, t_path, _, _ = oracle_mod.accept_tree(st.target_logits, st.draft_probs, tree_tokens, st.parents,
                                                        st.uniforms, st.spec_lens, st.temperature,
                                                        logits_dtype=st.logits_dtype, probs_dtype=st.probs_dtype)
    assert np.array_equal(out("out_tree_tokens", np.int32, t_tok.shape), t_tok)
    assert np.array_equal(out("out_tree_accept_len", np.int32), t_len)
    assert np.array_equal(out("out_tree_path", np.int32, t_path.shape), t_path)
    dq, dtok, _, _ = oracle_mod.draft_sample(st.target_logits[:B], st.temperature, st.uniforms[:B, 1].copy(),
                                             logits_dtype=st.logits_dtype, probs_dtype=st.probs_dtype)
    assert np.array_equal(out("out_draft_tokens", np.int32), dtok)
    assert np.array_equal(out("out_draft_q", np.float64, dq.shape), dq)
    # policy: the sanitizer build against the library's build and against the oracle
    om = OP.TimeModel(m.alpha_d, m.gamma_d, m.delta_d, m.alpha_v, m.gamma_v, m.delta_v, True)
    steps, ar, g = PP.adaptive_draft(m, C_committed, conf, 0.7, 1e30)
    k, g2 = PP.eliminate(m, C_committed, steps, ar, 1e30)
    res = out("out_policy", np.float64)
    assert int(res[0]) == steps and res[1] == g and res[2] == g2
    assert np.array_equal(out("out_policy_spec_lens", np.int32), k)
    o_steps, o_ars, _ = OP.adaptive_drafter(om, C_committed, conf, 0.7, 1e30)
    o_k, _ = OP.eliminate(om, C_committed, o_steps, o_ars, 1e30)
    assert o_steps == steps and np.array_equal(o_k, k)
    assert res[3] == PP.estimate_time(m, C_committed, steps, k) and res[4] == PP.goodput(m, C_committed, steps, k, ar, 1e30)
    assert (res[5], res[6]) == tuple(float(v) for v in OP.count_tokens(C_committed, k))
    np.testing.assert_allclose(out("out_policy_fit", np.float64), [3e-9, 2e-6, 1e-4], rtol=1e-6)
