"""The loop the policy exists for, closed on the GPU: the offline analyzer measures this library's own
kernels and fits the forward-time model (Sec. 6, Eq. 2-4); the policy (Alg. 1-3) turns those MI355X
coefficients and the drafter's confidences into per-request draft lengths; the verification step of
exactly that ragged batch is then held to the parity bar."""
import math
import sys

import numpy as np
import pytest

import workloads as W
from oracle import policy as OP
from tests.harness import compare_accept, compare_attention, to_device

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[case] {msg}", file=sys.stderr, flush=True)


def test_analyzer_measures_and_fits_on_this_gpu():
    """A small grid through the analyzer's own code path: the counts come from the library's C ABI
    (checked against the oracle's), times are positive, the fits exist and explain the measurements."""
    from paper_2503_05096_amd import analyzer
    grid = [(B, ctx, k) for B in (4, 24) for ctx in (128, 1536) for k in (0, 4)]
    _say(f"analyzer grid {grid}")
    rec = analyzer.run_grid(grid, iters=3, layers=2, draft_layers=1, log=lambda s: None)
    for p in rec["points"]:
        assert p["t_verify"] > 0 and p["t_draft"] > 0
        assert p["n_b"] >= p["B"] and p["n_c"] >= p["n_c_once"] - p["n_b"]
    for f in (rec["verify"]["ctx_per_position"], rec["verify"]["ctx_once_per_request"], rec["draft"]):
        assert all(math.isfinite(f[key]) for key in ("alpha_s_per_context_token", "gamma_s_per_batch_token", "delta_s"))
        assert f["r2"] <= 1.0
    # reading a request's cache once is the cost shape of this library's attention kernel
    assert rec["verify"]["ctx_once_per_request"]["r2"] > 0.8
    _say(f"analyzer fits r2: {rec['verify']['ctx_per_position']['r2']:.3f} (per position) "
         f"{rec['verify']['ctx_once_per_request']['r2']:.3f} (once per request) {rec['draft']['r2']:.3f} (draft)")


@pytest.mark.parametrize("tpot", [float("inf"), 2.2e-3])
def test_policy_shaped_step_parity(tpot, oracle_mod):
    """spec_lens = Alg. 1 + Alg. 2 on the shipped MI355X coefficients (library == oracle, decision for
    decision); then attention and acceptance of that batch against the oracle."""
    import torch
    import paper_2503_05096_amd as pkg
    from paper_2503_05096_amd import analyzer, policy as PP
    lm = analyzer.load_time_model(verify_ctx_once=True)
    om = OP.TimeModel(lm.alpha_d, lm.gamma_d, lm.delta_d, lm.alpha_v, lm.gamma_v, lm.delta_v, True)
    pin = W.policy_inputs(3, batch=40, max_steps=8)
    steps, ar, _ = PP.adaptive_draft(lm, pin["ctx_committed"], pin["conf"], pin["prev_conf"], tpot)
    k_lib, g_lib = PP.eliminate(lm, pin["ctx_committed"], steps, ar, tpot)
    o_steps, o_ars, _ = OP.adaptive_drafter(om, pin["ctx_committed"], pin["conf"], pin["prev_conf"], tpot)
    k_ora, g_ora = OP.eliminate(om, pin["ctx_committed"], o_steps, o_ars, tpot)
    assert steps == o_steps and np.array_equal(k_lib, k_ora) and math.isclose(g_lib, g_ora, rel_tol=1e-12)
    _say(f"policy tpot={tpot}: {steps} draft steps, spec_lens histogram {np.bincount(k_ora, minlength=9).tolist()}")
    st = W.make_policy_step(pin, k_ora)                  # the ORACLE's lengths are the input of both sides
    assert st.max_spec_len <= 8 and st.total_q == int((k_ora + 1).sum())
    dev = to_device(st)
    out = pkg.verify_attn(dev.q, dev.k_pages, dev.v_pages, dev.block_table, dev.ctx_lens, dev.spec_lens,
                          max_spec_len=st.max_spec_len, out_dtype=0)
    toks, alen = pkg.accept(dev.target_logits, dev.draft_probs, dev.draft_tokens, dev.uniforms, dev.spec_lens,
                            dev.temperature, max_spec_len=st.max_spec_len)
    torch.cuda.synchronize()
    ref, _ = oracle_mod.verify_attn(st.q, st.k_pages, st.v_pages, st.block_table, st.ctx_lens, st.spec_lens,
                                    dtype=st.dtype, want_rounded=False)
    err = compare_attention(out, ref, None, st.dtype)
    assert err["nan"] == 0 and err["max_abs_vs_f64"] <= 2e-5, err
    rep = compare_accept(st, toks.cpu().numpy(), alen.cpu().numpy(), oracle_mod)
    assert rep["hard_mismatches"] == 0, rep["details"][:5]
    assert rep["ratio_near_ties"] + rep["cdf_near_ties"] <= 2, rep
