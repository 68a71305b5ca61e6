"""GPU parity of adaspec_draft_sample against the oracle.

  probability row  16-bit storage: every stored value within ONE unit in the last place of the
                   oracle's rounded value and at least 99.9 % of them bit-identical (the GPU
                   evaluates softmax in fp32, the oracle in fp64; the two can land on different
                   sides of a rounding boundary).  fp32 storage: relative error <= 2e-5: the
                   kernel's arithmetic IS fp32, and the exponent (l - m) / T * log2(e), of
                   magnitude up to ~100 for the smallest probabilities, carries a rounding
                   error of 2^-24 of itself, i.e. up to ~1e-5 relative in the result;
  greedy token     bit-exact;
  sampled token    equal, or a counted near-tie: u * Q within 1e-5 * Q of the interval the GPU's
                   token owns in the oracle's cumulative sum;
  confidence       exactly the stored q[token] of the GPU's own row.
"""
import os
import sys

import numpy as np
import pytest

import workloads as W
from tests.harness import _torch_from

pytestmark = pytest.mark.gpu
NEAR = 1e-5


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


def _as_f64(t, dt):
    a = t.cpu()
    if dt == "bf16":
        return W.bf16_bits_to_f32(a.view(__import__("torch").int16).numpy().view(np.uint16)).astype(np.float64)
    return a.numpy().astype(np.float64)


def _check(logits, ldt, pdt, T, u, oracle, pkg, out_rows=None, n_prob_rows=None, path="auto"):
    import torch
    dev = "cuda:0"
    R, V = logits.shape
    q_ref, tok_ref, conf_ref, info = oracle.draft_sample(logits, T, u, logits_dtype=ldt, probs_dtype=pdt)
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[pdt]
    probs = None
    rows_d = None
    if out_rows is not None:
        probs = torch.zeros((n_prob_rows, V), dtype=tdt, device=dev)
        rows_d = torch.from_numpy(out_rows).to(dev)
    _say(f"draft_sample R={R} V={V} logits={ldt} probs={pdt} path={path}")
    q_d, tok_d, conf_d = pkg.draft_sample(_torch_from(logits, ldt, dev), torch.from_numpy(T).to(dev),
                                          torch.from_numpy(u).to(dev), probs_dtype=tdt, draft_probs=probs,
                                          out_rows=rows_d, path=path)
    torch.cuda.synchronize()
    q = _as_f64(q_d, pdt)
    if out_rows is not None:
        untouched = np.setdiff1d(np.arange(n_prob_rows), out_rows)
        assert np.all(q[untouched] == 0)
        q = q[out_rows]
    tok, conf = tok_d.cpu().numpy(), conf_d.cpu().numpy().astype(np.float64)
    ulp_rel = {"f32": 2e-5, "bf16": 2.0 ** -7, "f16": 2.0 ** -10}[pdt]
    tiny = {"f32": 1e-44, "bf16": 1e-40, "f16": 6e-8}[pdt]            # subnormal quantum
    assert np.all(np.abs(q - q_ref) <= ulp_rel * np.maximum(q, q_ref) + tiny), "a stored probability is off by more than one ulp"
    frac = float(np.mean(q == q_ref))
    # 16-bit rows: at most one entry in a thousand may sit on the other side of a rounding boundary (the kernel
    # evaluates the softmax in fp32, the oracle in fp64); tiny cases are allowed two such entries
    if pdt != "f32":
        assert int(np.sum(q != q_ref)) <= max(2, 0.001 * q.size), (int(np.sum(q != q_ref)), q.size)
    near = 0
    for r in range(R):
        assert 0 <= tok[r] < V and conf[r] == q[r, tok[r]] and (T[r] == 0 or conf[r] > 0)
        if tok[r] == tok_ref[r]:
            continue
        assert T[r] != 0.0, f"greedy row {r}: {tok[r]} != {tok_ref[r]}"
        cs = np.cumsum(q_ref[r])
        Q = cs[-1]
        lo, hi = (cs[tok[r] - 1] if tok[r] else 0.0), cs[tok[r]]
        tau = float(u[r]) * Q
        assert lo - NEAR * Q <= tau < hi + NEAR * Q, f"row {r}: token {tok[r]} vs {tok_ref[r]} is not a near-tie"
        near += 1
    _say(f"draft_sample ok: bit-equal fraction {frac:.6f}, near-ties {near}/{R}")
    assert near <= max(2, 0.025 * R)          # measured: none on these shapes
    return frac, near


@pytest.mark.parametrize("cfg", [1, 2, 3])
def test_draft_sample_on_config_logits(cfg, oracle_mod, pkg):
    st = W.make_verify_step(cfg, attention=False)
    R = min(st.total_q, 96)
    logits = np.ascontiguousarray(st.target_logits[:R])
    rng = np.random.default_rng(40 + cfg)
    T = rng.choice(np.array([0.0, 0.7, 1.0, 1.2], np.float32), R).astype(np.float32)
    u = rng.random(R).astype(np.float32)
    if st.logits_dtype == "f32":
        _check(logits, st.logits_dtype, st.probs_dtype, T, u, oracle_mod, pkg)
    else:
        _check(logits, st.logits_dtype, st.probs_dtype, T, u, oracle_mod, pkg, path="fast")
        _check(logits, st.logits_dtype, st.probs_dtype, T, u, oracle_mod, pkg, path="split")
        _check(logits, st.logits_dtype, st.probs_dtype, T, u, oracle_mod, pkg, path="vector")


def test_draft_sample_dtype_mixes_strides_and_row_map(oracle_mod, pkg):
    rng = np.random.default_rng(77)
    R, V = 9, 40000                                                   # five steps of 8192, ragged tail
    base = (2.5 * rng.standard_normal((R, V))).astype(np.float32)
    T = np.array([1.0, 0.0, 0.5, 1.0, 2.0, 0.0, 0.9, 1.0, 1.1], np.float32)
    u = rng.random(R).astype(np.float32)
    u[0], u[3] = 0.0, np.float32(1.0 - 2.0 ** -24)                    # the ends of the range
    for ldt, pdt in [("f32", "f32"), ("f32", "bf16"), ("bf16", "f16"), ("f16", "bf16")]:
        lg = base if ldt == "f32" else (W.f32_to_bf16_bits(base) if ldt == "bf16" else base.astype(np.float16))
        for path in (["vector"] if ldt == "f32" else ["fast", "split", "vector"]):
            _check(lg, ldt, pdt, T, u, oracle_mod, pkg, path=path)
    _check(W.f32_to_bf16_bits(base), "bf16", "f32", T, u, oracle_mod, pkg, path="fast")
    _check(W.f32_to_bf16_bits(base), "bf16", "f32", T, u, oracle_mod, pkg, path="split")
    # scattered destination rows (the ragged layout the acceptance call reads)
    out_rows = np.array([3, 0, 11, 4, 5, 9, 1, 12, 7], np.int32)
    for path in ("fast", "split", "vector"):
        _check(W.f32_to_bf16_bits(base), "bf16", "bf16", T, u, oracle_mod, pkg, out_rows=out_rows, n_prob_rows=13, path=path)
    # a row with no positive logit takes the exact-maximum branch of the register-resident kernel
    neg = W.f32_to_bf16_bits(-np.abs(base[:3]) - 0.5)
    _check(neg, "bf16", "bf16", T[:3], u[:3], oracle_mod, pkg, path="fast")
    _check(neg, "bf16", "bf16", T[:3], u[:3], oracle_mod, pkg, path="split")


def test_draft_sample_small_vocab_and_planted_ties(oracle_mod, pkg):
    rng = np.random.default_rng(5)
    R, V = 6, 8
    lg = rng.standard_normal((R, V)).astype(np.float32)
    lg[1, [2, 6]] = 5.0                                               # tie for the maximum
    lg[4, :] = 0.25                                                   # all equal
    T = np.array([1.0, 0.0, 0.3, 1.0, 0.0, 1.0], np.float32)
    u = rng.random(R).astype(np.float32)
    _check(lg, "f32", "f32", T, u, oracle_mod, pkg)
    # one chunk only: three of the four parts of the split form are empty
    _check(W.f32_to_bf16_bits(lg), "bf16", "bf16", T, u, oracle_mod, pkg, path="split")
    _check(lg.astype(np.float16), "f16", "f16", T, u, oracle_mod, pkg, path="split")


def test_draft_then_accept_roundtrip(oracle_mod, pkg):
    """The rows written by the draft step feed the acceptance step directly: drafting from the TARGET's
    own logits at the target's temperature makes q == p up to rounding, so every draft must be accepted
    for any uniform that is not within rounding of 1."""
    import torch
    dev = "cuda:0"
    rng = np.random.default_rng(31)
    B, V = 12, 32000
    spec = rng.integers(1, 4, B).astype(np.int32)
    TQ, TD = int((spec + 1).sum()), int(spec.sum())
    logits = W.f32_to_bf16_bits((3 * rng.standard_normal((TQ, V))).astype(np.float32))
    cu = np.concatenate([[0], np.cumsum(spec + 1)]).astype(np.int64)
    draft_rows = np.concatenate([np.arange(cu[i], cu[i] + spec[i]) for i in range(B)])   # logits rows judged by drafts
    temp_req = np.full(B, 0.8, np.float32)
    lg_d = _torch_from(logits, "bf16", dev)
    q_d, tok_d, conf_d = pkg.draft_sample(lg_d[torch.from_numpy(draft_rows).to(dev)].contiguous(),
                                          torch.full((TD,), 0.8, device=dev), torch.from_numpy(rng.random(TD).astype(np.float32)).to(dev),
                                          probs_dtype=torch.float32)
    uni = rng.random((TQ, 2)).astype(np.float32) * 0.98
    toks, alen = pkg.accept(lg_d, q_d, tok_d, torch.from_numpy(uni).to(dev), torch.from_numpy(spec).to(dev),
                            torch.from_numpy(temp_req).to(dev), max_spec_len=3)
    torch.cuda.synchronize()
    assert np.array_equal(alen.cpu().numpy(), spec)
    assert torch.all(conf_d > 0)


@pytest.mark.parametrize("path", ["fast", "split", "vector"])
def test_draft_sample_with_masked_logits(path, oracle_mod, pkg):
    """A share of every draft-logits row is -inf (masked tokens), whole aligned stretches included: their
    stored probability is exactly 0 and they are never drawn."""
    st = W.make_custom_step(650, ctx_lens=[1] * 40, spec_lens=[0] * 40, vocab=40000, logits_dtype="bf16",
                            attention=False, masked_frac=0.3)
    logits = np.ascontiguousarray(st.target_logits)
    logits[:, 8192:24576] = np.uint16(0xFF80)
    rng = np.random.default_rng(9)
    T = rng.choice(np.array([0.0, 0.7, 1.0], np.float32), 40).astype(np.float32)
    u = rng.random(40).astype(np.float32)
    _check(logits, "bf16", "bf16", T, u, oracle_mod, pkg, path=path)
