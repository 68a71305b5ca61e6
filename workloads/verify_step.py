"""Generators for the five synthetic verification-step workloads.

Shapes follow the benchmark configs (batch, heads, head_dim, page size, vocab,
dtypes); the ragged structure follows what the paper reports about its
speculative lengths (Table 2: mean 3-3.6 draft tokens under the adaptive
policy, up to 8 under the threshold baseline; Sec. 7.4: lengths shrink as the
batch grows).  Nothing here computes attention or the acceptance rule: the
softmax below only manufactures a plausible *draft distribution* input.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, Optional, Sequence

import numpy as np

PAGE_SIZE = 16
_CHUNK = 1 << 23  # elements per independently seeded chunk of a big tensor
_THREADS = 8

_ITEMSIZE = {"f32": 4, "f16": 2, "bf16": 2}


# --------------------------------------------------------------------------
# dtype helpers (storage only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest-even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    r = (u + (0x7FFF + ((u >> 16) & 1))) >> 16
    r = np.where(nan, (u >> 16) | 0x0040, r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def _store(x32: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(x32, dtype=np.float32)
    if dtype == "f16":
        return x32.astype(np.float16)
    if dtype == "bf16":
        return f32_to_bf16_bits(x32)
    raise ValueError(dtype)


def to_f64(x: np.ndarray, dtype: str) -> np.ndarray:
    """Exact upcast of a stored tensor to float64."""
    if dtype == "bf16":
        return bf16_bits_to_f32(x).astype(np.float64)
    return x.astype(np.float64)


def _nan_like(dtype: str):
    if dtype == "bf16":
        return np.uint16(0x7FC0)
    return np.nan


def _normal(ss: np.random.SeedSequence, shape, sigma: float, dtype: str,
            add_to: Optional[np.ndarray] = None, add_dtype: str = "f32",
            as_f32: bool = False) -> np.ndarray:
    """sigma * N(0,1) of `shape`, drawn in fixed-size chunks each with its own
    child seed so the result does not depend on the thread count."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32 if (as_f32 or dtype == "f32") else
                   (np.float16 if dtype == "f16" else np.uint16))
    n_chunks = max(1, (n + _CHUNK - 1) // _CHUNK)
    kids = ss.spawn(n_chunks)
    base = None if add_to is None else add_to.reshape(-1)

    def fill(c):
        lo, hi = c * _CHUNK, min(n, (c + 1) * _CHUNK)
        g = np.random.Generator(np.random.PCG64(kids[c]))
        x = g.standard_normal(hi - lo, dtype=np.float32)
        if sigma != 1.0:
            x *= np.float32(sigma)
        if base is not None:
            x += to_f64(base[lo:hi], add_dtype).astype(np.float32)
        out[lo:hi] = x if (as_f32 or dtype == "f32") else _store(x, dtype)

    if n_chunks == 1:
        fill(0)
    else:
        with ThreadPoolExecutor(_THREADS) as ex:
            list(ex.map(fill, range(n_chunks)))
    return out.reshape(shape)


# --------------------------------------------------------------------------
# the workload record
# --------------------------------------------------------------------------
@dataclass
class VerifyStep:
    name: str
    seed: int
    # attention half
    dtype: str = "bf16"
    n_q_heads: int = 0
    n_kv_heads: int = 0
    head_dim: int = 0
    page_size: int = PAGE_SIZE
    num_pages: int = 0
    max_pages_per_req: int = 0
    ctx_lens: np.ndarray = None      # int32 [B]   KV tokens incl. the n_i new ones
    spec_lens: np.ndarray = None     # int32 [B]   k_i
    q: np.ndarray = None             # [TQ][Hq][d]
    k_pages: np.ndarray = None       # [num_pages][Hkv][P][d]
    v_pages: np.ndarray = None
    block_table: np.ndarray = None   # int32 [B][max_pages_per_req], unused = -1
    # acceptance half
    vocab: int = 0
    logits_dtype: str = "bf16"
    probs_dtype: str = "bf16"
    target_logits: np.ndarray = None  # [TQ][V]
    draft_probs: np.ndarray = None    # [TD][V]
    draft_tokens: np.ndarray = None   # int32 [TD]
    uniforms: np.ndarray = None       # float32 [TQ][2]
    temperature: np.ndarray = None    # float32 [B]
    parents: np.ndarray = None        # int32 [TQ], only for draft TREES: parent node inside the request
    notes: Dict[str, object] = field(default_factory=dict)

    @property
    def batch(self) -> int:
        return int(self.spec_lens.shape[0])

    @property
    def total_q(self) -> int:
        return int(self.spec_lens.sum()) + self.batch

    @property
    def total_draft(self) -> int:
        return int(self.spec_lens.sum())

    @property
    def max_spec_len(self) -> int:
        return int(self.spec_lens.max()) if self.batch else 0

    @property
    def cu_q(self) -> np.ndarray:
        c = np.zeros(self.batch + 1, dtype=np.int64)
        np.cumsum(self.spec_lens.astype(np.int64) + 1, out=c[1:])
        return c


# --------------------------------------------------------------------------
# builders
# --------------------------------------------------------------------------
def _build(name: str, seed: int, ctx_lens, spec_lens, temperature, *,
           n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: str,
           vocab: int, logits_dtype: str, logits_sigma: float,
           noise_sigma: float, draft_temp: float,
           streams: Sequence[np.random.SeedSequence],
           attention: bool = True, acceptance: bool = True,
           poison: bool = True, pool_slack: float = 1.25,
           sharp_key: bool = False, planted_ties: bool = False, masked_frac: float = 0.0) -> VerifyStep:
    (s_q, s_k, s_v, s_bt, s_logit, s_noise, s_tok, s_uni) = streams
    ctx_lens = np.asarray(ctx_lens, dtype=np.int32)
    spec_lens = np.asarray(spec_lens, dtype=np.int32)
    temperature = np.asarray(temperature, dtype=np.float32)
    B = int(spec_lens.shape[0])
    assert ctx_lens.shape == (B,) and temperature.shape == (B,)
    n = spec_lens.astype(np.int64) + 1
    assert np.all(ctx_lens >= n), "context must include the query tokens"
    TQ, TD = int(n.sum()), int(spec_lens.sum())
    P = PAGE_SIZE
    st = VerifyStep(name=name, seed=seed, dtype=dtype, n_q_heads=n_q_heads,
                    n_kv_heads=n_kv_heads, head_dim=head_dim, vocab=vocab,
                    logits_dtype=logits_dtype, probs_dtype=logits_dtype,
                    ctx_lens=ctx_lens, spec_lens=spec_lens,
                    temperature=temperature)
    cu_q = st.cu_q

    if attention:
        pages_per = (ctx_lens.astype(np.int64) + P - 1) // P
        needed = int(pages_per.sum())
        num_pages = max(1, int(np.ceil(pool_slack * needed)))
        max_pages = max(1, int(pages_per.max()) if B else 1)
        st.num_pages, st.max_pages_per_req = num_pages, max_pages
        g_bt = np.random.Generator(np.random.PCG64(s_bt))
        perm = g_bt.permutation(num_pages).astype(np.int32)
        bt = np.full((B, max_pages), -1, dtype=np.int32)
        off = 0
        for i in range(B):
            bt[i, :pages_per[i]] = perm[off:off + pages_per[i]]
            off += int(pages_per[i])
        st.block_table = bt
        st.q = _normal(s_q, (TQ, n_q_heads, head_dim), 1.0, dtype)
        shape = (num_pages, n_kv_heads, P, head_dim)
        st.k_pages = _normal(s_k, shape, 1.0, dtype)
        st.v_pages = _normal(s_v, shape, 1.0, dtype)
        if sharp_key:
            # one key per (request, kv head) aligned with a query row: a sharp softmax peak
            G = n_q_heads // n_kv_heads
            g_sk = np.random.Generator(np.random.PCG64(s_bt.spawn(1)[0]))
            for i in range(B):
                hi = max(1, int(ctx_lens[i] - n[i]))
                t = int(g_sk.integers(0, hi))
                page, slot = bt[i, t // P], t % P
                for g in range(n_kv_heads):
                    qrow = to_f64(st.q[cu_q[i], g * G], dtype).astype(np.float32)
                    st.k_pages[page, g, slot] = _store(4.0 * qrow, dtype)
        if poison:
            bad = _nan_like(dtype)
            used = np.zeros(num_pages, dtype=bool)
            used[perm[:needed]] = True
            st.k_pages[~used] = bad
            st.v_pages[~used] = bad
            for i in range(B):
                tail = int(ctx_lens[i]) % P
                if tail:
                    page = bt[i, pages_per[i] - 1]
                    st.k_pages[page, :, tail:] = bad
                    st.v_pages[page, :, tail:] = bad

    if acceptance:
        st.target_logits = _normal(s_logit, (TQ, vocab), logits_sigma, logits_dtype)
        if masked_frac > 0.0:
            # logit masking as a serving stack applies it (banned tokens, grammar constraints): a random subset
            # of every row is -inf in the target logits; the draft distribution built below is 0 there
            g_m = np.random.Generator(np.random.PCG64(s_logit.spawn(2)[1]))
            neg_inf = {"f32": np.float32(-np.inf), "f16": np.float16(-np.inf), "bf16": np.uint16(0xFF80)}[logits_dtype]
            for r in range(TQ):
                cols = g_m.random(vocab) < masked_frac
                cols[int(g_m.integers(0, vocab))] = False              # at least one finite entry
                st.target_logits[r][cols] = neg_inf
        if planted_ties:
            g_t = np.random.Generator(np.random.PCG64(s_logit.spawn(1)[0]))
            for r in range(TQ):
                row = st.target_logits[r]
                top = int(np.argmax(to_f64(row, logits_dtype)))
                for v in g_t.integers(0, vocab, size=2):
                    row[int(v)] = row[top]
        # draft rows: the logits rows that judge a draft token (all but the bonus rows)
        keep = np.ones(TQ, dtype=bool)
        keep[cu_q[1:] - 1] = False
        draft_rows = np.nonzero(keep)[0]
        assert draft_rows.shape[0] == TD
        if TD:
            noisy = _normal(s_noise, (TD, vocab), noise_sigma, "f32",
                            add_to=st.target_logits[draft_rows], add_dtype=logits_dtype,
                            as_f32=True)
            noisy /= np.float32(draft_temp)
            noisy -= noisy.max(axis=1, keepdims=True)
            np.exp(noisy, out=noisy)
            noisy /= noisy.sum(axis=1, keepdims=True, dtype=np.float64).astype(np.float32)
            st.draft_probs = _store(noisy, logits_dtype)
            del noisy
        else:
            st.draft_probs = np.zeros((0, vocab), dtype=_store(np.zeros(1, np.float32), logits_dtype).dtype)
        g_tok = np.random.Generator(np.random.PCG64(s_tok))
        u_tok = g_tok.random(TD)
        toks = np.zeros(TD, dtype=np.int32)
        req_of_draft = np.repeat(np.arange(B), spec_lens)
        for d in range(TD):
            qrow = to_f64(st.draft_probs[d], logits_dtype)
            if temperature[req_of_draft[d]] == 0.0:
                toks[d] = int(np.argmax(qrow))           # greedy drafter
            else:
                c = np.cumsum(qrow)
                t = int(np.searchsorted(c, u_tok[d] * c[-1], side="right"))
                t = min(t, vocab - 1)
                while qrow[t] == 0.0 and t > 0:          # never hand out a zero-mass token
                    t -= 1
                toks[d] = t
        st.draft_tokens = toks
        g_u = np.random.Generator(np.random.PCG64(s_uni))
        st.uniforms = g_u.random((TQ, 2), dtype=np.float32)
    return st


CONFIGS = {
    1: dict(name="cfg1-tiny", n_q_heads=8, n_kv_heads=8, head_dim=64, dtype="f32",
            vocab=1024, logits_dtype="f32", logits_sigma=2.0, noise_sigma=1.0, draft_temp=1.0),
    2: dict(name="cfg2-llama2-7b-mha", n_q_heads=32, n_kv_heads=32, head_dim=128, dtype="f16",
            vocab=32000, logits_dtype="bf16", logits_sigma=3.0, noise_sigma=1.5, draft_temp=1.2),
    3: dict(name="cfg3-llama3-8b-gqa", n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16",
            vocab=128256, logits_dtype="bf16", logits_sigma=3.0, noise_sigma=1.5, draft_temp=1.2),
    4: dict(name="cfg4-70b-gqa", n_q_heads=64, n_kv_heads=8, head_dim=128, dtype="bf16",
            vocab=128256, logits_dtype="bf16", logits_sigma=3.0, noise_sigma=1.5, draft_temp=1.2),
    5: dict(name="cfg5-shrink", n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16",
            vocab=128256, logits_dtype="bf16", logits_sigma=3.0, noise_sigma=1.5, draft_temp=1.2),
}

_K_PMF_CFG3 = np.array([.05, .10, .25, .25, .20, .10, .05])


def _ragged(cfg: int, greedy: bool, s_ctx, s_spec, s_temp, batch: Optional[int]):
    g_c = np.random.Generator(np.random.PCG64(s_ctx))
    g_s = np.random.Generator(np.random.PCG64(s_spec))
    g_t = np.random.Generator(np.random.PCG64(s_temp))
    if cfg == 1:
        B = 4
        ctx = np.array([128, 256, 384, 512]); k = np.array([1, 2, 3, 4]); T = np.full(B, 1.0)
    elif cfg == 2:
        B = batch or 32
        ctx = g_c.integers(256, 2049, size=B); k = g_s.integers(0, 9, size=B); T = np.full(B, 1.0)
    elif cfg == 3:
        B = batch or 128
        ctx = np.clip(np.rint(np.exp(np.log(1024.0) + 0.7 * g_c.standard_normal(B))), 128, 4096)
        k = g_s.choice(7, size=B, p=_K_PMF_CFG3); T = np.full(B, 0.8)
    elif cfg == 4:
        B = batch or 64
        ctx = g_c.integers(2048, 8193, size=B); k = g_s.integers(0, 6, size=B)
        T = np.full(B, 0.0 if greedy else 1.0)
    elif cfg == 5:
        B = batch or 256
        ctx = g_c.integers(1024, 2049, size=B); k = g_s.integers(0, 2, size=B)
        T = g_t.choice(np.array([0.0, 0.7, 1.0]), size=B)
    else:
        raise ValueError(f"unknown config {cfg}")
    return ctx.astype(np.int32), k.astype(np.int32), T.astype(np.float32)


def make_verify_step(cfg: int, *, greedy: bool = False, batch: Optional[int] = None,
                     seed: Optional[int] = None, attention: bool = True,
                     acceptance: bool = True, poison: bool = True,
                     sharp_key: bool = False, planted_ties: bool = False, masked_frac: float = 0.0) -> VerifyStep:
    """One seeded draw of benchmark config `cfg` (1..5).  `greedy` selects the
    temperature-0 variant of config 4; `batch` shrinks the batch for quick tests."""
    seed = 5096000 + cfg if seed is None else seed
    ss = np.random.SeedSequence(seed).spawn(11)
    ctx, k, T = _ragged(cfg, greedy, ss[0], ss[1], ss[2], batch)
    spec = {kk: v for kk, v in CONFIGS[cfg].items() if kk != "name"}
    name = CONFIGS[cfg]["name"] + ("-greedy" if greedy else "")
    return _build(name, seed, ctx, k, T, streams=ss[3:], attention=attention,
                  acceptance=acceptance, poison=poison, sharp_key=sharp_key,
                  planted_ties=planted_ties, masked_frac=masked_frac, **spec)


def policy_inputs(cfg: int = 3, *, batch: Optional[int] = None, max_steps: int = 8,
                  seed: Optional[int] = None) -> Dict[str, object]:
    """Synthetic inputs of the speculative-length policy for one step of config `cfg` (random draws only;
    the policy itself is not evaluated here): the committed context lengths C_i (the config's context
    distribution, read as the cache BEFORE the step), the temperatures, and a table of draft-model
    confidences conf[s][i] for up to max_steps draft steps.  Every request has its own draft quality
    a_i ~ U(0.35, 0.97); its confidences are Beta(8 a_i, 8 (1 - a_i)) draws, so acceptance rates fall off
    at different speeds across the batch, which is what makes per-request lengths differ."""
    seed = 5096100 + cfg if seed is None else seed
    ss = np.random.SeedSequence(seed).spawn(5)
    ctx, _, T = _ragged(cfg, False, ss[0], ss[1], ss[2], batch)
    B = len(ctx)
    g = np.random.Generator(np.random.PCG64(ss[3]))
    quality = g.uniform(0.35, 0.97, B)
    conf = np.clip(g.beta(8.0 * quality, 8.0 * (1.0 - quality), size=(max_steps, B)), 1e-3, 1.0)
    return {"ctx_committed": ctx.astype(np.int32), "temperature": T, "conf": conf.astype(np.float64),
            "prev_conf": float(quality.mean()), "seed": seed, "cfg": cfg}


def make_policy_step(pin: Dict[str, object], spec_lens, **kw) -> VerifyStep:
    """The verification step of a batch whose per-request draft lengths `spec_lens` came out of the policy
    for the inputs `pin` (policy_inputs): the config's tensors, ctx_lens = C_i + k_i + 1."""
    cfg = int(pin["cfg"])
    k = np.asarray(spec_lens, dtype=np.int32)
    ctx = (np.asarray(pin["ctx_committed"]) + k + 1).astype(np.int32)
    ss = np.random.SeedSequence(int(pin["seed"]) + 7).spawn(11)
    spec = {kk: v for kk, v in CONFIGS[cfg].items() if kk != "name"}
    return _build(CONFIGS[cfg]["name"] + "-policy", int(pin["seed"]), ctx, k, np.asarray(pin["temperature"], np.float32),
                  streams=ss[3:], **spec, **kw)


def make_custom_step(seed: int, ctx_lens, spec_lens, *, n_q_heads=8, n_kv_heads=8, head_dim=64,
                     dtype="f32", vocab=1024, logits_dtype="f32", temperature=1.0,
                     logits_sigma=2.0, noise_sigma=1.0, draft_temp=1.0, name="custom",
                     **kw) -> VerifyStep:
    """Arbitrary small shapes for edge-case tests."""
    ss = np.random.SeedSequence(seed).spawn(11)
    B = len(spec_lens)
    T = np.broadcast_to(np.asarray(temperature, dtype=np.float32), (B,)).copy()
    return _build(name, seed, ctx_lens, spec_lens, T, streams=ss[3:], n_q_heads=n_q_heads,
                  n_kv_heads=n_kv_heads, head_dim=head_dim, dtype=dtype, vocab=vocab,
                  logits_dtype=logits_dtype, logits_sigma=logits_sigma,
                  noise_sigma=noise_sigma, draft_temp=draft_temp, **kw)


def attach_tree(st: VerifyStep, max_width: int = 3, seed: Optional[int] = None,
                chain: bool = False) -> VerifyStep:
    """Turn the drafts of every request into a token TREE (in place; returns `st`).

    Node 0 of a request is its root (the last committed token), nodes 1..k_i its drafts; a
    node's parent is drawn among the earlier nodes that still have fewer than `max_width`
    children (half of the time the most recent one, so that the trees have depth), which keeps
    every parent before its children.  `chain=True` gives parent = previous node.  The draft
    tokens are drawn again so that they fit the tree: node c's token comes from the draft
    distribution AT its parent (draft_probs row of the parent node); siblings are independent
    draws, and for a greedy (temperature 0) request the m-th child is the m-th most probable
    token.  Nothing else of the step changes."""
    seed = st.seed + 77 if seed is None else seed
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence(seed)))
    cu = st.cu_q
    parents = np.full(st.total_q, -1, dtype=np.int32)
    toks = None if st.draft_tokens is None else st.draft_tokens.copy()
    for i in range(st.batch):
        k = int(st.spec_lens[i])
        par = np.full(k + 1, -1, dtype=np.int32)
        n_child = np.zeros(k + 1, dtype=np.int64)
        for c in range(1, k + 1):
            if chain:
                par[c] = c - 1
            else:
                free = np.nonzero(n_child[:c] < max_width)[0]
                par[c] = free[-1] if g.random() < 0.5 else free[int(g.integers(0, free.shape[0]))]
            rank = int(n_child[par[c]])
            n_child[par[c]] += 1
            if toks is None:
                continue
            qrow = to_f64(st.draft_probs[cu[i] - i + par[c]], st.probs_dtype)
            if st.temperature[i] == 0.0:
                t = int(np.argsort(-qrow, kind="stable")[rank])
            else:
                cdf = np.cumsum(qrow)
                t = min(int(np.searchsorted(cdf, g.random() * cdf[-1], side="right")), st.vocab - 1)
                while qrow[t] == 0.0 and t > 0:
                    t -= 1
            toks[cu[i] - i + c - 1] = t
        parents[cu[i]:cu[i] + k + 1] = par
    st.parents = parents
    if toks is not None:
        st.draft_tokens = toks
    st.notes["tree_max_width"] = 1 if chain else max_width
    return st


def algorithmic_bytes(st: VerifyStep) -> Dict[str, int]:
    """Bytes the method has to move once (one HBM pass), split by stream.

    attention: every K and V element of a request once (not once per query
    row or q head), Q in and the output once, the used block-table entries.
    acceptance: a sampled draft row reads its logits row and its draft-prob
    row; a bonus row or a greedy row reads only the logits row."""
    out: Dict[str, int] = {}
    n = st.spec_lens.astype(np.int64) + 1
    if st.q is not None:
        isz = _ITEMSIZE[st.dtype]
        out["kv"] = int(st.ctx_lens.astype(np.int64).sum()) * 2 * st.n_kv_heads * st.head_dim * isz
        out["q_out"] = int(n.sum()) * st.n_q_heads * st.head_dim * isz * 2
        out["block_table"] = int(((st.ctx_lens.astype(np.int64) + st.page_size - 1) // st.page_size).sum()) * 4
        out["attn"] = out["kv"] + out["q_out"] + out["block_table"]
    if st.target_logits is not None:
        lsz, psz = _ITEMSIZE[st.logits_dtype], _ITEMSIZE[st.probs_dtype]
        out["logits"] = int(n.sum()) * st.vocab * lsz
        sampled = st.spec_lens.astype(np.int64)[st.temperature != 0.0].sum()
        out["probs"] = int(sampled) * st.vocab * psz
        out["accept"] = out["logits"] + out["probs"]
    out["total"] = out.get("attn", 0) + out.get("accept", 0)
    return out


def tree_internal_nodes(st: VerifyStep) -> np.ndarray:
    """bool [TQ]: the node of this row has at least one child (needs st.parents)."""
    cu = st.cu_q
    has = np.zeros(st.total_q, dtype=bool)
    for i in range(st.batch):
        par = st.parents[cu[i] + 1:cu[i + 1]]
        has[cu[i] + par] = True
    return has


def algorithmic_bytes_tree(st: VerifyStep) -> Dict[str, int]:
    """As algorithmic_bytes, for a draft tree evaluated node by node: the attention moves the same
    bytes (every node is a query row, its K/V row a cached token); the acceptance reads the logits
    row of every node once, and the draft-probability row of every sampled (temperature > 0) node
    that has children once."""
    out = algorithmic_bytes(st)
    if st.target_logits is not None:
        psz = _ITEMSIZE[st.probs_dtype]
        sampled_row = np.repeat(st.temperature != 0.0, st.spec_lens.astype(np.int64) + 1)
        out["probs"] = int((tree_internal_nodes(st) & sampled_row).sum()) * st.vocab * psz
        out["accept"] = out["logits"] + out["probs"]
        out["total"] = out.get("attn", 0) + out["accept"]
    return out


def tree_accept_bytes_walk_form(st: VerifyStep, path, accept_len) -> Dict[str, int]:
    """Bytes of a tree acceptance that walks while it works: the logits row of every node once (its
    maximum, arg-max and normaliser); then, only at the nodes the walk reaches and only if at least
    one child is rejected there, the logits row and the draft-probability row once more (all residual
    stages of a node are functions of these two rows).  Greedy requests stop at the first part.
    `path[i]`, `accept_len[i]`: the acceptance's own outputs (node indices of the accepted nodes)."""
    lsz, psz = _ITEMSIZE[st.logits_dtype], _ITEMSIZE[st.probs_dtype]
    cu = st.cu_q
    path = np.asarray(path)
    a = np.asarray(accept_len).astype(np.int64)
    rejecting = 0
    for i in range(st.batch):
        if st.temperature[i] == 0.0:
            continue
        par = st.parents[cu[i]:cu[i + 1]]
        walk = [0] + [int(x) for x in path[i, :a[i]]]
        for d, u in enumerate(walk):
            kids = np.nonzero(par[1:] == u)[0] + 1
            nxt = walk[d + 1] if d + 1 < len(walk) else None
            if (nxt is None and kids.size) or (nxt is not None and (kids < nxt).any()):
                rejecting += 1
    stats = st.total_q * st.vocab * lsz
    resid = rejecting * st.vocab * (lsz + psz)
    return {"stats_logits": stats, "walk_rows": resid, "rejecting_nodes_on_walks": rejecting,
            "accept": stats + resid}


def accept_bytes_skipping_form(st: VerifyStep, accept_len) -> Dict[str, int]:
    """Bytes of an acceptance that applies the sequential rule while it works (rows behind a
    request's first rejection are not read, and only the row that decides the request's token is
    sampled from): every draft row's logits row once for the accept test; then per request the
    deciding row once more -- with its draft-probability row if it is a rejected sampled draft,
    not at all if it is a rejected greedy draft (the arg-max of the test is the token).
    `accept_len[i]` = accepted drafts of request i (the acceptance's own output)."""
    lsz, psz = _ITEMSIZE[st.logits_dtype], _ITEMSIZE[st.probs_dtype]
    k = st.spec_lens.astype(np.int64)
    a = np.asarray(accept_len).astype(np.int64)
    sampled = st.temperature != 0.0
    rejected = a < k
    test = int(k.sum()) * st.vocab * lsz
    decide_logits = int((sampled | ~rejected).sum()) * st.vocab * lsz
    decide_probs = int((sampled & rejected).sum()) * st.vocab * psz
    return {"test_logits": test, "decide_logits": decide_logits, "decide_probs": decide_probs,
            "accept": test + decide_logits + decide_probs}
