"""CPU oracle of the two steps around a verification step: writing the new
tokens' K/V rows into the paged cache, and committing the accepted tokens
(paper Sec. 6: paged KV cache; the results of one speculative step are the
input of the next).

TEST INFRASTRUCTURE ONLY (see the package docstring).  Plain loops over numpy
arrays; byte and integer work, so every result is exact.
"""
from __future__ import annotations

import numpy as np


def kv_append(k_new, v_new, k_pages, v_pages, block_table, ctx_lens, spec_lens):
    """Returns copies of (k_pages, v_pages) with the new rows written.

    k_new, v_new: [TQ][Hkv][d], request-major rows (row j of request i is at
    sum_{r<i} (k_r + 1) + j).  Row j of request i is token position
    ctx_lens[i] - (k_i + 1) + j of that request: page block_table[i][pos // P],
    slot pos % P, every kv head.
    """
    assert k_new.dtype == k_pages.dtype and v_new.dtype == v_pages.dtype      # a copy, never a conversion
    kp, vp = k_pages.copy(), v_pages.copy()
    P = kp.shape[2]
    row = 0
    for i in range(len(spec_lens)):
        n = int(spec_lens[i]) + 1
        L = int(ctx_lens[i])
        assert L >= n
        for j in range(n):
            pos = L - n + j
            page = int(block_table[i, pos // P])
            assert 0 <= page < kp.shape[0]
            kp[page, :, pos % P, :] = k_new[row]
            vp[page, :, pos % P, :] = v_new[row]
            row += 1
    assert row == k_new.shape[0]
    return kp, vp


def commit(out_tokens, out_accept_len, spec_lens, ctx_lens, next_spec_lens=None,
           seq_tokens=None, seq_lens=None):
    """Returns a dict: committed_lens, next_ctx_lens (or None), last_token, seq_tokens, seq_lens.

    The cache keeps the last committed token and the a_i accepted drafts:
    committed = L_i - k_i + a_i.  The token emitted last (recovered or bonus)
    is the next step's first query row; it has no cache entry yet.
    """
    B = len(spec_lens)
    committed = np.zeros(B, np.int32)
    last = np.zeros(B, np.int32)
    nxt = None if next_spec_lens is None else np.zeros(B, np.int32)
    st = None if seq_tokens is None else seq_tokens.copy()
    sl = None if seq_lens is None else seq_lens.copy()
    for i in range(B):
        k, a = int(spec_lens[i]), int(out_accept_len[i])
        assert 0 <= a <= k
        committed[i] = int(ctx_lens[i]) - k + a
        last[i] = out_tokens[i, a]
        if nxt is not None:
            nxt[i] = committed[i] + int(next_spec_lens[i]) + 1
        if st is not None:
            cap = st.shape[1]
            for t in range(a + 1):
                if sl[i] < cap:
                    st[i, sl[i]] = out_tokens[i, t]
                    sl[i] += 1
    return dict(committed_lens=committed, next_ctx_lens=nxt, last_token=last, seq_tokens=st, seq_lens=sl)


def kv_compact_path(k_pages, v_pages, block_table, ctx_lens, spec_lens, out_path, out_accept_len):
    """After TREE acceptance: returns copies of (k_pages, v_pages) in which the K/V rows of the
    accepted nodes sit where a chain would have put them.

    The n_i = k_i + 1 nodes of request i were appended at positions base + j, base = L_i - n_i,
    in node order.  The walk accepted the nodes out_path[i][0 .. a_i-1] (a root-to-node path, so
    strictly increasing and out_path[i][j] >= j + 1).  Afterwards position base + 1 + j holds the
    row of node out_path[i][j]; the root stays at base; positions from base + 1 + a_i on are dead
    (whatever they hold is never read again once `commit` has shortened the request)."""
    kp, vp = k_pages.copy(), v_pages.copy()
    P = kp.shape[2]
    for i in range(len(spec_lens)):
        n, a = int(spec_lens[i]) + 1, int(out_accept_len[i])
        base = int(ctx_lens[i]) - n
        prev = 0
        for j in range(a):
            node = int(out_path[i, j])
            assert prev < node < n and node >= j + 1
            prev = node
            src, dst = base + node, base + 1 + j
            ps, pd = int(block_table[i, src // P]), int(block_table[i, dst // P])
            # taken from the ORIGINAL pages: a destination never overwrites a source still needed
            kp[pd, :, dst % P, :] = k_pages[ps, :, src % P, :]
            vp[pd, :, dst % P, :] = v_pages[ps, :, src % P, :]
    return kp, vp
