"""Host workload -> device tensors (plumbing only: no arithmetic of the method).

Used by the tests, by __graft_entry__.smoke() and by bench.py; torch is imported lazily so that the
generators stay usable without it."""
from __future__ import annotations

from types import SimpleNamespace

import numpy as np


def _torch_from(arr: np.ndarray, dtype: str, device):
    import torch
    if dtype == "bf16":
        return torch.from_numpy(arr.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(arr).to(device)


def to_device(st, device="cuda:0", attention=True, acceptance=True):
    import torch
    d = SimpleNamespace()
    d.spec_lens = torch.from_numpy(st.spec_lens).to(device)
    if getattr(st, "parents", None) is not None:
        d.parents = torch.from_numpy(st.parents).to(device)
    if attention and st.q is not None:
        d.ctx_lens = torch.from_numpy(st.ctx_lens).to(device)
        d.block_table = torch.from_numpy(st.block_table).to(device)
        d.q = _torch_from(st.q, st.dtype, device)
        d.k_pages = _torch_from(st.k_pages, st.dtype, device)
        d.v_pages = _torch_from(st.v_pages, st.dtype, device)
    if acceptance and st.target_logits is not None:
        d.target_logits = _torch_from(st.target_logits, st.logits_dtype, device)
        d.draft_probs = _torch_from(st.draft_probs, st.probs_dtype, device)
        d.draft_tokens = torch.from_numpy(st.draft_tokens).to(device)
        d.uniforms = torch.from_numpy(st.uniforms).to(device)
        d.temperature = torch.from_numpy(st.temperature).to(device)
    return d
