"""MI355X-native ragged verification step (attention + acceptance) behind a C ABI.

``binding`` wraps ``libadaspec.so``; ``build`` compiles it.  Nothing here falls
back to a CPU or PyTorch implementation.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    AdaspecError, AttnDims, AcceptDims, CommitDims, accept, accept_noalloc, accept_resolved_path, verify_attn, check_ragged_inputs,
    kv_append, commit, draft_sample, DraftDims, accept_tree, kv_compact_path, check_tree_parents, check_accept_inputs,
    status_string, version, lib, accept_dims, attn_dims,
)
