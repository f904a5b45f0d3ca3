"""MI355X (gfx950) library for one EAGLE-3 speculative-decoding step: feature fusion, draft-tree
expansion, tree-masked verification and acceptance, as hand-written HIP kernels behind a C ABI
(include/eagle3.h).  This package is the thin Python binding; see `build.py` for the in-tree build."""
from .binding import (  # noqa: F401
    EXPORTS, LIB_PATH, Eagle3Context, Eagle3Error, KVCache, eagle3_accept, eagle3_accept_static, eagle3_commit, eagle3_draft_chain, eagle3_draft_expand, eagle3_prefill,
    eagle3_fuse_features, eagle3_tree_verify, eagle3_tree_verify_layers, eagle3_ttt_attention, lib,
)
