"""MI355X-native hot path of retrieval-based Draft-then-Verify decoding (LASER, arxiv 2408.05676).

Thin ctypes binding over liblaser.so: argument marshalling only.  Every step of the path
(pool index lookup, verify forward, fused output head + acceptance, KV commit) runs in the
library's HIP kernels; PyTorch supplies device memory and the stream.
"""
from .binding import (  # noqa: F401
    LaserError, lib, lib_path, Pool, Model, KVCache,
    retrieve_drafts, retrieve_drafts_temp, own_text_append, verify_step, verify_head, verify_head_static, kv_commit, retrieve_tree, verify_tree, kv_commit_tree, generate, ctx_advance, probe_hbm, probe_mfma_f16, probe_launch, probe_exchange,
    MODE_RV, MODE_RV_OR_TOP1, MODE_TOPK_ONLY, MODE_TOPP_ONLY,
)
