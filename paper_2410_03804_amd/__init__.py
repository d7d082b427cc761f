"""MI355X-native hot path of the Mixture-of-Attentions draft step (LSA, CA, tree verification).

The package is a thin ctypes binding over ``libmoa.so`` (hand-written HIP for gfx950, C ABI in
``include/moa.h``).  Importing it loads the library; there is no fallback of any kind -- if the
library is missing the import fails.  Build it with ``python -m paper_2410_03804_amd.build``.
"""
from .binding import (  # noqa: F401
    BF16, F32, DecoderCfg, DEV_BAD_LENGTH, DEV_BAD_MESSAGE, DEV_BAD_PARENT, DEV_CACHE_FULL, DEV_EMPTY_KEYS, MAX_TREE, MoaError, Shape,
    ca_kv_append, cross_attn_draft, debug_force_attn_kernel, debug_force_lsa_kernel, linear, linear_workspace_bytes, lm_head_argmax, lm_head_workspace_bytes, msg_accept_bytes, msg_gunzip, msg_gzip, msg_pack_accept, msg_pack_tree, msg_unpack_accept, msg_unpack_tree, draft_step, draft_step_plan, exported_symbols, fold_projection, last_error, library_path, lsa, lsa_pack_weights, lsa_packed, lsa_packed_weight_bytes, mlp_block, mlp_block_workspace_bytes, profile_collect,
    probe_mfma, probe_read, profile_enable, rmsnorm, self_attn_draft, status_str, SCHED_GROUPED, SCHED_SEQUENTIAL, SCHED_TWO_STREAM,
    tli_decoder_layer, tli_workspace_bytes, topk_logprob, topk_workspace_bytes, tree_accept, tree_build, tree_expand_level, tree_finalize, tree_verify_attn, tree_verify_attn_noalloc, workspace_bytes,
)
