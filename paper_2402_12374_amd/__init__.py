"""Sequoia tree-verify hot path for AMD MI355X: tree-masked GQA attention and the
sampling-without-replacement verification walk, as HIP kernels behind a C ABI."""
from .binding import (SEQ_ERR_ALGORITHM, SEQ_ERR_ALIGN, SEQ_ERR_DTYPE, SEQ_ERR_FULL, SEQ_ERR_CAPTURE, SEQ_MAX_PLANS, SEQ_MAX_STREAMS, SEQ_ERR_HIP, SEQ_ERR_NULL, SEQ_ERR_SHAPE,  # noqa: F401
                      SEQ_ERR_TEMPERATURE, SEQ_ERR_TREE, SEQ_ERR_WORKSPACE, SEQ_MAX_CHILDREN,
                      SEQ_VERIFY_SEQUOIA, SEQ_VERIFY_SPECINFER, SEQ_VERIFY_TOPK,
                      SeqTreeError, lib, read_verify_trace, seq_build_tree, seq_draft_sample,
                      seq_draft_sample_workspace, seq_kv_append, seq_pick_tree_shape, seq_top_p_filter, seq_tree_attn, seq_tree_attn_batched, seq_tree_attn_noalloc,
                      seq_tree_attn_workspace, seq_tree_expected_tokens,
                      seq_tree_plan_host, seq_verify, seq_verify_batched, seq_verify_with,
                      seq_verify_workspace, shutdown, strerror,
                      version)
