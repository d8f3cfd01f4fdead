"""Sequoia tree-verify hot path for AMD MI355X: tree-masked GQA attention and the
sampling-without-replacement verification walk, as HIP kernels behind a C ABI."""
from .binding import (SeqTreeError, lib, read_verify_trace, seq_tree_attn,  # noqa: F401
                      seq_tree_attn_workspace, seq_tree_plan_host, seq_verify,
                      seq_verify_workspace, shutdown, strerror, version)
