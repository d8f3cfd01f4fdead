"""seq_tree_attn_noalloc -- the entry point for callers that cannot allocate device memory --
against seq_tree_attn through the C ABI: the same kernels on the same schedule must leave the
same bits, and both must agree with the CPU checker within the attention tolerance.  Calls come in
a row on one GPU, later ones smaller than earlier ones, so that whatever an earlier call left in
the static device array (bitset rows, arrival counters, partial results) is there to trip over."""
import numpy as np
import pytest
import torch

import paper_2402_12374_amd as S
import workloads as W

from gpu_util import TOL, oracle_attn, run_attn, to_dev

pytestmark = pytest.mark.gpu


def run_noalloc(a: W.AttnInputs) -> np.ndarray:
    tensors = [to_dev(x, a.dtype) for x in (a.q, a.k_cache, a.v_cache, a.k_tree, a.v_tree)]
    out = torch.full_like(tensors[0], float("nan"))
    S.seq_tree_attn_noalloc(*tensors, a.parent, a.prefix_len, out)
    torch.cuda.synchronize()
    return out.float().cpu().numpy().astype(np.float64)


def test_two_calls_in_a_row_the_second_smaller():
    big = W.attn_inputs_for("C2")      # 32 units x several key ranges: counters and partial results in use
    small = W.make_attn_inputs(8, 2, 128, 300, W.geometric_tree(24, 5), W.BF16, seed=5, prefix_cap=310)
    assert S.seq_tree_attn_workspace(big.prefix_len, 64, 32, 32, 128, S.binding.SEQ_BF16) > 256
    got_big = run_noalloc(big)
    got_small = run_noalloc(small)
    for a, got in ((big, got_big), (small, got_small)):
        assert np.isfinite(got).all()
        assert np.array_equal(got, run_attn(a))
        assert np.abs(got - oracle_attn(a)).max() <= TOL[a.dtype]


def test_a_run_of_shapes_trees_and_dtypes():
    rng = np.random.default_rng(12)
    cases = [
        W.make_attn_inputs(16, 2, 128, 1500, W.random_topological_tree(300, rng), W.BF16, seed=1),   # ten bitset words per row
        W.attn_inputs_for("C1"),                                                                     # fp32 path
        W.make_attn_inputs(4, 4, 64, 777, W.chain_tree(1024), W.BF16, seed=2, prefix_cap=800),       # the largest and deepest tree
        W.make_attn_inputs(3, 3, 128, 300, W.chain_tree(1), W.BF16, seed=3),                         # one node
        W.make_attn_inputs(2, 2, 128, 0, W.star_tree(5), W.BF16, seed=4),                            # no prefix
        W.make_attn_inputs(8, 1, 64, 77, W.random_topological_tree(130, rng), W.F32, seed=5),
        W.attn_inputs_for("C3"),
        W.make_attn_inputs(4, 2, 128, 200, W.geometric_tree(37, 9), W.BF16, seed=6, prefix_cap=205),
    ]
    got = [run_noalloc(a) for a in cases]            # all of them first, one after the other
    for a, g in zip(cases, got):
        assert np.array_equal(g, run_attn(a)), (a.q.shape, a.prefix_len)
        assert np.abs(g - oracle_attn(a)).max() <= TOL[a.dtype]


def test_what_exceeds_the_static_array_is_refused_and_the_ordinary_call_goes_on_working():
    a = W.make_attn_inputs(4, 2, 128, 100, W.geometric_tree(20, 4), W.BF16, seed=9)
    tensors = [to_dev(x, a.dtype) for x in (a.q, a.k_cache, a.v_cache, a.k_tree, a.v_tree)]
    out = torch.empty_like(tensors[0])
    # 8 KV heads x 7168 query rows over a prefix of 131072 keys: 119 MiB of partial results
    assert S.seq_tree_attn_workspace(131072, 1024, 56, 8, 128, S.binding.SEQ_BF16) > S.binding.SEQ_NOALLOC_MAX_PARTIAL_BYTES
    parent = np.ascontiguousarray(W.geometric_tree(1024, 12), np.int32)
    rc = S.lib().seq_tree_attn_noalloc(tensors[0].data_ptr(), tensors[1].data_ptr(), tensors[2].data_ptr(),
                                       tensors[3].data_ptr(), tensors[4].data_ptr(), parent.ctypes.data, 131072, 1024,
                                       56, 8, 128, out.data_ptr(), 131072, S.binding.SEQ_BF16, None)
    assert rc == S.binding.SEQ_ERR_WORKSPACE     # refused on the host: nothing was launched on these small buffers
    assert np.array_equal(run_noalloc(a), run_attn(a))


def test_the_largest_configuration_fits_the_static_array():
    a = W.attn_inputs_for("C5")      # 192 units x 2 key ranges of two sizes: 25.5 MiB of partial results
    need = S.seq_tree_attn_workspace(a.prefix_len, 768, 64, 8, 128, S.binding.SEQ_BF16)
    assert 16 << 20 < need <= S.binding.SEQ_NOALLOC_MAX_PARTIAL_BYTES
    small = W.make_attn_inputs(8, 2, 128, 300, W.geometric_tree(24, 5), W.BF16, seed=15, prefix_cap=310)
    got, got_small = run_noalloc(a), run_noalloc(small)
    assert np.array_equal(got, run_attn(a))
    assert np.array_equal(got_small, run_attn(small))
    assert np.abs(got_small - oracle_attn(small)).max() <= TOL[small.dtype]
