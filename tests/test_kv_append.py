"""seq_kv_append: the checker's definition is pinned through the (already pinned) attention
checker -- a new token decoding over the extended cache must see exactly what a child of the last
accepted node saw in the tree -- and the library is held to the checker bit for bit."""
import numpy as np
import pytest

import oracle
import paper_2402_12374_amd as S
from paper_2402_12374_amd import binding as B
import workloads as W


def test_decoding_over_the_extended_cache_equals_attention_in_the_tree():
    rng = np.random.default_rng(3)
    H, Hk, d, P = 4, 2, 64, 37
    parent = np.array([-1, 0, 0, 1, 1, 3, 3, 5], dtype=np.int32)     # accepted path: 1 -> 3 -> 5
    a = W.make_attn_inputs(H, Hk, d, P, parent, W.F32, seed=11, prefix_cap=P + 8)
    path = np.array([1, 3, 5, -1, -1, -1, -1, -1], dtype=np.int32)
    kc, vc, new_len = oracle.kv_append(a.k_tree, a.v_tree, path, a.k_cache, a.v_cache, P)
    assert new_len == P + 4
    # node 7 is a child of node 5: in the tree it attends to the prefix, 0, 1, 3, 5 and itself
    in_tree = oracle.tree_attn(a.q, a.k_cache, a.v_cache, a.k_tree, a.v_tree, parent, P)[7]
    # the same token decoding alone over the extended cache
    alone = oracle.tree_attn(a.q[7:8], kc, vc, a.k_tree[7:8], a.v_tree[7:8], np.array([-1], np.int32), new_len)[0]
    np.testing.assert_allclose(alone, in_tree, rtol=1e-12, atol=1e-14)
    # rows before the prefix end and after the appended ones are untouched
    assert np.array_equal(kc[:, :P], a.k_cache[:, :P]) and np.array_equal(kc[:, new_len:], a.k_cache[:, new_len:])
    # the wrong order, or forgetting the root, would not pass the comparison above
    bad_k, bad_v, _ = oracle.kv_append(a.k_tree, a.v_tree, np.array([3, 1, 5, -1], np.int32), a.k_cache, a.v_cache, P)
    assert not np.array_equal(bad_k, kc)


def test_empty_path_and_full_cache():
    rng = np.random.default_rng(4)
    k_tree, v_tree = rng.standard_normal((5, 2, 64)).astype(np.float32), rng.standard_normal((5, 2, 64)).astype(np.float32)
    kc, vc = np.zeros((2, 10, 64), np.float32), np.zeros((2, 10, 64), np.float32)
    k2, v2, n2 = oracle.kv_append(k_tree, v_tree, np.full(5, -1, np.int32), kc, vc, 6)
    assert n2 == 7 and np.array_equal(k2[:, 6], k_tree[0]) and not k2[:, 7:].any()
    k3, v3, n3 = oracle.kv_append(k_tree, v_tree, np.array([1, 2, 4, -1, -1], np.int32), kc, vc, 8)
    assert n3 == 10 and np.array_equal(k3[:, 9], k_tree[1]) and np.array_equal(v3[:, 8], v_tree[0])


def test_argument_errors_need_no_gpu():
    par = np.array([-1, 0, 0], dtype=np.int32)

    def call(kt=0x1000, path=0x1000, parent=par.ctypes.data, kc=0x1000, prefix_len=4, n=3, Hk=2, d=64, cap=16, dtype=B.SEQ_BF16):
        return S.lib().seq_kv_append(kt, 0x1000, path, parent, kc, 0x1000, prefix_len, n, Hk, d, cap, dtype, None, None)

    assert call(kt=None) == B.SEQ_ERR_NULL and call(path=None) == B.SEQ_ERR_NULL and call(parent=None) == B.SEQ_ERR_NULL
    assert call(dtype=9) == B.SEQ_ERR_DTYPE
    assert call(d=96) == B.SEQ_ERR_SHAPE and call(prefix_len=17) == B.SEQ_ERR_SHAPE and call(prefix_len=-1) == B.SEQ_ERR_SHAPE
    assert call(n=0) == B.SEQ_ERR_SHAPE and call(Hk=0) == B.SEQ_ERR_SHAPE and call(kc=0x1008) == B.SEQ_ERR_SHAPE
    bad = np.array([-1, 1, 0], dtype=np.int32)
    assert call(parent=bad.ctypes.data) == B.SEQ_ERR_TREE


@pytest.mark.gpu
@pytest.mark.parametrize("dtype,Hk,d", [(W.BF16, 32, 128), (W.F32, 2, 64), (W.BF16, 8, 128), (W.F32, 5, 128)])
def test_library_equals_the_checker_bit_for_bit(dtype, Hk, d):
    import torch
    from gpu_util import DEV, to_dev
    rng = np.random.default_rng(Hk)
    parent = W.geometric_tree(40, 6)
    a = W.make_attn_inputs(Hk, Hk, d, 50, parent, dtype, seed=d, prefix_cap=64)
    depth = W.depths(parent)
    paths = []
    for leaf in (int(np.argmax(depth)), 1):
        p, v = [], leaf
        while v != 0:
            p.append(v)
            v = int(parent[v])
        paths.append(p[::-1])
    paths += [[], [39], [1, 999], [200]]                                   # empty; not a real path but legal ids; bad ids end it
    for prefix_len in (50, 61):                                            # 61: the deepest path overflows the cache
        for path in paths:
            full = np.full(40, -1, dtype=np.int32)
            full[: len(path)] = path
            kc, vc = to_dev(a.k_cache, dtype), to_dev(a.v_cache, dtype)
            new_len = S.seq_kv_append(to_dev(a.k_tree, dtype), to_dev(a.v_tree, dtype), torch.from_numpy(full).to(DEV),
                                      parent, kc, vc, prefix_len)
            torch.cuda.synchronize()
            want_k, want_v, want_len = oracle.kv_append(a.k_tree, a.v_tree, full, a.k_cache, a.v_cache, prefix_len)
            assert int(new_len.item()) == want_len, (prefix_len, path)
            assert np.array_equal(kc.float().cpu().numpy(), want_k) and np.array_equal(vc.float().cpu().numpy(), want_v), (prefix_len, path)
