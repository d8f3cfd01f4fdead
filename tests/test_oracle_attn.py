"""Pins for the CPU checker of tree attention: every test compares it with something that
does not go through its own formula (a dense textbook routine, a hand computation, an
invariance, brute force on tiny trees)."""
import itertools

import numpy as np
import pytest

import oracle
import workloads as W


def dense_masked_attention(q, keys, vals, allowed):
    """Textbook attention for one head.  q [m,d], keys/vals [L,d], allowed [m,L] bool."""
    d = q.shape[1]
    s = (q.astype(np.float64) @ keys.astype(np.float64).T) / np.sqrt(d)
    s = np.where(allowed, s, -np.inf)
    s = s - s.max(axis=1, keepdims=True)
    w = np.exp(s)
    w /= w.sum(axis=1, keepdims=True)
    return w @ vals.astype(np.float64), w


def inputs(n_or_parent, H=2, Hk=2, d=8, P=5, seed=0, dtype=W.F32, cap=None):
    parent = W.chain_tree(n_or_parent) if np.isscalar(n_or_parent) else n_or_parent
    return W.make_attn_inputs(H, Hk, d, P, parent, dtype, seed, prefix_cap=cap)


def run(a):
    return oracle.tree_attn(a.q, a.k_cache, a.v_cache, a.k_tree, a.v_tree, a.parent, a.prefix_len)


@pytest.mark.parametrize("P,n,d", [(0, 6, 4), (7, 9, 8), (33, 17, 16)])
def test_chain_tree_is_causal_attention(P, n, d):
    a = inputs(n, H=3, Hk=3, d=d, P=P, seed=1, cap=P + 3)
    got = run(a)
    L = P + n
    allowed = np.zeros((n, L), dtype=bool)
    for i in range(n):
        allowed[i, : P + i + 1] = True  # lower-triangular over the concatenated sequence
    for h in range(3):
        keys = np.concatenate([a.k_cache[h, :P], a.k_tree[:, h]], axis=0)
        vals = np.concatenate([a.v_cache[h, :P], a.v_tree[:, h]], axis=0)
        want, _ = dense_masked_attention(a.q[:, h], keys, vals, allowed)
        np.testing.assert_allclose(got[:, h], want, rtol=0, atol=1e-12)


def test_single_node_is_decode_attention():
    a = inputs(1, H=4, Hk=2, d=16, P=40, seed=2)
    got = run(a)
    for h in range(4):
        g = h // 2
        keys = np.concatenate([a.k_cache[g, :40], a.k_tree[:, g]], axis=0)
        vals = np.concatenate([a.v_cache[g, :40], a.v_tree[:, g]], axis=0)
        want, _ = dense_masked_attention(a.q[:, h], keys, vals, np.ones((1, 41), dtype=bool))
        np.testing.assert_allclose(got[:, h], want, rtol=0, atol=1e-12)


def test_star_tree_by_hand_d2():
    # root + 3 leaves, one prefix key, d = 2, numbers small enough to do on paper
    parent = W.star_tree(4)
    q = np.array([[[1.0, 0.0]], [[0.0, 2.0]], [[1.0, 1.0]], [[-1.0, 0.5]]], dtype=np.float32)
    k_cache = np.array([[[0.5, -0.5]]], dtype=np.float32)
    v_cache = np.array([[[10.0, 20.0]]], dtype=np.float32)
    k_tree = np.array([[[1.0, 1.0]], [[2.0, 0.0]], [[0.0, 3.0]], [[-2.0, -2.0]]], dtype=np.float32)
    v_tree = np.array([[[1.0, 0.0]], [[0.0, 1.0]], [[2.0, 2.0]], [[-1.0, 3.0]]], dtype=np.float32)
    got = oracle.tree_attn(q, k_cache, v_cache, k_tree, v_tree, parent, 1)
    r2 = np.sqrt(2.0)
    # node 2 sees: prefix key, root, itself (not nodes 1 and 3)
    s = np.array([(1 * 0.5 + 1 * -0.5) / r2, (1 * 1 + 1 * 1) / r2, (1 * 0 + 1 * 3) / r2])
    w = np.exp(s - s.max())
    w /= w.sum()
    want2 = w[0] * np.array([10.0, 20.0]) + w[1] * np.array([1.0, 0.0]) + w[2] * np.array([2.0, 2.0])
    np.testing.assert_allclose(got[2, 0], want2, atol=1e-13)
    # root sees: prefix key and itself
    s = np.array([(1 * 0.5) / r2, (1 * 1) / r2])
    w = np.exp(s - s.max())
    w /= w.sum()
    want0 = w[0] * np.array([10.0, 20.0]) + w[1] * np.array([1.0, 0.0])
    np.testing.assert_allclose(got[0, 0], want0, atol=1e-13)


def test_gqa_equals_mha_with_repeated_kv_heads():
    parent = W.geometric_tree(12, 5)
    a = inputs(parent, H=6, Hk=2, d=8, P=9, seed=3)
    got = run(a)
    rep = 3
    b_kc = np.repeat(a.k_cache, rep, axis=0)
    b_vc = np.repeat(a.v_cache, rep, axis=0)
    b_kt = np.repeat(a.k_tree, rep, axis=1)
    b_vt = np.repeat(a.v_tree, rep, axis=1)
    want = oracle.tree_attn(a.q, b_kc, b_vc, b_kt, b_vt, parent, a.prefix_len)
    np.testing.assert_array_equal(got, want)
    # and the repeated-head layout really is the contiguous-group mapping: head 4 uses KV head 1
    keys = np.concatenate([a.k_cache[1, :9], a.k_tree[:, 1]], axis=0)
    vals = np.concatenate([a.v_cache[1, :9], a.v_tree[:, 1]], axis=0)
    allowed = np.ones((1, 9 + 12), dtype=bool)
    allowed[0, 9 + 1:] = False  # row 0 = root sees prefix + itself
    want0, _ = dense_masked_attention(a.q[0:1, 4], keys, vals, allowed)
    np.testing.assert_allclose(got[0, 4], want0[0], atol=1e-12)


def test_relabelling_nodes_permutes_rows_only():
    rng = np.random.default_rng(5)
    parent = W.random_topological_tree(14, rng)
    a = inputs(parent, H=2, Hk=1, d=8, P=6, seed=4)
    got = run(a)
    # another topological order: sort by (depth, -id) keeps parents before children
    dep = W.depths(parent)
    order = sorted(range(14), key=lambda i: (dep[i], -i))
    new_id = {old: new for new, old in enumerate(order)}
    parent2 = np.array([-1 if parent[o] < 0 else new_id[int(parent[o])] for o in order], dtype=np.int32)
    assert all(parent2[i] < i for i in range(1, 14))
    got2 = oracle.tree_attn(a.q[order], a.k_cache, a.v_cache, a.k_tree[order], a.v_tree[order],
                            parent2, a.prefix_len)
    np.testing.assert_allclose(got2, got[order], atol=1e-13)


def test_weights_sum_to_one_and_masked_weights_are_exactly_zero():
    parent = W.geometric_tree(20, 6)
    a = inputs(parent, H=2, Hk=2, d=8, P=11, seed=6)
    for i in range(20):
        anc = set()
        j = i
        while j >= 0:
            anc.add(j)
            j = int(parent[j])
        _, wp, wt = oracle.tree_attn_row(a.q, a.k_cache, a.v_cache, a.k_tree, a.v_tree, parent,
                                         a.prefix_len, i, 1, want_weights=True)
        assert abs(wp.sum() + wt.sum() - 1.0) < 1e-13
        for j in range(20):
            if j in anc:
                assert wt[j] > 0.0
            else:
                assert wt[j] == 0.0


def test_poisoned_masked_rows_leave_output_bit_identical():
    parent = W.geometric_tree(16, 5)
    a = inputs(parent, H=2, Hk=2, d=8, P=4, seed=7, cap=9)
    base = run(a)
    # poison every cache row beyond prefix_len, then per node every non-ancestor tree row
    kc, vc = a.k_cache.copy(), a.v_cache.copy()
    kc[:, 4:] = np.nan
    vc[:, 4:] = 1e30
    again = oracle.tree_attn(a.q, kc, vc, a.k_tree, a.v_tree, parent, 4)
    assert np.array_equal(base, again)
    for i in range(16):
        anc = set()
        j = i
        while j >= 0:
            anc.add(j)
            j = int(parent[j])
        kt, vt = a.k_tree.copy(), a.v_tree.copy()
        for j in range(16):
            if j not in anc:
                kt[j] = np.nan
                vt[j] = 1e30
        row = oracle.tree_attn_row(a.q, a.k_cache, a.v_cache, kt, vt, parent, 4, i, 0)
        assert np.array_equal(row, base[i, 0])


def test_empty_prefix():
    parent = W.geometric_tree(7, 4)
    a = inputs(parent, H=1, Hk=1, d=4, P=0, seed=8, cap=1)
    got = run(a)
    # root attends only to itself => output is its own value row
    np.testing.assert_allclose(got[0, 0], a.v_tree[0, 0].astype(np.float64), atol=1e-15)


def _reachability(parent):
    """Ancestor-or-self relation via transitive closure of the parent edges (no tree walk)."""
    n = len(parent)
    adj = np.eye(n, dtype=np.int64)
    for i in range(1, n):
        adj[i, parent[i]] = 1
    reach = adj.copy()
    for _ in range(n):
        reach = ((reach @ adj) > 0).astype(np.int64)
    return reach.astype(bool)


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5])
def test_brute_force_every_tree_shape(n):
    rng = np.random.default_rng(100 + n)
    for parents in itertools.product(*[range(i) for i in range(1, n)]):
        parent = np.array((-1,) + parents, dtype=np.int32)
        for P in (0, 1, 3):
            a = W.make_attn_inputs(2, 1, 2, P, parent, W.F32, int(rng.integers(1 << 30)), prefix_cap=P + 1)
            got = run(a)
            reach = _reachability(parent)
            allowed = np.concatenate([np.ones((n, P), dtype=bool), reach], axis=1)
            keys = np.concatenate([a.k_cache[0, :P], a.k_tree[:, 0]], axis=0)
            vals = np.concatenate([a.v_cache[0, :P], a.v_tree[:, 0]], axis=0)
            for h in range(2):
                want, _ = dense_masked_attention(a.q[:, h], keys, vals, allowed)
                np.testing.assert_allclose(got[:, h], want, atol=1e-12)


def test_scale_is_one_over_sqrt_head_dim():
    # doubling d by zero-padding must change the result exactly as a 1/sqrt(2) score scaling does
    a = inputs(3, H=1, Hk=1, d=4, P=2, seed=9)
    pad = lambda x: np.concatenate([x, np.zeros_like(x)], axis=-1)
    got = oracle.tree_attn(pad(a.q), pad(a.k_cache), pad(a.v_cache), pad(a.k_tree), pad(a.v_tree),
                           a.parent, 2)
    keys = np.concatenate([a.k_cache[0, :2], a.k_tree[:, 0]], axis=0)
    vals = np.concatenate([a.v_cache[0, :2], a.v_tree[:, 0]], axis=0)
    allowed = np.tril(np.ones((3, 5), dtype=bool), k=2)
    s = (a.q[:, 0].astype(np.float64) @ keys.astype(np.float64).T) / np.sqrt(8.0)
    s = np.where(allowed, s, -np.inf)
    w = np.exp(s - s.max(axis=1, keepdims=True))
    w /= w.sum(axis=1, keepdims=True)
    np.testing.assert_allclose(got[:, 0, :4], w @ vals.astype(np.float64), atol=1e-13)
    assert np.all(got[:, 0, 4:] == 0.0)
