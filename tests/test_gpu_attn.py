"""GPU parity of seq_tree_attn against the CPU checker (element by element, through the C ABI)."""
import numpy as np
import pytest
import torch

import oracle
import workloads as W

from gpu_util import TOL, oracle_attn, oracle_attn_all_rows, run_attn, to_dev

pytestmark = pytest.mark.gpu


def test_toy_config_fp32_full():
    a = W.attn_inputs_for("C1")
    err = np.abs(run_attn(a) - oracle_attn(a)).max()
    assert err <= TOL[W.F32], err


@pytest.mark.parametrize("H,Hk,d,P,n,tree", [
    (4, 2, 128, 200, 37, "geo"),      # ragged prefix tile, ragged tree tile
    (8, 1, 64, 77, 130, "rand"),      # G = 8, d = 64, three tree tiles
    (2, 2, 128, 0, 5, "chain"),       # empty prefix
    (3, 3, 128, 300, 1, "chain"),     # single node = decode attention
    (2, 1, 128, 64, 64, "star"),      # exact tile multiples
    (5, 5, 64, 1, 200, "geo"),
    (16, 2, 128, 513, 96, "rand"),
])
def test_small_shapes_bf16_and_fp32(H, Hk, d, P, n, tree):
    rng = np.random.default_rng(P * 1000 + n)
    parent = {"geo": lambda: W.geometric_tree(n, 9), "rand": lambda: W.random_topological_tree(n, rng),
              "chain": lambda: W.chain_tree(n), "star": lambda: W.star_tree(n)}[tree]()
    for dtype in (W.BF16, W.F32):
        a = W.make_attn_inputs(H, Hk, d, P, parent, dtype, seed=n + P, prefix_cap=P + 5)
        err = np.abs(run_attn(a) - oracle_attn(a)).max()
        assert err <= TOL[dtype], (dtype, err)


@pytest.mark.parametrize("key", ["C2", "C3"])
def test_full_config_all_rows(key):
    a = W.attn_inputs_for(key)
    got, want = run_attn(a), oracle_attn(a)
    err = np.abs(got - want).max()
    assert err <= TOL[a.dtype], err


@pytest.mark.parametrize("key", ["C4", "C5"])
def test_largest_configs_all_rows(key):
    """Every one of the 13 312 (C4) and 49 152 (C5) output rows against the checker, whose rows
    are shared out over the host's cores (about 6 s and 45 s of work for one core)."""
    a = W.attn_inputs_for(key)
    got = run_attn(a)
    assert np.isfinite(got).all()
    want = oracle_attn_all_rows(a)
    err = np.abs(got - want).max()
    assert err <= TOL[a.dtype], err


@pytest.mark.parametrize("dtype", [W.BF16, W.F32])
def test_masked_keys_have_exactly_zero_weight(dtype):
    parent = W.geometric_tree(70, 7)
    a = W.make_attn_inputs(4, 2, 128, 100, parent, dtype, seed=3, prefix_cap=140)
    base = run_attn(a)
    # cache rows past prefix_len: anything at all, NaN included
    a.k_cache[:, 100:] = np.nan
    a.v_cache[:, 100:] = np.nan
    assert np.array_equal(run_attn(a), base)
    # tree rows that one query may not see: NaN keys, huge values -> that query's row unchanged
    for i in (0, 13, 69):
        anc = set()
        j = i
        while j >= 0:
            anc.add(j)
            j = int(parent[j])
        b = W.make_attn_inputs(4, 2, 128, 100, parent, dtype, seed=3, prefix_cap=140)
        for j in range(70):
            if j not in anc:
                b.k_tree[j] = np.nan
                b.v_tree[j] = 1e30
        got = run_attn(b)
        assert np.array_equal(got[i], base[i]), i


def test_repeated_calls_are_bit_identical_and_cached_plan_is_reused():
    a = W.attn_inputs_for("C2")
    first = run_attn(a)
    for _ in range(3):
        assert np.array_equal(run_attn(a), first)


@pytest.mark.parametrize("H,Hk,P,n", [(32, 32, 1024, 64), (64, 8, 3000, 640), (52, 52, 4096, 320)])
def test_launches_on_changing_inputs_share_a_workspace_without_reading_each_other(H, Hk, P, n):
    """The partial results of the key ranges go through one workspace, call after call, and the
    workgroup that merges them learns from a counter that they have arrived.  If it could read
    them before they had landed it would merge the previous call's: 300 launches back to back on
    three input sets in turn, each set's output bit for bit what it was the first time.  (Five
    equal ranges; a long and a short one with the long ones of one length; two of two sizes.)"""
    import torch
    import paper_2402_12374_amd as S
    dev = torch.device("cuda:0")
    parent = W.geometric_tree(n, 9)
    sets = []
    for k in range(3):
        a = W.make_attn_inputs(H, Hk, 128, P, parent, W.BF16, seed=50 + k)
        sets.append([to_dev(x, a.dtype) for x in (a.q, a.k_cache, a.v_cache, a.k_tree, a.v_tree)])
    ws = torch.empty(S.seq_tree_attn_workspace(P, n, H, Hk, 128, 1), dtype=torch.uint8, device=dev)
    outs = [torch.empty(n, H, 128, dtype=torch.bfloat16, device=dev) for _ in range(300)]
    for i, out in enumerate(outs):
        S.seq_tree_attn(*sets[i % 3], parent, P, out=out, workspace=ws)
    torch.cuda.synchronize()
    for i, out in enumerate(outs):
        assert torch.equal(out, outs[i % 3]), i
    assert not torch.equal(outs[0], outs[1])


def test_chain_tree_matches_torch_causal_attention():
    # independent of the checker: PyTorch's own causal attention on the GPU
    P, n, H, d = 96, 40, 4, 128
    a = W.make_attn_inputs(H, H, d, P, W.chain_tree(n), W.BF16, seed=11)
    got = run_attn(a)
    k = torch.cat([torch.from_numpy(a.k_cache[:, :P]), torch.from_numpy(a.k_tree).permute(1, 0, 2)], 1).double()
    v = torch.cat([torch.from_numpy(a.v_cache[:, :P]), torch.from_numpy(a.v_tree).permute(1, 0, 2)], 1).double()
    q = torch.from_numpy(a.q).permute(1, 0, 2).double()
    mask = torch.ones(n, P + n, dtype=torch.bool).tril(diagonal=P)
    want = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=mask).permute(1, 0, 2).numpy()
    assert np.abs(got - want).max() <= TOL[W.BF16]


@pytest.mark.parametrize("d", [64, 128])
def test_every_workgroup_shape_and_range_count(d):
    """The library chooses row blocks per workgroup and key ranges per unit by a cost model; force
    every combination the kernels are built for on one shape with ragged tiles, so that no
    variant goes untested because the model happens not to pick it."""
    import paper_2402_12374_amd as S
    rng = np.random.default_rng(11)
    # 9 x 4 = 36 query rows per KV head would take wq = 2; 70 x 4 = 280 rows lets every wq apply
    parent = W.random_topological_tree(70, rng)
    # 1101 prefix keys + 70 tree keys = 38 tiles: up to 9 ranges with wq = 2 and all 16 with wq = 4, 8
    # (the merge of the ranges is compiled once per number of ranges up to 8, then for 10, 12, 16)
    a = W.make_attn_inputs(8, 2, d, 1101, parent, W.BF16, seed=d, prefix_cap=1110)
    ref = oracle_attn(a)
    try:
        for wq in (2, 4, 8):
            for splits in range(1, 17):
                S.lib().seqtree_internal_set_attn_wq(wq)
                S.lib().seqtree_internal_set_attn_splits(splits)
                err = np.abs(run_attn(a) - ref).max()
                assert err <= TOL[W.BF16], (wq, splits, err)
    finally:
        S.lib().seqtree_internal_set_attn_wq(0)
        S.lib().seqtree_internal_set_attn_splits(0)


@pytest.mark.parametrize("shape", ["star", "two_chains", "late_root_children"])
def test_tree_tiles_without_an_ancestor_of_a_row_block(shape):
    """A wavefront leaves out a tree tile none of whose 32 keys is an ancestor of any of its
    queries.  Trees in which that is most tiles, in which a block's only live tiles are the first
    and its own, and in which live tiles lie far apart; every workgroup shape, with the tree tiles
    in one key range and spread over several; no prefix at all as well (every tile a tree tile)."""
    import paper_2402_12374_amd as S
    n = 300
    if shape == "star":
        parent = W.star_tree(n)
    elif shape == "two_chains":
        # nodes alternate between two chains hanging off the root: a node's ancestors are every
        # other node below it, so every tile below it is live for it
        parent = np.array([-1, 0, 0] + list(range(1, n - 2)), np.int32)
    else:
        # the first 200 nodes are a star; the last 100 are children of node 199: their ancestors
        # sit in tiles 0 and 6 only
        parent = np.array([-1] + [0] * 199 + [199] * 100, np.int32)
    for P in (0, 333):
        a = W.make_attn_inputs(8, 2, 128, P, parent, W.BF16, seed=17 + P, prefix_cap=max(P, 1) + 5)
        ref = oracle_attn_all_rows(a)
        try:
            for wq in (2, 4, 8):
                for splits in (1, 2, 5):
                    S.lib().seqtree_internal_set_attn_wq(wq)
                    S.lib().seqtree_internal_set_attn_splits(splits)
                    err = np.abs(run_attn(a) - ref).max()
                    assert err <= TOL[W.BF16], (shape, P, wq, splits, err)
        finally:
            S.lib().seqtree_internal_set_attn_wq(0)
            S.lib().seqtree_internal_set_attn_splits(0)


@pytest.mark.parametrize("d", [64, 128])
def test_key_ranges_of_two_sizes(d):
    """Where the units leave compute units over, the library cuts a unit's keys into long ranges and
    short ones (several short ones then run in a row on the units left over).  Forced here on a
    small ragged shape: any number of short ranges, weights from nearly equal to so lopsided that
    short ranges get a single tile or none."""
    import paper_2402_12374_amd as S
    rng = np.random.default_rng(12)
    a = W.make_attn_inputs(8, 2, d, 1101, W.random_topological_tree(70, rng), W.BF16, seed=d + 1, prefix_cap=1110)
    ref = oracle_attn(a)
    try:
        for wq, splits, shorts, short_w, long_w in ((8, 2, 1, 1, 3), (8, 2, 1, 15, 49), (4, 3, 1, 12, 26), (2, 3, 2, 1, 5),
                                                    (8, 4, 3, 1, 61), (4, 5, 1, 1, 1), (8, 6, 2, 3, 7), (2, 2, 1, 1, 63),
                                                    (8, 16, 15, 1, 49), (4, 8, 4, 2, 3)):
            S.lib().seqtree_internal_set_attn_wq(wq)
            S.lib().seqtree_internal_set_attn_splits(splits)
            S.lib().seqtree_internal_set_attn_uneven(shorts, short_w, long_w)
            err = np.abs(run_attn(a) - ref).max()
            assert err <= TOL[W.BF16], (wq, splits, shorts, short_w, long_w, err)
    finally:
        S.lib().seqtree_internal_set_attn_wq(0)
        S.lib().seqtree_internal_set_attn_splits(0)
        S.lib().seqtree_internal_set_attn_uneven(-1, 1, 1)


def test_long_ranges_of_one_length_for_all_units():
    """Where a KV head has many units the long ranges get one length for all of them, counted from
    the end of each unit's tiles, and the short ranges what is left (the units differ in their
    tree tiles).  Forced here on a small shape whose units have 36 to 45 tiles: lengths from one
    tile to more than a unit has (short ranges, and then long ones, come out empty)."""
    import paper_2402_12374_amd as S
    rng = np.random.default_rng(21)
    a = W.make_attn_inputs(8, 2, 128, 1101, W.random_topological_tree(300, rng), W.BF16, seed=5, prefix_cap=1110)
    ref = oracle_attn_all_rows(a)
    try:
        for wq, splits, shorts in ((2, 2, 1), (4, 3, 1), (8, 3, 2), (8, 5, 1), (2, 4, 3)):
            S.lib().seqtree_internal_set_attn_wq(wq)
            S.lib().seqtree_internal_set_attn_splits(splits)
            S.lib().seqtree_internal_set_attn_uneven(shorts, 1, 3)
            for length in (1, 7, 18, 30, 1000):
                S.lib().seqtree_internal_set_attn_long_tiles(length)
                err = np.abs(run_attn(a) - ref).max()
                assert err <= TOL[W.BF16], (wq, splits, shorts, length, err)
    finally:
        S.lib().seqtree_internal_set_attn_wq(0)
        S.lib().seqtree_internal_set_attn_splits(0)
        S.lib().seqtree_internal_set_attn_uneven(-1, 1, 1)
        S.lib().seqtree_internal_set_attn_long_tiles(-1)


def test_the_shapes_that_take_ranges_of_two_sizes_by_themselves():
    """Shapes at which the library's own choice is ranges of two sizes (one or two long ranges per
    unit, workgroups of 8 or 4 row blocks; long ranges of one length where a KV head has many
    units, in proportion to their unit's tiles where it has few), all rows against the checker."""
    import ctypes
    import paper_2402_12374_amd as S
    five = (ctypes.c_int * 5)()
    for H, Hk, P, n, one_length in ((64, 8, 3000, 640, True), (88, 88, 4096, 256, False), (52, 52, 4096, 320, False)):
        S.lib().seqtree_internal_attn_schedule(P, n, H, Hk, 128, five)
        assert five[2] >= 1, (H, Hk, P, n, list(five))
        assert (S.lib().seqtree_internal_attn_long_tiles(P, n, H, Hk, 128) > 0) == one_length, (H, Hk, P, n)
        a = W.make_attn_inputs(H, Hk, 128, P, W.geometric_tree(n, 10), W.BF16, seed=n)
        got = run_attn(a)
        assert np.abs(got - oracle_attn_all_rows(a)).max() <= TOL[W.BF16], (H, Hk, P, n)
        # a long range's workgroup that finds all the others arrived keeps its partial result in
        # registers; whether it does depends on timing, the bits of the result must not
        try:
            S.lib().seqtree_internal_set_attn_keep_own(0)
            assert np.array_equal(run_attn(a), got), (H, Hk, P, n)
        finally:
            S.lib().seqtree_internal_set_attn_keep_own(1)
        assert np.array_equal(run_attn(a), got), (H, Hk, P, n)


def test_seeded_random_shapes_under_the_library_s_own_schedule():
    """Heads, group size, head dimension, prefix and tree drawn at random (seeded): whatever
    workgroup shape, range count and range sizes the library picks for them by itself, every row
    agrees with the checker.  The draw is checked to exercise several schedules, among them
    ranges of two sizes, so that a change of the cost figures cannot quietly narrow the test."""
    import ctypes
    import paper_2402_12374_amd as S
    rng, tree_rng = np.random.default_rng(2436), np.random.default_rng(12374)
    five = (ctypes.c_int * 5)()
    picks = []
    for case in range(14):
        Hk = int(rng.choice([1, 2, 4, 8, 12, 20, 24, 32]))
        G = int(rng.choice([1, 1, 2, 4, 8]))
        d = int(rng.choice([64, 128]))
        n = int(rng.integers(1, 420))
        P = int(rng.integers(0, 3600))
        S.lib().seqtree_internal_attn_schedule(P, n, Hk * G, Hk, d, five)
        picks.append(tuple(five) + (S.lib().seqtree_internal_attn_long_tiles(P, n, Hk * G, Hk, d),))
        parent = W.random_topological_tree(n, tree_rng) if case % 2 else W.geometric_tree(n, 9)
        a = W.make_attn_inputs(Hk * G, Hk, d, P, parent, W.BF16, seed=100 + case, prefix_cap=P + 1 + case)
        err = np.abs(run_attn(a) - oracle_attn_all_rows(a)).max()
        assert err <= TOL[W.BF16], (case, (Hk * G, Hk, d, P, n), picks[-1], err)
    assert sum(1 for k in picks if k[2] > 0) >= 2, picks           # ranges of two sizes
    assert sum(1 for k in picks if k[5] > 0) >= 1, picks           # long ranges of one length
    assert len({k[:2] for k in picks}) >= 6, picks                  # (row blocks, ranges) pairs
    assert {k[0] for k in picks} == {2, 4, 8}, picks


@pytest.mark.parametrize("H,Hk,d,P,n", [(28, 4, 64, 5648, 593), (30, 6, 128, 2876, 452), (120, 10, 128, 2552, 222),
                                        (14, 2, 64, 440, 239), (24, 3, 128, 3430, 580), (50, 10, 128, 4227, 387)])
def test_group_sizes_that_are_not_powers_of_two(H, Hk, d, P, n):
    """Query heads per KV head of 7, 5, 12, 7, 8 and 5: a row block of 32 query rows then straddles
    nodes unevenly, and every division by the group size (which node and head a row is, which
    tree tiles a unit sees, where a merged row goes) is a multiplication prepared on the host.
    All rows against the checker, under the library's own schedule (the first shape takes four key
    ranges of two sizes with long ranges of one length)."""
    rng = np.random.default_rng(n)
    a = W.make_attn_inputs(H, Hk, d, P, W.random_topological_tree(n, rng), W.BF16, seed=P, prefix_cap=P + 3)
    err = np.abs(run_attn(a) - oracle_attn_all_rows(a)).max()
    assert err <= TOL[W.BF16], (H, Hk, d, P, n, err)


@pytest.mark.parametrize("H,Hk,P,n", [(4, 4, 700, 40), (16, 2, 1500, 300)])
@pytest.mark.parametrize("order", ["rising", "falling", "spiky"])
def test_scores_of_large_and_moving_magnitude(H, Hk, P, n, order):
    """The running reference of the softmax has to follow scores that keep growing along the key
    axis (every tile raises the maximum by more than the slack the kernel allows itself), must
    not lose keys far below it when they come first, and must survive isolated huge scores."""
    d = 128
    rng = np.random.default_rng(P + n)
    parent = W.geometric_tree(n, 9)
    a = W.make_attn_inputs(H, Hk, d, P, parent, W.BF16, seed=3 * P + n)
    # keys get a component along one direction every query shares: score = base + ramp(key)
    u = np.zeros(d, dtype=np.float32)
    u[:8] = 1.0
    a.q[:] = W.quantize(a.q * 0.25 + 4.0 * u, W.BF16)          # q.u = 32, so q.k = 32 ramp + noise
    keys = P + n
    if order == "rising":
        ramp = np.linspace(-8.0, 8.0, keys)                      # q.k/sqrt(d) from about -23 to +23
    elif order == "falling":
        ramp = np.linspace(8.0, -8.0, keys)
    else:
        ramp = np.where(rng.random(keys) < 0.02, 8.0, -2.0) * rng.random(keys)
    ramp = ramp.astype(np.float32)
    a.k_cache[:, :P, :] = W.quantize(a.k_cache[:, :P, :] * 0.25 + ramp[None, :P, None] * u[None, None, :], W.BF16)
    a.k_tree[:] = W.quantize(a.k_tree * 0.25 + ramp[P:, None, None] * u[None, None, :], W.BF16)
    got, want = run_attn(a), oracle_attn(a)
    assert np.isfinite(got).all()
    err = np.abs(got - want).max()
    assert err <= TOL[a.dtype], err


def test_a_batch_of_sequences_is_a_call_with_more_heads():
    """B sequences that share the tree and the prefix length: heads = B*H, kv_heads = B*Hk on
    tensors laid out [n, B, H, d] and [B, Hk, cap, d].  Query head b*H + h maps to KV head
    b*Hk + h/G, i.e. sequence b only ever sees its own cache and tree rows."""
    B, H, Hk, d, P, n = 3, 8, 2, 128, 333, 40
    parent = W.geometric_tree(n, 6)
    seqs = [W.make_attn_inputs(H, Hk, d, P, parent, W.BF16, seed=90 + b) for b in range(B)]
    folded = W.AttnInputs(q=np.stack([s.q for s in seqs], axis=1).reshape(n, B * H, d),
                          k_cache=np.concatenate([s.k_cache for s in seqs], axis=0),
                          v_cache=np.concatenate([s.v_cache for s in seqs], axis=0),
                          k_tree=np.stack([s.k_tree for s in seqs], axis=1).reshape(n, B * Hk, d),
                          v_tree=np.stack([s.v_tree for s in seqs], axis=1).reshape(n, B * Hk, d),
                          parent=parent, prefix_len=P, prefix_cap=seqs[0].prefix_cap, dtype=W.BF16)
    got = run_attn(folded).reshape(n, B, H, d)
    for b, s in enumerate(seqs):
        assert np.abs(got[:, b] - oracle_attn(s)).max() <= TOL[W.BF16], b
        assert np.abs(got[:, b] - run_attn(s)).max() <= 2 ** -6, b      # the same numbers up to the schedule's rounding


def _batched_case(B, H, Hk, d, cap, n, lens, dtype, seed, tree):
    """A batch that shares the tree; sequence b uses the first lens[b] rows of its own cache."""
    import paper_2402_12374_amd as S
    from gpu_util import DEV, to_dev
    seqs = [W.make_attn_inputs(H, Hk, d, int(lens[b]), tree, dtype, seed=seed + b, prefix_cap=cap) for b in range(B)]
    q = np.stack([s.q for s in seqs], axis=1)
    kt = np.stack([s.k_tree for s in seqs], axis=1)
    vt = np.stack([s.v_tree for s in seqs], axis=1)
    kc = np.stack([s.k_cache for s in seqs], axis=0)
    vc = np.stack([s.v_cache for s in seqs], axis=0)
    dev_lens = torch.from_numpy(np.asarray(lens, np.int32)).to(DEV)
    return seqs, (to_dev(q, dtype), to_dev(kc, dtype), to_dev(vc, dtype), to_dev(kt, dtype), to_dev(vt, dtype)), dev_lens


@pytest.mark.parametrize("B,H,Hk,d,cap,n,lens,dtype", [
    (4, 8, 2, 128, 700, 40, [700, 0, 333, 31], W.BF16),          # full, empty, ragged and one-tile prefixes side by side
    (3, 32, 32, 128, 1100, 64, [1024, 17, 1100], W.BF16),        # C2's head shape: key ranges cut for 1100, one sequence has 17 keys
    (6, 4, 1, 64, 300, 130, [300, 299, 1, 64, 150, 0], W.BF16),  # d = 64, grouped heads, five bitset words
    (5, 2, 2, 64, 256, 16, [256, 3, 0, 100, 255], W.F32),        # the fp32 path
    (2, 64, 8, 128, 2100, 96, [2100, 5], W.BF16),                # many query rows per KV head
])
def test_a_batch_whose_sequences_differ_in_prefix_length(B, H, Hk, d, cap, n, lens, dtype):
    """seq_tree_attn_batched against one checker call per sequence, element by element; then the
    lengths change in device memory and the same call (same arguments, same plan) must follow."""
    import paper_2402_12374_amd as S
    tree = W.geometric_tree(n, 7) if n != 130 else W.random_topological_tree(n, np.random.default_rng(4))
    seqs, tensors, dev_lens = _batched_case(B, H, Hk, d, cap, n, lens, dtype, seed=31 * B + n, tree=tree)
    out = S.seq_tree_attn_batched(*tensors, tree, dev_lens, max(lens))
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    for b, s in enumerate(seqs):
        err = np.abs(got[:, b] - oracle_attn(s)).max()
        assert err <= TOL[dtype], (b, lens[b], err)
    # shorter histories in the same buffers: rows at and beyond the new lengths must have no weight
    shorter = [max(0, x - 7 * (b + 1)) for b, x in enumerate(lens)]
    dev_lens.copy_(torch.from_numpy(np.asarray(shorter, np.int32)))
    out = S.seq_tree_attn_batched(*tensors, tree, dev_lens, max(lens))
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    for b, s in enumerate(seqs):
        s.prefix_len = shorter[b]
        err = np.abs(got[:, b] - oracle_attn(s)).max()
        assert err <= TOL[dtype], (b, shorter[b], err)


def test_a_batch_with_key_ranges_of_two_sizes():
    """Sequences of different prefix lengths under a long and a short key range per unit: the
    ranges are shares of each sequence's own tiles, so a sequence with a handful of keys gets a
    short range that is empty."""
    import paper_2402_12374_amd as S
    B, H, Hk, d, cap, n, lens = 3, 16, 2, 128, 1300, 96, [1300, 40, 611]
    tree = W.geometric_tree(n, 7)
    seqs, tensors, dev_lens = _batched_case(B, H, Hk, d, cap, n, lens, W.BF16, seed=77, tree=tree)
    try:
        for wq, splits, shorts, short_w, long_w in ((8, 2, 1, 15, 49), (4, 3, 1, 12, 26), (8, 2, 1, 1, 63)):
            S.lib().seqtree_internal_set_attn_wq(wq)
            S.lib().seqtree_internal_set_attn_splits(splits)
            S.lib().seqtree_internal_set_attn_uneven(shorts, short_w, long_w)
            out = S.seq_tree_attn_batched(*tensors, tree, dev_lens, max(lens))
            torch.cuda.synchronize()
            got = out.float().cpu().numpy().astype(np.float64)
            for b, s in enumerate(seqs):
                err = np.abs(got[:, b] - oracle_attn(s)).max()
                assert err <= TOL[W.BF16], (wq, splits, short_w, long_w, b, err)
    finally:
        S.lib().seqtree_internal_set_attn_wq(0)
        S.lib().seqtree_internal_set_attn_splits(0)
        S.lib().seqtree_internal_set_attn_uneven(-1, 1, 1)


def test_batched_lengths_are_held_to_the_bound_and_equal_lengths_match_the_folded_call():
    import paper_2402_12374_amd as S
    B, H, Hk, d, cap, n = 3, 8, 2, 128, 400, 40
    tree = W.geometric_tree(n, 6)
    seqs, tensors, dev_lens = _batched_case(B, H, Hk, d, cap, n, [400, 400, 400], W.BF16, seed=77, tree=tree)
    batched = S.seq_tree_attn_batched(*tensors, tree, dev_lens, 400)
    q, kc, vc, kt, vt = tensors
    folded = S.seq_tree_attn(q.view(n, B * H, d), kc.view(B * Hk, cap, d), vc.view(B * Hk, cap, d),
                             kt.view(n, B * Hk, d), vt.view(n, B * Hk, d), tree, 400)
    torch.cuda.synchronize()
    assert torch.equal(batched.view(n, B * H, d), folded)          # same kernel, same schedule, same bits
    # lengths outside [0, bound] are read as the nearest legal value
    dev_lens.copy_(torch.tensor([9999, -5, 123], dtype=torch.int32))
    out = S.seq_tree_attn_batched(*tensors, tree, dev_lens, 400)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    for b, plen in enumerate([400, 0, 123]):
        seqs[b].prefix_len = plen
        assert np.abs(got[:, b] - oracle_attn(seqs[b])).max() <= TOL[W.BF16], b
