"""The library's tree construction (host code, no GPU) against the CPU checker: the value F of
the returned tree equals the checker's optimum (dynamic program; exhaustive search for small
sizes), the tree is valid and in the order the other calls expect, and the hardware-aware choice
of size and depth is the arg-max of the checker's Speedup(n, d)."""
import json
import os

import numpy as np
import pytest

import paper_2402_12374_amd as S
from oracle import tree_build_oracle as TB
from paper_2402_12374_amd import binding as B

PAPER_P = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_acceptance_vector.json")))["acceptance"]
POWER_LAW = [0.6 / k ** 1.5 for k in range(1, 12)]
RISING = [0.1, 0.3, 0.25]


def check_tree(parent, n, max_branch, max_depth):
    parent = [int(x) for x in parent]
    assert len(parent) == n and parent[0] == -1
    assert all(0 <= parent[i] < i for i in range(1, n))
    assert all(parent[i] <= parent[i + 1] for i in range(1, n - 1)), "breadth-first: parents never decrease"
    assert TB.depth_of(parent) <= max_depth and TB.max_branch_of(parent) <= max_branch
    d, _, _, _ = S.seq_tree_plan_host(parent)          # the other calls accept it
    assert int(d.max()) == TB.depth_of(parent)


@pytest.mark.parametrize("p", [PAPER_P, POWER_LAW, RISING])
def test_small_trees_equal_exhaustive_search(p):
    for branches in (1, 2, 3):
        for depth in (0, 1, 2, 3, 7):
            for n in range(1, 9):
                best, _ = TB.best_tree_brute_force(p[:branches], n, branches, depth)
                if best == TB.NEG_INF:
                    with pytest.raises(S.SeqTreeError) as e:
                        S.seq_build_tree(p[:branches], n, depth)
                    assert e.value.code == S.SEQ_ERR_SHAPE
                    continue
                parent, f = S.seq_build_tree(p[:branches], n, depth)
                check_tree(parent, n, branches, depth)
                assert f == pytest.approx(best, rel=1e-12)
                assert TB.tree_score(parent.tolist(), p[:branches]) == pytest.approx(best, rel=1e-12)


@pytest.mark.parametrize("p,n,depth", [(PAPER_P, 64, 8), (PAPER_P, 128, 10), (POWER_LAW, 100, 6), (RISING, 40, 12),
                                       (PAPER_P[:4], 90, 5)])
def test_larger_trees_equal_the_dynamic_program(p, n, depth):
    parent, f = S.seq_build_tree(p, n, depth)
    check_tree(parent, n, len(p), depth)
    assert f == pytest.approx(TB.expected_tokens(p, n, len(p), depth), rel=1e-12)
    assert TB.tree_score(parent.tolist(), p) == pytest.approx(f, rel=1e-12)
    assert S.seq_tree_expected_tokens(parent, p) == pytest.approx(f, rel=1e-12)


def test_benchmark_sized_trees_are_valid_and_score_what_they_claim():
    for n, depth in ((256, 12), (768, 16), (1024, 32)):
        parent, f = S.seq_build_tree(PAPER_P, n, depth)
        check_tree(parent, n, len(PAPER_P), depth)
        assert TB.tree_score(parent.tolist(), PAPER_P) == pytest.approx(f, rel=1e-12)
    small, _ = S.seq_build_tree(PAPER_P, 64, 8)
    assert S.seq_build_tree(PAPER_P, 768, 16)[1] > S.seq_build_tree(PAPER_P, 64, 8)[1]
    fan = np.bincount(small[1:], minlength=64)
    assert fan[0] == fan.max() > 2 and fan[1] >= fan[2]        # wide at the root, widest below the first child


def test_score_of_given_trees():
    rng = np.random.default_rng(9)
    for n in (1, 2, 17, 200):
        parent = np.array([-1] + [int(rng.integers(0, i)) for i in range(1, n)], dtype=np.int32)
        assert S.seq_tree_expected_tokens(parent, POWER_LAW) == pytest.approx(TB.tree_score(parent.tolist(), POWER_LAW), rel=1e-13)
    with pytest.raises(S.SeqTreeError) as e:
        S.seq_tree_expected_tokens([-1, 1, 0], POWER_LAW)
    assert e.value.code == S.SEQ_ERR_TREE


def test_hardware_aware_choice_is_the_arg_max_of_speedup():
    p = PAPER_P[:8]
    sizes = [1, 4, 8, 16, 32, 48]
    verify_time = [20.0, 20.5, 21.0, 22.0, 26.0, 33.0]        # flat, then rising (the shape of t(n) in Sec. 4.1)
    for draft_time, max_depth in ((1.0, 6), (6.0, 6), (0.0, 3), (40.0, 5)):
        n, d, s = S.seq_pick_tree_shape(p, sizes, verify_time, max_depth, decode_time=20.0, draft_time=draft_time)
        grid = {}
        for size, t in zip(sizes, verify_time):
            for depth in range(0, min(max_depth, size - 1) + 1):
                if TB.expected_tokens(p, size, len(p), depth) != TB.NEG_INF:
                    grid[(size, depth)] = TB.speedup(p, len(p), size, depth, t, 20.0, draft_time)
        best = max(grid.values())
        assert s == pytest.approx(best, rel=1e-12)
        assert grid[(n, d)] == pytest.approx(best, rel=1e-12)
    # drafting that costs more than it can ever gain: do not speculate at all
    n, d, s = S.seq_pick_tree_shape(p, sizes, verify_time, 6, decode_time=20.0, draft_time=400.0)
    assert (n, d) == (1, 0) and s == pytest.approx(1.0)


def test_argument_errors():
    lib = S.lib()
    rates = np.array([0.5, 0.2], dtype=np.float64)
    out = np.zeros(8, np.int32)
    assert lib.seq_build_tree(None, 2, 8, 3, out.ctypes.data, None) == B.SEQ_ERR_NULL
    assert lib.seq_build_tree(rates.ctypes.data, 2, 8, 3, None, None) == B.SEQ_ERR_NULL
    assert lib.seq_build_tree(rates.ctypes.data, 0, 8, 3, out.ctypes.data, None) == B.SEQ_ERR_SHAPE
    assert lib.seq_build_tree(rates.ctypes.data, B.SEQ_MAX_CHILDREN + 1, 8, 3, out.ctypes.data, None) == B.SEQ_ERR_SHAPE
    assert lib.seq_build_tree(rates.ctypes.data, 2, 0, 3, out.ctypes.data, None) == B.SEQ_ERR_SHAPE
    assert lib.seq_build_tree(rates.ctypes.data, 2, B.SEQ_MAX_TREE + 1, 3, out.ctypes.data, None) == B.SEQ_ERR_SHAPE
    assert lib.seq_build_tree(rates.ctypes.data, 2, 8, -1, out.ctypes.data, None) == B.SEQ_ERR_SHAPE
    for bad in (-0.1, 1.5, float("nan")):
        r = np.array([0.5, bad], dtype=np.float64)
        assert lib.seq_build_tree(r.ctypes.data, 2, 8, 3, out.ctypes.data, None) == B.SEQ_ERR_SHAPE
    assert lib.seq_build_tree(rates.ctypes.data, 2, 8, 3, out.ctypes.data, None) == B.SEQ_OK
    with pytest.raises(S.SeqTreeError):
        S.seq_pick_tree_shape(rates, [4], [0.0], 3, 1.0, 1.0)


def k_sequences(k, length):
    """k independent chains of `length` nodes below the root (the tree SpecInfer uses)."""
    parent = [-1]
    for _ in range(k):
        parent.append(0)
    tails = list(range(1, k + 1))
    for _ in range(length - 1):
        for j in range(k):
            parent.append(tails[j])
            tails[j] = len(parent) - 1
    return parent


def binary_tree(n):
    return [-1] + [(i - 1) // 2 for i in range(1, n)]


def test_sequoia_tree_beats_the_baseline_shapes_and_their_bounds_hold():
    """Sec. 3.1.3: one sequence generates at most 1/(1 - p1) tokens, k sequences at most one more,
    a binary tree at most 1/(1 - p1 - p2) however deep; the tree of the dynamic program is at
    least as good as each of them at equal size."""
    p = PAPER_P
    for n in (16, 41, 64, 128):
        _, best = S.seq_build_tree(p, n, n - 1)
        chain = S.seq_tree_expected_tokens(list(range(-1, n - 1)), p)
        assert chain < 1 / (1 - p[0]) and best >= chain
        binary = S.seq_tree_expected_tokens(binary_tree(n), p)
        assert binary < 1 / (1 - p[0] - p[1]) and best >= binary
    for k, length in ((5, 8), (3, 21), (8, 5)):
        seqs = k_sequences(k, length)
        f = S.seq_tree_expected_tokens(seqs, p)
        assert f < 1 / (1 - p[0]) + 1
        _, best = S.seq_build_tree(p, len(seqs), len(seqs) - 1)
        assert best >= f
    # and it keeps growing where they have levelled off
    _, g64 = S.seq_build_tree(p, 64, 63)
    _, g512 = S.seq_build_tree(p, 512, 511)
    assert g512 > g64 + 1.5 and g64 > 1 / (1 - p[0]) + 1
