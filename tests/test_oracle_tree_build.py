"""Pins for the CPU checker of Sequoia's tree construction (Sec. 3.1.2, Algorithm 1 and the depth
bound of its appendix).

The score F(T) is held against a simulation of the verification under the positional acceptance
assumption and against hand-computed examples; the dynamic program against the plain definition
of the problem (every tree generated and scored) and against closed forms for chains and stars.
"""
import json
import os

import numpy as np
import pytest

from oracle import tree_build_oracle as TB

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_acceptance_vector.json")
PAPER_P = json.load(open(GOLDEN))["acceptance"]
POWER_LAW = [0.6 / k ** 1.5 for k in range(1, 12)]
FLAT = [0.2, 0.2, 0.2, 0.2]
RISING = [0.1, 0.3, 0.25]          # not monotone: the program must not assume it is


def simulate_generated_tokens(parent, p, trials, seed):
    """Under the positional acceptance assumption an accepted node hands on to its k-th child with
    probability p[k] (at most one child); every accepted node, the root included, yields a token."""
    rng = np.random.default_rng(seed)
    children = [[] for _ in parent]
    for i in range(1, len(parent)):
        children[parent[i]].append(i)
    total = 0
    for _ in range(trials):
        v, count = 0, 1
        while True:
            u, acc, nxt = rng.random(), 0.0, None
            for k, c in enumerate(children[v]):
                acc += p[k] if k < len(p) else 0.0
                if u < acc:
                    nxt = c
                    break
            if nxt is None:
                break
            v, count = nxt, count + 1
        total += count
    return total / trials


def test_score_of_hand_examples():
    p = [0.5, 0.25, 0.125]
    assert TB.tree_score([-1], p) == 1.0
    assert TB.tree_score([-1, 0, 1, 2], p) == pytest.approx(1 + 0.5 + 0.25 + 0.125)        # a chain
    assert TB.tree_score([-1, 0, 0, 0], p) == pytest.approx(1 + 0.5 + 0.25 + 0.125)        # a star
    assert TB.tree_score([-1, 0, 0, 0, 0], p) == pytest.approx(1 + 0.875)                  # a 4th child adds 0
    # the example of the score function's definition: the 3rd child of the root's 2nd child has path [2, 3]
    parent = [-1, 0, 0, 2, 2, 2]
    assert TB.tree_score(parent, p) == pytest.approx(1 + 0.5 + 0.25 + 0.25 * (0.5 + 0.25 + 0.125))
    assert TB.child_positions(parent) == [0, 1, 2, 1, 2, 3]


def test_score_is_the_expected_number_of_generated_tokens():
    rng = np.random.default_rng(3)
    p = [0.45, 0.2, 0.1, 0.05]
    for n in (7, 20):
        parent = [-1] + [int(rng.integers(0, i)) for i in range(1, n)]
        want = TB.tree_score(parent, p)
        got = simulate_generated_tokens(parent, p, 200000, n)
        assert abs(got - want) < 0.01, (got, want)


@pytest.mark.parametrize("p", [PAPER_P, POWER_LAW, FLAT, RISING])
def test_dynamic_program_equals_exhaustive_search(p):
    for B in (1, 2, 3, 8):
        for depth_limit in (1, 2, 3, 8):
            T, Tmax = TB.dynamic_program(p, 8, B, depth_limit)
            for n in range(1, 9):
                best, tree = TB.best_tree_brute_force(p, n, B, depth_limit)
                assert Tmax[n][depth_limit + 1] == pytest.approx(best, rel=1e-12, abs=0) or \
                    (best == TB.NEG_INF and Tmax[n][depth_limit + 1] == TB.NEG_INF), (B, depth_limit, n)
                if tree is not None:
                    assert len(tree) == n and TB.depth_of(tree) <= depth_limit and TB.max_branch_of(tree) <= B
                    assert TB.tree_score(tree, p) == pytest.approx(best, rel=1e-12)


def test_a_planted_mistake_is_caught_by_the_exhaustive_search():
    """Giving tree #2 the same number of levels as the whole tree (a plausible slip in the
    recursion) breaks the depth bound and the comparison above would see it."""
    p, B, depth_limit, n = POWER_LAW, 3, 2, 8
    best, _ = TB.best_tree_brute_force(p, n, B, depth_limit)
    deeper, _ = TB.best_tree_brute_force(p, n, B, depth_limit + 1)
    assert deeper > best * (1 + 1e-6)


def test_chains_and_stars_have_closed_forms():
    p = PAPER_P
    for n in range(1, 12):
        # one child per node: the only tree is the chain, and it needs n levels
        assert TB.expected_tokens(p, n, 1, 20) == pytest.approx(sum(p[0] ** i for i in range(n)))
        assert TB.expected_tokens(p, n, 1, n - 1) > 0
        if n >= 2:
            assert TB.expected_tokens(p, n, 1, n - 2) == TB.NEG_INF
        # one level below the root: the only tree is the star
        assert TB.expected_tokens(p, n, 31, 1 if n > 1 else 0) == pytest.approx(1 + sum(p[: n - 1]))
    # a single sequence never generates more than 1 / (1 - p_1) tokens (Sec. 3.1.2)
    assert TB.expected_tokens(p, 200, 1, 400) < 1 / (1 - p[0])


def test_more_room_never_hurts():
    p = POWER_LAW
    for B, d in ((2, 3), (4, 6), (11, 12)):
        _, Tmax = TB.dynamic_program(p, 40, B, d)
        vals = [Tmax[n][d + 1] for n in range(1, 41)]
        finite = [v for v in vals if v != TB.NEG_INF]
        assert all(b >= a - 1e-15 for a, b in zip(finite, finite[1:]))
    assert TB.expected_tokens(p, 30, 4, 6) <= TB.expected_tokens(p, 30, 5, 6) <= TB.expected_tokens(p, 30, 5, 7)


def test_paper_vector_grows_a_wide_root_and_a_long_first_chain():
    """With the printed acceptance vector (p_1 = 0.77, then a fast decay) the best 64-node tree is
    neither a chain nor a star, beats both, and generates more tokens than the bound of a
    single sequence allows... which it cannot exceed by much: a sanity bracket, not a printed figure."""
    p = PAPER_P
    g = TB.expected_tokens(p, 64, 31, 63)
    chain = sum(p[0] ** i for i in range(64))
    star = 1 + sum(p[:31])
    assert g > chain and g > star
    assert g < 1 / (1 - sum(p))           # every accepted node hands on with probability at most sum(p)


def test_speedup_formula():
    p = POWER_LAW
    g = TB.expected_tokens(p, 16, 8, 4)
    assert TB.speedup(p, 8, 16, 4, verify_time_n=30.0, decode_time=20.0, draft_time=2.0) == pytest.approx(g / (1.5 + 4 * 0.1))
