"""CPU checker for Sequoia's tree construction.  TEST INFRASTRUCTURE ONLY: nothing in the
product path may import this.

What is computed (Sec. 3.1.2).  Under the positional acceptance assumption a token at child
position k of an accepted node is accepted with probability p[k]; the score of a node is the
product of the p's along its path from the root (the root scores 1), and the expected number of
tokens one verification generates is F(T) = sum of the scores of T's nodes (the proposition of
that section).  The construction problem: among all trees with n nodes, at most B children per
node and at most D levels, find one that maximises F.

Three things live here, from the most literal to the fastest:

  tree_score             F(T) written out from the definition of the score function.
  best_tree_brute_force  the plain definition of the problem: every tree is generated and scored
                         (sizes up to about 10).
  dynamic_program        the paper's dynamic program (Algorithm 1, with the depth bound its
                         appendix adds), in the paper's notation:
                             T[1, d, 0] = 1
                             T[n, d, b] = max over 1 <= m <= n-1 of
                                          T[n-m, d, b-1] + P[b] * Tmax[m, d-1]
                             Tmax[n, d] = max over b of T[n, d, b]
                         where "tree #1" is the root with its first b-1 children and "tree #2",
                         of m nodes and one level less, hangs below the root's b-th child.

Trees are parent arrays in this repository's convention: node 0 is the root, parent[i] < i, and
the children of a node in ascending id are its child positions 1, 2, ... (the drafting order).
`depth_limit` counts edges below the root (the paper's D counts levels: D = depth_limit + 1).
Arithmetic is Python floats (fp64).
"""
from __future__ import annotations

from functools import lru_cache
from typing import List, Optional, Sequence, Tuple

NEG_INF = float("-inf")


def child_positions(parent: Sequence[int]) -> List[int]:
    """position[i] = k if node i is the k-th child (1-based, ascending id) of its parent; 0 for the root."""
    seen = {}
    pos = [0] * len(parent)
    for i in range(1, len(parent)):
        seen[parent[i]] = seen.get(parent[i], 0) + 1
        pos[i] = seen[parent[i]]
    return pos


def tree_score(parent: Sequence[int], p: Sequence[float]) -> float:
    """F(T): the sum over nodes of the product of acceptance rates along the node's path."""
    pos = child_positions(parent)
    f = [0.0] * len(parent)
    f[0] = 1.0
    for i in range(1, len(parent)):
        rate = p[pos[i] - 1] if pos[i] <= len(p) else 0.0
        f[i] = f[parent[i]] * rate
    return sum(f)


def _shapes(n: int, levels: int, max_branch: int):
    """Every ordered tree with n nodes, at most `levels` levels and at most max_branch children per
    node, as a nested tuple of its children's shapes."""
    if n == 1:
        yield ()
        return
    if levels <= 1:
        return

    def forests(budget: int, slots: int):
        # ordered sequences of at most `slots` non-empty trees with `budget` nodes in all
        if budget == 0:
            yield ()
            return
        if slots == 0:
            return
        for first in range(1, budget + 1):
            for head in _shapes(first, levels - 1, max_branch):
                for rest in forests(budget - first, slots - 1):
                    yield (head,) + rest

    for forest in forests(n - 1, max_branch):
        yield forest


def _score_of_shape(shape, p: Sequence[float]) -> float:
    total = 1.0
    for k, child in enumerate(shape):
        rate = p[k] if k < len(p) else 0.0
        total += rate * _score_of_shape(child, p)
    return total


def shape_to_parent(shape) -> List[int]:
    """Breadth-first numbering: parent[i] < i, siblings in ascending id = child positions."""
    parent = [-1]
    queue = [(0, shape)]
    while queue:
        node, sh = queue.pop(0)
        for child in sh:
            parent.append(node)
            queue.append((len(parent) - 1, child))
    return parent


def best_tree_brute_force(p: Sequence[float], n: int, max_branch: int, depth_limit: int
                          ) -> Tuple[float, Optional[List[int]]]:
    """max F over every tree with exactly n nodes within the bounds; (-inf, None) if there is none."""
    best, best_shape = NEG_INF, None
    for shape in _shapes(n, depth_limit + 1, max_branch):
        s = _score_of_shape(shape, p)
        if s > best:
            best, best_shape = s, shape
    return best, (shape_to_parent(best_shape) if best_shape is not None else None)


def dynamic_program(p: Sequence[float], N: int, B: int, depth_limit: int):
    """Returns (T, Tmax) as nested lists: T[n][d][b], Tmax[n][d], d = 1..D levels (index 0 unused)."""
    D = depth_limit + 1
    P = [0.0] + [p[b - 1] if b <= len(p) else 0.0 for b in range(1, B + 1)]
    T = [[[NEG_INF] * (B + 1) for _ in range(D + 1)] for _ in range(N + 1)]
    Tmax = [[NEG_INF] * (D + 1) for _ in range(N + 1)]
    if N >= 1:
        for d in range(1, D + 1):
            T[1][d][0] = 1.0
            Tmax[1][d] = 1.0
    for n in range(2, N + 1):
        for d in range(2, D + 1):
            for b in range(1, B + 1):
                best = NEG_INF
                for m in range(1, n):
                    tree1, tree2 = T[n - m][d][b - 1], Tmax[m][d - 1]
                    if tree1 == NEG_INF or tree2 == NEG_INF:
                        continue
                    best = max(best, tree1 + P[b] * tree2)
                T[n][d][b] = best
            Tmax[n][d] = max(T[n][d])
    return T, Tmax


def expected_tokens(p: Sequence[float], n: int, B: int, depth_limit: int) -> float:
    """G(n, d) of Sec. 4.1: the best F over trees of exactly n nodes within the bounds."""
    _, Tmax = dynamic_program(p, n, B, depth_limit)
    return Tmax[n][depth_limit + 1]


def depth_of(parent: Sequence[int]) -> int:
    d = [0] * len(parent)
    for i in range(1, len(parent)):
        d[i] = d[parent[i]] + 1
    return max(d)


def max_branch_of(parent: Sequence[int]) -> int:
    fan = [0] * len(parent)
    for i in range(1, len(parent)):
        fan[parent[i]] += 1
    return max(fan) if fan else 0


def speedup(p: Sequence[float], B: int, n: int, d: int, verify_time_n: float, decode_time: float,
            draft_time: float) -> float:
    """Speedup(n, d) = G(n, d) / (t(n) + d c) of Sec. 4.1 with t(n) = verify_time_n / decode_time and
    c = draft_time / decode_time."""
    return expected_tokens(p, n, B, d) / (verify_time_n / decode_time + d * draft_time / decode_time)
