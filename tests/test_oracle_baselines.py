"""Pins for the CPU checker of the baseline verification algorithms (Sec. 2.2: SpecInfer; naive /
top-k sampling).

Held against: the theorem that both emit the target distribution (exhaustive enumeration over
every tuple of children drawn WITH replacement for SpecInfer; a scan over the uniform for
top-k); the two numbers the paper prints for its counter-examples; the one-child case, where
SpecInfer and Algorithm 2 coincide with the already pinned checker of Algorithm 2; and the closed
relation between the two algorithms' second accept ratio.
"""
import itertools
import json
import os

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

import oracle
import workloads as W

GOLDEN = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_worked_examples.json")))
ALMOST_ONE = np.float32(1.0 - 2.0 ** -24)


def logits_of(p):
    with np.errstate(divide="ignore"):
        return np.log(np.asarray(p, dtype=np.float64)).astype(np.float32)


def star(P, Q, tokens, uniforms=None):
    k = len(tokens)
    parent = W.star_tree(k + 1)
    tl = np.tile(logits_of(P), (k + 1, 1))
    dl = np.tile(logits_of(Q), (k + 1, 1))
    tok = np.zeros(k + 1, dtype=np.int32)
    tok[1:] = tokens
    un = np.full(k + 1, ALMOST_ONE, dtype=np.float32) if uniforms is None else np.asarray(uniforms, np.float32)
    return tl, dl, tok, parent, un


def run(algorithm, inputs, T=1.0):
    tl, dl, tok, parent, un = inputs
    return oracle.verify_baseline(algorithm, tl, dl, tok, parent, T, un)


def seen(p):
    """The distribution the checker itself sees: softmax of the float32 log-probabilities."""
    return sp_softmax(logits_of(p).astype(np.float64))


def residual_after(P, Q, rejections):
    R = np.array(P, dtype=np.float64)
    for _ in range(rejections):
        R = np.maximum(R - Q, 0.0)
        R /= R.sum()
    return R


@pytest.mark.parametrize("k", [1, 2, 3])
def test_specinfer_emits_the_target_distribution(k):
    """Every k-tuple of children drawn independently from Q (repeats allowed): the accept
    probabilities are the checker's ratios, the bonus law is the residual after k rejections."""
    rng = np.random.default_rng(20 + k)
    V = 6
    P, Q = seen(rng.dirichlet(np.ones(V))), seen(rng.dirichlet(np.ones(V)))
    out = np.zeros(V)
    for tup in itertools.product(range(V), repeat=k):
        pr = float(np.prod([Q[s] for s in tup]))
        res = run(oracle.SPECINFER, star(P, Q, tup))
        alive = 1.0                                              # uniforms just below 1 reject everything rejectable
        for rec in res.records:
            a = min(1.0, rec[5])
            out[int(rec[1])] += pr * alive * a
            alive *= 1.0 - a
        if alive > 0.0:
            assert res.path == [] and len(res.records) == k
            out += pr * alive * residual_after(P, Q, k)
    np.testing.assert_allclose(out, P, atol=1e-12)


def test_specinfer_bonus_is_drawn_from_the_residual():
    rng = np.random.default_rng(31)
    V = 7
    P, Q = seen(rng.dirichlet(np.ones(V))), seen(rng.dirichlet(np.ones(V)))
    tokens = (2, 2, 5)                                           # a repeated child: allowed with replacement
    R = residual_after(P, Q, 3)
    cdf = np.cumsum(R)
    for u0 in (0.0, 0.1, 0.37, 0.5, 0.81, 0.999):
        un = np.array([u0, ALMOST_ONE, ALMOST_ONE, ALMOST_ONE], dtype=np.float32)
        res = run(oracle.SPECINFER, star(P, Q, tokens, un))
        if all(rec[5] < 1 for rec in res.records):
            assert res.bonus_token == int(np.searchsorted(cdf, np.float32(u0) * cdf[-1], side="right"))


def test_cover_counter_example_of_the_paper():
    """Q = [0.5, 0.5], P = [1, 0], two children: SpecInfer rejects both with probability 0.25
    (the printed figure) -- whenever both children are the token the target never emits."""
    ex = GOLDEN["cover_counterexample"]
    P, Q = ex["P"], ex["Q"]
    reject_both = 0.0
    for tup in itertools.product(range(2), repeat=2):
        pr = Q[tup[0]] * Q[tup[1]]
        for u in (0.0, 0.3, 0.9):                                # the outcome does not depend on the uniforms here
            un = np.array([0.5, u, u], dtype=np.float32)
            res = run(oracle.SPECINFER, star(P, Q, tup, un))
            rejected = res.path == []
            assert rejected == (tup == (1, 1))
        reject_both += pr * (tup == (1, 1))
    assert reject_both == pytest.approx(ex["specinfer_reject_both_probability"])


def test_optimal_transport_counter_example_of_the_paper():
    """P = Q = [0.6, 0.4], one child (the top-1 token): top-k sampling accepts with probability
    0.6 (the printed figure), SpecInfer and Algorithm 2 always."""
    ex = GOLDEN["optimal_transport_counterexample"]
    P, Q = ex["P"], ex["Q"]
    us = (np.arange(1000) + 0.5) / 1000
    accepted = 0
    for u in us:
        un = np.array([u, 0.5], dtype=np.float32)
        res = run(oracle.TOPK, star(P, Q, (0,), un))
        accepted += res.path == [1]
        if res.path == []:
            assert res.bonus_token == 1
    assert accepted / len(us) == pytest.approx(ex["topk_acceptance"], abs=1e-3)
    for u in (0.0, 0.5, 0.999):
        un = np.array([0.2, u], dtype=np.float32)
        assert run(oracle.SPECINFER, star(P, Q, (0,), un)).path == [1]


def test_topk_emits_a_sample_of_the_target_whatever_the_tree():
    rng = np.random.default_rng(41)
    V = 9
    parent = np.array([-1, 0, 0, 1, 1, 2], dtype=np.int32)
    tl = rng.standard_normal((6, V)).astype(np.float32)
    dl = rng.standard_normal((6, V)).astype(np.float32)
    tok = np.array([0, 3, 5, 1, 3, 8], dtype=np.int32)
    P0 = sp_softmax(tl[0].astype(np.float64) / 0.7)
    cdf = np.cumsum(P0)
    counts = np.zeros(V)
    us = (np.arange(4000) + 0.5) / 4000
    for u in us:
        un = np.full(6, 0.5, dtype=np.float32)
        un[0] = u
        res = oracle.verify_baseline(oracle.TOPK, tl, dl, tok, parent, 0.7, un)
        first = tok[res.path[0]] if res.path else res.bonus_token
        assert first == int(np.searchsorted(cdf, np.float32(u) * cdf[-1], side="right"))
        counts[first] += 1
        # the walk goes on exactly while the drawn token is among the children
        assert (len(res.path) >= 1) == (first in (3, 5))
    np.testing.assert_allclose(counts / len(us), P0, atol=2e-3)
    # the second draw uses the uniform of the node the walk stands on
    un = np.full(6, 0.5, dtype=np.float32)
    un[0] = np.float32((cdf[2] + cdf[3]) / 2)                    # draws token 3 -> node 1
    P1 = np.cumsum(sp_softmax(tl[1].astype(np.float64) / 0.7))
    for u1 in (0.05, 0.5, 0.95):
        un[1] = u1
        res = oracle.verify_baseline(oracle.TOPK, tl, dl, tok, parent, 0.7, un)
        x1 = int(np.searchsorted(P1, np.float32(u1) * P1[-1], side="right"))
        assert res.path[0] == 1
        assert (res.path[1:] == [{1: 3, 3: 4}[x1]]) if x1 in (1, 3) else (res.path[1:] == [] and res.bonus_token == x1)


def test_one_child_per_node_specinfer_is_algorithm_2():
    """With a single child the blue lines of Algorithm 2 never matter for the accept tests, and
    after the rejection the residual is the same: the pinned checker of Algorithm 2 decides."""
    for rep in range(20):
        rng = np.random.default_rng(rep)
        n, V = 6, 12
        parent = W.chain_tree(n)
        tl = (2 * rng.standard_normal((n, V))).astype(np.float32)
        dl = (tl + rng.standard_normal((n, V))).astype(np.float32)
        tok = rng.integers(0, V, size=n).astype(np.int32)
        un = rng.random(n, dtype=np.float32)
        a = oracle.verify_baseline(oracle.SPECINFER, tl, dl, tok, parent, 0.8, un)
        b = oracle.verify(tl, dl, tok, parent, 0.8, un)
        assert a.path == b.path and a.bonus_token == b.bonus_token
        assert [r[5] for r in a.records] == pytest.approx([d.ratio for d in b.decisions], rel=1e-13)


def test_second_ratio_differs_from_algorithm_2_by_the_mass_left():
    """After rejecting token s1, Algorithm 2 renormalises the draft over what is left, SpecInfer
    does not: ratio_SpecInfer(s2) * (1 - Q[s1]) = ratio_Algorithm2(s2) for s2 != s1."""
    rng = np.random.default_rng(51)
    V = 8
    P, Q = seen(rng.dirichlet(np.ones(V))), seen(rng.dirichlet(np.ones(V)))
    for s1, s2 in ((0, 3), (5, 1), (2, 7)):
        a = run(oracle.SPECINFER, star(P, Q, (s1, s2)))
        b = oracle.verify(*star(P, Q, (s1, s2))[:4], 1.0, star(P, Q, (s1, s2))[4])
        if len(a.records) == 2 and len(b.decisions) == 2:
            assert a.records[1][5] * (1 - Q[s1]) == pytest.approx(b.decisions[1].ratio, rel=1e-12)


def test_zero_temperature_walks_along_the_arg_max():
    rng = np.random.default_rng(61)
    n, V = 7, 10
    parent = np.array([-1, 0, 0, 1, 1, 3, 3], dtype=np.int32)
    tl = rng.standard_normal((n, V)).astype(np.float32)
    dl = rng.standard_normal((n, V)).astype(np.float32)
    tok = np.zeros(n, dtype=np.int32)
    tok[2] = np.argmax(tl[0]); tok[1] = (tok[2] + 1) % V
    un = rng.random(n, dtype=np.float32)
    for alg in (oracle.SPECINFER, oracle.TOPK):
        res = oracle.verify_baseline(alg, tl, dl, tok, parent, 0.0, un)
        assert res.path == [2] and res.bonus_token == int(np.argmax(tl[2]))
