"""Pins for the CPU checker of the verification walk (Algorithm 2 applied down the tree).

None of these re-types the checker's update rule: they use the theorem that the emitted token
follows the target distribution (exhaustive enumeration and a chi-square test), the two
robustness properties with their closed forms, the paper's two-token worked examples, and
special cases that reduce to routines written here independently.
"""
import itertools
import json
import os

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

import oracle
import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_worked_examples.json")
ALMOST_ONE = np.float32(1.0 - 2.0 ** -24)  # largest float32 below 1: rejects unless ratio >= 1


def logits_of(p):
    p = np.asarray(p, dtype=np.float64)
    with np.errstate(divide="ignore"):
        return np.log(p).astype(np.float32)


def star_inputs(P, Q, tokens, uniforms=None):
    """Root with len(tokens) children, all leaves."""
    k = len(tokens)
    V = len(P)
    parent = W.star_tree(k + 1)
    tl = np.tile(logits_of(P), (k + 1, 1))
    dl = np.tile(logits_of(Q), (k + 1, 1))
    tok = np.zeros(k + 1, dtype=np.int32)
    tok[1:] = tokens
    un = np.full(k + 1, ALMOST_ONE, dtype=np.float32) if uniforms is None else np.asarray(uniforms, np.float32)
    return tl, dl, tok, parent, un


def ordered_draw_probability(Q, tup):
    """Probability of drawing the ordered tuple by sequential sampling without replacement from
    Q, continuing uniformly over the not-yet-drawn tokens once Q's support is exhausted
    (the sampling scheme of Sec. 3.2.1)."""
    Q = np.asarray(Q, dtype=np.float64)
    V = len(Q)
    prob, used_mass, used = 1.0, 0.0, set()
    support = int((Q > 0).sum())
    for s in tup:
        if len([t for t in used if Q[t] > 0]) < support:
            prob *= Q[s] / (1.0 - used_mass)
        else:
            prob *= 1.0 / (V - len(used))
        if prob == 0.0:
            return 0.0
        used.add(s)
        used_mass += Q[s]
    return prob


def output_distribution_by_enumeration(P, Q, k):
    """Law of the emitted token when the root has k children: sum over every ordered k-tuple of
    distinct tokens; per tuple the checker's ratios give the accept probabilities and its final
    residual gives the bonus law."""
    V = len(P)
    out = np.zeros(V)
    total_prob = 0.0
    for tup in itertools.permutations(range(V), k):
        pr = ordered_draw_probability(Q, tup)
        if pr == 0.0:
            continue
        total_prob += pr
        res = oracle.verify(*star_inputs(P, Q, tup)[:4], 1.0, star_inputs(P, Q, tup)[4], want_final=True)
        alive = 1.0
        for dec in res.decisions:
            a = min(1.0, dec.ratio)
            out[dec.token] += pr * alive * a
            alive *= 1.0 - a
        if alive > 0.0:
            assert res.path == []
            out += pr * alive * res.final_R
    assert abs(total_prob - 1.0) < 1e-12
    return out


def random_dist(rng, V, zeros=0):
    p = rng.dirichlet(np.ones(V))
    if zeros:
        idx = rng.choice(V, size=zeros, replace=False)
        p[idx] = 0.0
        p /= p.sum()
    # make it exactly representable after log/exp round trip irrelevant: compare with what the
    # checker itself sees, i.e. softmax of the float32 log-probabilities
    return sp_softmax(logits_of(p).astype(np.float64))


@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_exhaustive_enumeration_emits_target_distribution_v8(k):
    rng = np.random.default_rng(10 + k)
    V = 8
    P, Q = random_dist(rng, V), random_dist(rng, V)
    out = output_distribution_by_enumeration(P, Q, k)
    np.testing.assert_allclose(out, P, atol=1e-12)


@pytest.mark.parametrize("k,qzeros,pzeros", [(3, 6, 0), (4, 5, 2), (4, 6, 5)])
def test_exhaustive_enumeration_with_small_draft_support(k, qzeros, pzeros):
    """Draft support smaller than k, or not covering the target's: exercises D[s] <- 0 until
    sum(D) = 0 and the uniform fallback."""
    rng = np.random.default_rng(50 + k + qzeros)
    V = 8
    P, Q = random_dist(rng, V, zeros=pzeros), random_dist(rng, V, zeros=qzeros)
    out = output_distribution_by_enumeration(P, Q, k)
    np.testing.assert_allclose(out, P, atol=1e-12)


def gumbel_children(draft_logits_row, k, T, rng, trials):
    key = draft_logits_row.astype(np.float64)[None, :] / T + rng.gumbel(size=(trials, len(draft_logits_row)))
    return np.argsort(-key, axis=1)[:, :k].astype(np.int32)


def test_chi_square_first_emitted_token_follows_target_million_trials():
    V, trials, T = 8, 1_000_000, 0.8
    rng = np.random.default_rng(2402)
    # two-level tree: root with 3 children, each child with 2 children
    parent = np.array([-1, 0, 0, 0, 1, 1, 2, 2, 3, 3], dtype=np.int32)
    n = len(parent)
    tl = (rng.standard_normal((n, V)) * 1.5).astype(np.float32)
    dl = (tl + rng.standard_normal((n, V))).astype(np.float32)
    tok = np.zeros((trials, n), dtype=np.int32)
    tok[:, 1:4] = gumbel_children(dl[0], 3, T, rng, trials)
    for c, (a, b) in zip((1, 2, 3), ((4, 5), (6, 7), (8, 9))):
        tok[:, [a, b]] = gumbel_children(dl[c], 2, T, rng, trials)
    un = rng.random((trials, n), dtype=np.float32)
    plen, first, bonus = oracle.verify_trials(tl, dl, tok, parent, T, un)
    expected = trials * sp_softmax(tl[0].astype(np.float64) / T)
    counts = np.bincount(first, minlength=V)
    chi2 = float(((counts - expected) ** 2 / expected).sum())
    assert chi2 < 24.32, chi2  # 7 degrees of freedom, alpha = 1e-3
    # second level: given that root child at node 1 was accepted, the next emitted token
    # (token of the accepted grandchild, else the bonus) follows the target at node 1
    sel = (plen >= 1)
    path_first_is_1 = np.zeros(trials, dtype=bool)
    # recover which child was accepted from the first emitted token and the child tokens
    path_first_is_1[sel] = tok[sel, 1] == first[sel]
    idx = np.flatnonzero(path_first_is_1)
    sub_un = un[idx][:, [0, 4, 5]]  # walk restarted at node 1: bonus draw + its two children
    sub_tok = np.zeros((len(idx), 3), dtype=np.int32)
    sub_tok[:, 1:] = tok[idx][:, [4, 5]]
    _, first2, _ = oracle.verify_trials(tl[[1, 4, 5]], dl[[1, 4, 5]], sub_tok,
                                        np.array([-1, 0, 0], dtype=np.int32), T, sub_un)
    exp2 = len(idx) * sp_softmax(tl[1].astype(np.float64) / T)
    chi2b = float(((np.bincount(first2, minlength=V) - exp2) ** 2 / exp2).sum())
    assert chi2b < 24.32, chi2b
    # sanity: the walk does accept sometimes and reject sometimes
    assert 0.05 < (plen > 0).mean() < 0.999


def test_k1_acceptance_is_one_minus_half_l1_distance():
    """Optimal-transport property (Sec. 3.2.2)."""
    rng = np.random.default_rng(7)
    V = 8
    for _ in range(5):
        P, Q = random_dist(rng, V), random_dist(rng, V)
        acc = 0.0
        for s in range(V):
            tl, dl, tok, parent, un = star_inputs(P, Q, [s])
            res = oracle.verify(tl, dl, tok, parent, 1.0, un)
            acc += Q[s] * min(1.0, res.decisions[0].ratio)
        assert abs(acc - (1.0 - 0.5 * np.abs(P - Q).sum())) < 1e-12


def test_reject_mass_lemma_at_later_iterations():
    """Lemma (App. proof of correctness): P(no accept at iteration i) = sum_x max(0, t_i - d_i),
    with t_i, d_i the residual and draft after i-1 rejections."""
    rng = np.random.default_rng(8)
    V = 8
    P, Q = random_dist(rng, V), random_dist(rng, V)
    for rejected in [(3,), (3, 5), (0, 6, 2)]:
        tl, dl, tok, parent, un = star_inputs(P, Q, list(rejected))
        res = oracle.verify(tl, dl, tok, parent, 1.0, un, want_final=True)
        if res.path:  # some ratio >= 1: the forced rejection did not happen, not this case
            continue
        t_i, d_i = res.final_R, res.final_D
        assert abs(d_i.sum() - 1.0) < 1e-12 and abs(t_i.sum() - 1.0) < 1e-12
        assert all(d_i[s] == 0.0 for s in rejected)
        reject = 0.0
        for s in range(V):
            if d_i[s] == 0.0:
                continue
            tl2, dl2, tok2, parent2, un2 = star_inputs(P, Q, list(rejected) + [s])
            r2 = oracle.verify(tl2, dl2, tok2, parent2, 1.0, un2)
            reject += d_i[s] * (1.0 - min(1.0, r2.decisions[-1].ratio))
        assert abs(reject - np.maximum(0.0, t_i - d_i).sum()) < 1e-12


def test_cover_property_support_of_size_k():
    """|supp Q| = k and supp Q contains supp P: some child is accepted within k, whatever the
    uniforms (Sec. 3.2.2, cover property)."""
    rng = np.random.default_rng(9)
    V, k = 8, 4
    supp = [1, 2, 5, 7]
    Q = np.zeros(V); Q[supp] = rng.dirichlet(np.ones(k))
    P = np.zeros(V); P[[2, 7]] = [0.3, 0.7]
    P, Q = sp_softmax(logits_of(P).astype(np.float64)), sp_softmax(logits_of(Q).astype(np.float64))
    for tup in itertools.permutations(supp, k):
        res = oracle.verify(*star_inputs(P, Q, tup)[:4], 1.0, star_inputs(P, Q, tup)[4])
        assert len(res.path) == 1, tup
        assert P[res.decisions[-1].token] > 0


def test_cover_property_k_equals_vocab_uses_uniform_fallback():
    rng = np.random.default_rng(11)
    V = 5
    P = rng.dirichlet(np.ones(V))
    Q = np.zeros(V); Q[[0, 3]] = [0.4, 0.6]          # support of size 2, does not cover P
    P, Q = sp_softmax(logits_of(P).astype(np.float64)), sp_softmax(logits_of(Q).astype(np.float64))
    seen_fallback = False
    for head in itertools.permutations([0, 3]):
        for tail in itertools.permutations([1, 2, 4]):
            tup = list(head) + list(tail)
            res = oracle.verify(*star_inputs(P, Q, tup)[:4], 1.0, star_inputs(P, Q, tup)[4])
            assert len(res.path) == 1, tup
            seen_fallback |= res.fallbacks > 0
    assert seen_fallback


def test_paper_worked_examples():
    g = json.load(open(GOLDEN))
    ex = g["cover_counterexample"]
    P, Q = ex["P"], ex["Q"]
    # Sequoia accepts within two children for either drafting order, for every uniform
    acc = 0.0
    for tup in ([0, 1], [1, 0]):
        pr = ordered_draw_probability(Q, tup)
        for u in (0.0, 0.3, float(ALMOST_ONE)):
            tl, dl, tok, parent, _ = star_inputs(P, Q, tup)
            res = oracle.verify(tl, dl, tok, parent, 1.0, np.array([0.5, u, u], np.float32))
            assert len(res.path) == 1 and tok[res.path[0]] == 0
        acc += pr
    assert acc == ex["sequoia_acceptance_within_2"]
    # the order (1, 0): first ratio 0 (rejected), then the residual is one-hot and so is the
    # renormalised draft: ratio exactly 1
    tl, dl, tok, parent, un = star_inputs(P, Q, [1, 0])
    res = oracle.verify(tl, dl, tok, parent, 1.0, un)
    assert [d.ratio for d in res.decisions] == [0.0, 1.0]
    ex = g["optimal_transport_counterexample"]
    P, Q = np.array(ex["P"]), np.array(ex["Q"])
    acc = 0.0
    for s in range(2):
        tl, dl, tok, parent, un = star_inputs(P, Q, [s])
        acc += Q[s] * min(1.0, oracle.verify(tl, dl, tok, parent, 1.0, un).decisions[0].ratio)
    assert abs(acc - ex["optimal_transport_acceptance"]) < 1e-7


def test_residual_support_never_grows_and_rejected_tokens_leave_it():
    rng = np.random.default_rng(12)
    V = 8
    P, Q = random_dist(rng, V, zeros=2), random_dist(rng, V)
    prev_support = set(np.flatnonzero(P > 0))
    order = [int(x) for x in np.argsort(-(Q - P))]  # most over-drafted first: these get rejected
    for k in range(1, 6):
        tl, dl, tok, parent, un = star_inputs(P, Q, order[:k])
        res = oracle.verify(tl, dl, tok, parent, 1.0, un, want_final=True)
        if res.path:
            break
        supp = set(np.flatnonzero(res.final_R > 0))
        assert supp <= prev_support
        assert not (supp & set(order[:k]))
        prev_support = supp


def test_greedy_is_argmax_matching():
    rng = np.random.default_rng(13)
    for trial in range(30):
        n, V = 12, 9
        parent = W.random_topological_tree(n, rng)
        tl = rng.standard_normal((n, V)).astype(np.float32)
        dl = rng.standard_normal((n, V)).astype(np.float32)
        if trial % 3 == 0:
            tl[:, 3] = tl[:, 5] = 4.0  # ties: lowest index wins
        tok = rng.integers(0, V, size=n).astype(np.int32)
        un = rng.random(n, dtype=np.float32)
        res = oracle.verify(tl, dl, tok, parent, 0.0, un)
        # independent routine
        v, path = 0, []
        while True:
            top = int(np.argmax(tl[v]))
            nxt = [c for c in range(v + 1, n) if parent[c] == v and tok[c] == top]
            if not nxt:
                break
            path.append(nxt[0])
            v = nxt[0]
        assert res.path == path
        assert res.bonus_token == int(np.argmax(tl[v]))


def test_chain_tree_is_sequence_speculative_decoding():
    """k = 1 everywhere: accept while u < p(x)/q(x); on the first rejection emit a sample of
    norm(max(p - q, 0)); if everything is accepted emit a sample of the last target row."""
    rng = np.random.default_rng(14)
    T = 0.7
    for _ in range(40):
        n, V = 6, 7
        parent = W.chain_tree(n)
        tl = (rng.standard_normal((n, V)) * 2).astype(np.float32)
        dl = (tl + rng.standard_normal((n, V))).astype(np.float32)
        tok = rng.integers(0, V, size=n).astype(np.int32)
        un = rng.random(n, dtype=np.float32)
        res = oracle.verify(tl, dl, tok, parent, T, un)
        path, law = [], None
        for c in range(1, n):
            p = sp_softmax(tl[c - 1].astype(np.float64) / T)
            q = sp_softmax(dl[c - 1].astype(np.float64) / T)
            if float(un[c]) < p[tok[c]] / q[tok[c]]:
                path.append(c)
            else:
                law = np.maximum(p - q, 0.0)
                break
        if law is None:
            law = sp_softmax(tl[n - 1].astype(np.float64) / T)
        cdf = np.cumsum(law)
        bonus = int(np.searchsorted(cdf, float(un[0]) * cdf[-1], side="right"))
        assert res.path == path
        if res.bonus_margin > 1e-9:
            assert res.bonus_token == bonus


def test_single_node_samples_from_target_by_inverse_cdf():
    rng = np.random.default_rng(15)
    V, T = 11, 1.3
    tl = rng.standard_normal((1, V)).astype(np.float32)
    dl = rng.standard_normal((1, V)).astype(np.float32)
    p = sp_softmax(tl[0].astype(np.float64) / T)
    cdf = np.cumsum(p)
    hits = np.zeros(V)
    grid = (np.arange(4000) + 0.5) / 4000
    for u in grid:
        res = oracle.verify(tl, dl, np.zeros(1, np.int32), np.array([-1], np.int32), T,
                            np.array([u], np.float32))
        assert res.path == []
        if res.bonus_margin > 1e-9:
            assert res.bonus_token == int(np.searchsorted(cdf, float(np.float32(u)), side="right"))
        hits[res.bonus_token] += 1
    np.testing.assert_allclose(hits / len(grid), p, atol=1.0 / 2000)


def test_strict_inequality_and_ratio_above_one():
    # P == Q: ratio exactly 1 -> every u in [0,1) accepts; ratio 0 -> even u = 0 rejects
    P = np.array([0.25, 0.25, 0.5])
    tl, dl, tok, parent, _ = star_inputs(P, P, [2])
    for u in (0.0, float(ALMOST_ONE)):
        res = oracle.verify(tl, dl, tok, parent, 1.0, np.array([0.1, u], np.float32))
        assert res.path == [1] and res.decisions[0].ratio == 1.0
    tl, dl, tok, parent, _ = star_inputs([1.0, 0.0, 0.0], [0.5, 0.5, 0.0], [1])
    res = oracle.verify(tl, dl, tok, parent, 1.0, np.array([0.1, 0.0], np.float32))
    assert res.path == [] and res.decisions[0].ratio == 0.0 and res.bonus_token == 0


def test_zero_draft_probability_conventions():
    # token outside the draft support: accepted iff the residual has mass there
    tl, dl, tok, parent, un = star_inputs([0.5, 0.5, 0.0], [1.0, 0.0, 0.0], [1])
    res = oracle.verify(tl, dl, tok, parent, 1.0, un)
    assert res.path == [1] and np.isinf(res.decisions[0].ratio)
    tl, dl, tok, parent, un = star_inputs([0.5, 0.5, 0.0], [1.0, 0.0, 0.0], [2])
    res = oracle.verify(tl, dl, tok, parent, 1.0, un)
    assert res.path == [] and res.decisions[0].ratio == 0.0
    # duplicate sibling: the second copy has D = 0 and R = 0 -> rejected
    tl, dl, tok, parent, un = star_inputs([0.1, 0.9, 0.0], [0.8, 0.1, 0.1], [0, 0])
    res = oracle.verify(tl, dl, tok, parent, 1.0, un)
    assert res.path == [] and res.decisions[1].ratio == 0.0


def test_temperature_tempers_both_models():
    rng = np.random.default_rng(16)
    V = 6
    tl = rng.standard_normal((2, V)).astype(np.float32) * 3
    dl = rng.standard_normal((2, V)).astype(np.float32) * 3
    parent = np.array([-1, 0], np.int32)
    for T in (0.2, 0.6, 1.0, 2.5):
        p = sp_softmax(tl[0].astype(np.float64) / T)
        q = sp_softmax(dl[0].astype(np.float64) / T)
        for s in range(V):
            res = oracle.verify(tl, dl, np.array([0, s], np.int32), parent, T,
                                np.array([0.5, 0.5], np.float32))
            assert abs(res.decisions[0].ratio - p[s] / q[s]) < 1e-12 * max(1.0, p[s] / q[s])


def test_bonus_draw_never_emits_a_zero_probability_token():
    # u = 0 with a leading zero-mass token: the first token whose cumulative mass EXCEEDS 0
    tl = logits_of([0.0, 0.5, 0.5])[None, :]
    res = oracle.verify(tl, tl, np.zeros(1, np.int32), np.array([-1], np.int32), 1.0,
                        np.array([0.0], np.float32))
    assert res.bonus_token == 1
    # u at an interior CDF edge belongs to the next token (half-open intervals [lo, hi))
    tl = np.zeros((1, 2), np.float32)  # P = [0.5, 0.5] exactly
    res = oracle.verify(tl, tl, np.zeros(1, np.int32), np.array([-1], np.int32), 1.0,
                        np.array([0.5], np.float32))
    assert res.bonus_token == 1
