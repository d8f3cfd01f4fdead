"""Pins for the CPU checker of the drafter's ordered draw (sampling without replacement by
exponential sort, Sec. 3.2.1 and the implementation details of Sec. 4.1).

The checker sorts keys; none of these tests sorts keys.  They hold it against: the published
known answers of the Philox4x32-10 generator; the uniform and exponential laws of its variates;
the closed form of an ordered draw without replacement (each next token in proportion to its
probability among those left, uniform once the support is used up) by chi-square over every
ordered tuple; the arg-max/top-k limit at T = 0 through numpy's own sort; and invariances.
"""
import itertools

import numpy as np
import pytest
from scipy import stats
from scipy.special import softmax as sp_softmax

import oracle


# --------------------------------------------------------------------------------------
# the generator
# --------------------------------------------------------------------------------------
# Known answers of Philox4x32-10 from the reference test vectors published with the generator
# (Salmon et al., SC'11): counter, key -> output.
PHILOX_KNOWN_ANSWERS = [
    ((0x00000000, 0x00000000, 0x00000000, 0x00000000), (0x00000000, 0x00000000),
     (0x6627E8D5, 0xE169C58D, 0xBC57AC4C, 0x9B00DBD8)),
    ((0xFFFFFFFF, 0xFFFFFFFF, 0xFFFFFFFF, 0xFFFFFFFF), (0xFFFFFFFF, 0xFFFFFFFF),
     (0x408F276D, 0x41C83B0E, 0xA20BC7C6, 0x6D5451FD)),
    ((0x243F6A88, 0x85A308D3, 0x13198A2E, 0x03707344), (0xA4093822, 0x299F31D0),
     (0xD16CFE09, 0x94FDCCEB, 0x5001E420, 0x24126EA1)),
]


@pytest.mark.parametrize("counter,key,expected", PHILOX_KNOWN_ANSWERS)
def test_philox_known_answers(counter, key, expected):
    assert tuple(int(v) for v in oracle.philox4x32_10(counter, key)) == expected


def test_token_takes_its_own_word_of_its_own_block():
    seed, step, row = 0x0123456789ABCDEF, 0xFEDCBA9876543210, 37
    for x in (0, 1, 2, 3, 4, 7, 1001, 128255):
        out = oracle.philox4x32_10([x // 4, row, step & 0xFFFFFFFF, step >> 32],
                                   [seed & 0xFFFFFFFF, seed >> 32])
        w = ((int(out[x % 4]) >> 9) + 0.5) * 2.0 ** -23
        assert oracle.draft_uniform(seed, step, row, x) == w


def test_variates_are_uniform_and_exponential():
    rng = np.random.default_rng(5)
    w = np.array([oracle.draft_uniform(int(rng.integers(1 << 62)), int(rng.integers(1 << 62)),
                                       int(rng.integers(1024)), int(rng.integers(128256)))
                  for _ in range(20000)])
    assert w.min() > 0.0 and w.max() < 1.0
    assert np.all(w.astype(np.float32).astype(np.float64) == w)       # exact in fp32
    assert stats.kstest(w, "uniform").pvalue > 1e-3
    assert stats.kstest(-np.log(w), "expon").pvalue > 1e-3
    # neighbouring tokens, rows and steps are not correlated
    a = np.array([[oracle.draft_uniform(9, s, r, x) for x in range(64)] for s in range(4) for r in range(4)])
    for shifted in (a[:, 1:], ):
        assert abs(np.corrcoef(a[:, :-1].ravel(), shifted.ravel())[0, 1]) < 0.1
    assert abs(np.corrcoef(a[0], a[1])[0, 1]) < 0.4 and abs(np.corrcoef(a[0], a[4])[0, 1]) < 0.4


# --------------------------------------------------------------------------------------
# the law of the ordered draw
# --------------------------------------------------------------------------------------
def ordered_draw_probability(q, tup):
    """Closed form: the next token is drawn in proportion to q among the tokens not drawn yet;
    once the tokens of non-zero q are used up, uniformly among the rest."""
    q = np.asarray(q, dtype=np.float64)
    prob, left = 1.0, 1.0
    drawn = []
    for s in tup:
        support_left = sum(1 for t in range(len(q)) if q[t] > 0 and t not in drawn)
        if support_left:
            prob *= q[s] / left
            left -= q[s]
        else:
            prob *= 1.0 / (len(q) - len(drawn))
        if prob == 0.0:
            return 0.0
        drawn.append(s)
    return prob


def chi_square_of_tuples(logits, k, T, trials, seed):
    logits = np.asarray(logits, dtype=np.float32)
    V = len(logits)
    res = oracle.draft_sample(np.tile(logits, (trials, 1)), np.full(trials, k), T, seed, 3)
    with np.errstate(divide="ignore"):
        q = sp_softmax(logits.astype(np.float64) / T)
    tuples = list(itertools.permutations(range(V), k))
    expected = np.array([ordered_draw_probability(q, t) for t in tuples])
    assert abs(expected.sum() - 1.0) < 1e-12
    index = {t: i for i, t in enumerate(tuples)}
    counts = np.zeros(len(tuples))
    for row in res.tokens:
        counts[index[tuple(int(v) for v in row[:k])]] += 1
    assert counts[expected == 0].sum() == 0          # impossible tuples never appear
    live = expected > 0
    return stats.chisquare(counts[live], expected[live] * trials).pvalue


def test_first_token_follows_the_tempered_softmax():
    logits = [0.3, -1.2, 2.0, 0.0, 1.1, -0.4, 0.9, -2.5]
    for T, seed in ((0.6, 11), (1.0, 12), (2.5, 13)):
        assert chi_square_of_tuples(logits, 1, T, 40000, seed) > 1e-3


def test_ordered_tuples_follow_sampling_without_replacement():
    logits = [1.0, -0.5, 0.2, 2.2, -1.0]
    assert chi_square_of_tuples(logits, 3, 0.7, 120000, 21) > 1e-3
    assert chi_square_of_tuples(logits, 5, 1.3, 240000, 22) > 1e-3    # whole permutations


def test_a_planted_mistake_in_the_law_is_caught():
    """The same statistic rejects a draw WITH replacement-like law (second token independent of
    the first apart from being different) -- the test above is not vacuous."""
    logits = np.array([1.0, -0.5, 0.2, 2.2, -1.0], dtype=np.float32)
    q = sp_softmax(logits.astype(np.float64) / 0.7)
    res = oracle.draft_sample(np.tile(logits, (60000, 1)), np.full(60000, 2), 0.7, 23, 3)
    tuples = list(itertools.permutations(range(5), 2))
    wrong = np.array([q[a] * q[b] for a, b in tuples])
    wrong /= wrong.sum()
    counts = np.array([np.sum((res.tokens[:, 0] == a) & (res.tokens[:, 1] == b)) for a, b in tuples])
    assert stats.chisquare(counts, wrong * 60000).pvalue < 1e-6


def test_zero_probability_tokens_come_last_in_uniform_order():
    ninf = -np.inf
    logits = [0.5, ninf, 1.5, ninf, ninf]          # support of two tokens, three without mass
    assert chi_square_of_tuples(logits, 4, 0.8, 120000, 31) > 1e-3
    res = oracle.draft_sample(np.tile(np.float32(logits), (2000, 1)), np.full(2000, 5), 0.8, 32, 0)
    assert np.all(np.isin(res.tokens[:, :2], [0, 2])) and np.all(np.isin(res.tokens[:, 2:], [1, 3, 4]))
    nan_row = np.array([[0.5, np.nan, 1.5, ninf, ninf]], dtype=np.float32)   # NaN reads as -inf
    a = oracle.draft_sample(nan_row, [5], 0.8, 33, 7).tokens
    b = oracle.draft_sample(np.float32([logits]), [5], 0.8, 33, 7).tokens
    assert np.array_equal(a, b)


# --------------------------------------------------------------------------------------
# special cases and invariances
# --------------------------------------------------------------------------------------
def test_zero_temperature_is_top_k_by_numpy_sort():
    rng = np.random.default_rng(41)
    logits = rng.standard_normal((6, 300)).astype(np.float32)
    logits[1, 10:20] = logits[1, 5]                 # ties: lower id first
    logits[2, ::3] = -np.inf
    logits[3] = 0.25                                # all equal
    ks = np.array([1, 12, 7, 9, 0, 300])
    res = oracle.draft_sample(logits, ks, 0.0, 1, 2, k_stride=300)
    for r, k in enumerate(ks):
        order = np.lexsort((np.arange(300), -logits[r].astype(np.float64)))
        assert np.array_equal(res.tokens[r, :k], order[:k]), r
        assert np.all(res.tokens[r, k:] == -1)
    assert np.array_equal(res.tokens[5], np.lexsort((np.arange(300), -logits[5].astype(np.float64))))


def test_seed_and_step_do_not_matter_at_zero_temperature():
    logits = np.random.default_rng(42).standard_normal((2, 50)).astype(np.float32)
    a = oracle.draft_sample(logits, [5, 5], 0.0, 1, 2).tokens
    b = oracle.draft_sample(logits, [5, 5], 0.0, 99, 77).tokens
    assert np.array_equal(a, b)


def test_shorter_draw_is_a_prefix_and_full_draw_is_a_permutation():
    logits = np.random.default_rng(43).standard_normal((3, 40)).astype(np.float32)
    full = oracle.draft_sample(logits, [40, 40, 40], 0.9, 5, 6).tokens
    for r in range(3):
        assert sorted(full[r].tolist()) == list(range(40))
    for k in (1, 2, 17):
        part = oracle.draft_sample(logits, [k, k, k], 0.9, 5, 6).tokens
        assert np.array_equal(part[:, :k], full[:, :k])


def test_adding_a_constant_to_a_row_changes_nothing():
    logits = np.random.default_rng(44).integers(-8, 8, size=(2, 64)).astype(np.float32)
    a = oracle.draft_sample(logits, [6, 6], 0.5, 7, 8).tokens       # T = 0.5: exact in floating point
    b = oracle.draft_sample(logits + np.float32(16.0), [6, 6], 0.5, 7, 8).tokens
    assert np.array_equal(a, b)


def test_rows_and_steps_draw_independently_and_reproducibly():
    logits = np.zeros((8, 1000), dtype=np.float32)                  # flat: the noise decides
    a = oracle.draft_sample(logits, np.full(8, 3), 1.0, 50, 0).tokens
    assert len({tuple(r) for r in a.tolist()}) == 8                 # every row its own draw
    assert np.array_equal(a, oracle.draft_sample(logits, np.full(8, 3), 1.0, 50, 0).tokens)
    assert not np.array_equal(a, oracle.draft_sample(logits, np.full(8, 3), 1.0, 50, 1).tokens)
    assert not np.array_equal(a, oracle.draft_sample(logits, np.full(8, 3), 1.0, 51, 0).tokens)
    other = logits.copy()
    other[:4] = np.random.default_rng(45).standard_normal((4, 1000))
    b = oracle.draft_sample(other, np.full(8, 3), 1.0, 50, 0).tokens
    assert np.array_equal(a[4:], b[4:])                             # a row depends on itself only
    c = oracle.draft_sample(logits[[5, 2]], [3, 3], 1.0, 50, 0, row_ids=[5, 2]).tokens
    assert np.array_equal(c, a[[5, 2]])                             # single rows of a larger call


def test_keys_reported_in_descending_order_with_their_gap():
    logits = np.random.default_rng(46).standard_normal((4, 500)).astype(np.float32)
    res = oracle.draft_sample(logits, [4, 4, 4, 4], 0.6, 1, 1)
    for r in range(4):
        keys = res.order_keys[r, :5]
        assert np.all(np.diff(keys) <= 0)
        assert res.closest_call(r, 4) == pytest.approx(np.min(-np.diff(keys)))
        # the key of a drawn token is its tempered logit plus the Gumbel variate of its uniform
        x = int(res.tokens[r, 0])
        g = -np.log(-np.log(oracle.draft_uniform(1, 1, r, x)))
        assert keys[0] == pytest.approx(float(logits[r, x]) / 0.6 + g, rel=1e-14)


def test_bad_arguments_are_refused():
    logits = np.zeros((2, 10), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.draft_sample(logits, [11, 1], 1.0, 0, 0, k_stride=16)    # more children than tokens
    with pytest.raises(ValueError):
        oracle.draft_sample(logits, [1, 1], -1.0, 0, 0)
    with pytest.raises(ValueError):
        oracle.draft_sample(logits, [-1, 1], 1.0, 0, 0)
