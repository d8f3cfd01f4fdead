"""GPU parity of seq_draft_sample against the CPU checker: drawn tokens bit-exact and in the same
order, except in rows where two neighbouring keys among the first k+1 of the checker's order are
closer than a few fp32 roundings of the key; there the library's tokens must still be a valid
order within that tolerance.  Such rows are counted and must stay rare.  T = 0 is always exact."""
import numpy as np
import pytest
import torch

import oracle
import paper_2402_12374_amd as S
import workloads as W

from gpu_util import DEV, to_dev

pytestmark = pytest.mark.gpu


def key_tolerance(key: float) -> float:
    """Eight roundings of an fp32 key of this magnitude (at least of magnitude 16): the library
    forms logit * (1/T) + g in fp32 from hardware logarithms."""
    return 2.0 ** -20 * max(16.0, abs(key))


def rng_tensor(seed: int, step: int):
    return torch.from_numpy(np.array([seed, step], dtype=np.uint64).view(np.int64)).to(DEV)


def run_draft(logits, n_children, T, seed, step, dtype, k_max, chunks=0):
    S.lib().seqtree_internal_set_draft_chunks(chunks)
    try:
        tokens, _ = S.seq_draft_sample(to_dev(logits, dtype), torch.from_numpy(np.asarray(n_children, np.int32)).to(DEV),
                                       T, rng_tensor(seed, step), k_max)
        torch.cuda.synchronize()
    finally:
        S.lib().seqtree_internal_set_draft_chunks(0)
    return tokens.cpu().numpy()


def key_of(logits_row, T, seed, step, row, x):
    """What the checker's order would report for token x: (class, key)."""
    l = float(logits_row[x])
    g = -np.log(-np.log(oracle.draft_uniform(seed, step, row, x)))
    if np.isnan(l) or l == -np.inf:
        return 1, g
    return 0, l / T + g


def check_draft(logits, n_children, T, seed, step, dtype, k_max, chunks=0, rows=None):
    """Returns the number of rows that were too close to call.  rows: check only these."""
    logits = W.quantize(np.asarray(logits, np.float32), dtype)
    n_children = np.asarray(n_children, np.int32)
    got = run_draft(logits, n_children, T, seed, step, dtype, k_max, chunks)
    assert got.shape == (len(logits), k_max)
    ids = np.arange(len(logits)) if rows is None else np.asarray(rows)
    ref = oracle.draft_sample(logits[ids], n_children[ids], T, seed, step, k_stride=k_max, row_ids=ids)
    flagged = 0
    for j, r in enumerate(ids):
        k = int(n_children[r])
        assert np.all(got[r, k:] == -1), r
        if np.array_equal(got[r], ref.tokens[j]):
            continue
        assert T > 0, (r, got[r], ref.tokens[j])
        # not the checker's order: allowed only as another valid order within the tolerance
        tol = key_tolerance(np.nanmax(np.abs(ref.order_keys[j, : k + 1])))
        assert ref.closest_call(j, k) < tol, (r, got[r], ref.tokens[j], ref.closest_call(j, k))
        toks = got[r, :k]
        assert len(set(toks.tolist())) == k and toks.min() >= 0 and toks.max() < logits.shape[1]
        for pos, x in enumerate(toks):
            cls, key = key_of(logits[r], T, seed, step, int(r), int(x))
            assert cls == ref.order_class[j, pos] and abs(key - ref.order_keys[j, pos]) < tol, (r, pos, x)
        flagged += 1
    return flagged


@pytest.mark.parametrize("V,rows,dtype,T", [
    (2, 3, W.F32, 1.0), (5, 4, W.F32, 0.7), (63, 7, W.BF16, 0.6), (64, 5, W.F32, 0.3),
    (1001, 9, W.BF16, 1.5), (2048, 3, W.F32, 1.0), (2049, 6, W.BF16, 0.6), (5000, 33, W.F32, 0.6),
    (32000, 16, W.BF16, 0.6), (50257, 5, W.F32, 1.0), (128256, 4, W.BF16, 0.6),
])
def test_shapes_dtypes_and_temperatures(V, rows, dtype, T):
    rng = np.random.default_rng(V + rows)
    k_max = min(V, 12)
    flagged = 0
    for rep in range(3):
        logits = 3.0 * rng.standard_normal((rows, V), dtype=np.float32)
        ks = rng.integers(0, k_max + 1, size=rows)
        ks[rep % rows] = k_max
        flagged += check_draft(logits, ks, T, 1000 + rep, rep, dtype, k_max)
    assert flagged <= 1


def test_tree_of_the_benchmark_configuration():
    """C2: every node of the 64-node tree draws as many children as it has, from its own row."""
    v = W.verify_inputs_for("C2")
    fan = np.bincount(v.parent[1:], minlength=len(v.parent)).astype(np.int32)
    assert check_draft(v.draft_logits, fan, v.temperature, 2024, 7, v.dtype, int(fan.max())) <= 1


def test_largest_configuration_on_sampled_rows():
    """C5 (768 rows of 128256 bf16 logits) in the launch shape the benchmark times; the checker
    takes 96 of its rows, among them the root with the largest fan-out."""
    v = W.verify_inputs_for("C5")
    fan = np.bincount(v.parent[1:], minlength=len(v.parent)).astype(np.int32)
    rows = np.unique(np.concatenate([[0, 1, 767], np.random.default_rng(5).choice(768, 93, replace=False)]))
    assert check_draft(v.draft_logits, fan, v.temperature, 99, 3, v.dtype, int(fan.max()), rows=rows) <= 2


@pytest.mark.parametrize("chunks", [1, 2, 3, 5, 16])
def test_any_number_of_workgroups_per_row(chunks):
    rng = np.random.default_rng(chunks)
    for V, rows in ((32000, 6), (128256, 2), (4100, 3)):
        logits = 2.0 * rng.standard_normal((rows, V), dtype=np.float32)
        ks = rng.integers(1, 21, size=rows)
        assert check_draft(logits, ks, 0.8, 5, chunks, W.BF16, 20, chunks=chunks) <= 1


@pytest.mark.parametrize("groups", [1, 7, 64])
def test_workgroups_that_take_many_runs(groups):
    """A grid much smaller than the number of runs: every workgroup works through several rows
    and parts of rows, and finishes rows whose other parts it or others computed earlier."""
    rng = np.random.default_rng(groups)
    logits = 2.0 * rng.standard_normal((40, 9000), dtype=np.float32)
    ks = rng.integers(0, 9, size=40)
    S.lib().seqtree_internal_set_draft_max_groups(groups)
    try:
        for chunks in (1, 3, 5):
            assert check_draft(logits, ks, 0.7, 3, groups, W.BF16, 8, chunks=chunks) <= 1
    finally:
        S.lib().seqtree_internal_set_draft_max_groups(0)


def test_most_children_per_node():
    rng = np.random.default_rng(64)
    logits = 2.0 * rng.standard_normal((5, 9000), dtype=np.float32)
    assert check_draft(logits, [64, 64, 1, 63, 0], 1.0, 64, 64, W.F32, 64) <= 1
    small = rng.standard_normal((3, 64), dtype=np.float32)       # every token of the row is drawn
    assert check_draft(small, [64, 64, 64], 1.0, 65, 1, W.F32, 64) <= 1
    got = run_draft(small, [64, 64, 64], 1.0, 65, 1, W.F32, 64)
    assert all(sorted(r.tolist()) == list(range(64)) for r in got)


def test_zero_temperature_is_exact_with_ties_and_missing_tokens():
    rng = np.random.default_rng(70)
    logits = rng.standard_normal((6, 32000), dtype=np.float32)
    logits[1] = np.round(logits[1] * 2) / 2          # many equal logits: lower id first
    logits[2, ::2] = -np.inf
    logits[3] = 0.0
    logits[3, 100:] = -0.0                           # the two zeros are one value
    logits[4, 5:] = -np.inf                          # fewer finite logits than children
    logits[5, 17] = np.nan
    for dtype in (W.BF16, W.F32):
        for chunks in (0, 1, 3):
            assert check_draft(logits, [20, 20, 20, 20, 20, 20], 0.0, 1, 1, dtype, 20, chunks=chunks) == 0


def test_tokens_without_probability_come_last():
    rng = np.random.default_rng(71)
    logits = rng.standard_normal((4, 3000), dtype=np.float32)
    logits[0, 3:] = -np.inf                          # support of 3, ten children
    logits[1, ::2] = -np.inf
    logits[2, 7] = np.nan
    logits[3, :] = -np.inf                           # no support at all: uniform order
    flagged = check_draft(logits, [10, 10, 10, 10], 0.6, 8, 9, W.F32, 10)
    assert flagged <= 1
    got = run_draft(logits, [10, 10, 10, 10], 0.6, 8, 9, W.F32, 10)
    assert set(got[0, :3].tolist()) == {0, 1, 2} and got[0, 3:].min() >= 3
    assert np.all(got[1] % 2 == 1) and 7 not in got[2]


def test_seed_and_step_live_on_the_device():
    """Full 64-bit seed and step; another step gives another draw, the same step the same one."""
    logits = np.zeros((4, 4096), dtype=np.float32)
    seed, step = 0xFEDCBA9876543210, 0x0123456789ABCDEF
    assert check_draft(logits, [4, 4, 4, 4], 1.0, seed, step, W.F32, 4) == 0
    a = run_draft(logits, [4, 4, 4, 4], 1.0, seed, step, W.F32, 4)
    b = run_draft(logits, [4, 4, 4, 4], 1.0, seed, step + 1, W.F32, 4)
    assert np.array_equal(a, run_draft(logits, [4, 4, 4, 4], 1.0, seed, step, W.F32, 4))
    assert not np.array_equal(a, b)
    # advancing the step on the device between two launches of the same arguments
    dl, nc, rng = to_dev(logits, W.F32), torch.full((4,), 4, dtype=torch.int32, device=DEV), rng_tensor(seed, step)
    first, ws = S.seq_draft_sample(dl, nc, 1.0, rng, 4)
    first = first.clone()
    rng[1] += 1
    second, _ = S.seq_draft_sample(dl, nc, 1.0, rng, 4, workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(first.cpu().numpy(), a) and np.array_equal(second.cpu().numpy(), b)


def test_first_children_follow_the_draft_distribution():
    """Chi-square of the first drawn token against softmax(logits / T), on the GPU's own draws."""
    from scipy import stats
    from scipy.special import softmax
    logits = np.float32([0.3, -1.2, 2.0, 0.0, 1.1, -0.4, 0.9, -2.5, 0.5, 0.1])
    rows = 1024
    counts = np.zeros(10)
    for step in range(20):
        got = run_draft(np.tile(logits, (rows, 1)), np.full(rows, 1), 0.7, 77, step, W.F32, 1)
        counts += np.bincount(got[:, 0], minlength=10)
    expected = softmax(logits.astype(np.float64) / 0.7) * rows * 20
    assert stats.chisquare(counts, expected).pvalue > 1e-3


def test_bad_arguments_are_refused_on_the_gpu_box_too():
    logits = torch.zeros((2, 16), dtype=torch.float32, device=DEV)
    nc = torch.ones(2, dtype=torch.int32, device=DEV)
    with pytest.raises(S.SeqTreeError) as e:
        S.seq_draft_sample(logits, nc, 1.0, rng_tensor(0, 0), 65)
    assert e.value.code == S.SEQ_ERR_SHAPE
    with pytest.raises(S.SeqTreeError) as e:
        S.seq_draft_sample(logits, nc, -1.0, rng_tensor(0, 0), 4)
    assert e.value.code == S.SEQ_ERR_TEMPERATURE
