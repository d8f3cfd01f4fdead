"""seq_top_p_filter.  The checker is the definition (sort by probability, shortest prefix reaching
top_p); it is pinned by closed forms (uniform and geometric rows, top_p = 1, T = 0) and by the
defining properties on random rows.  The library must keep the same tokens, or -- where the cut
falls within fp32 precision of top_p or between probabilities that agree to fp32 precision --
another set that has the defining properties within that precision."""
import numpy as np
import pytest

import oracle
import paper_2402_12374_amd as S
from paper_2402_12374_amd import binding as B
import workloads as W


def test_uniform_and_geometric_rows_have_closed_forms():
    V = 50
    out, prob, keep = oracle.top_p_filter(np.zeros((1, V), np.float32), 0.3, 1.0)
    assert keep[0].tolist() == [i < 15 for i in range(V)]                # 15/50 = 0.3 exactly reached by the first 15 ids
    out, prob, keep = oracle.top_p_filter(np.zeros((1, V), np.float32), 0.301, 1.0)
    assert keep[0].sum() == 16
    # probabilities 1/2, 1/4, 1/8, ...: top_p = 0.9 needs 4 tokens (0.9375), whatever their positions
    logits = np.full((1, 12), -np.inf, np.float32)
    places = [7, 2, 9, 0, 5, 11, 3]
    for j, x in enumerate(places):
        logits[0, x] = -np.log(2.0) * (j + 1)
    out, prob, keep = oracle.top_p_filter(logits, 0.9, 1.0)
    assert sorted(np.nonzero(keep[0])[0].tolist()) == sorted(places[:4])
    assert np.array_equal(out[0, keep[0]], logits[0, keep[0]]) and np.all(np.isneginf(out[0, ~keep[0]]))
    # temperature scales the logits first: T = 0.5 squares the probability ratios
    out, prob, keep = oracle.top_p_filter(logits, 0.9, 0.5)
    assert sorted(np.nonzero(keep[0])[0].tolist()) == sorted(places[:2])  # 1/4 + 1/16 + ... : 0.75, then 0.9375


def test_limits():
    rng = np.random.default_rng(1)
    logits = rng.standard_normal((3, 40)).astype(np.float32)
    logits[1, 5] = -np.inf
    logits[2, 6] = np.nan
    out, prob, keep = oracle.top_p_filter(logits, 1.0, 0.8)
    assert keep[0].all() and keep[1].sum() == 39 and not keep[1, 5] and not keep[2, 6]
    wide = np.array([[0.0, -50.0, -100.0, -700.0, -np.inf]], dtype=np.float32)     # the tail is below fp64's epsilon
    assert oracle.top_p_filter(wide, 1.0, 1.0)[2][0].tolist() == [True, True, True, True, False]
    out, prob, keep = oracle.top_p_filter(logits, 0.5, 0.0)
    assert keep.sum(axis=1).tolist() == [1, 1, 1] and keep[0, int(np.argmax(logits[0]))]
    out, prob, keep = oracle.top_p_filter(logits, 1e-6, 1.0)
    assert keep.sum(axis=1).tolist() == [1, 1, 1]


def has_defining_properties(prob, keep, top_p, tol):
    """Kept tokens are at least as probable as dropped ones, reach top_p, and would not without
    the least probable kept token (all within tol)."""
    if keep.sum() == 0:
        return False
    kept, dropped = prob[keep], prob[~keep]
    if len(dropped) and dropped.max() > kept.min() * (1 + tol) + 1e-30:
        return False
    total = kept.sum()
    return total >= min(top_p, prob.sum()) - tol and total - kept.min() < top_p + tol


def test_defining_properties_on_random_rows():
    rng = np.random.default_rng(2)
    logits = (3 * rng.standard_normal((20, 500))).astype(np.float32)
    for top_p in (0.1, 0.5, 0.9, 0.99):
        out, prob, keep = oracle.top_p_filter(logits, top_p, 0.7)
        for r in range(20):
            assert has_defining_properties(prob[r], keep[r], top_p, 1e-12)
            assert not has_defining_properties(prob[r], np.roll(keep[r], 1), top_p, 1e-12) or np.array_equal(np.roll(keep[r], 1), keep[r])


def test_argument_errors_need_no_gpu():
    def call(logits=0x1000, out=0x1000, top_p=0.9, T=1.0, rows=2, V=100, dtype=B.SEQ_F32):
        return S.lib().seq_top_p_filter(logits, out, top_p, T, rows, V, dtype, None, None)
    assert call(logits=None) == B.SEQ_ERR_NULL and call(out=None) == B.SEQ_ERR_NULL
    assert call(dtype=0) == B.SEQ_ERR_DTYPE
    for bad in (0.0, -0.1, 1.01, float("nan")):
        assert call(top_p=bad) == B.SEQ_ERR_SHAPE
    assert call(rows=0) == B.SEQ_ERR_SHAPE and call(V=1) == B.SEQ_ERR_SHAPE
    assert call(T=-1.0) == B.SEQ_ERR_TEMPERATURE and call(T=float("inf")) == B.SEQ_ERR_TEMPERATURE


@pytest.mark.gpu
@pytest.mark.parametrize("V,rows,dtype,T", [(64, 5, W.F32, 1.0), (1001, 7, W.BF16, 0.6), (8192, 3, W.F32, 0.8), (32000, 12, W.BF16, 0.6),
                                            (32768, 2, W.F32, 1.0), (50257, 3, W.BF16, 1.0), (128256, 2, W.BF16, 0.6)])
def test_library_against_the_checker(V, rows, dtype, T):
    import torch
    from gpu_util import DEV, to_dev
    rng = np.random.default_rng(V)
    logits = W.quantize((3.0 * rng.standard_normal((rows, V))).astype(np.float32), dtype)
    logits[0, ::7] = -np.inf
    if rows > 2:
        logits[2] = W.quantize(np.round(logits[2]), dtype)                 # many equal probabilities
    differing = 0
    for top_p in (0.05, 0.5, 0.9, 1.0):
        got, kept = S.seq_top_p_filter(to_dev(logits, dtype), top_p, T)
        torch.cuda.synchronize()
        got = got.float().cpu().numpy()
        want, prob, keep = oracle.top_p_filter(logits, top_p, T)
        got_keep = ~np.isneginf(got)
        assert np.array_equal(kept.cpu().numpy(), got_keep.sum(axis=1))
        for r in range(rows):
            assert np.array_equal(got[r, got_keep[r]], logits[r, got_keep[r]])          # kept logits unchanged
            if np.array_equal(got_keep[r], keep[r]):
                continue
            assert has_defining_properties(prob[r], got_keep[r], top_p, 2e-6), (top_p, r, got_keep[r].sum(), keep[r].sum())
            differing += 1
            if top_p == 1.0:
                # no search at all: every token whose fp32 probability is not zero is kept (1e-37:
                # above the smallest normal float), and no token of probability exactly zero is
                assert not ((prob[r] > 1e-37) & ~got_keep[r]).any()
                assert not ((prob[r] == 0.0) & got_keep[r]).any()
    assert differing <= 4 * rows // 2


@pytest.mark.gpu
def test_zero_temperature_in_place_and_downstream_calls():
    import torch
    from gpu_util import DEV, to_dev, check_verify
    rng = np.random.default_rng(5)
    logits = W.quantize(rng.standard_normal((4, 3000)).astype(np.float32), W.BF16)
    dev = to_dev(logits, W.BF16)
    S.seq_top_p_filter(dev, 0.7, 0.0, filtered=dev)                                     # in place
    torch.cuda.synchronize()
    got = dev.float().cpu().numpy()
    for r in range(4):
        assert np.nonzero(~np.isneginf(got[r]))[0].tolist() == [int(np.argmax(logits[r]))]
    # filtered rows through the drafter's draw and the verification walk: children come from the
    # nucleus only, and the walk (whose uniform fallback is now reachable) agrees with the checker
    flagged = 0
    for rep in range(6):
        parent = W.geometric_tree(24, 4)
        v = W.make_verify_inputs(parent, 2000, 3.0, 1.0, 0.8, W.BF16, seed=70 + rep)
        tl, _ = S.seq_top_p_filter(to_dev(v.target_logits, W.BF16), 0.8, 0.8)
        dl, kept = S.seq_top_p_filter(to_dev(v.draft_logits, W.BF16), 0.3, 0.8)
        fan = np.bincount(parent[1:], minlength=24).astype(np.int32)
        rngt = torch.tensor([9, rep], dtype=torch.int64, device=DEV)
        drawn, _ = S.seq_draft_sample(dl, torch.from_numpy(fan).to(DEV), 0.8, rngt, int(fan.max()))
        torch.cuda.synchronize()
        v.target_logits, v.draft_logits = tl.float().cpu().numpy(), dl.float().cpu().numpy()
        drawn = drawn.cpu().numpy()
        for node, ch in enumerate(W.children_lists(parent)):
            if ch:
                v.tree_tokens[ch] = drawn[node, : len(ch)]
        nucleus = ~np.isneginf(v.draft_logits)
        for node, ch in enumerate(W.children_lists(parent)):
            inside = [bool(nucleus[node, t]) for t in v.tree_tokens[ch]]
            assert inside[: min(len(ch), int(nucleus[node].sum()))] == [True] * min(len(ch), int(nucleus[node].sum()))
        flagged += check_verify(v) == "flagged"
    assert flagged <= 1
