"""GPU parity of seq_verify_with for the baseline algorithms of Sec. 2.2 (SpecInfer; naive / top-k
sampling) against their CPU checker: accepted paths and emitted tokens bit-exact, except where a
uniform falls within 1e-5 of an accept ratio or of a CDF edge; those cases are counted and must
stay rare."""
import numpy as np
import pytest
import torch

import oracle
import paper_2402_12374_amd as S
import workloads as W

from gpu_util import DEV, FLAG_MARGIN, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=["draws at once", "draws along the walk"])
def topk_kernel_choice(request):
    """Top-k sampling has two kernels (every node draws at once; one workgroup draws where the walk
    goes): every case runs with each forced."""
    S.lib().seqtree_internal_set_topk_mode(1 if request.param == "draws at once" else 2)
    yield request.param
    S.lib().seqtree_internal_set_topk_mode(0)


@pytest.fixture(autouse=True, params=["auto", "lazy"])
def walk_kernel_choice(request):
    """SpecInfer runs on both kernels of the walk (the per-node one where temperature, vocabulary
    and tree size allow it): every case runs with the library's choice and with the lazy walk forced."""
    S.lib().seqtree_internal_set_verify_mode(0 if request.param == "auto" else 1)
    yield request.param
    S.lib().seqtree_internal_set_verify_mode(0)


def inputs_for(algorithm, parent, V, T, dtype, seed, sigma_d=1.5):
    """Logits as for the Sequoia tests; children drawn the way the algorithm assumes: independent
    draws from the draft distribution (repeats allowed) for SpecInfer, its top-k tokens for top-k."""
    v = W.make_verify_inputs(parent, V, 3.0, sigma_d, T, dtype, seed)
    rng = np.random.default_rng(seed + 77)
    for node, ch in enumerate(W.children_lists(parent)):
        if not ch:
            continue
        if algorithm == S.SEQ_VERIFY_SPECINFER and T > 0:
            q = np.exp((v.draft_logits[node].astype(np.float64) - v.draft_logits[node].max()) / T)
            v.tree_tokens[ch] = rng.choice(V, size=len(ch), p=q / q.sum())
        else:
            v.tree_tokens[ch] = W.draw_children_tokens(v.draft_logits[node], len(ch), 0.0, rng)
    return v


def run(algorithm, v, draft=True):
    path, bonus, ws = S.seq_verify_with(algorithm, to_dev(v.target_logits, v.dtype),
                                        to_dev(v.draft_logits, v.dtype) if draft else None,
                                        torch.from_numpy(v.tree_tokens).to(DEV), v.parent, v.temperature,
                                        torch.from_numpy(v.uniforms).to(DEV))
    torch.cuda.synchronize()
    return path.cpu().numpy(), int(bonus.item()), S.read_verify_trace(ws)


def check(algorithm, v, draft=True, got=None):
    p, bonus, trace = run(algorithm, v, draft) if got is None else got
    assert trace["status"] == 0
    ref = oracle.verify_baseline(algorithm, v.target_logits, v.draft_logits, v.tree_tokens, v.parent,
                                 v.temperature, v.uniforms)
    k = int(np.argmax(p < 0)) if (p < 0).any() else len(p)
    assert (p[k:] == -1).all()
    got_path = [int(x) for x in p[:k]]
    if v.temperature == 0:
        assert got_path == ref.path and bonus == ref.bonus_token
        return "exact"
    if algorithm == S.SEQ_VERIFY_SPECINFER:
        for j, rec in enumerate(ref.records):
            node, u, ratio, accepted = int(rec[0]), rec[2], rec[5], bool(rec[6])
            if abs(u - ratio) < FLAG_MARGIN:
                return "flagged"
            assert int(trace["nodes"][j]) == node and bool(trace["accepted"][j]) == accepted, (j, rec)
            if np.isfinite(ratio):
                assert abs(float(trace["ratios"][j]) - ratio) <= 1e-5 * max(1.0, ratio), (j, rec)
        assert len(trace["nodes"]) == len(ref.records)
    else:
        for j, rec in enumerate(ref.records):
            node, drawn, margin, child = int(rec[0]), int(rec[1]), rec[5], int(rec[6])
            if margin < FLAG_MARGIN:
                return "flagged"
            assert int(trace["nodes"][j]) == node and int(trace["drawn"][j]) == drawn and int(trace["children"][j]) == child, (j, rec)
        assert len(trace["nodes"]) == len(ref.records)
    assert got_path == ref.path and trace["stop_node"] == ref.stop_node
    if ref.bonus_margin < FLAG_MARGIN:
        return "flagged"
    assert bonus == ref.bonus_token
    return "exact"


ALGORITHMS = [S.SEQ_VERIFY_SPECINFER, S.SEQ_VERIFY_TOPK]


@pytest.mark.parametrize("algorithm", ALGORITHMS)
@pytest.mark.parametrize("V,n,dtype,T", [
    (8, 6, W.F32, 1.0), (64, 16, W.BF16, 0.6), (1000, 33, W.F32, 0.3), (2049, 20, W.BF16, 1.5),
    (32000, 64, W.BF16, 0.6), (50257, 12, W.F32, 1.0),
])
def test_shapes_and_temperatures(algorithm, V, n, dtype, T):
    flagged = 0
    for rep in range(6):
        parent = W.geometric_tree(n, 6) if rep % 2 == 0 else W.random_topological_tree(n, np.random.default_rng(rep))
        flagged += check(algorithm, inputs_for(algorithm, parent, V, T, dtype, seed=V + rep)) == "flagged"
    assert flagged <= 1


@pytest.mark.parametrize("algorithm", ALGORITHMS)
def test_good_drafters_walk_deep(algorithm):
    """A draft close to the target: long accepted paths, acceptance at later siblings too."""
    flagged, lengths = 0, []
    for rep in range(8):
        parent = W.geometric_tree(64, 8)
        v = inputs_for(algorithm, parent, 5000, 0.6, W.BF16, seed=900 + rep, sigma_d=0.3)
        flagged += check(algorithm, v) == "flagged"
        lengths.append(int((run(algorithm, v)[0] >= 0).sum()))
    assert flagged <= 1 and max(lengths) >= 2


@pytest.mark.parametrize("algorithm", ALGORITHMS)
def test_zero_temperature(algorithm):
    for rep in range(6):
        parent = W.geometric_tree(40, 6)
        v = inputs_for(algorithm, parent, 3000, 0.0, W.BF16, seed=300 + rep, sigma_d=0.4)
        assert check(algorithm, v) == "exact"


def test_specinfer_takes_repeated_children():
    parent = W.star_tree(6)
    v = inputs_for(S.SEQ_VERIFY_SPECINFER, parent, 500, 1.0, W.F32, seed=5)
    v.tree_tokens[1:] = [7, 7, 9, 7, 9]
    v.uniforms[1:] = np.float32(1.0 - 2.0 ** -24)
    assert check(S.SEQ_VERIFY_SPECINFER, v) in ("exact", "flagged")


def test_topk_needs_no_draft_logits_and_handles_the_largest_shape():
    cfg = W.CONFIGS["C5"]
    parent = W.make_tree(cfg, W.seed_for(5))
    v = inputs_for(S.SEQ_VERIFY_TOPK, parent, cfg.vocab, 0.6, W.BF16, seed=55, sigma_d=0.5)
    assert check(S.SEQ_VERIFY_TOPK, v, draft=False) in ("exact", "flagged")


def test_unknown_algorithm_is_refused():
    v = inputs_for(S.SEQ_VERIFY_TOPK, W.star_tree(3), 16, 1.0, W.F32, seed=1)
    with pytest.raises(S.SeqTreeError) as e:
        run(7, v)
    assert e.value.code == S.SEQ_ERR_ALGORITHM


@pytest.mark.parametrize("algorithm", ALGORITHMS)
@pytest.mark.parametrize("V,n,B,T", [(3000, 20, 9, 0.8), (32000, 64, 3, 0.6), (40000, 7, 70, 1.0), (2049, 12, 5, 0.0)])
def test_a_batch_of_sequences(algorithm, V, n, B, T):
    """seq_verify_batched with the baselines' rules: every sequence gets what it gets alone."""
    parent = W.geometric_tree(n, 5)
    vs = [inputs_for(algorithm, parent, V, T, W.BF16, seed=3000 + 13 * b + n) for b in range(B)]
    stack = lambda key: torch.from_numpy(np.stack([getattr(v, key) for v in vs])).to(DEV)
    path, bonus, ws = S.seq_verify_batched(algorithm, stack("target_logits").to(torch.bfloat16),
                                           stack("draft_logits").to(torch.bfloat16), stack("tree_tokens"), parent, T,
                                           stack("uniforms"))
    torch.cuda.synchronize()
    flagged = 0
    for b, v in enumerate(vs):
        got = (path[b].cpu().numpy(), int(bonus[b].item()), S.read_verify_trace(ws[b]))
        flagged += check(algorithm, v, got=got) == "flagged"
    assert flagged <= max(1, B // 3)


def test_random_batches_equal_one_call_per_sequence():
    """Random trees, vocabularies, batch sizes, temperatures and algorithms: what seq_verify_batched
    gives a sequence is what seq_verify_with gives it alone (the checker is not involved here; the
    single calls are held against it everywhere else)."""
    rng = np.random.default_rng(11)
    for case in range(12):
        n = int(rng.integers(1, 80))
        V = int(rng.choice([64, 777, 2049, 9000, 32000, 40000]))
        B = max(1, min(int(rng.integers(1, 30)), int(4e7 // (n * V))))
        T = float(rng.choice([0.0, 0.6, 1.0]))
        alg = int(rng.choice([S.SEQ_VERIFY_SEQUOIA, S.SEQ_VERIFY_SPECINFER, S.SEQ_VERIFY_TOPK]))
        parent = W.random_topological_tree(n, np.random.default_rng(case)) if n > 1 else np.array([-1], np.int32)
        vs = [W.make_verify_inputs(parent, V, 3.0, 1.5, T, W.BF16, seed=7000 + 50 * case + b) for b in range(B)]
        stack = lambda key: torch.from_numpy(np.stack([getattr(v, key) for v in vs])).to(DEV)
        tl, dl = stack("target_logits").to(torch.bfloat16), stack("draft_logits").to(torch.bfloat16)
        tok, un = stack("tree_tokens"), stack("uniforms")
        path, bonus, ws = S.seq_verify_batched(alg, tl, dl, tok, parent, T, un)
        torch.cuda.synchronize()
        for b in range(B):
            p1, b1, w1 = S.seq_verify_with(alg, tl[b], dl[b], tok[b], parent, T, un[b])
            torch.cuda.synchronize()
            assert S.read_verify_trace(ws[b])["status"] == 0 and S.read_verify_trace(w1)["status"] == 0, (case, n, V, B, T, alg, b)
            assert torch.equal(path[b], p1) and int(bonus[b].item()) == int(b1.item()), (case, n, V, B, T, alg, b)
