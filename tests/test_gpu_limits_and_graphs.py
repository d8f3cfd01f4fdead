"""Largest sizes the header allows, and replay of both calls from a captured HIP graph."""
import numpy as np
import pytest
import torch

import oracle
import paper_2402_12374_amd as S
import workloads as W

from gpu_util import DEV, TOL, check_verify, oracle_attn, run_attn, to_dev

pytestmark = pytest.mark.gpu


def test_attention_at_the_largest_tree():
    n = S.binding.SEQ_MAX_TREE
    rng = np.random.default_rng(1)
    for parent in (W.random_topological_tree(n, rng), W.chain_tree(n)):
        a = W.make_attn_inputs(2, 1, 64, 45, parent, W.BF16, seed=7, prefix_cap=45)
        err = np.abs(run_attn(a) - oracle_attn(a)).max()
        assert err <= TOL[W.BF16], err


@pytest.mark.parametrize("mode", [1, 2])   # lazy walk, per-node kernel
@pytest.mark.parametrize("shape", ["star", "chain", "random"])
def test_verification_at_the_largest_tree(mode, shape):
    n, V = S.binding.SEQ_MAX_TREE, 300
    rng = np.random.default_rng(2)
    parent = {"star": W.star_tree(n), "chain": W.chain_tree(n), "random": W.random_topological_tree(n, rng)}[shape]
    if shape == "star":
        # 1023 children of the root cannot carry distinct tokens out of 300: draw them with
        # repetition, which Algorithm 2 must survive (a repeated token has residual zero)
        v = W.make_verify_inputs(W.star_tree(V // 2), V, 2.0, 1.0, 0.8, W.F32, seed=3)
        tl = np.tile(v.target_logits[:1], (n, 1))
        dl = np.tile(v.draft_logits[:1], (n, 1))
        tok = rng.integers(0, V, size=n).astype(np.int32)
        un = rng.random(n, dtype=np.float32)
        un[1:600] = 0.999999   # reject for a long while
        v = W.VerifyInputs(tl, dl, tok, parent, un, 0.8, W.F32)
    else:
        v = W.make_verify_inputs(parent, V, 2.0, 1.0, 0.8, W.F32, seed=4)
        if shape == "chain":   # a draft equal to the target accepts all the way down
            v.draft_logits[:] = v.target_logits
            for node in range(n - 1):
                v.tree_tokens[node + 1] = W.draw_children_tokens(v.draft_logits[node], 1, 0.8, rng)[0]
    S.lib().seqtree_internal_set_verify_mode(mode)
    try:
        assert check_verify(v) in ("exact", "flagged")
    finally:
        S.lib().seqtree_internal_set_verify_mode(0)


def test_verification_at_the_largest_vocabulary():
    V = S.binding.SEQ_MAX_VOCAB
    parent = W.geometric_tree(5, 3)
    for dtype in (W.BF16, W.F32):
        v = W.make_verify_inputs(parent, V, 4.0, 2.0, 0.7, dtype, seed=9)
        assert check_verify(v) in ("exact", "flagged")


def test_graph_replays_match_eager_results():
    """Capture one attention call and one verification call in a HIP graph; replay it several
    times with new data copied into the same buffers and the program's own eager calls and
    synchronisations in between; every replay must give what the eager call gives."""
    cfg = W.CONFIGS["C2"]
    n, H, Hk, d, P, V, T = cfg.n_tree, cfg.heads, cfg.kv_heads, cfg.head_dim, 300, 4096, 0.6
    parent = W.geometric_tree(n, cfg.max_depth)
    first_a = W.make_attn_inputs(H, Hk, d, P, parent, W.BF16, seed=0, prefix_cap=P)
    first_v = W.make_verify_inputs(parent, V, 3.0, 1.5, T, W.BF16, seed=0)
    buf = dict(q=to_dev(first_a.q, W.BF16), kc=to_dev(first_a.k_cache, W.BF16), vc=to_dev(first_a.v_cache, W.BF16),
               kt=to_dev(first_a.k_tree, W.BF16), vt=to_dev(first_a.v_tree, W.BF16),
               tl=to_dev(first_v.target_logits, W.BF16), dl=to_dev(first_v.draft_logits, W.BF16),
               tok=torch.from_numpy(first_v.tree_tokens).to(DEV), un=torch.from_numpy(first_v.uniforms).to(DEV))
    out = torch.empty_like(buf["q"])
    path = torch.empty(n, dtype=torch.int32, device=DEV)
    bonus = torch.empty(1, dtype=torch.int32, device=DEV)
    code = 1
    aws = torch.empty(S.seq_tree_attn_workspace(P, n, H, Hk, d, code), dtype=torch.uint8, device=DEV)
    vws = torch.empty(S.seq_verify_workspace(n, V, code), dtype=torch.uint8, device=DEV)

    def step():
        S.seq_tree_attn(buf["q"], buf["kc"], buf["vc"], buf["kt"], buf["vt"], parent, P, out=out, workspace=aws)
        S.seq_verify(buf["tl"], buf["dl"], buf["tok"], parent, T, buf["un"], accepted_path=path,
                     bonus_token=bonus, workspace=vws)

    step()   # builds the plan and the library's synchronisation area outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(1, 5):
        a = W.make_attn_inputs(H, Hk, d, P, parent, W.BF16, seed=rep, prefix_cap=P)
        v = W.make_verify_inputs(parent, V, 3.0, 1.5, T, W.BF16, seed=rep)
        for key, arr in (("q", a.q), ("kc", a.k_cache), ("vc", a.v_cache), ("kt", a.k_tree), ("vt", a.v_tree),
                         ("tl", v.target_logits), ("dl", v.draft_logits)):
            buf[key].copy_(to_dev(arr, W.BF16))
        buf["tok"].copy_(torch.from_numpy(v.tree_tokens).to(DEV))
        buf["un"].copy_(torch.from_numpy(v.uniforms).to(DEV))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got_out = out.float().cpu().numpy()
        got_path, got_bonus = path.cpu().numpy().copy(), int(bonus.item())
        trace = S.read_verify_trace(vws)
        # the same inputs through eager calls with buffers of their own
        eager_out = run_attn(a)
        assert np.array_equal(got_out, eager_out.astype(np.float32))
        assert check_verify(v, (got_path, got_bonus, trace)) in ("exact", "flagged")
        assert np.abs(got_out - oracle_attn(a)).max() <= TOL[W.BF16]


def test_batched_walk_in_a_graph():
    """seq_verify_batched with the teams of several sequences in one launch, captured once and
    replayed with new logits and uniforms in the same buffers: every replay gives every sequence
    what the checker gives it, and no team reports a timeout."""
    n, V, B, T = 24, 20000, 7, 0.7          # three workgroups per team
    parent = W.geometric_tree(n, 5)
    make = lambda rep: [W.make_verify_inputs(parent, V, 3.0, 1.0, T, W.BF16, seed=40 * rep + b) for b in range(B)]
    stack = lambda vs, key: torch.from_numpy(np.stack([getattr(v, key) for v in vs])).to(DEV)
    vs = make(0)
    buf = dict(tl=stack(vs, "target_logits").to(torch.bfloat16), dl=stack(vs, "draft_logits").to(torch.bfloat16),
               tok=stack(vs, "tree_tokens"), un=stack(vs, "uniforms"))
    path = torch.empty((B, n), dtype=torch.int32, device=DEV)
    bonus = torch.empty(B, dtype=torch.int32, device=DEV)
    ws = torch.empty((B, S.seq_verify_workspace(n, V, 1)), dtype=torch.uint8, device=DEV)

    def step():
        S.seq_verify_batched(S.SEQ_VERIFY_SEQUOIA, buf["tl"], buf["dl"], buf["tok"], parent, T, buf["un"],
                             accepted_path=path, bonus_token=bonus, workspace=ws)

    S.lib().seqtree_internal_set_verify_mode(1)
    try:
        step()
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for rep in range(1, 4):
            vs = make(rep)
            buf["tl"].copy_(stack(vs, "target_logits").to(torch.bfloat16))
            buf["dl"].copy_(stack(vs, "draft_logits").to(torch.bfloat16))
            buf["tok"].copy_(stack(vs, "tree_tokens"))
            buf["un"].copy_(stack(vs, "uniforms"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for b, v in enumerate(vs):
                got = (path[b].cpu().numpy(), int(bonus[b].item()), S.read_verify_trace(ws[b]))
                assert check_verify(v, got) in ("exact", "flagged"), (rep, b)
    finally:
        S.lib().seqtree_internal_set_verify_mode(0)


def test_whole_iteration_in_one_graph():
    """Draw the root's children, verify the tree with each of the three algorithms, append the
    accepted path to the cache -- captured once, replayed with the step counter advanced on the
    device and new logits copied in; every replay must equal what the checker computes for that
    step number (no host value is baked into the graph except sizes and pointers)."""
    n, V, T, Hk, d, P, cap = 6, 4096, 0.8, 4, 64, 20, 32
    parent = W.star_tree(n)
    k = n - 1
    seed = 31337
    rng = torch.tensor([seed, 0], dtype=torch.int64, device=DEV)
    nc = torch.tensor([k], dtype=torch.int32, device=DEV)
    tokens = torch.zeros(n, dtype=torch.int32, device=DEV)
    tl = torch.zeros((n, V), dtype=torch.bfloat16, device=DEV)
    dl = torch.zeros((n, V), dtype=torch.bfloat16, device=DEV)
    un = torch.zeros(n, dtype=torch.float32, device=DEV)
    outs = {alg: (torch.empty(n, dtype=torch.int32, device=DEV), torch.empty(1, dtype=torch.int32, device=DEV),
                  torch.empty(S.seq_verify_workspace(n, V, 1), dtype=torch.uint8, device=DEV))
            for alg in (S.SEQ_VERIFY_SEQUOIA, S.SEQ_VERIFY_SPECINFER, S.SEQ_VERIFY_TOPK)}
    a0 = W.make_attn_inputs(Hk, Hk, d, P, parent, W.BF16, seed=1, prefix_cap=cap)
    kt, vt = to_dev(a0.k_tree, W.BF16), to_dev(a0.v_tree, W.BF16)
    kc, vc = to_dev(a0.k_cache, W.BF16), to_dev(a0.v_cache, W.BF16)
    new_len = torch.zeros(1, dtype=torch.int32, device=DEV)
    dws = torch.empty(S.seq_draft_sample_workspace(1, V, k, 1), dtype=torch.uint8, device=DEV)

    def iteration():
        S.seq_draft_sample(dl[:1], nc, T, rng, k, tokens=tokens[1:].view(1, k), workspace=dws)
        for alg, (path, bonus, ws) in outs.items():
            S.seq_verify_with(alg, tl, dl, tokens, parent, T, un, accepted_path=path, bonus_token=bonus, workspace=ws)
        S.seq_kv_append(kt, vt, outs[S.SEQ_VERIFY_SEQUOIA][0], parent, kc, vc, P, new_prefix_len=new_len)
        rng[1] += 1          # the next replay draws with the next step number

    iteration()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        iteration()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        iteration()
    step = int(rng[1].item())
    for rep in range(4):
        v = W.make_verify_inputs(parent, V, 3.0, 0.6, T, W.BF16, seed=40 + rep)
        tl.copy_(to_dev(v.target_logits, W.BF16)); dl.copy_(to_dev(v.draft_logits, W.BF16))
        un.copy_(torch.from_numpy(v.uniforms).to(DEV))
        kc.copy_(to_dev(a0.k_cache, W.BF16)); vc.copy_(to_dev(a0.v_cache, W.BF16))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        drawn = oracle.draft_sample(v.draft_logits[:1], [k], T, seed, step, k_stride=k)
        if drawn.closest_call(0, k) < 1e-4:
            step += 1
            continue
        assert np.array_equal(tokens[1:].cpu().numpy(), drawn.tokens[0]), rep
        v.tree_tokens[1:] = drawn.tokens[0]
        ref = oracle.verify(v.target_logits, v.draft_logits, v.tree_tokens, parent, T, v.uniforms)
        if all(dec.margin > 1e-5 for dec in ref.decisions) and ref.bonus_margin > 1e-5:
            path, bonus, _ = outs[S.SEQ_VERIFY_SEQUOIA]
            assert [int(x) for x in path.cpu().numpy() if x >= 0] == ref.path and int(bonus.item()) == ref.bonus_token
            want_k, want_v, want_len = oracle.kv_append(a0.k_tree, a0.v_tree, path.cpu().numpy(), a0.k_cache, a0.v_cache, P)
            assert int(new_len.item()) == want_len
            assert np.array_equal(kc.float().cpu().numpy(), want_k) and np.array_equal(vc.float().cpu().numpy(), want_v)
        for alg in (S.SEQ_VERIFY_SPECINFER, S.SEQ_VERIFY_TOPK):
            refb = oracle.verify_baseline(alg, v.target_logits, v.draft_logits, v.tree_tokens, parent, T, v.uniforms)
            margins = [abs(r[2] - r[5]) for r in refb.records] if alg == S.SEQ_VERIFY_SPECINFER else [r[5] for r in refb.records]
            if min(margins + [refb.bonus_margin]) > 1e-5:
                path, bonus, _ = outs[alg]
                assert [int(x) for x in path.cpu().numpy() if x >= 0] == refb.path and int(bonus.item()) == refb.bonus_token, (rep, alg)
        step += 1
    assert int(rng[1].item()) == step


def test_new_calls_at_their_largest_sizes():
    """The largest vocabulary (524288) and row count (1024) for the drafter's draw and the top-p
    filter, the largest tree for the KV append and the top-k walk."""
    from test_gpu_draft import check_draft
    rng = np.random.default_rng(99)
    big = 3.0 * rng.standard_normal((2, S.binding.SEQ_MAX_VOCAB), dtype=np.float32)
    assert check_draft(big, [64, 5], 0.7, 1, 2, W.BF16, 64) <= 1
    many = rng.standard_normal((1024, 512), dtype=np.float32)
    assert check_draft(many, rng.integers(0, 5, size=1024), 1.0, 3, 4, W.F32, 4) <= 3
    # top-p on the largest row: the kept set has the defining properties
    from test_top_p import has_defining_properties
    logits = W.quantize(big[:1], W.BF16)
    got, kept = S.seq_top_p_filter(to_dev(logits, W.BF16), 0.9, 0.8)
    torch.cuda.synchronize()
    want, prob, keep = oracle.top_p_filter(logits, 0.9, 0.8)
    got_keep = ~np.isneginf(got.float().cpu().numpy())
    assert int(kept.item()) == got_keep.sum()
    assert np.array_equal(got_keep, keep) or has_defining_properties(prob[0], got_keep[0], 0.9, 2e-6)
    # a chain of 1024 nodes: the deepest possible path, all of it accepted
    n, Hk, d = 1024, 2, 64
    parent = W.chain_tree(n)
    a = W.make_attn_inputs(Hk, Hk, d, 8, parent, W.F32, seed=5, prefix_cap=8 + n)
    path = np.full(n, -1, dtype=np.int32)
    path[: n - 1] = np.arange(1, n)
    kc, vc = to_dev(a.k_cache, W.F32), to_dev(a.v_cache, W.F32)
    new_len = S.seq_kv_append(to_dev(a.k_tree, W.F32), to_dev(a.v_tree, W.F32), torch.from_numpy(path).to(DEV), parent, kc, vc, 8)
    torch.cuda.synchronize()
    want_k, want_v, want_len = oracle.kv_append(a.k_tree, a.v_tree, path, a.k_cache, a.v_cache, 8)
    assert int(new_len.item()) == want_len == 8 + n
    assert np.array_equal(kc.cpu().numpy(), want_k) and np.array_equal(vc.cpu().numpy(), want_v)
