"""GPU parity of all three calls on trees built by the Sequoia dynamic program from the paper's
printed acceptance vector (wide at the root, a long first chain): the second tree workload,
beside the geometric trees of the configurations."""
import json
import os

import numpy as np
import pytest

import oracle
import paper_2402_12374_amd as S
import workloads as W

from gpu_util import TOL, check_verify, oracle_attn, run_attn
from test_gpu_draft import check_draft

pytestmark = pytest.mark.gpu

PAPER_P = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_acceptance_vector.json")))["acceptance"]


def sequoia_tree(n, depth):
    parent, _ = S.seq_build_tree(PAPER_P, n, depth)
    return parent


@pytest.mark.parametrize("n,depth,cfg_key,P", [(64, 8, "C2", 300), (128, 10, "C3", 513), (256, 12, "C4", 200)])
def test_attention_all_rows(n, depth, cfg_key, P):
    cfg = W.CONFIGS[cfg_key]
    a = W.make_attn_inputs(cfg.heads, cfg.kv_heads, cfg.head_dim, P, sequoia_tree(n, depth), cfg.dtype, seed=n)
    err = np.abs(run_attn(a) - oracle_attn(a)).max()
    assert err <= TOL[a.dtype], err


def test_attention_largest_tree_sampled_rows():
    cfg = W.CONFIGS["C5"]
    a = W.make_attn_inputs(cfg.heads, cfg.kv_heads, cfg.head_dim, cfg.prefix_len, sequoia_tree(768, 16), cfg.dtype, seed=768)
    got = run_attn(a)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(8)
    rows = {(0, 0), (767, cfg.heads - 1)}
    while len(rows) < 48:
        rows.add((int(rng.integers(768)), int(rng.integers(cfg.heads))))
    worst = max(float(np.abs(got[i, h] - oracle.tree_attn_row(a.q, a.k_cache, a.v_cache, a.k_tree, a.v_tree, a.parent,
                                                              a.prefix_len, i, h)).max()) for i, h in sorted(rows))
    assert worst <= TOL[a.dtype], worst


@pytest.mark.parametrize("n,depth,V,sigma_d", [(64, 8, 32000, 1.5), (64, 8, 32000, 0.3), (128, 10, 5000, 0.5), (256, 12, 2048, 0.3)])
def test_verification_walk(n, depth, V, sigma_d):
    """Both kernels (the per-node one where it applies, the lazy walk otherwise and when forced)."""
    parent = sequoia_tree(n, depth)
    flagged = 0
    for mode in (0, 1):
        S.lib().seqtree_internal_set_verify_mode(mode)
        try:
            for rep in range(3):
                v = W.make_verify_inputs(parent, V, 3.0, sigma_d, 0.6, W.BF16, seed=n + rep)
                flagged += check_verify(v) == "flagged"
        finally:
            S.lib().seqtree_internal_set_verify_mode(0)
    assert flagged <= 1


@pytest.mark.parametrize("n,depth,V", [(64, 8, 32000), (256, 12, 32000), (768, 16, 128256)])
def test_drafting_the_children(n, depth, V):
    """Every internal node of the tree draws its children in one call."""
    parent = sequoia_tree(n, depth)
    fan = np.bincount(parent[1:], minlength=n).astype(np.int32)
    rows = np.nonzero(fan > 0)[0]
    rng = np.random.default_rng(n)
    logits = 3.0 * rng.standard_normal((len(rows), V), dtype=np.float32)
    sample = None if len(rows) * V < 2 ** 23 else np.unique(np.concatenate([[0], rng.choice(len(rows), 40, replace=False)]))
    assert check_draft(logits, fan[rows], 0.6, 11, n, W.BF16, int(fan.max()), rows=sample) <= 2
