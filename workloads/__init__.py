"""Seeded synthetic inputs for the tree-verify hot path.

This module only *draws* inputs: tree shapes, Gaussian Q/K/V and logits, child
tokens and uniforms.  It holds none of the method's arithmetic (no attention,
no softmax, no accept test), so both the HIP path and the CPU checker can be fed
from it without sharing any computation.

The shapes stand in for the paper's workloads (Sec. 4.1 "Setup": Llama2-7B /
Llama2-13B / Vicuna-33B on device, Llama3-70B offloaded; tree sizes from Sec. 4.1
"Analysis": 64-128 on device, 768 offloaded).  The datasets and model weights the
paper measured on are replaced by Gaussian tensors of the same shape.

Child tokens are an ordered sample without replacement from the draft
distribution (Sec. 3.2.1, Algorithm 2 step "sample s_i ~ D").  They are drawn
with the exponential-sort / Gumbel-top-k device the paper names in Sec. 4.1
"Implementation Details": perturb ``logit / T`` with i.i.d. Gumbel noise and take
the top entries in descending order.  That needs no normalised probabilities.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

BF16 = "bf16"
F32 = "f32"


@dataclass(frozen=True)
class Config:
    name: str
    heads: int
    kv_heads: int
    head_dim: int
    dtype: str
    prefix_len: int
    n_tree: int
    max_depth: int
    vocab: int
    sigma_target: float
    sigma_draft: float
    temperatures: tuple
    layers: int  # number of distinct K/V sets a real forward pass would touch
    tree: str = "geometric"


# BASELINE configs, in order (index 1 is the one the headline metric is quoted on).
CONFIGS: Dict[str, Config] = {
    "C1": Config("C1-toy", 2, 2, 64, F32, 256, 16, 4, 64, 2.0, 1.0, (1.0,), 64, "uniform"),
    "C2": Config("C2-llama2-7b", 32, 32, 128, BF16, 1024, 64, 8, 32000, 3.0, 1.5, (0.6,), 32),
    "C3": Config("C3-llama2-13b", 40, 40, 128, BF16, 2048, 128, 10, 32000, 3.0, 1.5, (1.0, 0.0), 40),
    "C4": Config("C4-vicuna-33b", 52, 52, 128, BF16, 4096, 256, 12, 32000, 3.0, 2.0, (0.6,), 60),
    "C5": Config("C5-llama3-70b", 64, 8, 128, BF16, 8192, 768, 16, 128256, 4.0, 2.0, (0.6,), 80),
}


def seed_for(config_index: int, rep: int = 0) -> int:
    return 1000 * config_index + rep


# --------------------------------------------------------------------------
# dtype helpers (storage only)
# --------------------------------------------------------------------------
def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    bits = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        bits = np.where(nan, np.uint16(0x7FC0), bits)
    inf = np.isinf(x)
    if inf.any():
        bits = np.where(inf, (u >> np.uint32(16)).astype(np.uint16), bits)
    return bits


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> the float32 holding exactly the same value."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round a float array to the storage dtype, returned as float32 (exact container)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == F32:
        return x
    if dtype == BF16:
        return bf16_bits_to_f32(to_bf16_bits(x))
    raise ValueError(dtype)


# --------------------------------------------------------------------------
# tree shapes: parent[0] = -1, parent[i] < i
# --------------------------------------------------------------------------
def chain_tree(n: int) -> np.ndarray:
    return np.arange(-1, n - 1, dtype=np.int32)


def star_tree(n: int) -> np.ndarray:
    p = np.zeros(n, dtype=np.int32)
    p[0] = -1
    return p


def depths(parent: np.ndarray) -> np.ndarray:
    d = np.zeros(len(parent), dtype=np.int32)
    for i in range(1, len(parent)):
        d[i] = d[parent[i]] + 1
    return d


def uniform_tree(n: int, max_depth: int, rng: np.random.Generator) -> np.ndarray:
    """parent[i] uniform over earlier nodes whose depth is < max_depth (toy config)."""
    parent = np.full(n, -1, dtype=np.int32)
    depth = np.zeros(n, dtype=np.int32)
    for i in range(1, n):
        cand = np.flatnonzero(depth[:i] < max_depth)
        p = int(cand[rng.integers(len(cand))])
        parent[i] = p
        depth[i] = depth[p] + 1
    return parent


def geometric_tree(n: int, max_depth: int, ratio: float = 0.5) -> np.ndarray:
    """Deterministic 'Sequoia-like' tree: a node with budget m keeps one slot and deals the
    remaining m-1 to its children; child k receives ceil(ratio * what is still undealt) (at
    least 1), so first children carry the large subtrees.  A node whose children would sit at
    ``max_depth`` makes all of them leaves.  Nodes are numbered breadth-first with siblings in
    deal order, hence ascending node id among siblings is the drafting order.
    """
    if n < 1:
        raise ValueError("n >= 1")
    # build as nested budgets, breadth-first
    parent: List[int] = [-1]
    budget: List[int] = [n]
    depth: List[int] = [0]
    head = 0
    while head < len(parent):
        m, dep = budget[head], depth[head]
        left = m - 1
        while left > 0:
            if dep + 1 >= max_depth:
                share = 1
            else:
                share = max(1, int(np.ceil(left * ratio)))
            share = min(share, left)
            parent.append(head)
            budget.append(share)
            depth.append(dep + 1)
            left -= share
        head += 1
    out = np.asarray(parent, dtype=np.int32)
    assert len(out) == n, (len(out), n)
    return out


def random_topological_tree(n: int, rng: np.random.Generator) -> np.ndarray:
    """Any tree with parent[i] < i, siblings not contiguous (edge-case generator)."""
    parent = np.full(n, -1, dtype=np.int32)
    for i in range(1, n):
        parent[i] = int(rng.integers(0, i))
    return parent


def make_tree(cfg: Config, seed: int, n_tree: Optional[int] = None) -> np.ndarray:
    n = cfg.n_tree if n_tree is None else n_tree
    if cfg.tree == "uniform":
        return uniform_tree(n, cfg.max_depth, np.random.Generator(np.random.PCG64(seed + 7)))
    return geometric_tree(n, cfg.max_depth)


def children_lists(parent: np.ndarray) -> List[List[int]]:
    ch: List[List[int]] = [[] for _ in range(len(parent))]
    for i in range(1, len(parent)):
        ch[int(parent[i])].append(i)
    return ch


# --------------------------------------------------------------------------
# attention inputs
# --------------------------------------------------------------------------
@dataclass
class AttnInputs:
    q: np.ndarray        # [n, H, d]       float32 holding dtype-exact values
    k_cache: np.ndarray  # [Hk, cap, d]
    v_cache: np.ndarray  # [Hk, cap, d]
    k_tree: np.ndarray   # [n, Hk, d]
    v_tree: np.ndarray   # [n, Hk, d]
    parent: np.ndarray   # [n] int32
    prefix_len: int
    prefix_cap: int
    dtype: str


def make_attn_inputs(heads: int, kv_heads: int, head_dim: int, prefix_len: int, parent: np.ndarray,
                     dtype: str, seed: int, prefix_cap: Optional[int] = None) -> AttnInputs:
    rng = np.random.Generator(np.random.PCG64(seed))
    n = len(parent)
    cap = prefix_len if prefix_cap is None else prefix_cap
    cap = max(cap, 1)

    def normal(*shape):
        return quantize(rng.standard_normal(shape, dtype=np.float32), dtype)

    q = normal(n, heads, head_dim)
    k_cache = normal(kv_heads, cap, head_dim)
    v_cache = normal(kv_heads, cap, head_dim)
    k_tree = normal(n, kv_heads, head_dim)
    v_tree = normal(n, kv_heads, head_dim)
    return AttnInputs(q, k_cache, v_cache, k_tree, v_tree, np.asarray(parent, dtype=np.int32),
                      int(prefix_len), int(cap), dtype)


# The acceptance rate vector the paper prints in its appendix "Examples of Sequoia trees" (Llama3-70B
# target, Llama3-8B draft, CNN daily news): entry k-1 = probability that the token at child position k
# of an accepted node is accepted.  Input data for the tree construction, nothing is computed here.
PAPER_ACCEPTANCE_VECTOR = (
    0.7732, 0.1039, 0.0402, 0.0206, 0.0128, 0.0081, 0.0064, 0.0043, 0.0035, 0.0026, 0.0025, 0.0021,
    0.0016, 0.0014, 0.0010, 0.0010, 0.0010, 0.0007, 0.0007, 0.0006, 0.0007, 0.0006, 0.0004, 0.0004,
    0.0005, 0.0006, 0.0004, 0.0003, 0.0002, 0.0004, 0.0001)


# --------------------------------------------------------------------------
# verification inputs
# --------------------------------------------------------------------------
@dataclass
class VerifyInputs:
    target_logits: np.ndarray  # [n, V] float32 holding dtype-exact values
    draft_logits: np.ndarray   # [n, V]
    tree_tokens: np.ndarray    # [n] int32, [0] unused (set to 0)
    parent: np.ndarray         # [n] int32
    uniforms: np.ndarray       # [n] float32 in [0,1)
    temperature: float
    dtype: str


def draw_children_tokens(draft_row: np.ndarray, k: int, temperature: float,
                         rng: np.random.Generator) -> np.ndarray:
    """Ordered sample of k distinct tokens.  T>0: Gumbel-top-k on logit/T (an ordered draw
    without replacement from the tempered draft distribution).  T==0: the k largest logits,
    ties to the lower index (the paper's top-k drafting, Sec. 2.2)."""
    v = len(draft_row)
    k = min(k, v)
    if k == 0:
        return np.zeros(0, dtype=np.int32)
    if temperature > 0:
        key = draft_row.astype(np.float64) / temperature + rng.gumbel(size=v)
    else:
        key = draft_row.astype(np.float64)
    order = np.lexsort((np.arange(v), -key))  # descending key, lower index first on ties
    return order[:k].astype(np.int32)


def make_verify_inputs(parent: np.ndarray, vocab: int, sigma_target: float, sigma_draft: float,
                       temperature: float, dtype: str, seed: int) -> VerifyInputs:
    rng = np.random.Generator(np.random.PCG64(seed + 500))
    n = len(parent)
    target = rng.standard_normal((n, vocab), dtype=np.float32)
    target *= np.float32(sigma_target)
    draft = rng.standard_normal((n, vocab), dtype=np.float32)
    draft *= np.float32(sigma_draft)
    draft += target
    target = quantize(target, dtype)
    draft = quantize(draft, dtype)
    tokens = np.zeros(n, dtype=np.int32)
    for v, ch in enumerate(children_lists(parent)):
        if ch:
            tokens[ch] = draw_children_tokens(draft[v], len(ch), temperature, rng)
    uniforms = rng.random(n, dtype=np.float32)
    uniforms = np.minimum(uniforms, np.float32(1.0 - 2.0 ** -24))
    return VerifyInputs(target, draft, tokens, np.asarray(parent, dtype=np.int32), uniforms,
                        float(temperature), dtype)


def attn_inputs_for(cfg_key: str, rep: int = 0, n_tree: Optional[int] = None,
                    prefix_len: Optional[int] = None) -> AttnInputs:
    cfg = CONFIGS[cfg_key]
    idx = list(CONFIGS).index(cfg_key) + 1
    seed = seed_for(idx, rep)
    parent = make_tree(cfg, seed, n_tree)
    return make_attn_inputs(cfg.heads, cfg.kv_heads, cfg.head_dim,
                            cfg.prefix_len if prefix_len is None else prefix_len,
                            parent, cfg.dtype, seed)


def verify_inputs_for(cfg_key: str, rep: int = 0, temperature: Optional[float] = None,
                      n_tree: Optional[int] = None, vocab: Optional[int] = None) -> VerifyInputs:
    cfg = CONFIGS[cfg_key]
    idx = list(CONFIGS).index(cfg_key) + 1
    seed = seed_for(idx, rep)
    parent = make_tree(cfg, seed, n_tree)
    t = cfg.temperatures[0] if temperature is None else temperature
    return make_verify_inputs(parent, cfg.vocab if vocab is None else vocab, cfg.sigma_target,
                              cfg.sigma_draft, t, cfg.dtype, seed)


def tree_summary(parent: np.ndarray) -> dict:
    d = depths(parent)
    fan = np.bincount(parent[1:], minlength=len(parent)) if len(parent) > 1 else np.zeros(1, int)
    return {"n": int(len(parent)), "max_depth": int(d.max()),
            "depth_hist": np.bincount(d).tolist(), "max_fanout": int(fan.max())}
