"""CPU checker for the Sequoia tree-verify step.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import this package.
It wraps the plain-C fp64 routines in this directory with ctypes; it shares no code with the
HIP library and never imports it.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np

from . import build as _build

_LIB: Optional[C.CDLL] = None
_f32p = np.ctypeslib.ndpointer(dtype=np.float32, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(dtype=np.int32, flags="C_CONTIGUOUS")
_f64p = np.ctypeslib.ndpointer(dtype=np.float64, flags="C_CONTIGUOUS")


def lib() -> C.CDLL:
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        _LIB = C.CDLL(path)
        _LIB.oracle_tree_attn_row.restype = C.c_int
        _LIB.oracle_tree_attn.restype = C.c_int
        _LIB.oracle_draft_sample.restype = C.c_int
        _LIB.oracle_verify_baseline.restype = C.c_int
        _LIB.oracle_draft_uniform.restype = C.c_double
        _LIB.oracle_philox4x32_10.restype = None
        _LIB.oracle_verify.restype = C.c_int
        _LIB.oracle_verify_trials.restype = C.c_int
    return _LIB


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def tree_attn(q, k_cache, v_cache, k_tree, v_tree, parent, prefix_len: int) -> np.ndarray:
    """All rows.  q [n,H,d]; k_cache/v_cache [Hk,cap,d]; k_tree/v_tree [n,Hk,d] -> fp64 [n,H,d]."""
    q, k_cache, v_cache, k_tree, v_tree = map(_f32, (q, k_cache, v_cache, k_tree, v_tree))
    parent = _i32(parent)
    n, H, d = q.shape
    Hk, cap, _ = k_cache.shape
    out = np.zeros((n, H, d), dtype=np.float64)
    rc = lib().oracle_tree_attn(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_tree), _ptr(v_tree),
                                _ptr(parent), C.c_int32(prefix_len), C.c_int32(cap), C.c_int32(n),
                                C.c_int32(H), C.c_int32(Hk), C.c_int32(d), _ptr(out))
    if rc:
        raise ValueError(f"oracle_tree_attn rc={rc}")
    return out


def tree_attn_row(q, k_cache, v_cache, k_tree, v_tree, parent, prefix_len: int, i: int, h: int,
                  want_weights: bool = False):
    """One output row (node i, head h) -> fp64 [d] (and the softmax weights if asked)."""
    q, k_cache, v_cache, k_tree, v_tree = map(_f32, (q, k_cache, v_cache, k_tree, v_tree))
    parent = _i32(parent)
    n, H, d = q.shape
    Hk, cap, _ = k_cache.shape
    out = np.zeros(d, dtype=np.float64)
    wp = np.zeros(max(prefix_len, 1), dtype=np.float64) if want_weights else None
    wt = np.zeros(n, dtype=np.float64) if want_weights else None
    rc = lib().oracle_tree_attn_row(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_tree),
                                    _ptr(v_tree), _ptr(parent), C.c_int32(prefix_len),
                                    C.c_int32(cap), C.c_int32(n), C.c_int32(H), C.c_int32(Hk),
                                    C.c_int32(d), C.c_int32(i), C.c_int32(h), _ptr(out),
                                    _ptr(wp), _ptr(wt))
    if rc:
        raise ValueError(f"oracle_tree_attn_row rc={rc}")
    if want_weights:
        return out, wp[:prefix_len], wt
    return out


@dataclass
class Decision:
    node: int
    token: int
    u: float
    R_s: float
    D_s: float
    ratio: float
    accepted: bool
    parent: int

    @property
    def margin(self) -> float:
        return abs(self.u - self.ratio)


@dataclass
class VerifyResult:
    accepted_path: np.ndarray  # [n] int32, -1 terminated
    bonus_token: int
    decisions: List[Decision]
    stop_node: int
    bonus_u: float
    bonus_total: float
    bonus_cdf_lo: float
    bonus_cdf_hi: float
    bonus_margin: float        # distance of u*sum(R) to the nearer CDF edge, relative to sum(R)
    final_R: Optional[np.ndarray]
    final_D: Optional[np.ndarray]
    degenerate: int
    fallbacks: int

    @property
    def path(self) -> List[int]:
        return [int(x) for x in self.accepted_path if x >= 0]


def verify(target_logits, draft_logits, tree_tokens, parent, temperature: float, uniforms,
           want_final: bool = False) -> VerifyResult:
    tl, dl, un = _f32(target_logits), _f32(draft_logits), _f32(uniforms)
    tok, par = _i32(tree_tokens), _i32(parent)
    n, V = tl.shape
    path = np.full(n, -1, dtype=np.int32)
    bonus = np.zeros(1, dtype=np.int32)
    dec = np.zeros((max(n - 1, 1), 8), dtype=np.float64)
    ndec = np.zeros(1, dtype=np.int32)
    binfo = np.zeros(8, dtype=np.float64)
    fR = np.zeros(V, dtype=np.float64) if want_final else None
    fD = np.zeros(V, dtype=np.float64) if want_final else None
    counters = np.zeros(2, dtype=np.int32)
    rc = lib().oracle_verify(_ptr(tl), _ptr(dl), _ptr(tok), _ptr(par), C.c_double(temperature),
                             _ptr(un), C.c_int32(n), C.c_int32(V), _ptr(path), _ptr(bonus),
                             _ptr(dec), _ptr(ndec), _ptr(binfo), _ptr(fR), _ptr(fD), _ptr(counters))
    if rc:
        raise ValueError(f"oracle_verify rc={rc}")
    decisions = [Decision(int(r[0]), int(r[1]), float(r[2]), float(r[3]), float(r[4]), float(r[5]),
                          bool(r[6]), int(r[7])) for r in dec[: int(ndec[0])]]
    return VerifyResult(path, int(bonus[0]), decisions, int(binfo[0]), float(binfo[1]),
                        float(binfo[2]), float(binfo[3]), float(binfo[4]), float(binfo[5]),
                        fR, fD, int(counters[0]), int(counters[1]))


def verify_trials(target_logits, draft_logits, tree_tokens, parent, temperature: float, uniforms
                  ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Independent walks.  tree_tokens, uniforms [trials, n]; logits [n,V] (shared) or
    [trials,n,V].  Returns (path_len, first_token, bonus) per trial."""
    tl, dl, un = _f32(target_logits), _f32(draft_logits), _f32(uniforms)
    tok, par = _i32(tree_tokens), _i32(parent)
    trials, n = tok.shape
    shared = tl.ndim == 2
    V = tl.shape[-1]
    plen = np.zeros(trials, dtype=np.int32)
    first = np.zeros(trials, dtype=np.int32)
    bonus = np.zeros(trials, dtype=np.int32)
    rc = lib().oracle_verify_trials(C.c_int64(trials), C.c_int32(1 if shared else 0), _ptr(tl),
                                    _ptr(dl), _ptr(tok), _ptr(par), C.c_double(temperature),
                                    _ptr(un), C.c_int32(n), C.c_int32(V), _ptr(plen), _ptr(first),
                                    _ptr(bonus))
    if rc:
        raise ValueError(f"oracle_verify_trials rc={rc}")
    return plen, first, bonus


# --------------------------------------------------------------------------
# the drafter's ordered draw of child tokens (sampling without replacement, Sec. 3.2.1 / 4.1)
# --------------------------------------------------------------------------
@dataclass
class DraftSample:
    tokens: np.ndarray       # [rows, k_stride] int32: the drawn tokens in order, then -1
    order_keys: np.ndarray   # [rows, k_stride + 1] float64: keys of the first k+1 tokens of the order
    order_class: np.ndarray  # [rows, k_stride + 1] int32: 1 where that token had zero probability

    def closest_call(self, r: int, k: int) -> float:
        """Smallest gap between neighbours among the first k+1 keys of row r's order (inf if
        the neighbours are of different classes): how far the order is from flipping."""
        keys, cls = self.order_keys[r, : k + 1], self.order_class[r, : k + 1]
        gaps = [keys[j] - keys[j + 1] for j in range(len(keys) - 1)
                if cls[j] == cls[j + 1] and np.isfinite(keys[j]) and np.isfinite(keys[j + 1])]
        return min(gaps) if gaps else float("inf")


def philox4x32_10(counter, key) -> np.ndarray:
    c = np.ascontiguousarray(counter, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(c.ctypes.data_as(C.c_void_p), k.ctypes.data_as(C.c_void_p),
                               out.ctypes.data_as(C.c_void_p))
    return out


def draft_uniform(seed: int, step: int, row: int, x: int) -> float:
    return float(lib().oracle_draft_uniform(C.c_uint64(seed), C.c_uint64(step), C.c_int32(row), C.c_int32(x)))


def draft_sample(draft_logits, n_children, temperature: float, seed: int, step: int,
                 k_stride: Optional[int] = None, row_ids=None) -> DraftSample:
    """row_ids: the row numbers the given rows have in the call being checked (default 0, 1, ...)."""
    dl = _f32(draft_logits)
    nc = _i32(n_children)
    ids = None if row_ids is None else _i32(row_ids)
    rows, V = dl.shape
    ks = int(max(1, nc.max())) if k_stride is None else int(k_stride)
    tokens = np.full((rows, ks), -1, dtype=np.int32)
    keys = np.zeros((rows, ks + 1), dtype=np.float64)
    cls = np.zeros((rows, ks + 1), dtype=np.int32)
    rc = lib().oracle_draft_sample(_ptr(dl), _ptr(ids), C.c_int32(rows), C.c_int32(V), _ptr(nc),
                                   C.c_double(temperature), C.c_uint64(seed), C.c_uint64(step),
                                   C.c_int32(ks), _ptr(tokens), _ptr(keys), _ptr(cls))
    if rc:
        raise ValueError(f"oracle_draft_sample rc={rc}")
    return DraftSample(tokens, keys, cls)


# --------------------------------------------------------------------------
# the baseline verification algorithms of Sec. 2.2 (SpecInfer; naive / top-k sampling)
# --------------------------------------------------------------------------
SPECINFER, TOPK = 1, 2


@dataclass
class BaselineResult:
    accepted_path: np.ndarray   # [n] int32, -1 terminated
    bonus_token: int
    records: np.ndarray         # [m, 8] float64, see verify_baselines_oracle.c
    stop_node: int
    bonus_u: float
    bonus_total: float
    bonus_cdf_lo: float
    bonus_cdf_hi: float
    bonus_margin: float

    @property
    def path(self) -> List[int]:
        return [int(x) for x in self.accepted_path if x >= 0]


def verify_baseline(algorithm: int, target_logits, draft_logits, tree_tokens, parent, temperature: float,
                    uniforms) -> BaselineResult:
    tl, dl, un = _f32(target_logits), _f32(draft_logits), _f32(uniforms)
    tok, par = _i32(tree_tokens), _i32(parent)
    n, V = tl.shape
    path = np.full(n, -1, dtype=np.int32)
    bonus = np.zeros(1, dtype=np.int32)
    rec = np.zeros((n, 8), dtype=np.float64)
    nrec = np.zeros(1, dtype=np.int32)
    binfo = np.zeros(8, dtype=np.float64)
    rc = lib().oracle_verify_baseline(C.c_int32(algorithm), _ptr(tl), _ptr(dl), _ptr(tok), _ptr(par),
                                      C.c_double(temperature), _ptr(un), C.c_int32(n), C.c_int32(V),
                                      _ptr(path), _ptr(bonus), _ptr(rec), _ptr(nrec), _ptr(binfo))
    if rc:
        raise ValueError(f"oracle_verify_baseline rc={rc}")
    return BaselineResult(path, int(bonus[0]), rec[: int(nrec[0])].copy(), int(binfo[0]), float(binfo[1]),
                          float(binfo[2]), float(binfo[3]), float(binfo[4]), float(binfo[5]))


# --------------------------------------------------------------------------
# loop glue: the accepted path's K/V rows join the prefix
# --------------------------------------------------------------------------
def kv_append(k_tree, v_tree, accepted_path, k_cache, v_cache, prefix_len: int):
    """The caches after a step: the root's rows, then the accepted nodes' rows in path order, behind
    the prefix_len valid rows of every head.  Returns (k_cache, v_cache, new_prefix_len); rows that
    do not fit the cache are dropped."""
    kc, vc = np.array(k_cache, copy=True), np.array(v_cache, copy=True)
    nodes = [0]
    for x in np.asarray(accepted_path):
        if x < 0 or x >= len(k_tree):
            break
        nodes.append(int(x))
    cap = kc.shape[1]
    for j, node in enumerate(nodes):
        if prefix_len + j < cap:
            kc[:, prefix_len + j, :] = k_tree[node]
            vc[:, prefix_len + j, :] = v_tree[node]
    return kc, vc, min(prefix_len + len(nodes), cap)


def top_p_filter(logits, top_p: float, temperature: float):
    """Nucleus filtering by its definition: sort the tokens of a row by probability (descending,
    lower id first among equals), keep the shortest prefix whose probabilities sum to at least
    top_p, set every other logit to -inf.  fp64.  Returns (filtered [rows,V] float32, probabilities
    [rows,V] float64, kept mask [rows,V] bool)."""
    x = np.asarray(logits, dtype=np.float64)
    x = np.where(np.isnan(x), -np.inf, x)
    rows, V = x.shape
    prob = np.zeros_like(x)
    keep = np.zeros(x.shape, dtype=bool)
    for r in range(rows):
        if not np.isfinite(x[r]).any() and not (x[r] == np.inf).any():
            keep[r] = temperature > 0          # a row without mass is left as it is
            continue
        if temperature == 0:
            prob[r, int(np.argmax(x[r]))] = 1.0
        else:
            z = np.exp((x[r] - x[r].max()) / temperature)
            prob[r] = z / z.sum()
        order = np.lexsort((np.arange(V), -prob[r]))
        cum = np.cumsum(prob[r][order])
        reach = np.nonzero(cum >= top_p)[0]
        # top_p = 1 is the whole support in exact arithmetic: the rounding of the running sum
        # (which reaches 1.0 a little early in fp64) must not cut it short
        n_keep = int(reach[0]) + 1 if len(reach) and top_p < 1.0 else int((prob[r] > 0).sum())
        n_keep = min(n_keep, int((prob[r] > 0).sum()))
        keep[r, order[:n_keep]] = True
    out = np.where(keep, np.asarray(logits, dtype=np.float32), np.float32(-np.inf)).astype(np.float32)
    return out, prob, keep
