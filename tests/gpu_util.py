"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch

import oracle
import paper_2402_12374_amd as S
import workloads as W

DEV = "cuda:0"
TOL = {W.F32: 1e-5, W.BF16: 2e-2}          # max-abs bound on attention outputs
FLAG_MARGIN = 1e-5                         # |u - R[s]/D[s]| below this: decision not compared


def to_dev(x: np.ndarray, dtype: str):
    t = torch.from_numpy(np.ascontiguousarray(x)).to(DEV)
    return (t.to(torch.bfloat16) if dtype == W.BF16 else t.to(torch.float32)).contiguous()


def run_attn(a: W.AttnInputs, **kw) -> np.ndarray:
    out = S.seq_tree_attn(to_dev(a.q, a.dtype), to_dev(a.k_cache, a.dtype), to_dev(a.v_cache, a.dtype),
                          to_dev(a.k_tree, a.dtype), to_dev(a.v_tree, a.dtype), a.parent, a.prefix_len, **kw)
    torch.cuda.synchronize()
    return out.float().cpu().numpy().astype(np.float64)


def oracle_attn(a: W.AttnInputs) -> np.ndarray:
    return oracle.tree_attn(a.q, a.k_cache, a.v_cache, a.k_tree, a.v_tree, a.parent, a.prefix_len)


def oracle_attn_all_rows(a: W.AttnInputs, workers: int = 0) -> np.ndarray:
    """Every row of the checker's answer, one call of its row routine per (node, head), spread
    over host threads (the routine is reentrant and the foreign call releases the interpreter
    lock).  The arithmetic is the checker's own, row by row; only the outer loop is shared out."""
    import ctypes as C
    import os
    from concurrent.futures import ThreadPoolExecutor
    n, H, d = a.q.shape
    Hk, cap, _ = a.k_cache.shape
    out = np.zeros((n, H, d), dtype=np.float64)
    workers = workers or min(16, os.cpu_count() or 1)
    arrays = [np.ascontiguousarray(x, dtype=np.float32) for x in (a.q, a.k_cache, a.v_cache, a.k_tree, a.v_tree)]
    parent = np.ascontiguousarray(a.parent, dtype=np.int32)
    ptrs = [x.ctypes.data_as(C.c_void_p) for x in arrays] + [parent.ctypes.data_as(C.c_void_p)]
    row = oracle.lib().oracle_tree_attn_row
    sizes = [C.c_int32(x) for x in (a.prefix_len, cap, n, H, Hk, d)]

    def rows_of(i):
        for h in range(H):
            rc = row(*ptrs, *sizes, C.c_int32(i), C.c_int32(h), C.c_void_p(out[i, h].ctypes.data), None, None)
            assert rc == 0

    with ThreadPoolExecutor(max_workers=workers) as pool:
        list(pool.map(rows_of, range(n)))
    return out


def run_verify(v: W.VerifyInputs):
    path, bonus, ws = S.seq_verify(to_dev(v.target_logits, v.dtype), to_dev(v.draft_logits, v.dtype),
                                   torch.from_numpy(v.tree_tokens).to(DEV), v.parent, v.temperature,
                                   torch.from_numpy(v.uniforms).to(DEV))
    torch.cuda.synchronize()
    trace = S.read_verify_trace(ws)
    p = path.cpu().numpy()
    return p, int(bonus.item()), trace


def check_verify(v: W.VerifyInputs, got=None):
    """Compare the library with the checker on one input.  Returns 'exact' or 'flagged'."""
    p, bonus, trace = run_verify(v) if got is None else got
    assert trace["status"] == 0
    ref = oracle.verify(v.target_logits, v.draft_logits, v.tree_tokens, v.parent, v.temperature, v.uniforms)
    n = len(v.parent)
    k = int(np.argmax(p < 0)) if (p < 0).any() else n
    assert (p[k:] == -1).all(), "tail of accepted_path must be -1"
    got_path = [int(x) for x in p[:k]]
    # decision by decision, until the first one too close to call
    for j, dec in enumerate(ref.decisions):
        if v.temperature > 0 and dec.margin < FLAG_MARGIN:
            return "flagged"
        assert j < len(trace["nodes"]), "library took fewer accept tests than the checker"
        assert int(trace["nodes"][j]) == dec.node
        assert bool(trace["accepted"][j]) == dec.accepted, (j, dec, float(trace["ratios"][j]))
        if v.temperature > 0 and np.isfinite(dec.ratio):
            assert abs(float(trace["ratios"][j]) - dec.ratio) <= 1e-5 * max(1.0, dec.ratio), (j, dec)
    assert len(trace["nodes"]) == len(ref.decisions)
    assert got_path == ref.path
    assert trace["stop_node"] == ref.stop_node
    if v.temperature > 0 and ref.bonus_margin < FLAG_MARGIN:
        return "flagged"
    assert bonus == ref.bonus_token, (bonus, ref.bonus_token, ref.bonus_margin)
    return "exact"
