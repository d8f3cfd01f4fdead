"""Thin ctypes binding of libseqtree.so: argument marshalling only.

Every step of the path runs inside the library's HIP kernels; PyTorch is used for device
memory and for the stream the work is enqueued on.  There is no CPU fallback: if the library
has not been built, loading fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libseqtree.so")

SEQ_BF16, SEQ_F32 = 1, 2
SEQ_OK = 0
SEQ_ERR_NULL, SEQ_ERR_SHAPE, SEQ_ERR_TREE, SEQ_ERR_DTYPE = -1, -2, -3, -4
SEQ_ERR_TEMPERATURE, SEQ_ERR_WORKSPACE, SEQ_ERR_HIP, SEQ_ERR_ALGORITHM, SEQ_ERR_FULL, SEQ_ERR_CAPTURE = -5, -6, -7, -8, -9, -10
SEQ_ERR_ALIGN = -11
SEQ_VERIFY_SEQUOIA, SEQ_VERIFY_SPECINFER, SEQ_VERIFY_TOPK = 0, 1, 2
SEQ_MAX_TREE = 1024
SEQ_MAX_VOCAB = 524288
SEQ_MAX_CHILDREN = 64
SEQ_MAX_PLANS = 1024
SEQ_MAX_STREAMS = 16
SEQ_MAX_BATCH = 4096
SEQ_NOALLOC_MAX_PARTIAL_BYTES = 32 << 20
TRACE_HEADER_INTS, TRACE_RECORD_WORDS = 8, 4

EXPORTS = ("seq_tree_attn", "seq_tree_attn_noalloc", "seq_tree_attn_batched", "seq_tree_attn_batched_workspace", "seq_verify", "seq_verify_with", "seq_verify_batched", "seq_draft_sample", "seq_kv_append", "seq_top_p_filter", "seq_tree_attn_workspace",
           "seq_verify_workspace", "seq_draft_sample_workspace", "seq_tree_plan_host",
           "seq_build_tree", "seq_tree_expected_tokens", "seq_pick_tree_shape",
           "seq_shutdown", "seq_strerror", "seq_version")

_lib: Optional[C.CDLL] = None


class SeqTreeError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} (code {code})")


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'"
                " or python paper_2402_12374_amd/build.py); there is no fallback path")
        l = C.CDLL(LIB_PATH)
        vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        l.seq_tree_attn.restype = C.c_int
        l.seq_tree_attn.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, i32, i32, vp, sz, vp]
        l.seq_tree_attn_noalloc.restype = C.c_int
        l.seq_tree_attn_noalloc.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, i32, i32, vp]
        l.seq_tree_attn_batched.restype = C.c_int
        l.seq_tree_attn_batched.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, i32, i32, vp, sz, vp]
        l.seq_tree_attn_batched_workspace.restype = sz
        l.seq_tree_attn_batched_workspace.argtypes = [i32] * 7
        l.seq_verify.restype = C.c_int
        l.seq_verify.argtypes = [vp, vp, vp, vp, C.c_float, vp, vp, vp, i32, i32, i32, vp, sz, vp]
        l.seq_verify_batched.restype = C.c_int
        l.seq_verify_batched.argtypes = [i32, i32, vp, vp, vp, vp, C.c_float, vp, vp, vp, i32, i32, i32, vp, sz, vp]
        l.seq_verify_with.restype = C.c_int
        l.seq_verify_with.argtypes = [i32, vp, vp, vp, vp, C.c_float, vp, vp, vp, i32, i32, i32, vp, sz, vp]
        l.seq_top_p_filter.restype = C.c_int
        l.seq_top_p_filter.argtypes = [vp, vp, C.c_float, C.c_float, i32, i32, i32, vp, vp]
        l.seq_kv_append.restype = C.c_int
        l.seq_kv_append.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp]
        l.seq_tree_attn_workspace.restype = sz
        l.seq_tree_attn_workspace.argtypes = [i32] * 6
        l.seq_verify_workspace.restype = sz
        l.seq_verify_workspace.argtypes = [i32] * 3
        l.seq_draft_sample.restype = C.c_int
        l.seq_draft_sample.argtypes = [vp, vp, C.c_float, vp, vp, i32, i32, i32, i32, vp, sz, vp]
        l.seq_draft_sample_workspace.restype = sz
        l.seq_draft_sample_workspace.argtypes = [i32] * 4
        l.seqtree_internal_set_topk_mode.restype = None
        l.seqtree_internal_set_topk_mode.argtypes = [C.c_int]
        l.seqtree_internal_set_draft_chunks.restype = None
        l.seqtree_internal_set_draft_chunks.argtypes = [C.c_int]
        l.seqtree_internal_set_draft_max_groups.restype = None
        l.seqtree_internal_set_draft_max_groups.argtypes = [C.c_int]
        l.seq_tree_plan_host.restype = C.c_int
        l.seq_tree_plan_host.argtypes = [vp, i32, vp, vp, vp, vp]
        l.seq_build_tree.restype = C.c_int
        l.seq_build_tree.argtypes = [vp, i32, i32, i32, vp, vp]
        l.seq_tree_expected_tokens.restype = C.c_int
        l.seq_tree_expected_tokens.argtypes = [vp, i32, vp, i32, vp]
        l.seq_pick_tree_shape.restype = C.c_int
        l.seq_pick_tree_shape.argtypes = [vp, i32, vp, vp, i32, i32, C.c_double, C.c_double, vp, vp, vp]
        l.seq_shutdown.restype = C.c_int
        l.seq_strerror.restype = C.c_char_p
        l.seq_strerror.argtypes = [C.c_int]
        l.seq_version.restype = C.c_int
        l.seqtree_internal_copy_probe.restype = C.c_int
        l.seqtree_internal_copy_probe.argtypes = [vp, vp, sz, vp]
        l.seqtree_internal_use_host_memory.restype = None
        l.seqtree_internal_use_host_memory.argtypes = [C.c_int]
        l.seqtree_internal_plan_pointers.restype = C.c_int
        l.seqtree_internal_plan_pointers.argtypes = [vp, i32, vp, vp]
        l.seqtree_internal_sync_area_of.restype = C.c_int
        l.seqtree_internal_sync_area_of.argtypes = [vp, vp]
        l.seqtree_internal_fast_div.restype = C.c_uint32
        l.seqtree_internal_fast_div.argtypes = [C.c_uint32, C.c_uint32]
        _lib = l
    return _lib


def strerror(code: int) -> str:
    return lib().seq_strerror(code).decode()


def version() -> int:
    return lib().seq_version()


def shutdown() -> None:
    lib().seq_shutdown()


def _parent_array(parent) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(parent), dtype=np.int32)


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return SEQ_BF16
    if t.dtype == torch.float32:
        return SEQ_F32
    raise SeqTreeError(SEQ_ERR_DTYPE, "dtype")


def _stream_ptr(stream=None) -> int:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def seq_tree_plan_host(parent):
    """(depth, child_start, child_list, anc_words[n, words_per_row]) computed on the host."""
    par = _parent_array(parent)
    n = len(par)
    wpr = 2 * ((n + 63) // 64)
    depth = np.zeros(n, np.int32)
    cstart = np.zeros(n + 1, np.int32)
    clist = np.zeros(max(n - 1, 1), np.int32)
    anc = np.zeros((n, wpr), np.uint32)
    rc = lib().seq_tree_plan_host(par.ctypes.data, n, depth.ctypes.data, cstart.ctypes.data,
                                  clist.ctypes.data, anc.ctypes.data)
    if rc != SEQ_OK:
        raise SeqTreeError(rc, "seq_tree_plan_host")
    return depth, cstart, clist[: n - 1], anc


def _rates(acceptance) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(acceptance, dtype=np.float64))


def seq_build_tree(acceptance, n_tree: int, max_depth: int):
    """The Sequoia tree of n_tree nodes and depth <= max_depth for this acceptance vector (host
    only).  Returns (parent int32 [n_tree], expected tokens per verification)."""
    p = _rates(acceptance)
    parent = np.zeros(max(int(n_tree), 1), np.int32)
    f = C.c_double(0.0)
    rc = lib().seq_build_tree(p.ctypes.data, len(p), int(n_tree), int(max_depth), parent.ctypes.data, C.byref(f))
    if rc != SEQ_OK:
        raise SeqTreeError(rc, "seq_build_tree")
    return parent, f.value


def seq_tree_expected_tokens(parent, acceptance) -> float:
    par, p = _parent_array(parent), _rates(acceptance)
    f = C.c_double(0.0)
    rc = lib().seq_tree_expected_tokens(par.ctypes.data, len(par), p.ctypes.data, len(p), C.byref(f))
    if rc != SEQ_OK:
        raise SeqTreeError(rc, "seq_tree_expected_tokens")
    return f.value


def seq_pick_tree_shape(acceptance, sizes, verify_time, max_depth: int, decode_time: float, draft_time: float):
    """(size, depth, speedup) maximising G(n, d) / (t(n) + d c) over the given sizes (host only)."""
    p = _rates(acceptance)
    sz = np.ascontiguousarray(np.asarray(sizes), dtype=np.int32)
    vt = np.ascontiguousarray(np.asarray(verify_time), dtype=np.float64)
    n, d, s = C.c_int32(0), C.c_int32(0), C.c_double(0.0)
    rc = lib().seq_pick_tree_shape(p.ctypes.data, len(p), sz.ctypes.data, vt.ctypes.data, len(sz), int(max_depth),
                                   float(decode_time), float(draft_time), C.byref(n), C.byref(d), C.byref(s))
    if rc != SEQ_OK:
        raise SeqTreeError(rc, "seq_pick_tree_shape")
    return n.value, d.value, s.value


def seq_tree_attn_workspace(prefix_len, n_tree, heads, kv_heads, head_dim, dtype_code) -> int:
    return int(lib().seq_tree_attn_workspace(prefix_len, n_tree, heads, kv_heads, head_dim, dtype_code))


def seq_verify_workspace(n_tree, vocab, dtype_code) -> int:
    return int(lib().seq_verify_workspace(n_tree, vocab, dtype_code))


def seq_tree_attn(q, k_cache, v_cache, k_tree, v_tree, parent, prefix_len: int, out=None,
                  workspace=None, stream=None):
    """q [n,H,d]; k_cache/v_cache [Hk,cap,d]; k_tree/v_tree [n,Hk,d] (torch, on the GPU);
    parent: host int array.  Returns out [n,H,d].  Asynchronous on the current stream."""
    import torch
    par = _parent_array(parent)
    n, H, d = q.shape
    Hk, cap = k_cache.shape[0], k_cache.shape[1]
    code = _dtype_code(q)
    for t in (q, k_cache, v_cache, k_tree, v_tree):
        if not t.is_contiguous() or not t.is_cuda or t.dtype != q.dtype:
            raise SeqTreeError(SEQ_ERR_SHAPE, "seq_tree_attn (tensors must be contiguous GPU tensors of one dtype)")
    if out is None:
        out = torch.empty_like(q)
    need = seq_tree_attn_workspace(prefix_len, n, H, Hk, d, code)
    if workspace is None or workspace.numel() * workspace.element_size() < need:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    rc = lib().seq_tree_attn(q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(), k_tree.data_ptr(),
                             v_tree.data_ptr(), par.ctypes.data, int(prefix_len), n, H, Hk, d,
                             out.data_ptr(), cap, code, workspace.data_ptr(),
                             workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    if rc != SEQ_OK:
        raise SeqTreeError(rc, "seq_tree_attn")
    return out


def seq_tree_attn_batched(q, k_cache, v_cache, k_tree, v_tree, parent, prefix_lens, max_prefix_len: int, out=None,
                          workspace=None, stream=None):
    """q [n,B,H,d]; k_cache/v_cache [B,Hk,cap,d]; k_tree/v_tree [n,B,Hk,d]; prefix_lens int32 [B] (all torch, on the
    GPU); parent: host int array.  Returns out [n,B,H,d].  Asynchronous on the current stream."""
    import torch
    par = _parent_array(parent)
    n, B, H, d = q.shape
    Hk, cap = k_cache.shape[1], k_cache.shape[2]
    code = _dtype_code(q)
    for t in (q, k_cache, v_cache, k_tree, v_tree):
        if not t.is_contiguous() or not t.is_cuda or t.dtype != q.dtype:
            raise SeqTreeError(SEQ_ERR_SHAPE, "seq_tree_attn_batched (tensors must be contiguous GPU tensors of one dtype)")
    if prefix_lens.dtype != torch.int32 or prefix_lens.numel() != B or not prefix_lens.is_cuda or not prefix_lens.is_contiguous():
        raise SeqTreeError(SEQ_ERR_SHAPE, "seq_tree_attn_batched (prefix_lens: int32 [batch] on the GPU)")
    if out is None:
        out = torch.empty_like(q)
    need = int(lib().seq_tree_attn_batched_workspace(int(max_prefix_len), B, n, H, Hk, d, code))
    if workspace is None or workspace.numel() * workspace.element_size() < need:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    rc = lib().seq_tree_attn_batched(q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(), k_tree.data_ptr(),
                                     v_tree.data_ptr(), par.ctypes.data, prefix_lens.data_ptr(), int(max_prefix_len), B, n, H, Hk, d,
                                     out.data_ptr(), cap, code, workspace.data_ptr(),
                                     workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    if rc != SEQ_OK:
        raise SeqTreeError(rc, "seq_tree_attn_batched")
    return out


def seq_tree_attn_noalloc(q, k_cache, v_cache, k_tree, v_tree, parent, prefix_len: int, out, stream=None):
    """seq_tree_attn through the entry point that allocates nothing: `out` [n,H,d] comes from the
    caller, there is no workspace.  Returns out.  Asynchronous on the current stream."""
    par = _parent_array(parent)
    n, H, d = q.shape
    Hk, cap = k_cache.shape[0], k_cache.shape[1]
    code = _dtype_code(q)
    for t in (q, k_cache, v_cache, k_tree, v_tree, out):
        if not t.is_contiguous() or not t.is_cuda or t.dtype != q.dtype:
            raise SeqTreeError(SEQ_ERR_SHAPE, "seq_tree_attn_noalloc (tensors must be contiguous GPU tensors of one dtype)")
    rc = lib().seq_tree_attn_noalloc(q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(), k_tree.data_ptr(),
                                     v_tree.data_ptr(), par.ctypes.data, int(prefix_len), n, H, Hk, d,
                                     out.data_ptr(), cap, code, _stream_ptr(stream))
    if rc != SEQ_OK:
        raise SeqTreeError(rc, "seq_tree_attn_noalloc")
    return out


def seq_verify(target_logits, draft_logits, tree_tokens, parent, temperature: float, uniforms,
               accepted_path=None, bonus_token=None, workspace=None, stream=None, algorithm: int = SEQ_VERIFY_SEQUOIA):
    """Logits [n,V] (bf16 or fp32), tree_tokens int32 [n], uniforms float32 [n] on the GPU; parent
    on the host.  Returns (accepted_path int32 [n], bonus_token int32 [1], workspace) -- device
    tensors, valid after the stream has been synchronised."""
    import torch
    par = _parent_array(parent)
    n, V = target_logits.shape
    code = _dtype_code(target_logits)
    if accepted_path is None:
        accepted_path = torch.empty(n, dtype=torch.int32, device=target_logits.device)
    if bonus_token is None:
        bonus_token = torch.empty(1, dtype=torch.int32, device=target_logits.device)
    need = seq_verify_workspace(n, V, code)
    if workspace is None or workspace.numel() * workspace.element_size() < need:
        workspace = torch.empty(need, dtype=torch.uint8, device=target_logits.device)
    for t in (target_logits, draft_logits, tree_tokens, uniforms):
        if t is not None and (not t.is_contiguous() or not t.is_cuda):
            raise SeqTreeError(SEQ_ERR_SHAPE, "seq_verify (tensors must be contiguous GPU tensors)")
    args = (target_logits.data_ptr(), None if draft_logits is None else draft_logits.data_ptr(),
            tree_tokens.data_ptr(), par.ctypes.data, float(temperature), uniforms.data_ptr(),
            accepted_path.data_ptr(), bonus_token.data_ptr(), n, V, code,
            workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    rc = lib().seq_verify(*args) if algorithm == SEQ_VERIFY_SEQUOIA else lib().seq_verify_with(int(algorithm), *args)
    if rc != SEQ_OK:
        raise SeqTreeError(rc, "seq_verify")
    return accepted_path, bonus_token, workspace


def seq_draft_sample_workspace(n_rows, vocab, k_max, dtype_code) -> int:
    return int(lib().seq_draft_sample_workspace(n_rows, vocab, k_max, dtype_code))


def seq_draft_sample(draft_logits, n_children, temperature: float, rng, k_max: int, tokens=None,
                     workspace=None, stream=None):
    """draft_logits [rows,V] (bf16 or fp32), n_children int32 [rows], rng int64 [2] = (seed, step),
    all on the GPU.  Returns (tokens int32 [rows,k_max], workspace)."""
    import torch
    rows, V = draft_logits.shape
    code = _dtype_code(draft_logits)
    for t in (draft_logits, n_children, rng):
        if not t.is_contiguous() or not t.is_cuda:
            raise SeqTreeError(SEQ_ERR_SHAPE, "seq_draft_sample (tensors must be contiguous GPU tensors)")
    if n_children.dtype != torch.int32 or n_children.numel() != rows or rng.element_size() != 8 or rng.numel() != 2:
        raise SeqTreeError(SEQ_ERR_SHAPE, "seq_draft_sample (n_children int32 [rows], rng 64-bit [2])")
    if tokens is None:
        tokens = torch.empty((rows, max(int(k_max), 1)), dtype=torch.int32, device=draft_logits.device)
    need = seq_draft_sample_workspace(rows, V, k_max, code)
    if workspace is None or workspace.numel() * workspace.element_size() < need:
        workspace = torch.empty(need, dtype=torch.uint8, device=draft_logits.device)
    rc = lib().seq_draft_sample(draft_logits.data_ptr(), n_children.data_ptr(), float(temperature),
                                rng.data_ptr(), tokens.data_ptr(), rows, V, int(k_max), code,
                                workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                _stream_ptr(stream))
    if rc != SEQ_OK:
        raise SeqTreeError(rc, "seq_draft_sample")
    return tokens, workspace


def seq_top_p_filter(logits, top_p: float, temperature: float, filtered=None, kept=None, stream=None):
    """logits [rows,V] (bf16 or fp32, GPU).  Returns (filtered logits, kept int32 [rows])."""
    import torch
    rows, V = logits.shape
    code = _dtype_code(logits)
    if not logits.is_contiguous() or not logits.is_cuda:
        raise SeqTreeError(SEQ_ERR_SHAPE, "seq_top_p_filter (logits must be a contiguous GPU tensor)")
    if filtered is None:
        filtered = torch.empty_like(logits)
    if kept is None:
        kept = torch.empty(rows, dtype=torch.int32, device=logits.device)
    rc = lib().seq_top_p_filter(logits.data_ptr(), filtered.data_ptr(), float(top_p), float(temperature), rows, V, code,
                                kept.data_ptr(), _stream_ptr(stream))
    if rc != SEQ_OK:
        raise SeqTreeError(rc, "seq_top_p_filter")
    return filtered, kept


def seq_kv_append(k_tree, v_tree, accepted_path, parent, k_cache, v_cache, prefix_len: int, new_prefix_len=None,
                  stream=None):
    """Appends the root's and the accepted nodes' K/V rows to the caches in place (GPU tensors;
    accepted_path int32 [n] on the GPU, parent on the host).  Returns new_prefix_len (int32 [1], GPU)."""
    import torch
    par = _parent_array(parent)
    n, Hk, d = k_tree.shape
    code = _dtype_code(k_tree)
    for t in (k_tree, v_tree, k_cache, v_cache, accepted_path):
        if not t.is_contiguous() or not t.is_cuda:
            raise SeqTreeError(SEQ_ERR_SHAPE, "seq_kv_append (tensors must be contiguous GPU tensors)")
    if new_prefix_len is None:
        new_prefix_len = torch.empty(1, dtype=torch.int32, device=k_tree.device)
    rc = lib().seq_kv_append(k_tree.data_ptr(), v_tree.data_ptr(), accepted_path.data_ptr(), par.ctypes.data,
                             k_cache.data_ptr(), v_cache.data_ptr(), int(prefix_len), n, Hk, d, k_cache.shape[1], code,
                             new_prefix_len.data_ptr(), _stream_ptr(stream))
    if rc != SEQ_OK:
        raise SeqTreeError(rc, "seq_kv_append")
    return new_prefix_len


def seq_verify_batched(algorithm: int, target_logits, draft_logits, tree_tokens, parent, temperature: float, uniforms,
                       accepted_path=None, bonus_token=None, workspace=None, stream=None):
    """Logits [B,n,V]; tree_tokens int32 [B,n]; uniforms float32 [B,n] (GPU); parent on the host.
    Returns (accepted_path int32 [B,n], bonus_token int32 [B], workspace uint8 [B, bytes per sequence])."""
    import torch
    par = _parent_array(parent)
    B, n, V = target_logits.shape
    code = _dtype_code(target_logits)
    dev = target_logits.device
    if accepted_path is None:
        accepted_path = torch.empty((B, n), dtype=torch.int32, device=dev)
    if bonus_token is None:
        bonus_token = torch.empty(B, dtype=torch.int32, device=dev)
    per = seq_verify_workspace(n, V, code)
    if workspace is None or workspace.numel() * workspace.element_size() < per * B:
        workspace = torch.empty((B, per), dtype=torch.uint8, device=dev)
    for t in (target_logits, draft_logits, tree_tokens, uniforms):
        if t is not None and (not t.is_contiguous() or not t.is_cuda):
            raise SeqTreeError(SEQ_ERR_SHAPE, "seq_verify_batched (tensors must be contiguous GPU tensors)")
    rc = lib().seq_verify_batched(int(algorithm), B, target_logits.data_ptr(),
                                  None if draft_logits is None else draft_logits.data_ptr(), tree_tokens.data_ptr(),
                                  par.ctypes.data, float(temperature), uniforms.data_ptr(), accepted_path.data_ptr(),
                                  bonus_token.data_ptr(), n, V, code, workspace.data_ptr(),
                                  workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    if rc != SEQ_OK:
        raise SeqTreeError(rc, "seq_verify_batched")
    return accepted_path, bonus_token, workspace


def seq_verify_with(algorithm: int, target_logits, draft_logits, tree_tokens, parent, temperature: float, uniforms,
                    **kw):
    """seq_verify with one of SEQ_VERIFY_SEQUOIA / SEQ_VERIFY_SPECINFER / SEQ_VERIFY_TOPK at every node."""
    return seq_verify(target_logits, draft_logits, tree_tokens, parent, temperature, uniforms,
                      algorithm=algorithm, **kw)


def read_verify_trace(workspace) -> dict:
    """Decode the trace seq_verify leaves at the start of its workspace (synchronises).  For
    SEQ_VERIFY_TOPK at T > 0 the records read: nodes = visited node, accepted = a child matched,
    and raw[:, 1] / raw[:, 2] (kept as 'children' / 'drawn') the accepted child or -1 and the drawn token."""
    raw = workspace.cpu().numpy().view(np.int32)
    n_dec, status, stop, fallbacks, degenerate = (int(x) for x in raw[:5])
    rec = raw[TRACE_HEADER_INTS: TRACE_HEADER_INTS + n_dec * TRACE_RECORD_WORDS].reshape(-1, 4)
    binfo = raw[TRACE_HEADER_INTS + SEQ_MAX_TREE * TRACE_RECORD_WORDS:][:4].view(np.float32)
    return {
        "status": status, "stop_node": stop, "fallbacks": fallbacks, "degenerate": degenerate,
        "nodes": rec[:, 0].copy(), "accepted": rec[:, 1].astype(bool), "children": rec[:, 1].copy(), "drawn": rec[:, 2].copy(),
        "ratios": rec[:, 2].copy().view(np.float32), "uniforms": rec[:, 3].copy().view(np.float32),
        "bonus_u": float(binfo[0]), "bonus_total": float(binfo[1]),
        "bonus_cdf_lo": float(binfo[2]), "bonus_cdf_hi": float(binfo[3]),
    }
