"""CPU-side checks of the C-ABI library: it loads, exports what the header declares, rejects
bad arguments before touching a GPU, and builds the tree plan correctly."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2402_12374_amd as S
from paper_2402_12374_amd import binding as B
import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "seqtree.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(seq_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)
    lib = S.lib()
    for name in declared:
        assert getattr(lib, name) is not None


def test_version_and_strerror():
    assert S.version() >= 100
    assert S.strerror(0) == "ok"
    for code in range(-11, 0):
        assert "unknown" not in S.strerror(code)
    assert "unknown" in S.strerror(-99)


def _attn(parent, prefix_len=4, n=None, heads=2, kv_heads=2, head_dim=64, cap=8, dtype=B.SEQ_F32,
          ptr=0x1000, ws=0x1000, ws_bytes=1 << 30, q=0x1000, out=0x1000):
    par = np.asarray(parent, np.int32)
    n = len(par) if n is None else n
    return S.lib().seq_tree_attn(q, ptr, ptr, ptr, ptr, par.ctypes.data, prefix_len, n, heads, kv_heads,
                                 head_dim, out, cap, dtype, ws, ws_bytes, None)


def test_attn_argument_errors_need_no_gpu():
    good = [-1, 0, 0, 1]
    assert _attn(good, q=None) == B.SEQ_ERR_NULL
    assert _attn(good, out=None) == B.SEQ_ERR_NULL
    assert _attn(good, head_dim=96) == B.SEQ_ERR_SHAPE
    assert _attn(good, heads=3, kv_heads=2) == B.SEQ_ERR_SHAPE
    assert _attn(good, prefix_len=9, cap=8) == B.SEQ_ERR_SHAPE
    assert _attn(good, prefix_len=-1) == B.SEQ_ERR_SHAPE
    assert _attn(good, n=0) == B.SEQ_ERR_SHAPE
    assert _attn(good, n=B.SEQ_MAX_TREE + 1) == B.SEQ_ERR_SHAPE
    assert _attn(good, dtype=7) == B.SEQ_ERR_DTYPE
    # the kernels move the tensors 16 bytes at a time
    assert _attn(good, q=0x1008) == B.SEQ_ERR_ALIGN
    assert _attn(good, out=0x1004) == B.SEQ_ERR_ALIGN
    assert _attn(good, ptr=0x1002) == B.SEQ_ERR_ALIGN
    assert _attn([0, 0, 0, 1]) == B.SEQ_ERR_TREE
    assert _attn([-1, 0, 2, 1]) == B.SEQ_ERR_TREE
    assert _attn([-1, 0, -1, 1]) == B.SEQ_ERR_TREE
    # bf16 with a split key axis needs the workspace it asks for
    par = W.geometric_tree(64, 8)
    need = S.seq_tree_attn_workspace(1024, 64, 32, 32, 128, B.SEQ_BF16)
    assert need > 256
    assert _attn(par, prefix_len=1024, cap=1024, heads=32, kv_heads=32, head_dim=128, dtype=B.SEQ_BF16,
                 ws_bytes=need - 1) == B.SEQ_ERR_WORKSPACE
    assert _attn(par, prefix_len=1024, cap=1024, heads=32, kv_heads=32, head_dim=128, dtype=B.SEQ_BF16,
                 ws=None) == B.SEQ_ERR_WORKSPACE


def _verify(parent, n=None, vocab=64, dtype=B.SEQ_F32, temperature=1.0, ptr=0x1000, ws=0x1000,
            ws_bytes=1 << 20, tl=0x1000):
    par = np.asarray(parent, np.int32)
    n = len(par) if n is None else n
    return S.lib().seq_verify(tl, ptr, ptr, par.ctypes.data, temperature, ptr, ptr, ptr, n, vocab, dtype,
                              ws, ws_bytes, None)


def test_verify_argument_errors_need_no_gpu():
    good = [-1, 0, 0]
    assert _verify(good, tl=None) == B.SEQ_ERR_NULL
    assert _verify(good, vocab=1) == B.SEQ_ERR_SHAPE
    assert _verify(good, vocab=(1 << 19) + 1) == B.SEQ_ERR_SHAPE
    assert _verify(good, n=0) == B.SEQ_ERR_SHAPE
    assert _verify(good, dtype=0) == B.SEQ_ERR_DTYPE
    assert _verify(good, temperature=-0.5) == B.SEQ_ERR_TEMPERATURE
    assert _verify(good, temperature=float("nan")) == B.SEQ_ERR_TEMPERATURE
    assert _verify(good, temperature=float("inf")) == B.SEQ_ERR_TEMPERATURE
    assert _verify([-1, 1, 0]) == B.SEQ_ERR_TREE
    assert _verify(good, ws=None) == B.SEQ_ERR_WORKSPACE
    assert _verify(good, ws_bytes=S.seq_verify_workspace(3, 64, B.SEQ_F32) - 1) == B.SEQ_ERR_WORKSPACE


def _draft(logits=0x1000, nc=0x1000, temperature=1.0, rng=0x1000, tokens=0x1000, rows=4, vocab=100,
           k_max=8, dtype=B.SEQ_F32, ws=0x1000, ws_bytes=1 << 24):
    return S.lib().seq_draft_sample(logits, nc, temperature, rng, tokens, rows, vocab, k_max, dtype,
                                    ws, ws_bytes, None)


def test_draft_sample_argument_errors_need_no_gpu():
    for missing in ("logits", "nc", "rng", "tokens"):
        assert _draft(**{missing: None}) == B.SEQ_ERR_NULL
    assert _draft(dtype=7) == B.SEQ_ERR_DTYPE
    assert _draft(rows=0) == B.SEQ_ERR_SHAPE
    assert _draft(rows=B.SEQ_MAX_TREE + 1) == B.SEQ_ERR_SHAPE
    assert _draft(vocab=1) == B.SEQ_ERR_SHAPE
    assert _draft(vocab=B.SEQ_MAX_VOCAB + 1) == B.SEQ_ERR_SHAPE
    assert _draft(k_max=0) == B.SEQ_ERR_SHAPE
    assert _draft(k_max=B.SEQ_MAX_CHILDREN + 1, vocab=1000) == B.SEQ_ERR_SHAPE
    assert _draft(k_max=9, vocab=8) == B.SEQ_ERR_SHAPE          # more children than tokens
    for t in (-0.5, float("nan"), float("inf")):
        assert _draft(temperature=t) == B.SEQ_ERR_TEMPERATURE
    assert _draft(ws=None) == B.SEQ_ERR_WORKSPACE
    assert _draft(ws=0x1008) == B.SEQ_ERR_WORKSPACE             # not 16-byte aligned
    assert _draft(ws_bytes=S.seq_draft_sample_workspace(4, 100, 8, B.SEQ_F32) - 1) == B.SEQ_ERR_WORKSPACE


def test_verify_with_argument_errors_need_no_gpu():
    par = np.array([-1, 0, 0], dtype=np.int32)
    ptr, ws = 0x1000, 0x1000
    need = S.seq_verify_workspace(3, 64, B.SEQ_F32)

    def call(algorithm, tl=ptr, dl=ptr, temperature=1.0):
        return S.lib().seq_verify_with(algorithm, tl, dl, ptr, par.ctypes.data, temperature, ptr, ptr, ptr, 3, 64,
                                       B.SEQ_F32, ws, need, None)

    for bad in (-1, 3, 99):
        assert call(bad) == B.SEQ_ERR_ALGORITHM
    for alg in (B.SEQ_VERIFY_SEQUOIA, B.SEQ_VERIFY_SPECINFER, B.SEQ_VERIFY_TOPK):
        assert call(alg, tl=None) == B.SEQ_ERR_NULL
        assert call(alg, temperature=-1.0) == B.SEQ_ERR_TEMPERATURE
    assert call(B.SEQ_VERIFY_SEQUOIA, dl=None) == B.SEQ_ERR_NULL
    assert call(B.SEQ_VERIFY_SPECINFER, dl=None) == B.SEQ_ERR_NULL
    assert S.strerror(B.SEQ_ERR_ALGORITHM) != S.strerror(-99)


def test_verify_batched_argument_errors_need_no_gpu():
    par = np.array([-1, 0, 0], dtype=np.int32)
    ptr = 0x1000
    need = S.seq_verify_workspace(3, 64, B.SEQ_F32)

    def call(batch, ws_bytes):
        return S.lib().seq_verify_batched(B.SEQ_VERIFY_SEQUOIA, batch, ptr, ptr, ptr, par.ctypes.data, 1.0, ptr, ptr, ptr, 3, 64,
                                          B.SEQ_F32, ptr, ws_bytes, None)

    assert call(0, need) == B.SEQ_ERR_SHAPE and call(257, 257 * need) == B.SEQ_ERR_SHAPE
    assert call(4, 4 * need - 1) == B.SEQ_ERR_WORKSPACE and call(2, need) == B.SEQ_ERR_WORKSPACE


def test_workspace_sizes():
    assert S.seq_draft_sample_workspace(1, 2, 1, B.SEQ_F32) >= 256
    assert S.seq_draft_sample_workspace(768, 128256, 10, B.SEQ_BF16) >= 256
    assert S.seq_tree_attn_workspace(256, 16, 2, 2, 64, B.SEQ_F32) >= 256
    assert S.seq_verify_workspace(768, 128256, B.SEQ_BF16) >= 4 * (8 + 4 * 1024 + 4)
    # bigger trees never need less attention scratch at the same head shape
    a = S.seq_tree_attn_workspace(8192, 768, 64, 8, 128, B.SEQ_BF16)
    assert a >= 256


@pytest.mark.parametrize("n,seed", [(1, 0), (2, 1), (17, 2), (64, 3), (65, 4), (200, 5), (1024, 6)])
def test_tree_plan_against_direct_definitions(n, seed):
    rng = np.random.default_rng(seed)
    parent = W.random_topological_tree(n, rng) if seed % 2 else W.geometric_tree(n, 12)
    depth, cstart, clist, anc = S.seq_tree_plan_host(parent)
    assert anc.shape == (n, 2 * ((n + 63) // 64))
    for i in range(n):
        # walk to the root
        want_bits = np.zeros(anc.shape[1] * 32, dtype=bool)
        j, dep = i, 0
        while j >= 0:
            want_bits[j] = True
            j = int(parent[j])
            dep += 1
        assert depth[i] == dep - 1
        got_bits = np.unpackbits(anc[i].view(np.uint8), bitorder="little").astype(bool)
        assert np.array_equal(got_bits, want_bits)
        kids = [c for c in range(n) if parent[c] == i]
        assert list(clist[cstart[i]:cstart[i + 1]]) == kids  # ascending id = drafting order
    assert cstart[0] == 0 and cstart[n] == n - 1


def test_tree_plan_rejects_bad_trees():
    with pytest.raises(S.SeqTreeError) as e:
        S.seq_tree_plan_host([-1, 0, 5])
    assert e.value.code == B.SEQ_ERR_TREE
    with pytest.raises(S.SeqTreeError):
        S.seq_tree_plan_host([0])


def test_workload_generators_are_seeded_and_shaped():
    a1, a2 = W.attn_inputs_for("C1"), W.attn_inputs_for("C1")
    assert np.array_equal(a1.q, a2.q) and np.array_equal(a1.parent, a2.parent)
    assert a1.q.shape == (16, 2, 64) and a1.k_cache.shape == (2, 256, 64)
    assert W.depths(a1.parent).max() <= 4
    for key in ("C2", "C3", "C4", "C5"):
        cfg = W.CONFIGS[key]
        par = W.make_tree(cfg, 0)
        assert len(par) == cfg.n_tree and W.depths(par).max() <= cfg.max_depth
        assert all(par[i] < i for i in range(1, len(par)))
    v = W.verify_inputs_for("C2", n_tree=16, vocab=512)
    # siblings carry distinct tokens (sampling without replacement)
    for ch in W.children_lists(v.parent):
        toks = v.tree_tokens[ch]
        assert len(set(toks.tolist())) == len(ch)
    # bf16 storage: values survive a bf16 round trip exactly
    assert np.array_equal(W.quantize(v.target_logits, W.BF16), v.target_logits)
    assert (v.uniforms >= 0).all() and (v.uniforms < 1).all()


def test_acceptance_vector_of_the_generators_is_the_printed_one():
    import json
    golden = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_acceptance_vector.json")))
    assert list(W.PAPER_ACCEPTANCE_VECTOR) == golden["acceptance"]


def test_division_by_multiplication_is_exact():
    """The attention kernel divides by per-launch constants with a host-prepared multiplier; the
    host evaluation of that formula must equal integer division for every dividend below 2^31."""
    fd = S.lib().seqtree_internal_fast_div
    rng = np.random.default_rng(5)
    divisors = list(range(1, 70)) + [127, 128, 129, 255, 256, 257, 1000, 1023, 1024, 1025, 4095, 4096, 4097,
                                     65535, 65536, 65537, (1 << 26) - 1, 1 << 26, (1 << 30) + 1, (1 << 31) - 1]
    divisors += [int(x) for x in rng.integers(2, 1 << 20, size=200)]
    top = (1 << 31) - 1
    for d in divisors:
        edge = [0, 1, d - 1, d, d + 1, 2 * d - 1, 2 * d, top, top - 1, top - d, (top // d) * d, (top // d) * d - 1]
        dividends = [n for n in edge if 0 <= n <= top] + [int(x) for x in rng.integers(0, top, size=64)]
        for n in dividends:
            assert fd(n, d) == n // d, (n, d)
    # small divisors, every dividend up to 2^16 (the row and workgroup indices of the kernel)
    for d in range(1, 33):
        n = np.arange(1 << 16, dtype=np.int64)
        got = np.array([fd(int(x), d) for x in n[:: 7]], dtype=np.int64)
        assert np.array_equal(got, n[:: 7] // d)


def test_noalloc_attn_argument_errors_and_size_limit_need_no_gpu():
    good = np.asarray([-1, 0, 0, 1], np.int32)
    def call(parent=good, prefix_len=4, n=None, heads=2, kv_heads=2, head_dim=64, cap=8, dtype=B.SEQ_BF16, q=0x1000, out=0x1000):
        par = np.asarray(parent, np.int32)
        return S.lib().seq_tree_attn_noalloc(q, 0x1000, 0x1000, 0x1000, 0x1000, par.ctypes.data, prefix_len,
                                             len(par) if n is None else n, heads, kv_heads, head_dim, out, cap, dtype, None)
    assert call(q=None) == B.SEQ_ERR_NULL
    assert call(out=None) == B.SEQ_ERR_NULL
    assert call(head_dim=96) == B.SEQ_ERR_SHAPE
    assert call(heads=3, kv_heads=2) == B.SEQ_ERR_SHAPE
    assert call(prefix_len=9, cap=8) == B.SEQ_ERR_SHAPE
    assert call(n=B.SEQ_MAX_TREE + 1) == B.SEQ_ERR_SHAPE
    assert call(dtype=7) == B.SEQ_ERR_DTYPE
    assert call(parent=[-1, 0, 2, 1]) == B.SEQ_ERR_TREE
    # more partial results than the static array holds: refused before anything touches a GPU
    par = W.geometric_tree(1024, 12)
    assert S.seq_tree_attn_workspace(131072, 1024, 56, 8, 128, B.SEQ_BF16) > B.SEQ_NOALLOC_MAX_PARTIAL_BYTES
    assert call(parent=par, prefix_len=131072, cap=131072, heads=56, kv_heads=8, head_dim=128) == B.SEQ_ERR_WORKSPACE


def test_batched_attn_argument_errors_need_no_gpu():
    good = np.asarray([-1, 0, 0, 1], np.int32)
    def call(parent=good, lens=0x1000, bound=4, batch=2, heads=2, kv_heads=2, head_dim=64, cap=8, dtype=B.SEQ_BF16, q=0x1000,
             ws=0x1000, ws_bytes=1 << 30):
        par = np.asarray(parent, np.int32)
        return S.lib().seq_tree_attn_batched(q, 0x1000, 0x1000, 0x1000, 0x1000, par.ctypes.data, lens, bound, batch, len(par),
                                             heads, kv_heads, head_dim, 0x1000, cap, dtype, ws, ws_bytes, None)
    assert call(q=None) == B.SEQ_ERR_NULL
    assert call(lens=None) == B.SEQ_ERR_NULL
    assert call(batch=0) == B.SEQ_ERR_SHAPE
    assert call(batch=B.SEQ_MAX_BATCH + 1) == B.SEQ_ERR_SHAPE
    assert call(bound=9, cap=8) == B.SEQ_ERR_SHAPE
    assert call(heads=3, kv_heads=2) == B.SEQ_ERR_SHAPE
    assert call(head_dim=100) == B.SEQ_ERR_SHAPE
    assert call(dtype=0) == B.SEQ_ERR_DTYPE
    assert call(parent=[-1, 1, 0]) == B.SEQ_ERR_TREE
    par = W.geometric_tree(64, 8)
    need = S.lib().seq_tree_attn_batched_workspace(1024, 2, 64, 16, 16, 128, B.SEQ_BF16)
    assert need == S.seq_tree_attn_workspace(1024, 64, 32, 32, 128, B.SEQ_BF16) > 256
    assert call(parent=par, bound=1024, cap=1024, heads=16, kv_heads=16, head_dim=128, ws_bytes=need - 1) == B.SEQ_ERR_WORKSPACE


@pytest.fixture
def host_memory():
    """The library's own allocations come from host memory for the duration of a test, so that
    the bookkeeping of plans and synchronisation areas can be exercised without a GPU."""
    S.lib().seqtree_internal_use_host_memory(1)
    yield S.lib()
    S.lib().seqtree_internal_use_host_memory(0)


def _plan_pointers(lib, parent, stream=None):
    par = np.ascontiguousarray(parent, np.int32)
    three = (C.c_void_p * 3)()
    rc = lib.seqtree_internal_plan_pointers(par.ctypes.data, len(par), C.c_void_p(stream), three)
    return rc, tuple(three)


def _read(ptr, count, ctype):
    return np.ctypeslib.as_array(C.cast(ptr, C.POINTER(ctype)), shape=(count,)).copy()


def test_a_plan_stays_where_it_is_however_many_trees_follow(host_memory):
    """A captured graph holds a plan's device pointers: no later tree may move, free or overwrite
    it, and the tree that no longer fits is refused instead of pushing another one out."""
    lib = host_memory
    first = W.geometric_tree(64, 8)
    rc, ptrs = _plan_pointers(lib, first)
    assert rc == B.SEQ_OK and all(ptrs)
    _, cstart, clist, anc = S.seq_tree_plan_host(first)
    def intact():
        assert np.array_equal(_read(ptrs[0], anc.size, C.c_uint32), anc.ravel())
        assert np.array_equal(_read(ptrs[1], 65, C.c_int32), cstart)
        assert np.array_equal(_read(ptrs[2], 63, C.c_int32), clist)
    intact()
    for n in range(2, B.SEQ_MAX_PLANS + 1):              # 1023 more distinct trees: the cache is full
        rc, other = _plan_pointers(lib, W.chain_tree(n))
        assert rc == B.SEQ_OK and not set(other) & set(ptrs)
        if n in (34, 35, 600):                           # (the old cache held 32)
            assert _plan_pointers(lib, first) == (B.SEQ_OK, ptrs)
            intact()
    assert _plan_pointers(lib, W.star_tree(7))[0] == B.SEQ_ERR_FULL
    assert "seq_shutdown" in S.strerror(B.SEQ_ERR_FULL)
    assert _plan_pointers(lib, first) == (B.SEQ_OK, ptrs)   # a cached tree is still served
    assert _plan_pointers(lib, W.chain_tree(500))[0] == B.SEQ_OK
    intact()
    S.shutdown()
    assert _plan_pointers(lib, W.star_tree(7))[0] == B.SEQ_OK


def test_every_stream_has_a_synchronisation_area_of_its_own(host_memory):
    lib = host_memory
    def area_of(stream):
        out = C.c_void_p()
        rc = lib.seqtree_internal_sync_area_of(C.c_void_p(stream), C.byref(out))
        return rc, out.value
    rc, null_stream = area_of(None)
    assert rc == B.SEQ_OK and null_stream
    areas = {null_stream}
    for k in range(1, B.SEQ_MAX_STREAMS):
        rc, a = area_of(0x1000 * k)
        assert rc == B.SEQ_OK and a not in areas
        areas.add(a)
        assert area_of(0x1000 * k) == (B.SEQ_OK, a)       # the same stream: the same area
    assert area_of(None) == (B.SEQ_OK, null_stream)
    assert area_of(0x99000)[0] == B.SEQ_ERR_FULL          # one stream too many is refused, nothing is recycled
    S.shutdown()
    assert area_of(0x99000)[0] == B.SEQ_OK


def test_nothing_is_allocated_under_stream_capture(host_memory):
    """With host memory standing in, odd stream handles count as capturing.  A capturing stream
    gets no area of its own (that would allocate): it records with the device's first area, and
    a tree that is not cached yet is refused instead of being uploaded."""
    lib = host_memory
    def area_of(stream):
        out = C.c_void_p()
        rc = lib.seqtree_internal_sync_area_of(C.c_void_p(stream), C.byref(out))
        return rc, out.value
    tree = W.geometric_tree(40, 6)
    assert area_of(0x2001)[0] == B.SEQ_ERR_CAPTURE             # no area on this device yet
    assert _plan_pointers(lib, tree, stream=0x2001)[0] == B.SEQ_ERR_CAPTURE
    rc, first = area_of(0x1000)
    assert rc == B.SEQ_OK
    assert area_of(0x3000)[0] == B.SEQ_OK
    assert area_of(0x2001) == (B.SEQ_OK, first)                # recorded with the first stream's area
    rc, ptrs = _plan_pointers(lib, tree)                       # one call outside capture ...
    assert rc == B.SEQ_OK
    assert _plan_pointers(lib, tree, stream=0x2001) == (B.SEQ_OK, ptrs)   # ... and the capture finds the plan
    assert "capture" in S.strerror(B.SEQ_ERR_CAPTURE)


def test_no_kernel_needs_the_dispatch_packet_or_scratch_memory(tmp_path):
    """Compiled as shipped, no kernel may ask for the pointer to its dispatch packet (the packet
    lives in host memory: reading the workgroup size from it -- which is what a per-thread array
    that ends up in shared memory makes the compiler do -- costs every launch several
    microseconds) and none may spill registers to scratch memory."""
    import re
    import subprocess
    from concurrent.futures import ThreadPoolExecutor
    from paper_2402_12374_amd import build as lib_build

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

    def assembly_of(src):
        out = tmp_path / (os.path.basename(src) + ".s")
        subprocess.run([hipcc] + lib_build.HIPCC_FLAGS + ["--cuda-device-only", "-S", src, "-o", str(out)], check=True,
                       stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
        return out.read_text()

    with ThreadPoolExecutor(max_workers=8) as pool:
        listings = list(pool.map(assembly_of, lib_build.sources()))
    kernels = 0
    for src, text in zip(lib_build.sources(), listings):
        for block in re.findall(r"\.amdhsa_kernel (\S+)(.*?)\.end_amdhsa_kernel", text, flags=re.S):
            name, body = block
            kernels += 1
            assert ".amdhsa_user_sgpr_dispatch_ptr 1" not in body, (src, name)
            assert ".amdhsa_user_sgpr_queue_ptr 1" not in body, (src, name)
            assert re.search(r"\.amdhsa_private_segment_fixed_size 0\b", body), (src, name)
    assert kernels >= 20


def schedule(P, n, H, Hk, d=128):
    """(row blocks per workgroup, key ranges, short ranges, short weight, long weight) the library would take."""
    import ctypes
    five = (ctypes.c_int * 5)()
    S.lib().seqtree_internal_attn_schedule(P, n, H, Hk, d, five)
    return tuple(five)


def test_attention_schedule_takes_ranges_of_two_sizes_where_units_leave_compute_units_over():
    # the four configurations: equal ranges for the Llama2 and Vicuna shapes; the Llama3-70B one
    # (192 units on 256 compute units) gets one long and one short range per unit, the long one
    # about three quarters of the tiles (three short ones run in a row on the 64 units left over)
    assert schedule(1024, 64, 32, 32)[2:] == (0, 1, 1)
    assert schedule(2048, 128, 40, 40)[2:] == (0, 1, 1)
    assert schedule(4096, 256, 52, 52)[2:] == (0, 1, 1)
    wq, ranges, shorts, short_w, long_w = schedule(8192, 768, 64, 8)
    assert (wq, ranges, shorts) == (8, 2, 1) and short_w + long_w == 64 and 0.70 <= long_w / 64 <= 0.80
    # 96 units: two long ranges each (192 compute units) and one short one, two in a row on the other 64
    wq, ranges, shorts, short_w, long_w = schedule(8192, 384, 64, 8)
    assert (wq, ranges, shorts) == (8, 3, 1) and short_w + 2 * long_w == 64 and long_w > short_w
    # short key axes stay with equal ranges: a short range of a few tiles would be all fixed cost
    assert schedule(512, 768, 64, 8)[2] == 0
    # a forced number of ranges means equal ranges
    S.lib().seqtree_internal_set_attn_splits(4)
    try:
        assert schedule(8192, 768, 64, 8)[1:] == (4, 0, 1, 1)
    finally:
        S.lib().seqtree_internal_set_attn_splits(0)


def test_key_ranges_of_either_kind_cut_the_tiles_into_consecutive_pieces():
    start = S.lib().seqtree_internal_attn_range_start
    for ranges, shorts, short_w, long_w in ((1, 0, 1, 1), (4, 0, 1, 1), (16, 0, 1, 1), (2, 1, 15, 49), (3, 1, 12, 26),
                                            (2, 1, 1, 63), (5, 2, 3, 7), (16, 15, 1, 49), (7, 3, 2, 5)):
        for tiles in list(range(1, 400)) + [1000, 4097, 65536, 1 << 20]:
            cuts = [start(tiles, r, ranges, shorts, short_w, long_w, 0) for r in range(ranges + 1)]
            assert cuts[0] == 0 and cuts[-1] == tiles, (ranges, shorts, tiles, cuts)
            assert all(a <= b for a, b in zip(cuts, cuts[1:])), (ranges, shorts, tiles, cuts)
            total = shorts * short_w + (ranges - shorts) * long_w
            for r in range(ranges):   # a range's length is its share of the tiles, to within one tile
                share = tiles * (short_w if r < shorts else long_w) / total
                assert abs((cuts[r + 1] - cuts[r]) - share) < 1.0 + 1e-9, (ranges, shorts, tiles, r, cuts)
    # long ranges of one length for all units, counted from the end; the short ones share the rest
    for ranges, shorts, length in ((2, 1, 206), (3, 1, 100), (2, 1, 1), (5, 2, 7), (16, 15, 3), (4, 3, 50)):
        for tiles in list(range(1, 400)) + [1000, 4097, 65536, 1 << 20]:
            cuts = [start(tiles, r, ranges, shorts, 1, 1, length) for r in range(ranges + 1)]
            assert cuts[0] == 0 and cuts[-1] == tiles, (ranges, shorts, length, tiles, cuts)
            assert all(a <= b for a, b in zip(cuts, cuts[1:])), (ranges, shorts, length, tiles, cuts)
            longs = ranges - shorts
            if tiles >= longs * length:
                assert all(cuts[r + 1] - cuts[r] == length for r in range(shorts, ranges)), (ranges, shorts, length, tiles, cuts)
            else:   # too few tiles for all of them: the last ones are whole, the one before takes what is left
                assert cuts[shorts] == 0
                assert all(cuts[r + 1] - cuts[r] in (0, length) or cuts[r] == 0 for r in range(shorts, ranges)), (tiles, cuts)
            rest = cuts[shorts]
            assert all(abs((cuts[r + 1] - cuts[r]) - rest / shorts) < 1.0 + 1e-9 for r in range(shorts)), (ranges, shorts, length, tiles, cuts)


def test_long_ranges_have_one_length_where_a_kv_head_has_many_units():
    length = S.lib().seqtree_internal_attn_long_tiles
    # C5: 24 units per KV head with 256 prefix tiles and 1..24 tree tiles, 268.5 on average; the
    # long share of that, within a tile or two of 64ths (measured optimum: 207 +- 1 tiles)
    wq, ranges, shorts, short_w, long_w = schedule(8192, 768, 64, 8)
    assert (wq, ranges, shorts) == (8, 2, 1)
    assert abs(length(8192, 768, 64, 8, 128) - 268.5 * long_w / 64) <= 2.5
    assert 205 <= length(8192, 768, 64, 8, 128) <= 210
    # few units per KV head: ranges of two sizes, each its share of its own unit's tiles
    assert schedule(4096, 256, 88, 88)[2] == 1 and length(4096, 256, 88, 88, 128) == 0
    assert schedule(8192, 640, 32, 32)[2] == 1 and length(8192, 640, 32, 32, 128) == 0
    # equal ranges: no such thing
    assert length(1024, 64, 32, 32, 128) == 0
    S.lib().seqtree_internal_set_attn_long_tiles(0)
    try:
        assert length(8192, 768, 64, 8, 128) == 0
        S.lib().seqtree_internal_set_attn_long_tiles(123)
        assert length(8192, 768, 64, 8, 128) == 123 and length(4096, 256, 88, 88, 128) == 123
    finally:
        S.lib().seqtree_internal_set_attn_long_tiles(-1)
