#!/usr/bin/env python3
"""Benchmark of the tree-verify step on one MI355X.

A step is one pass of the hot path over one set of synthetic inputs: one seq_tree_attn call
(one attention layer of the target's forward pass over the tree) followed by one seq_verify
call (the verification walk).  Consecutive steps use different input sets (as many K/V sets as
the model has layers), so no step finds its K/V or logits in a cache left by the previous one.
All inputs are in HBM before the timed region starts.

Prints ONE JSON line: `value` is the wall time per step at the largest configuration; `roofline`
prices that configuration's attention kernel (algorithmic flops over its launch time from HIP
events around graph replays, against the dense bf16 matrix peak), `verify` the verification kernel,
`configs` the other configurations, `cpu_baseline` the fp64 checker on the same workload.

Other modes print lines of their own instead of the benchmark line: --sweep (latency of both calls
over the tree size; --sweep-tree sequoia for trees built by seq_build_tree; --sweep-prefix for another
prefix length than the configurations'; --pick-tree for the hardware-aware choice fed with the measured times), --draft-sample (seq_draft_sample per
configuration), --rejection-curve (rejection rate against the number of children for the three
verification algorithms), --verify-batch (seq_verify_batched over the batch size).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0

TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "tree_attn_mfma_hbm_traffic_per_config.md")


def load_traffic_table():
    """HBM bytes per launch of the attention kernel for each configuration, as measured with rocprofv3 --pmc
    FETCH_SIZE / WRITE_SIZE and scaled by a copy kernel of known size.  Counters cannot be read from inside
    this process: the committed summary (which gives the commands and the raw counters) is the source, its
    table rows read `| C5 | ... | <total bytes> |`.  A configuration without a row reports null."""
    table = {}
    try:
        for row in open(TRAFFIC_TABLE):
            cells = [c.strip() for c in row.strip().strip("|").split("|")]
            if len(cells) >= 3 and cells[0] in ("C1", "C2", "C3", "C4", "C5") and cells[-1].replace(" ", "").isdigit():
                table[cells[0]] = int(cells[-1].replace(" ", ""))
    except OSError:
        pass
    return table


def attn_alg_bytes(cfg, n=None, P=None):
    e = 2 if cfg.dtype == "bf16" else 4
    n = cfg.n_tree if n is None else n
    P = cfg.prefix_len if P is None else P
    H, Hk, d = cfg.heads, cfg.kv_heads, cfg.head_dim
    return 2 * Hk * P * d * e + 2 * n * Hk * d * e + 2 * n * H * d * e + n * ((n + 63) // 64) * 8


def attn_alg_flops(cfg, parent):
    import workloads as W
    visible = int((W.depths(parent) + 1).sum())
    return 4 * cfg.head_dim * cfg.heads * (len(parent) * cfg.prefix_len + visible)


_SIDE_STREAM = None


def side_stream(torch):
    """One stream beside the default one for all warm-ups under capture rules: the library keeps a
    synchronisation area per stream it has been called on, and has room for a few of them."""
    global _SIDE_STREAM
    if _SIDE_STREAM is None:
        _SIDE_STREAM = torch.cuda.Stream()
    return _SIDE_STREAM


def graph_time_us(torch, fn, count, reps):
    """Average duration of one call of fn(i), i = 0..count-1 captured once as a HIP graph."""
    fn(0)
    torch.cuda.synchronize()
    side = side_stream(torch)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for i in range(count):
            fn(i)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for i in range(count):
            fn(i)
    for _ in range(3):
        graph.replay()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for _ in range(reps):
        graph.replay()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) * 1e3 / (reps * count)


def capture(torch, fn, indices):
    """fn(i) for i in indices as a HIP graph.  (The workload has made one eager call already: the tree's plan
    and the stream's synchronisation area exist, so nothing is allocated while recording.)"""
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for i in indices:
            fn(i)
    return graph


def percentiles(values):
    v = sorted(values)
    pick = lambda q: round(v[min(len(v) - 1, int(q * len(v)))], 3)
    return {"p10": pick(0.10), "p50": pick(0.50), "p90": pick(0.90), "blocks": len(v)}


def timed_replays(torch, graph, launches_per_replay, blocks):
    """Replays a graph `blocks` times with a HIP event (on the launching stream) between every two replays.
    Returns (average us per launch over all blocks, spread of the per-block averages)."""
    for _ in range(2):
        graph.replay()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(blocks + 1)]
    torch.cuda.synchronize()
    marks[0].record()
    for b in range(blocks):
        graph.replay()
        marks[b + 1].record()
    torch.cuda.synchronize()
    per_block = [marks[b].elapsed_time(marks[b + 1]) * 1e3 / launches_per_replay for b in range(blocks)]
    total = marks[0].elapsed_time(marks[blocks]) * 1e3 / (launches_per_replay * blocks)
    return total, percentiles(per_block)


class Workload:
    """One configuration's synthetic inputs, resident in HBM: as many K/V/Q sets as the model has layers (so
    that no call finds its inputs in a cache left by the one before) and as many logit sets as 2 GiB hold."""

    def __init__(self, key, torch, dev, sets=0, vocab=0):
        import dataclasses
        import paper_2402_12374_amd as S
        import workloads as W
        self.S, self.W, self.torch, self.key = S, W, torch, key
        cfg = self.cfg = W.CONFIGS[key] if vocab <= 0 else dataclasses.replace(W.CONFIGS[key], vocab=vocab)
        idx = list(W.CONFIGS).index(key) + 1
        self.tdt = tdt = torch.bfloat16 if cfg.dtype == W.BF16 else torch.float32
        self.code = 1 if tdt == torch.bfloat16 else 2
        self.T = T = cfg.temperatures[0]
        self.sets = sets = sets or cfg.layers
        self.parent = parent = W.make_tree(cfg, W.seed_for(idx))
        self.n, self.V = n, V = cfg.n_tree, cfg.vocab
        H, Hk, d, P = cfg.heads, cfg.kv_heads, cfg.head_dim, cfg.prefix_len
        g = torch.Generator(device=dev)
        g.manual_seed(W.seed_for(idx))

        def randn(*shape, scale=1.0):
            return (torch.randn(*shape, generator=g, device=dev, dtype=torch.float32) * scale).to(tdt).contiguous()

        self.attn_sets = [dict(q=randn(n, H, d), kc=randn(Hk, P, d), vc=randn(Hk, P, d), kt=randn(n, Hk, d), vt=randn(n, Hk, d),
                               out=torch.empty(n, H, d, device=dev, dtype=tdt)) for _ in range(sets)]
        e = 2 if tdt == torch.bfloat16 else 4
        self.n_vsets = max(1, min(sets, 32, (2 << 30) // (2 * n * V * e)))
        # set 0 comes from the seeded host generator
        self.host0 = W.verify_inputs_for(key) if vocab <= 0 else W.make_verify_inputs(
            parent, V, cfg.sigma_target, cfg.sigma_draft, T, cfg.dtype, seed=W.seed_for(idx))
        children = [(node, ch) for node, ch in enumerate(W.children_lists(parent)) if ch]
        self.verify_sets = []
        for s in range(self.n_vsets):
            if s == 0:
                tl = torch.from_numpy(self.host0.target_logits).to(dev).to(tdt)
                dl = torch.from_numpy(self.host0.draft_logits).to(dev).to(tdt)
                tok = torch.from_numpy(self.host0.tree_tokens).to(dev)
                un = torch.from_numpy(self.host0.uniforms).to(dev)
            else:
                tl = randn(n, V, scale=cfg.sigma_target)
                dl = (tl.float() + torch.randn(n, V, generator=g, device=dev) * cfg.sigma_draft).to(tdt)
                # ordered children without replacement: Gumbel-top-k on the tempered draft logits
                tok = torch.zeros(n, dtype=torch.int32, device=dev)
                for node, ch in children:
                    u = torch.rand(V, generator=g, device=dev).clamp_(1e-20, 1.0)
                    gumbel_key = dl[node].float() / max(T, 1e-6) - torch.log(-torch.log(u))
                    tok[torch.tensor(ch, device=dev)] = torch.topk(gumbel_key, len(ch)).indices.to(torch.int32)
                un = torch.rand(n, generator=g, device=dev, dtype=torch.float32).clamp_(0.0, 1.0 - 2.0 ** -24)
            self.verify_sets.append(dict(tl=tl.contiguous(), dl=dl.contiguous(), tok=tok, un=un,
                                         path=torch.empty(n, dtype=torch.int32, device=dev),
                                         bonus=torch.empty(1, dtype=torch.int32, device=dev),
                                         ws=torch.empty(S.seq_verify_workspace(n, V, self.code), dtype=torch.uint8, device=dev)))
        self.attn_ws = torch.empty(S.seq_tree_attn_workspace(P, n, H, Hk, d, self.code), dtype=torch.uint8, device=dev)
        torch.cuda.synchronize()
        self.step(0)   # builds the tree plan and the stream's synchronisation area (the library's only allocations)
        torch.cuda.synchronize()

    def attn_call(self, i):
        a = self.attn_sets[i % self.sets]
        self.S.seq_tree_attn(a["q"], a["kc"], a["vc"], a["kt"], a["vt"], self.parent, self.cfg.prefix_len, out=a["out"],
                             workspace=self.attn_ws)

    def verify_call(self, i, temperature=None):
        v = self.verify_sets[i % self.n_vsets]
        self.S.seq_verify(v["tl"], v["dl"], v["tok"], self.parent, self.T if temperature is None else temperature, v["un"],
                          accepted_path=v["path"], bonus_token=v["bonus"], workspace=v["ws"])

    def step(self, i):
        self.attn_call(i)
        self.verify_call(i)

    def describe(self):
        c, W = self.cfg, self.W
        return (f"{c.name}: H{c.heads}/Hk{c.kv_heads}/d{c.head_dim} {c.dtype}, prefix {c.prefix_len}, tree {self.n} "
                f"(geometric, depth {int(W.depths(self.parent).max())}), vocab {self.V}, T={self.T}")

    def release(self):
        self.attn_sets = self.verify_sets = self.attn_ws = None
        self.torch.cuda.empty_cache()

    def check_results(self):
        """The last verification of set 0 (the seeded, host-generated one) ended normally."""
        trace = self.S.read_verify_trace(self.verify_sets[0]["ws"])
        assert trace["status"] == 0
        self.path0 = [int(x) for x in self.verify_sets[0]["path"].cpu().numpy() if x >= 0]

    def measure_kernels(self, blocks, traffic):
        """Each kernel alone on the stream: one graph holding one launch per input set, replayed `blocks` times
        with an event between replays.  Returns the step time and a roofline object per kernel."""
        torch, cfg, W, n, V = self.torch, self.cfg, self.W, self.n, self.V
        idx = range(self.sets)
        attn_us, attn_spread = timed_replays(torch, capture(torch, self.attn_call, idx), self.sets, blocks)
        verify_us, verify_spread = timed_replays(torch, capture(torch, self.verify_call, idx), self.sets, blocks)
        step_us, step_spread = timed_replays(torch, capture(torch, self.step, idx), self.sets, blocks)
        self.check_results()

        bytes_alg, flops_alg = attn_alg_bytes(cfg), attn_alg_flops(cfg, self.parent)
        gbs = bytes_alg / (attn_us * 1e-6) / 1e9
        tflops = flops_alg / (attn_us * 1e-6) / 1e12
        hbm_bound = bytes_alg / (HBM_PEAK_GBS * 1e9) >= flops_alg / (MFMA_BF16_PEAK_TFLOPS * 1e12)
        sched_kernel = "tree_attn_mfma_kernel" if self.code == 1 else "tree_attn_rowwise_f32"
        common = {"kernel": sched_kernel, "traffic": traffic.get(self.key), "alg_bytes_per_launch": bytes_alg,
                  "alg_flops_per_launch": flops_alg, "avg_launch_us": round(attn_us, 3), "launch_us_spread": attn_spread,
                  "hbm_frac": round(gbs / HBM_PEAK_GBS, 4), "mfma_frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4)}
        if hbm_bound:
            attn = {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(gbs / HBM_PEAK_GBS, 4), **common}
        else:
            attn = {"bound": "mfma", "achieved": round(tflops, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4), **common}

        # The verification walk: two figures, never merged.  (1) The logit bytes the kernel that ran really reads
        # against the HBM peak; (2) the bytes of the method's minimum -- only the rows of the nodes the walk visits.
        e = 2 if self.tdt == torch.bfloat16 else 4
        lazy_bytes = (len(self.path0) + 1) * 2 * V * e
        kids = W.children_lists(self.parent)
        leaves = sum(1 for ch in kids if not ch)
        # the library's own choice of kernel (include/seqtree.h): a workgroup per node, a team per node with children, or the lazy walk
        per_node = self.T > 0 and V <= 32768 and n <= 256
        teams = self.T > 0 and V > 32768 and (n - leaves) * ((V + 16383) // 16384) <= 256 and n > leaves
        moved = ((n - leaves) * 2 + leaves) * V * e if per_node else (n - leaves) * 2 * V * e if teams else lazy_bytes
        moved_gbs = moved / (verify_us * 1e-6) / 1e9
        verify = {"kernel": "verify_chains_kernel" if per_node else "verify_chains_kernel (teams)" if teams else "verify_walk_kernel",
                  "bound": "hbm", "achieved": round(moved_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                  "frac": round(moved_gbs / HBM_PEAK_GBS, 5), "traffic": None,
                  "logit_bytes_read_per_launch": moved, "avg_launch_us": round(verify_us, 3), "launch_us_spread": verify_spread,
                  "alg_bytes_lazy_set0": lazy_bytes, "accepted_path_len_set0": len(self.path0),
                  "frac_lazy_set0": round(lazy_bytes / (verify_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 5)}
        if per_node:
            # bound by the vector unit of the ONE compute unit that holds the node with the longest sibling chain:
            # per vocabulary entry 2 x 8 instruction slots for the two softmaxes and 2 per rejection, on 64 lanes per
            # clock (4 SIMDs x 16 lanes) at 2.4 GHz -- a modelled figure, given beside the measured ones
            k_max = max(len(ch) for ch in kids)
            chain_us = V * (16 + 2 * k_max) / 64.0 / 2.4e9 * 1e6
            verify["note"] = ("one workgroup per node reads every row the tree can visit; limited by one compute unit's vector "
                              "rate over its node's sibling chain (modelled %.1f us for %d children), not by HBM" % (chain_us, k_max))
        else:
            verify["note"] = "reads only the rows of visited nodes: a chain of dependent steps, latency-bound by construction"
        if self.T > 0 and V > 32768 and not teams:
            # Beyond one workgroup's vocabulary the per-node kernel exists too (a team of workgroups per node that
            # has children); at this tree size the library does not pick it.  Forced here, to put its figure -- the
            # streaming efficiency on the bytes it really moves -- beside the lazy walk's.
            internal = n - leaves
            self.S.lib().seqtree_internal_set_verify_mode(2)
            try:
                self.verify_call(0)
                torch.cuda.synchronize()
                assert self.S.read_verify_trace(self.verify_sets[0]["ws"])["status"] == 0
                eager_us, eager_spread = timed_replays(torch, capture(torch, self.verify_call, idx), self.sets, blocks)
            finally:
                self.S.lib().seqtree_internal_set_verify_mode(0)
            eager_bytes = 2 * internal * V * e
            eager_gbs = eager_bytes / (eager_us * 1e-6) / 1e9
            verify["eager_per_node_teams"] = {
                "kernel": "verify_chains_kernel (teams of %d workgroups per node with children)" % ((V + 16383) // 16384),
                "bound": "hbm", "achieved": round(eager_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(eager_gbs / HBM_PEAK_GBS, 5), "logit_bytes_read_per_launch": eager_bytes,
                "avg_launch_us": round(eager_us, 3), "launch_us_spread": eager_spread,
                "note": "forced for this measurement; every row pair of an internal node is read once, then held in registers "
                        "for the node's chain of dependent steps"}
        report = {"step_us": round(step_us, 3), "step_us_spread": step_spread, "attn": attn, "verify": verify}
        if len(cfg.temperatures) > 1 and 0.0 in cfg.temperatures:
            greedy = lambda i: self.verify_call(i, temperature=0.0)
            greedy(0)
            report["verify_greedy_us"] = round(timed_replays(torch, capture(torch, greedy, idx), self.sets, blocks)[0], 3)
        return report


def small_tree_large_vocab(torch, dev, S, W, blocks, vocab, tree_key="C2"):
    """seq_verify for a small tree over a large vocabulary -- the case the per-node teams are picked for: the
    library's own choice against the lazy walk forced, on the same rotating inputs, with a drafter like the
    configurations' (short accepted paths) and with a good one (the walk runs several nodes deep)."""
    cfg = W.CONFIGS[tree_key]
    parent = W.make_tree(cfg, W.seed_for(list(W.CONFIGS).index(tree_key) + 1))
    n, T = len(parent), 0.6
    internal = sum(1 for ch in W.children_lists(parent) if ch)
    out = {"tree": "%s's (%d nodes, %d with children)" % (tree_key, n, internal), "vocab": vocab, "temperature": T}
    path = torch.empty(n, dtype=torch.int32, device=dev)
    bonus = torch.empty(1, dtype=torch.int32, device=dev)
    ws = torch.empty(S.seq_verify_workspace(n, vocab, 1), dtype=torch.uint8, device=dev)
    for label, sigma_d in (("synthetic_drafter", 2.0), ("good_drafter", 0.3)):
        sets = []
        for s_ in range(8):
            v = W.make_verify_inputs(parent, vocab, 4.0, sigma_d, T, W.BF16, seed=4242 + s_)
            sets.append((torch.from_numpy(v.target_logits).to(dev).to(torch.bfloat16), torch.from_numpy(v.draft_logits).to(dev).to(torch.bfloat16),
                         torch.from_numpy(v.tree_tokens).to(dev), torch.from_numpy(v.uniforms).to(dev)))

        def call(i):
            tl, dl, tok, un = sets[i % len(sets)]
            S.seq_verify(tl, dl, tok, parent, T, un, accepted_path=path, bonus_token=bonus, workspace=ws)

        row = {}
        for mode, name in ((0, "library_choice_us"), (1, "lazy_walk_us")):
            S.lib().seqtree_internal_set_verify_mode(mode)
            try:
                lengths = []
                for i in range(len(sets)):
                    call(i)
                    torch.cuda.synchronize()
                    assert S.read_verify_trace(ws)["status"] == 0
                    lengths.append(int((path >= 0).sum().item()))
                us, _ = timed_replays(torch, capture(torch, call, range(len(sets))), len(sets), blocks)
            finally:
                S.lib().seqtree_internal_set_verify_mode(0)
            row[name] = round(us, 3)
        row["mean_accepted_path"] = round(sum(lengths) / len(lengths), 2)
        eager_bytes = 2 * internal * vocab * 2
        row["per_node_bytes_read"] = eager_bytes
        row["per_node_frac_of_hbm_peak"] = round(eager_bytes / (row["library_choice_us"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 5)
        out[label] = row
        del sets
    return out


def yardstick_copy(torch, S, dev, mib):
    """Four launches of a plain copy kernel of known size: the reference HBM traffic counters are scaled by."""
    nbytes = mib << 20
    src = torch.full((nbytes,), 1, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(4):
        rc = S.lib().seqtree_internal_copy_probe(src.data_ptr(), dst.data_ptr(), nbytes, torch.cuda.current_stream().cuda_stream)
        assert rc == 0
    torch.cuda.synchronize()
    assert bool((dst == 1).all())
    return nbytes


def cpu_baseline(w, seconds):
    """The CPU checker as it stands on a bounded sample of the same workload: attention rows one by one (one
    thread, then one thread per host core -- the routine is reentrant and the foreign call releases the
    interpreter lock), and whole verification walks.  Scaled to one step; a baseline, not a target."""
    import ctypes as C
    from concurrent.futures import ThreadPoolExecutor

    import numpy as np

    import oracle
    W, cfg = w.W, w.cfg
    a0 = W.attn_inputs_for(w.key)
    n, H, d = a0.q.shape
    Hk, cap, _ = a0.k_cache.shape
    rows_per_step = n * H
    arrays = [np.ascontiguousarray(x, dtype=np.float32) for x in (a0.q, a0.k_cache, a0.v_cache, a0.k_tree, a0.v_tree)]
    parent = np.ascontiguousarray(a0.parent, dtype=np.int32)
    ptrs = [x.ctypes.data_as(C.c_void_p) for x in arrays] + [parent.ctypes.data_as(C.c_void_p)]
    sizes = [C.c_int32(x) for x in (a0.prefix_len, cap, n, H, Hk, d)]
    row_fn = oracle.lib().oracle_tree_attn_row

    def run_rows(rows):
        out = np.zeros(d, dtype=np.float64)
        for i, h in rows:
            assert row_fn(*ptrs, *sizes, C.c_int32(i), C.c_int32(h), C.c_void_p(out.ctypes.data), None, None) == 0

    rng = np.random.default_rng(0)
    t0 = time.perf_counter()
    run_rows([(0, 0)])
    row_s = max(time.perf_counter() - t0, 1e-6)
    cores = os.cpu_count() or 1

    def sample(count):
        if count >= rows_per_step:
            return [(r // H, r % H) for r in range(rows_per_step)]
        return [(int(rng.integers(n)), int(rng.integers(H))) for _ in range(count)]

    one = sample(int(max(8, seconds * 0.3 / row_s)))
    t0 = time.perf_counter()
    run_rows(one)
    attn_one_s = (time.perf_counter() - t0) * rows_per_step / len(one)
    many = sample(int(max(8 * cores, seconds * 0.5 * cores / row_s)))
    shares = [many[k::cores] for k in range(cores)]
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as pool:
        list(pool.map(run_rows, shares))
    attn_all_s = (time.perf_counter() - t0) * rows_per_step / len(many)
    h0 = w.host0
    t0, reps = time.perf_counter(), 0
    while reps < 3 or (time.perf_counter() - t0 < seconds * 0.2 and reps < 50):
        oracle.verify(h0.target_logits, h0.draft_logits, h0.tree_tokens, h0.parent, w.T, h0.uniforms)
        reps += 1
    verify_s = (time.perf_counter() - t0) / reps
    return {"value": round((attn_all_s + verify_s) * 1e6, 1), "unit": "us/step", "cores": cores, "kind": "oracle",
            "sample": f"{len(many)} of {rows_per_step} attention rows of {cfg.name} on {cores} threads (the checker's row routine, "
                      f"one row per call; scaled to all rows) + {reps} whole verification walks on one thread; fp64",
            "attn_us": round(attn_all_s * 1e6, 1), "verify_us": round(verify_s * 1e6, 1),
            "single_thread": {"value": round((attn_one_s + verify_s) * 1e6, 1), "unit": "us/step", "cores": 1,
                              "sample": f"{len(one)} of {rows_per_step} attention rows (scaled) + the same walks",
                              "attn_us": round(attn_one_s * 1e6, 1)}}


def run_sweep(args) -> int:
    """Latency of the two calls over the tree size, at each configuration's head shape, prefix
    length and vocabulary: one JSON line per (configuration, n).  Not the benchmark line."""
    import numpy as np
    import torch

    import paper_2402_12374_amd as S
    import workloads as W

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    sizes = [int(x) for x in args.sweep_sizes.split(",")]
    results = []
    for key in args.sweep_configs.split(","):
        cfg = W.CONFIGS[key]
        # a batch of sequences (same tree, same prefix length) is a call with more heads
        H, Hk, d, P, V = cfg.heads * args.sweep_batch, cfg.kv_heads * args.sweep_batch, cfg.head_dim, cfg.prefix_len, cfg.vocab
        if args.sweep_prefix > 0:
            P = args.sweep_prefix
        tdt = torch.bfloat16 if cfg.dtype == W.BF16 else torch.float32
        code = 1 if tdt == torch.bfloat16 else 2
        T = cfg.temperatures[0]
        sets = max(2, min(cfg.layers, 16) // args.sweep_batch)
        mk = lambda *shape: torch.randn(*shape, device=dev).to(tdt)
        caches = [(mk(Hk, P, d), mk(Hk, P, d)) for _ in range(sets)]
        for n in sizes:
            if args.sweep_tree == "sequoia":
                parent, _ = S.seq_build_tree(W.PAPER_ACCEPTANCE_VECTOR, n, cfg.max_depth)
            else:
                parent = W.geometric_tree(n, cfg.max_depth)
            q = [(mk(n, H, d), mk(n, Hk, d), mk(n, Hk, d), torch.empty(n, H, d, device=dev, dtype=tdt)) for _ in range(sets)]
            ws = torch.empty(S.seq_tree_attn_workspace(P, n, H, Hk, d, code), dtype=torch.uint8, device=dev)

            def attn_call(i):
                kc, vc = caches[i % sets]
                qq, kt, vt, out = q[i % sets]
                S.seq_tree_attn(qq, kc, vc, kt, vt, parent, P, out=out, workspace=ws)

            attn_us = graph_time_us(torch, attn_call, sets, 20)
            vsets = []
            for rep in range(2 if n * V > 2 ** 25 else 4):
                v = W.make_verify_inputs(parent, V, cfg.sigma_target, cfg.sigma_draft, T, cfg.dtype, seed=n + rep)
                vsets.append(dict(tl=torch.from_numpy(v.target_logits).to(dev).to(tdt), dl=torch.from_numpy(v.draft_logits).to(dev).to(tdt),
                                  tok=torch.from_numpy(v.tree_tokens).to(dev), un=torch.from_numpy(v.uniforms).to(dev),
                                  path=torch.empty(n, dtype=torch.int32, device=dev), bonus=torch.empty(1, dtype=torch.int32, device=dev),
                                  ws=torch.empty(S.seq_verify_workspace(n, V, code), dtype=torch.uint8, device=dev)))

            def verify_call(i):
                x = vsets[i % len(vsets)]
                S.seq_verify(x["tl"], x["dl"], x["tok"], parent, T, x["un"], accepted_path=x["path"],
                             bonus_token=x["bonus"], workspace=x["ws"])

            verify_us = graph_time_us(torch, verify_call, len(vsets), 20)
            cfg_n = type("C", (), dict(dtype=cfg.dtype, n_tree=n, prefix_len=P, heads=H, kv_heads=Hk, head_dim=d))
            bytes_alg, flops_alg = attn_alg_bytes(cfg_n), attn_alg_flops(cfg_n, parent)
            results.append((key, n, attn_us, verify_us))
            print(json.dumps({"config": cfg.name, "tree": args.sweep_tree, "batch": args.sweep_batch, "n_tree": n, "prefix_len": P, "vocab": V,
                              "attn_us_per_layer": round(attn_us, 2), "verify_us": round(verify_us, 2),
                              "attn_hbm_frac": round(bytes_alg / (attn_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                              "attn_mfma_frac": round(flops_alg / (attn_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}), flush=True)
            del q, vsets
        del caches
        torch.cuda.empty_cache()
        if args.pick_tree:
            # The hardware-aware choice of Sec. 4.1 fed with what was just measured.  t(n) here is the
            # part of the target's pass this library covers -- every layer's tree attention plus the
            # verification walk, not the linear layers -- relative to the same at the smallest size.
            mine = [(n, cfg.layers * a + v) for k, n, a, v in results if k == key]
            decode = mine[0][1]
            n_best, d_best, s_best = S.seq_pick_tree_shape(W.PAPER_ACCEPTANCE_VECTOR, [n for n, _ in mine], [t for _, t in mine],
                                                           cfg.max_depth, decode_time=decode, draft_time=args.draft_cost * decode)
            _, g_best = S.seq_build_tree(W.PAPER_ACCEPTANCE_VECTOR, n_best, d_best)
            print(json.dumps({"config": cfg.name, "pick_tree": {"size": n_best, "depth": d_best, "speedup": round(s_best, 3),
                              "expected_tokens": round(g_best, 3), "draft_cost": args.draft_cost,
                              "t_of_n": {str(n): round(t / decode, 3) for n, t in mine}}}), flush=True)
    S.shutdown()
    return 0


# Vector instructions the sampling kernel spends per token on its fast path, as compiled (Philox4x32-10:
# 4.5 64-bit multiplies and 9 logic operations; 3 to turn the word into a uniform; 2 logarithms and a
# multiply-add for the Gumbel variate; 4 for the key and the class of zero-probability tokens; unpacking the
# logit and the compare against the bar), and the chip's rate for them: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz.
DRAFT_LANE_INSTR_PER_TOKEN = 30.0
VALU_PEAK_T_LANE_INSTR = 256 * 4 * 16 * 2.4e9 / 1e12


def run_draft_sample(args) -> int:
    """Latency of seq_draft_sample (the drafter's ordered draw of child tokens): for each
    configuration, one call over every node of its tree that has children (rows = internal
    nodes, n_children = their fan-outs), and one call for a single level of the tree.  One JSON
    line per case.  Not the benchmark line."""
    import numpy as np
    import torch

    import paper_2402_12374_amd as S
    import workloads as W

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    first = True
    for key in args.sweep_configs.split(","):
        cfg = W.CONFIGS[key]
        idx = list(W.CONFIGS).index(key) + 1
        parent = W.make_tree(cfg, W.seed_for(idx))
        fan = np.bincount(parent[1:], minlength=len(parent))
        depth = W.depths(parent)
        level = int(np.argmax(np.bincount(depth[fan > 0])))     # the level with most internal nodes
        tdt = torch.bfloat16 if cfg.dtype == W.BF16 else torch.float32
        T = cfg.temperatures[0]
        for name, rows_of in (("tree", np.nonzero(fan > 0)[0]), (f"level{level}", np.nonzero((fan > 0) & (depth == level))[0])):
            ks = fan[rows_of].astype(np.int32)
            rows, V, k_max = len(ks), cfg.vocab, int(ks.max())
            n_sets = 2 if rows * V > 2 ** 24 else 8
            gen = np.random.Generator(np.random.PCG64(W.seed_for(idx) + 900))
            sets = []
            for _ in range(n_sets):
                x = gen.standard_normal((rows, V), dtype=np.float32) * np.float32(np.hypot(cfg.sigma_target, cfg.sigma_draft))
                sets.append(torch.from_numpy(x).to(dev).to(tdt))
            nc = torch.from_numpy(ks).to(dev)
            rng = torch.tensor([2024, 0], dtype=torch.int64, device=dev)
            tokens = torch.empty((rows, k_max), dtype=torch.int32, device=dev)
            ws = torch.empty(S.seq_draft_sample_workspace(rows, V, k_max, 1), dtype=torch.uint8, device=dev)

            def call(i):
                S.seq_draft_sample(sets[i % n_sets], nc, T, rng, k_max, tokens=tokens, workspace=ws)

            us = graph_time_us(torch, call, n_sets, 40)
            tok_per_s = rows * V / (us * 1e-6)
            achieved = tok_per_s * DRAFT_LANE_INSTR_PER_TOKEN / 1e12
            line = {"op": "seq_draft_sample", "config": cfg.name, "case": name, "rows": rows, "vocab": V,
                    "children": int(ks.sum()), "k_max": k_max, "temperature": T, "dtype": cfg.dtype,
                    "us": round(us, 2), "g_tokens_per_s": round(tok_per_s / 1e9, 1),
                    "roofline": {"bound": "alu", "achieved": round(achieved, 2), "peak": round(VALU_PEAK_T_LANE_INSTR, 1),
                                 "unit": "T lane-instr/s", "frac": round(achieved / VALU_PEAK_T_LANE_INSTR, 4),
                                 "hbm_frac": round(rows * V * (2 if tdt == torch.bfloat16 else 4) / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}}
            if first and not args.no_cpu_baseline:
                import oracle
                host = sets[0][: min(rows, 16)].float().cpu().numpy()
                t0 = time.perf_counter()
                oracle.draft_sample(host, ks[: len(host)], T, 2024, 0, k_stride=k_max)
                dt = time.perf_counter() - t0
                line["cpu_baseline"] = {"value": round(len(host) * V / dt / 1e9, 4), "unit": "G tokens/s", "cores": 1,
                                        "kind": "oracle", "sample": f"{len(host)} rows of {V} logits"}
                first = False
            print(json.dumps(line), flush=True)
            del sets
        torch.cuda.empty_cache()
    S.shutdown()
    return 0


def run_verify_batch(args) -> int:
    """Latency of seq_verify_batched over the number of sequences, per configuration (its tree,
    its vocabulary; --verify-batch-vocab overrides the vocabulary, --verify-batch-temperature
    the temperature).  Graph replay over two rotating input sets.  One JSON line per case.  Not
    the benchmark line."""
    import numpy as np
    import torch

    import paper_2402_12374_amd as S
    import workloads as W

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    for key in args.sweep_configs.split(","):
        cfg = W.CONFIGS[key]
        parent = W.make_tree(cfg, W.seed_for(list(W.CONFIGS).index(key) + 1))
        n = len(parent)
        V = args.verify_batch_vocab or cfg.vocab
        T = cfg.temperatures[0] if args.verify_batch_temperature < 0 else args.verify_batch_temperature
        for B in (int(x) for x in args.verify_batch.split(",")):
            if 2 * 2 * B * n * V * 2 > 24e9:      # two sets of two bf16 logit tensors
                continue
            sets = []
            for s in range(2):
                vs = [W.make_verify_inputs(parent, V, cfg.sigma_target, cfg.sigma_draft, T, W.BF16, seed=1000 * s + b)
                      for b in range(B)]
                stack = lambda k: torch.from_numpy(np.stack([getattr(v, k) for v in vs])).to(dev)
                sets.append((stack("target_logits").to(torch.bfloat16), stack("draft_logits").to(torch.bfloat16),
                             stack("tree_tokens"), stack("uniforms")))
                del vs
            path = torch.empty((B, n), dtype=torch.int32, device=dev)
            bonus = torch.empty(B, dtype=torch.int32, device=dev)
            ws = torch.empty((B, S.seq_verify_workspace(n, V, 1)), dtype=torch.uint8, device=dev)

            def call(i):
                tl, dl, tok, un = sets[i % 2]
                S.seq_verify_batched(S.SEQ_VERIFY_SEQUOIA, tl, dl, tok, parent, T, un, accepted_path=path,
                                     bonus_token=bonus, workspace=ws)

            us = graph_time_us(torch, call, 4, 30)
            print(json.dumps({"config": cfg.name, "n_tree": n, "vocab": V, "temperature": T, "batch": B,
                              "verify_us": round(us, 2), "us_per_sequence": round(us / B, 2)}), flush=True)
            del sets
    return 0


def run_rejection_curve(args) -> int:
    """Rejection rate at one node against the number of speculated children k, for Sequoia's
    algorithm and the two baselines of Sec. 2.2, each with children drawn the way it assumes
    (without replacement / independently / the draft's top k): the shape of the paper's figure
    "rejection rate vs. number of speculated tokens" on synthetic distributions (Gaussian target
    logits, draft = target + noise).  One JSON line per temperature.  Not the benchmark line."""
    import numpy as np
    import torch

    import paper_2402_12374_amd as S
    import workloads as W

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    V, pairs, trials, ks = 32000, 32, args.curve_trials, [1, 2, 3, 4, 6, 8, 12, 16]
    k_max = max(ks)
    g = torch.Generator(device=dev)
    g.manual_seed(2402)
    target_rows = (3.0 * torch.randn((pairs, V), device=dev, generator=g))
    draft_rows = target_rows + args.curve_draft_noise * torch.randn((pairs, V), device=dev, generator=g)
    # a star needs k+1 rows; only the root's matter for what happens at the root
    tl = target_rows.to(torch.bfloat16)[:, None, :].expand(pairs, k_max + 1, V).contiguous()
    dl = draft_rows.to(torch.bfloat16)[:, None, :].expand(pairs, k_max + 1, V).contiguous()
    ws = torch.empty(S.seq_verify_workspace(k_max + 1, V, 1), dtype=torch.uint8, device=dev)
    rng = torch.tensor([2402, 0], dtype=torch.int64, device=dev)
    for T in (0.2, 0.6, 1.0):
        out = {"rejection_curve": {"temperature": T, "vocab": V, "trials": trials, "draft_noise": args.curve_draft_noise, "k": ks}}
        for name, alg in (("sequoia", S.SEQ_VERIFY_SEQUOIA), ("specinfer", S.SEQ_VERIFY_SPECINFER), ("topk", S.SEQ_VERIFY_TOPK)):
            rates = []
            for k in ks:
                n = k + 1
                parent = W.star_tree(n)
                paths = torch.empty((trials, n), dtype=torch.int32, device=dev)
                bonus = torch.empty((trials, 1), dtype=torch.int32, device=dev)
                tokens = torch.zeros((trials, n), dtype=torch.int32, device=dev)
                uniforms = torch.rand((trials, n), device=dev, generator=g).clamp_(max=1.0 - 2.0 ** -24)
                nc = torch.full((1,), k, dtype=torch.int32, device=dev)
                for t in range(trials):
                    r = t % pairs
                    if alg == S.SEQ_VERIFY_SEQUOIA:
                        rng[1] += 1
                        S.seq_draft_sample(dl[r, :1], nc, T, rng, k, tokens=tokens[t, 1:].view(1, k))
                    elif alg == S.SEQ_VERIFY_SPECINFER:
                        q = torch.softmax(dl[r, 0].float() / T, dim=0)
                        tokens[t, 1:] = torch.multinomial(q, k, replacement=True, generator=g).to(torch.int32)
                    else:
                        tokens[t, 1:] = torch.topk(dl[r, 0].float(), k).indices.to(torch.int32)
                    S.seq_verify_with(alg, tl[r, :n], dl[r, :n], tokens[t], parent, T, uniforms[t],
                                      accepted_path=paths[t], bonus_token=bonus[t], workspace=ws)
                torch.cuda.synchronize()
                rates.append(round(float((paths[:, 0] < 0).float().mean().item()), 4))
                if k == k_max:
                    # the acceptance vector of Sec. 3.1.1 as measured here: how often the child at
                    # position j is the one accepted; and what Sequoia's dynamic program makes of it
                    first = paths[:, 0].cpu().numpy()
                    vector = [round(float((first == j).mean()), 4) for j in range(1, k + 1)]
                    _, g64 = S.seq_build_tree(vector, 64, 8)
                    out["rejection_curve"].setdefault("acceptance_vector", {})[name] = vector
                    out["rejection_curve"].setdefault("expected_tokens_64_nodes_depth_8", {})[name] = round(g64, 3)
            out["rejection_curve"][name] = rates
        print(json.dumps(out), flush=True)
    S.shutdown()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000, help="steps timed (exactly this many)")
    ap.add_argument("--warmup", type=int, default=200, help="untimed steps before them")
    ap.add_argument("--no-graph-upload", action="store_true",
                    help="leave each step graph's first launch (its upload to the device) to the warmup and timed steps")
    ap.add_argument("--config", default="C5",
                    help="workload of the headline figure (C5, the largest configuration that one GPU holds, unless told otherwise)")
    ap.add_argument("--also", default="C2,C3,C4",
                    help="configurations reported beside the headline, each with its own rooflines (empty: none)")
    ap.add_argument("--blocks", type=int, default=20,
                    help="replays (at least 20) of the per-kernel graphs that the kernel durations and their spread come from")
    ap.add_argument("--sets", type=int, default=0, help="distinct input sets to rotate over (0 = layer count)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--eager", action="store_true",
                    help="for profilers: launch --warmup + --steps steps of --config from Python, no HIP graph, print a short "
                         "line and stop (per-dispatch counters and kernel traces then see one dispatch per call)")
    ap.add_argument("--cpu-seconds", type=float, default=16.0)
    ap.add_argument("--vocab", type=int, default=0, help="vocabulary of the headline workload (0 = the configuration's)")
    ap.add_argument("--verify-kernel", choices=("auto", "lazy", "per-node"), default="auto",
                    help="force the lazy walk, or the per-node kernels wherever temperature and algorithm allow them")
    ap.add_argument("--yardstick-mib", type=int, default=0,
                    help="after the timed region, also launch a plain copy kernel of this many MiB four times "
                         "(the known-size reference for HBM traffic counters collected with rocprofv3 --pmc)")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark line: latency of both calls over the tree size (one line each)")
    ap.add_argument("--sweep-tree", choices=("geometric", "sequoia"), default="geometric",
                    help="tree of the sweep: the configurations' geometric tree, or the Sequoia tree of that size built "
                         "by seq_build_tree from the paper's printed acceptance vector")
    ap.add_argument("--sweep-batch", type=int, default=1,
                    help="with --sweep: attention over this many sequences per call (heads and KV heads times the batch; "
                         "the verification walk stays one sequence)")
    ap.add_argument("--pick-tree", action="store_true",
                    help="with --sweep: after each configuration, the tree size and depth that maximise Speedup(n, d) for "
                         "the measured t(n) (first sweep size = the decoding step)")
    ap.add_argument("--draft-cost", type=float, default=0.05, help="c of Speedup(n, d): one draft step relative to one decoding step")
    ap.add_argument("--rejection-curve", action="store_true",
                    help="instead of the benchmark line: rejection rate against the number of children for the three "
                         "verification algorithms (one line per temperature)")
    ap.add_argument("--curve-trials", type=int, default=512)
    ap.add_argument("--curve-draft-noise", type=float, default=1.0)
    ap.add_argument("--draft-sample", action="store_true",
                    help="instead of the benchmark line: latency of seq_draft_sample per configuration (one line each)")
    ap.add_argument("--verify-batch", default="",
                    help="instead of the benchmark line: latency of seq_verify_batched for these batch sizes, e.g. 1,2,4,8,16,64")
    ap.add_argument("--verify-batch-vocab", type=int, default=0, help="vocabulary for --verify-batch (0 = the configuration's)")
    ap.add_argument("--verify-batch-temperature", type=float, default=-1.0, help="temperature for --verify-batch (< 0 = the configuration's)")
    ap.add_argument("--sweep-configs", default="C2,C3,C4,C5")
    ap.add_argument("--sweep-prefix", type=int, default=0,
                    help="with --sweep: this prefix length instead of each configuration's (the paper's prompts are 128 tokens)")
    ap.add_argument("--sweep-sizes", default="16,32,64,128,256,512,768")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        return 2

    if args.sweep:
        return run_sweep(args)
    if args.draft_sample:
        return run_draft_sample(args)
    if args.rejection_curve:
        return run_rejection_curve(args)
    if args.verify_batch:
        return run_verify_batch(args)

    import torch

    import paper_2402_12374_amd as S

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    traffic = load_traffic_table()
    blocks = max(20, args.blocks)

    # ---- the headline workload: exactly --steps steps after --warmup steps ------------------
    head = Workload(args.config, torch, dev, sets=args.sets, vocab=args.vocab)
    if args.verify_kernel != "auto":
        S.lib().seqtree_internal_set_verify_mode({"lazy": 1, "per-node": 2}[args.verify_kernel])
    if args.eager:
        for i in range(args.warmup):
            head.step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            head.step(args.warmup + i)
        torch.cuda.synchronize()
        line = {"eager": True, "workload": head.describe(), "steps": args.steps,
                "us_per_step_from_python": round((time.perf_counter() - t0) / args.steps * 1e6, 2)}
        head.check_results()
        if args.yardstick_mib > 0:
            line["yardstick_copy_bytes"] = yardstick_copy(torch, S, dev, args.yardstick_mib)
        print(json.dumps(line))
        S.shutdown()
        return 0
    step_graphs = [capture(torch, head.step, [i]) for i in range(head.sets)]   # one graph per step and input set
    # (A graph's first launch uploads it to the device, tens of microseconds of host time each.  The
    # rotation over input sets is a device of this measurement -- a serving loop replays one graph --
    # so the upload belongs to building the graphs, not to the steps: every graph is launched once
    # here, before the warmup steps.)
    if not args.no_graph_upload:
        for g in step_graphs:
            g.replay()
        torch.cuda.synchronize()
    for i in range(args.warmup):
        step_graphs[i % head.sets].replay()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record()
    for i in range(args.steps):
        step_graphs[(args.warmup + i) % head.sets].replay()
    stop.record()
    torch.cuda.synchronize()
    wall_s = time.perf_counter() - t0
    step_us = wall_s / args.steps * 1e6
    event_step_us = start.elapsed_time(stop) * 1e3 / args.steps
    # spread of the step latency: at least 20 consecutive steps, an event between every two
    n_spread = max(20, min(args.steps, 400))
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(n_spread + 1)]
    marks[0].record()
    for i in range(n_spread):
        step_graphs[i % head.sets].replay()
        marks[i + 1].record()
    torch.cuda.synchronize()
    spread = percentiles([marks[i].elapsed_time(marks[i + 1]) * 1e3 for i in range(n_spread)])
    spread["timed_one_by_one"] = n_spread
    del step_graphs
    head_report = head.measure_kernels(blocks, traffic)
    head.check_results()
    if head.T > 0 and head.V > 32768:
        import workloads as W
        head_report["verify"]["small_tree_same_vocab"] = small_tree_large_vocab(torch, dev, S, W, blocks, head.V)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(head, args.cpu_seconds)
    head.release()

    # ---- the other configurations of the paper's models, each with its own rooflines --------
    others = {}
    for key in [k for k in args.also.split(",") if k and k != args.config]:
        w = Workload(key, torch, dev)
        rep = w.measure_kernels(blocks, traffic)
        w.check_results()
        others[key] = {"workload": w.describe(), "step_us": rep["step_us"], "tree_tokens_per_s": round(w.n / (rep["step_us"] * 1e-6), 1),
                       "attn": rep["attn"], "verify": rep["verify"]}
        if "verify_greedy_us" in rep:
            others[key]["verify_greedy_us"] = rep["verify_greedy_us"]
        w.release()

    line = {
        "metric": "tree-verify step latency", "value": round(step_us, 3), "unit": "us",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(step_us * 1e-3, 6),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if head.code == 1 else "f32", "data": "synthetic",
        "config": {"workload": head.describe(), "step": "1 x seq_tree_attn (one layer) + 1 x seq_verify",
                   "input_sets": head.sets, "launch": "one HIP graph per step, rotating over the input sets" + ("" if args.no_graph_upload else "; every graph launched once when built (its upload), before the warmup steps")},
        "tree_tokens_per_s": round(head.n / (step_us * 1e-6), 1),
        "attn_us_per_layer": head_report["attn"]["avg_launch_us"], "verify_us": head_report["verify"]["avg_launch_us"],
        "gpu_event_us_per_step": round(event_step_us, 3), "step_us_in_one_graph": head_report["step_us"],
        "step_us_spread": spread,
        "roofline": head_report["attn"], "verify": head_report["verify"],
        "configs": others, "cpu_baseline": cpu,
    }
    if args.yardstick_mib > 0:
        line["yardstick_copy_bytes"] = yardstick_copy(torch, S, dev, args.yardstick_mib)
    print(json.dumps(line))
    S.shutdown()
    return 0


if __name__ == "__main__":
    sys.exit(main())
