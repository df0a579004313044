"""Benchmark of the block-structured-pruning path on one MI355X.

Workload: the BERT-large / RoBERTa-large linear set (QKV 3072x1024, attention out 1024x1024,
FFN up 4096x1024, FFN down 1024x4096), bf16, 8192 tokens, row-blocks of R=16 rows, 5x
compression chosen by a matrix-scope percentile of the group norms of N(0, 0.02) weights.

One step = one pass of the whole path over the four matrices: group norms + reweighting
factors, regulariser gradient, percentile mask, pack (count + pack), layer plan, and the pruned
layer.  The four matrices are independent, so each matrix's share of the step is recorded into a HIP graph
and the four graphs are replayed side by side on four streams: a matrix's steps follow each other on
its stream, all streams are joined before the clock stops; `--launch serial` replays one graph with the matrices one after the other,
`--launch eager` launches every kernel from Python.  All inputs are resident in HBM before the timed region.  `value` is the useful
FLOP rate of the layers (2 * T * R * kept columns, pads excluded) over the whole step time.

Kernel durations (for `linear_only` and `roofline`) come from a second pass of the same number of
steps in which the layer launches of a step run back to back on one stream, each bracketed by
events on that stream.

    python bench.py --gpus 1 --steps K --warmup W
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import bsp_workloads as wl  # noqa: E402
import paper_2009_08065_amd as bsp  # noqa: E402

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published
LDS_PEAK_GBS = 256 * 256 * 2.4  # 256 compute units x 256 B/clk (ds_read_b128 measured at 246) x 2.4 GHz = 157 286 GB/s
# HBM bytes per launch of the dominant layer kernel on this workload (average of its launches), from the FETCH_SIZE /
# WRITE_SIZE counter runs summarised in profiles/layer_kernels_bert_large_r16_per_launch.md (QKV 80.2 MB and FFN-up
# 99.5 MB for the step-loop kernel, attention-out 41.6 MB and FFN-down 105.1 MB for the streaming one); None = not
# measured for the kernel as it stands.
DOMINANT_KERNEL_HBM_BYTES_PER_LAUNCH = {"linear_steploop16_kernel": 89.9e6, "linear_stream16_kernel": 73.4e6}


class Matrix:
    """Device-resident tensors and preallocated outputs of one layer of the set."""

    def __init__(self, d, k_align=32, path="planned"):
        self.name, self.M, self.N, self.R, self.T = d["name"], d["M"], d["N"], d["R"], d["T"]
        self.n_keep, self.k_align = d["n_keep"], k_align
        dev = "cuda"
        self.W = torch.from_numpy(d["W"]).to(torch.bfloat16).to(dev)
        self.X = torch.from_numpy(d["X"]).to(torch.bfloat16).to(dev)
        self.bias = torch.from_numpy(d["bias"]).to(torch.bfloat16).to(dev)
        B = self.M // self.R
        self.B = B
        f32 = dict(dtype=torch.float32, device=dev)
        self.sumsq, self.alpha = torch.empty((B, self.N), **f32), torch.empty((B, self.N), **f32)
        self.grad = torch.empty_like(self.W)
        self.keep = torch.empty((B, self.N), dtype=torch.uint8, device=dev)
        self.ws = torch.empty(bsp.lib().bsp_prune_mask_workspace_bytes(B, self.N, bsp.SCOPE_MATRIX),
                              dtype=torch.uint8, device=dev)
        self.blk_cnt = torch.empty(B, dtype=torch.int32, device=dev)
        self.blk_ptr = torch.empty(B + 1, dtype=torch.int32, device=dev)
        # at most n_keep groups survive a percentile, each block pads by < k_align columns
        self.capacity = self.n_keep + B * (k_align - 1)
        self.col_idx = torch.empty(self.capacity, dtype=torch.int32, device=dev)
        self.vals = torch.empty(self.R * self.capacity, dtype=torch.bfloat16, device=dev)
        self.Y = torch.empty((self.T, self.M), dtype=torch.bfloat16, device=dev)
        self.packed = bsp.Packed(self.M, self.N, self.R, k_align, self.blk_cnt, self.blk_ptr, self.col_idx,
                                 self.vals, self.capacity)
        self.kept_cols = None
        self.use_plan = path == "planned" and bsp.bsp_linear_plan_supported(torch.bfloat16, self.N, k_align)
        self.plan = None
        if self.use_plan:
            self.plan = torch.empty(bsp.lib().bsp_linear_plan_bytes(self.M, self.R, self.capacity), dtype=torch.uint8,
                                    device=dev)

    def prune_and_pack(self, eps=1e-6, lam=None):
        """Norms and factors (with lam: and the regulariser's gradient, in the same pass over W), mask, pack, plan."""
        if lam is None:
            bsp.bsp_group_norms(self.W, self.R, eps=eps, mode=bsp.ALPHA_SQNORM, sumsq=self.sumsq, alpha=self.alpha,
                                want=())
        else:
            bsp.bsp_group_norms_grad(self.W, self.R, lam, eps=eps, mode=bsp.ALPHA_SQNORM, sumsq=self.sumsq,
                                     alpha=self.alpha, grad=self.grad, want=())
        bsp.bsp_prune_mask_count(self.sumsq, n_keep=self.n_keep, scope=bsp.SCOPE_MATRIX, k_align=self.k_align,
                                 keep=self.keep, ws=self.ws, blk_cnt=self.blk_cnt, blk_ptr=self.blk_ptr)
        L = bsp.lib()
        st = L.bsp_pack(self.W.data_ptr(), bsp.BF16, self.M, self.N, self.R, self.keep.data_ptr(), self.k_align,
                        self.blk_cnt.data_ptr(), self.blk_ptr.data_ptr(), self.capacity, self.col_idx.data_ptr(),
                        self.vals.data_ptr(), bsp.BF16, torch.cuda.current_stream().cuda_stream)
        if st != 0:
            raise bsp.BspError(st, "bsp_pack")
        if self.use_plan:
            bsp.bsp_linear_plan(self.packed, plan=self.plan)

    def whole_step(self):
        """Norms and factors with the regulariser's gradient (one pass over W: Alg. 2 at a milestone), mask, pack,
        plan, layer.  A gradient launch of its own after the layer cost 15 us per step: every launch of a stream
        queues behind the layer kernels of the other streams."""
        self.prune_and_pack(lam=1e-4)
        self.linear()

    def linear(self):
        if self.use_plan:
            bsp.bsp_linear_planned(self.X, self.packed, self.plan, self.bias, Y=self.Y)
        else:
            bsp.bsp_linear(self.X, self.packed, self.bias, Y=self.Y)

    # algorithmic work of one layer call
    def useful_flops(self):
        return 2.0 * self.T * self.R * self.kept_cols

    def dense_flops(self):
        return 2.0 * self.T * self.M * self.N

    def linear_bytes(self):
        padded = int(self.blk_ptr[-1].item())
        return 2.0 * self.T * self.N + 2.0 * self.T * self.M + 2.0 * self.R * padded + 4.0 * padded + 2.0 * self.M


def streams_on_different_queues(want=4, candidates=12):
    """`want` streams (default priority) of which no two share a hardware queue, and what the probe saw.

    HIP deals its streams to a few hardware queues (4 per process here), and two streams on one queue run their
    kernels strictly one after the other.  Which streams share a queue is a property of the process (the order in
    which torch and HIP created them), not of the workload, so it is found before anything is timed, with a probe that
    knows nothing of the benchmark: a graph of 24 tiny dependent kernels takes t alone; replayed on two streams at the
    same time it takes 1.4 to 1.8 t when they are on different queues (the launches themselves do not overlap
    fully) and 2 t, to within 4 %, when they share one -- as two replays on one stream do, which is the yardstick:
    a pair below 0.955 of that is on two queues.  Streams are taken in creation order, each one kept if it overlaps with
    all those kept before."""
    pool = [torch.cuda.Stream() for _ in range(candidates)]
    bufs = [torch.zeros(256, device="cuda") for _ in range(2)]
    graphs = []
    for b in bufs:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(24):
                b.add_(1.0)
        graphs.append(g)

    def timed(pairs, reps=30):
        best = float("inf")
        for _ in range(5):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                for g, st in pairs:
                    with torch.cuda.stream(st):
                        g.replay()
            torch.cuda.synchronize()
            best = min(best, (time.perf_counter() - t0) / reps)
        return best

    for st in pool:                      # first use of a stream (queue set-up) stays out of the timings
        with torch.cuda.stream(st):
            graphs[0].replay()
    torch.cuda.synchronize()
    for _ in range(3):                   # and so do the clocks' first moments on a box that has just started
        timed([(graphs[0], pool[0]), (graphs[1], pool[0])])
    alone = timed([(graphs[0], pool[0])])

    def on_two_queues(a, b, yard):
        return timed([(graphs[0], a), (graphs[1], b)]) < 0.955 * yard

    # The yardstick is taken before and after the choice, and every chosen pair is checked once more against the
    # smaller of the two: a yardstick measured while the machine was still speeding up would let a pair that shares a
    # queue pass (the step is then two chains wide, 0.21 instead of 0.16 ms).  A choice that fails the check is made anew.
    for attempt in range(1, 4):
        serial = timed([(graphs[0], pool[0]), (graphs[1], pool[0])])    # one stream: one after the other by construction
        kept, shared = [pool[0]], []
        for i in range(1, candidates):
            if len(kept) == want:
                break
            if all(on_two_queues(k, pool[i], serial) for k in kept):
                kept.append(pool[i])
            else:
                shared.append(i)
        found = len(kept)
        serial = min(serial, timed([(graphs[0], pool[0]), (graphs[1], pool[0])]))
        if all(on_two_queues(kept[i], kept[j], serial) for i in range(found) for j in range(i + 1, found)):
            break
    for st in pool:                      # fewer queues than wanted: fill up in creation order
        if len(kept) == want:
            break
        if st not in kept:
            kept.append(st)
    return kept, {"streams_probed": candidates, "on_different_queues": found, "sharing_a_queue_with_an_earlier_one": shared,
                  "probe_us_alone": round(alone * 1e6, 1), "probe_us_two_on_one_stream": round(serial * 1e6, 1),
                  "choices_made": attempt}


def time_layers(mats, steps, warmup):
    """The layer launches of the set, in turn on the launch stream, each between two events: [steps, matrices] ms."""
    evs = [[[torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)] for _ in mats]
           for _ in range(steps)]
    for _ in range(warmup):
        for m in mats:
            m.linear()
    torch.cuda.synchronize()
    for s_i in range(steps):
        for i, m in enumerate(mats):
            evs[s_i][i][0].record()
            m.linear()
            evs[s_i][i][1].record()
    torch.cuda.synchronize()
    return np.array([[e[0].elapsed_time(e[1]) for e in ev] for ev in evs])


def time_set_back_to_back(mats, steps, warmup):
    """The same launches with no event between them: ms per pass over the set (what a stream of layers costs; the
    per-launch figures above each carry the few microseconds between an event and the start of a kernel)."""
    for _ in range(warmup):
        for m in mats:
            m.linear()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        for m in mats:
            m.linear()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def compact_storage_layers(mats, steps):
    """The same layers through bsp_linear, on the compact storage itself (no derived buffer): microseconds per launch,
    in turn, each between two events."""
    evs = [[[torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)] for _ in mats]
           for _ in range(steps)]
    for m in mats:
        bsp.bsp_linear(m.X, m.packed, m.bias, Y=m.Y)
    torch.cuda.synchronize()
    for s_i in range(steps):
        for i, m in enumerate(mats):
            evs[s_i][i][0].record()
            bsp.bsp_linear(m.X, m.packed, m.bias, Y=m.Y)
            evs[s_i][i][1].record()
    torch.cuda.synchronize()
    ms = np.array([[e[0].elapsed_time(e[1]) for e in ev] for ev in evs]).mean(axis=0)
    return {"entry_point": "bsp_linear", "ms": round(float(ms.sum()), 4),
            "us": {m.name: round(float(v) * 1e3, 2) for m, v in zip(mats, ms)}}


def per_matrix_report(mats, lin_avg_ms):
    out = {}
    for m, ms in zip(mats, lin_avg_ms):
        by = m.linear_bytes()
        out[m.name] = {
            "shape": [m.M, m.N], "kept_cols": m.kept_cols,
            "rate": round(bsp.bsp_compression_rate(m.M, m.N, m.R, m.kept_cols), 4),
            "us": round(float(ms) * 1e3, 2),
            "useful_tflops": round(m.useful_flops() / (ms * 1e-3) / 1e12, 2),
            "dense_equiv_tflops": round(m.dense_flops() / (ms * 1e-3) / 1e12, 2),
            "hbm_gbs": round(by / (ms * 1e-3) / 1e9, 1),
            "frac_mfma_peak": round(m.useful_flops() / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "frac_hbm_peak": round(by / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        }
    return out


def prepared_set(descs, scope=None):
    """Matrices of a workload with the storage and plan built once (kept counts read back for the accounting)."""
    mats = [Matrix(d) for d in descs]
    for m in mats:
        m.prune_and_pack()
        m.linear()
    torch.cuda.synchronize()
    for m in mats:
        m.kept_cols = int(m.blk_cnt.sum().item())
    return mats


def linear_only_set(descs, steps, warmup, label):
    """Layer-only timing of a whole set (one entry per matrix and the set's totals)."""
    mats = prepared_set(descs)
    ms = time_layers(mats, steps, warmup).mean(axis=0)
    useful = sum(m.useful_flops() for m in mats)
    tot = float(ms.sum())
    res = {"workload": label, "ms": round(tot, 4), "ms_back_to_back": round(time_set_back_to_back(mats, steps, 2), 4),
           "useful_tflops": round(useful / (tot * 1e-3) / 1e12, 2),
           "frac_mfma_peak": round(useful / (tot * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
           "frac_hbm_peak": round(sum(m.linear_bytes() for m in mats) / (tot * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
           "per_matrix": per_matrix_report(mats, ms)}
    del mats
    return res


def config1_latency(reps=5, launches=200):
    """Config 1 (BERT-base attention projection, fp32, 128 tokens, half of the columns kept per block): a
    latency case.  `launches` calls recorded into one HIP graph, the graph replayed `reps` times between two
    events; the median over the replays, per call."""
    c = wl.config1()
    W = torch.from_numpy(c["W"]).cuda()
    X = torch.from_numpy(c["X"]).cuda()
    b = torch.from_numpy(c["bias"]).cuda()
    p = bsp.bsp_pack(W, c["R"], torch.from_numpy(c["keep"]).cuda(), 32)
    Y = torch.empty((X.shape[0], W.shape[0]), dtype=torch.float32, device="cuda")
    bsp.bsp_linear(X, p, b, Y=Y)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(launches):
            bsp.bsp_linear(X, p, b, Y=Y)
    g.replay()
    torch.cuda.synchronize()
    us = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); g.replay(); e1.record()
        torch.cuda.synchronize()
        us.append(e0.elapsed_time(e1) * 1e3 / launches)
    kept = int(p.blk_cnt.sum().item())
    med = float(np.median(us))
    flops = 2.0 * X.shape[0] * c["R"] * kept
    return {"workload": "config 1: X 128x768, W 768x768, fp32, R = 16, 384 of 768 columns kept per block",
            "dtype": "f32", "us_per_call": round(med, 2), "useful_gflops": round(flops / med / 1e3, 1),
            "note": "launch-bound: 75 MFLOP of useful work per call"}


def config2_layer(c, steps):
    """Config 2 (BERT-base FFN up-projection, 4096 tokens, the top 256 of 768 groups of every row-block: 3x)."""
    d = dict(c)
    per_block = d["n_keep"]
    d["n_keep"] = per_block * (d["M"] // d["R"])     # what the storage has to hold
    m = Matrix(d)
    bsp.bsp_group_norms(m.W, m.R, eps=1e-6, mode=bsp.ALPHA_SQNORM, sumsq=m.sumsq, alpha=m.alpha, want=())
    bsp.bsp_prune_mask(m.sumsq, n_keep=per_block, scope=bsp.SCOPE_BLOCK, keep=m.keep)
    bsp.bsp_pack_count(m.keep, m.k_align, blk_cnt=m.blk_cnt, blk_ptr=m.blk_ptr)
    st = bsp.lib().bsp_pack(m.W.data_ptr(), bsp.BF16, m.M, m.N, m.R, m.keep.data_ptr(), m.k_align,
                            m.blk_cnt.data_ptr(), m.blk_ptr.data_ptr(), m.capacity, m.col_idx.data_ptr(),
                            m.vals.data_ptr(), bsp.BF16, torch.cuda.current_stream().cuda_stream)
    if st != 0:
        raise bsp.BspError(st, "bsp_pack")
    if m.use_plan:
        bsp.bsp_linear_plan(m.packed, plan=m.plan)
    m.linear()
    torch.cuda.synchronize()
    m.kept_cols = int(m.blk_cnt.sum().item())
    ms = time_layers([m], steps, 5).mean(axis=0)
    return {"workload": "config 2: X 4096x768, W 3072x768, bf16, R = 16, block-scope percentile, 256 of 768 kept (3x)",
            "per_matrix": per_matrix_report([m], ms)}


def fused_epilogue(mats, steps):
    """The layers with their epilogue inside the kernel (Sec. 4.4; Sec. 4.2's networks: GELU behind the FFN
    up-projection, a residual behind the attention output and the FFN down-projection) beside the plain layer:
    microseconds per call, and the bytes of the element-wise pass that the fusion saves."""
    by_name = {m.name: m for m in mats}
    out = {}
    for name, act, with_res in (("ffn_up", bsp.ACT_GELU, False), ("attn_out", bsp.ACT_NONE, True),
                                ("ffn_down", bsp.ACT_NONE, True)):
        m = by_name[name]
        res = torch.randn((m.T, m.M), device="cuda", generator=torch.Generator(device="cuda").manual_seed(77)
                          ).to(torch.bfloat16) if with_res else None
        def call():
            bsp.bsp_linear_planned_fused(m.X, m.packed, m.plan, m.bias, act=act, residual=res, Y=m.Y)
        us = {}
        for label, fn in (("plain", m.linear), ("fused", call)):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
            for e0, e1 in ev:       # the other layers pass in between: cold caches, as in `linear_only`
                for o in mats:
                    if o is not m:
                        o.linear()
                e0.record(); fn(); e1.record()
            torch.cuda.synchronize()
            us[label] = float(np.mean([e0.elapsed_time(e1) for e0, e1 in ev])) * 1e3
        saved = (2 + (1 if with_res else 0)) * 2.0 * m.T * m.M   # the pass it replaces: read Y (+ residual), write Y
        out[name] = {"epilogue": ("gelu" if act == bsp.ACT_GELU else "") + ("residual" if with_res else ""),
                     "us_plain": round(us["plain"], 2), "us_fused": round(us["fused"], 2),
                     "bytes_of_the_pass_saved": saved,
                     "us_of_that_pass_at_hbm_peak": round(saved / HBM_PEAK_GBS / 1e3, 2)}
    return out


def whole_block_mode(steps, Ct=32, R=16):
    """The comparison structure of Sec. 4.4 / Table 4 (a tile of R rows x Ct columns is kept or removed as a whole)
    on the BERT-large set at 5x, through the same storage, plan and layer kernels: kept columns then come in runs of
    Ct, and the layer's time is the bound the column-granular structure is measured against."""
    mats = []
    for d in wl.config4(R=R):
        m = Matrix(d)
        bsp.bsp_group_norms(m.W, m.R, eps=1e-6, mode=bsp.ALPHA_SQNORM, sumsq=m.sumsq, alpha=m.alpha, want=())
        ts = bsp.bsp_tile_sumsq(m.sumsq, Ct)
        tk, _ = bsp.bsp_prune_mask(ts, n_keep=ts.numel() // 5, scope=bsp.SCOPE_MATRIX)
        m.keep = bsp.bsp_expand_tile_mask(tk, Ct)
        bsp.bsp_pack_count(m.keep, m.k_align, blk_cnt=m.blk_cnt, blk_ptr=m.blk_ptr)
        st = bsp.lib().bsp_pack(m.W.data_ptr(), bsp.BF16, m.M, m.N, m.R, m.keep.data_ptr(), m.k_align,
                                m.blk_cnt.data_ptr(), m.blk_ptr.data_ptr(), m.capacity, m.col_idx.data_ptr(),
                                m.vals.data_ptr(), bsp.BF16, torch.cuda.current_stream().cuda_stream)
        if st != 0:
            raise bsp.BspError(st, "bsp_pack")
        bsp.bsp_linear_plan(m.packed, plan=m.plan)
        m.linear()
        torch.cuda.synchronize()
        m.kept_cols = int(m.blk_cnt.sum().item())
        mats.append(m)
    ms = time_layers(mats, steps, 3).mean(axis=0)
    return {"tile": [R, Ct], "ms": round(float(ms.sum()), 4), "per_matrix": per_matrix_report(mats, ms)}


def cpu_baseline(mats):
    """The CPU oracle's layer on the same workload (all four matrices, all tokens: about a
    second per matrix on this machine's host cores), timed as it stands."""
    from oracle import bsp_oracle as orc
    cores = min(len(os.sched_getaffinity(0)), 16)
    flops, secs = 0.0, 0.0
    for m in mats:
        W = m.W.float().cpu().numpy()
        X = m.X.float().cpu().numpy()
        bias = m.bias.float().cpu().numpy()
        p = orc.pack(W, m.R, m.keep.cpu().numpy(), m.k_align, orc.BF16)
        t = time.perf_counter()
        orc.linear_packed(X, p, bias, ydt=orc.BF16, n_threads=cores)
        secs += time.perf_counter() - t
        flops += 2.0 * m.T * m.R * int(p["blk_cnt"].sum())
    # one thread, on the first 256 tokens of the first matrix
    m = mats[0]
    p = orc.pack(m.W.float().cpu().numpy(), m.R, m.keep.cpu().numpy(), m.k_align, orc.BF16)
    X1 = m.X[:256].float().cpu().numpy()
    t = time.perf_counter()
    orc.linear_packed(X1, p, m.bias.float().cpu().numpy(), ydt=orc.BF16, n_threads=1)
    one = 2.0 * 256 * m.R * int(p["blk_cnt"].sum()) / (time.perf_counter() - t) / 1e12
    return {"value": round(flops / secs / 1e12, 5), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "single_thread_tflops": round(one, 5),
            "sample": f"oracle layer (fp64 accumulate, OpenMP over row-blocks) on the full set, all 8192 tokens; {secs:.1f} s "
                      f"on {cores} threads; single thread: 256 tokens of the QKV matrix"}


def transposed_product(mats, reps=10, with_cpu=True):
    """The transposed product Z = U Wp (input gradient of the layer; the layer of the row-segment variant on a
    transposed matrix) on the same four compact storages: U is a synthetic [tokens, M] bf16 tensor, every launch
    between two events on the launch stream.  Algorithmic bytes: U read once, Z written once, the storage read once."""
    out, tot_us, tot_flops, lds_bytes, hbm_bytes, tot_dense_us = {}, 0.0, 0.0, 0.0, 0.0, 0.0
    for m in mats:
        gen = torch.Generator(device="cuda").manual_seed(4200 + m.M + m.N)   # seeded: the stand-in for an output gradient
        U = torch.randn((m.T, m.M), device="cuda", generator=gen).to(torch.bfloat16)
        Z = torch.empty((m.T, m.N), dtype=torch.bfloat16, device="cuda")
        for _ in range(3):
            bsp.bsp_linear_transposed(U, m.packed, None, Z)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            bsp.bsp_linear_transposed(U, m.packed, None, Z)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / reps * 1e3
        # the same product as a dense one on the masked matrix (bsp_linear_transposed_dense: rocBLAS), which spends
        # 1 / density times the FLOPs
        Wm = m.W.clone()
        bsp.bsp_mask_weights(Wm, m.R, m.keep)
        for _ in range(3):
            bsp.bsp_linear_transposed_dense(U, Wm, None, Z)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            bsp.bsp_linear_transposed_dense(U, Wm, None, Z)
        e1.record()
        torch.cuda.synchronize()
        us_dense = e0.elapsed_time(e1) / reps * 1e3
        del Wm
        padded = int(m.blk_ptr[-1].item())
        by = 2.0 * m.T * m.M + 2.0 * m.T * m.N + 2.0 * m.R * padded + 4.0 * padded
        tf = m.useful_flops() / us / 1e6
        lds = 8.0 * m.T * m.kept_cols    # one fp32 cell read and written per token, kept column and row-block
        lds_bytes += lds
        hbm_bytes += by
        out[m.name] = {"shape": [m.M, m.N], "us": round(us, 1), "useful_tflops": round(tf, 2),
                       "dense_on_masked_matrix_us": round(us_dense, 1),
                       "dense_on_masked_matrix_useful_tflops": round(m.useful_flops() / us_dense / 1e6, 1),
                       "dense_on_masked_matrix_dense_tflops": round(m.dense_flops() / us_dense / 1e6, 1),
                       "lds_gbs": round(lds / us / 1e3, 1),
                       "frac_mfma_peak": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
                       "hbm_gbs": round(by / us / 1e3, 1), "frac_hbm_peak": round(by / us / 1e3 / HBM_PEAK_GBS, 4)}
        tot_us += us
        tot_dense_us += us_dense
        tot_flops += m.useful_flops()
        del U, Z
    res = {"kernel": "linear_t_mfma_kernel", "per_matrix": out, "us": round(tot_us, 1),
           "useful_tflops": round(tot_flops / tot_us / 1e6, 2),
           "dense_on_masked_matrix": {"entry_point": "bsp_linear_transposed_dense (rocBLAS)", "us": round(tot_dense_us, 1),
                                      "useful_tflops": round(tot_flops / tot_dense_us / 1e6, 2)},
           "frac_mfma_peak": round(tot_flops / tot_us / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4),
           # the method's traffic: U read once, Z written once, the storage read once (the same pair of roofs as the layer)
           "roofline": {"bound": "hbm", "achieved": round(hbm_bytes / tot_us / 1e3, 1), "peak": HBM_PEAK_GBS,
                        "unit": "GB/s", "frac": round(hbm_bytes / tot_us / 1e3 / HBM_PEAK_GBS, 4), "traffic": None},
           "lds_diagnostic": {"achieved_gbs": round(lds_bytes / tot_us / 1e3, 1), "peak_gbs": LDS_PEAK_GBS,
                              "frac": round(lds_bytes / tot_us / 1e3 / LDS_PEAK_GBS, 4),
                              "note": "what this design moves through LDS: one fp32 cell of the tile read and written per "
                                      "token, kept column and row-block; 256 compute units x 256 B/clk x 2.4 GHz"}}
    if with_cpu:
        from oracle import bsp_oracle as orc
        m = mats[2]
        cores = min(len(os.sched_getaffinity(0)), 16)
        p = orc.pack(m.W.float().cpu().numpy(), m.R, m.keep.cpu().numpy(), m.k_align, orc.BF16)
        rows = m.T
        U1 = np.random.default_rng(1).standard_normal((rows, m.M)).astype(np.float32)
        t = time.perf_counter()
        orc.linear_t_packed(U1, p, None, zdt=orc.BF16, n_threads=cores)
        secs = time.perf_counter() - t
        res["cpu_oracle"] = {"value": round(2.0 * rows * m.R * int(p["blk_cnt"].sum()) / secs / 1e12, 5),
                             "unit": "TFLOP/s", "cores": cores,
                             "sample": f"oracle transposed product (fp64, OpenMP over token rows), {rows} token rows of "
                                       f"the {m.name} matrix, {secs:.2f} s"}
    return res


def weight_gradient(mats, reps=10, with_cpu=True):
    """The gradient with respect to the kept weights, D = dY^T X on the kept positions (Alg. 2's weight update), on
    the same four compact storages: dY is a synthetic [tokens, M] bf16 tensor, bf16 output in the layout of the value
    panels.  `us` is a call that reuses the work list of its workspace (two launches: partial sums, ordered sum: the
    retraining loop of Alg. 2, where the mask is fixed), `us_first_call` one that builds the list too; ten calls between
    two events on the launch stream.  Algorithmic bytes: X and dY read once, the column indices read once, D written
    once."""
    out, tot_us, tot_flops, hbm_bytes = {}, 0.0, 0.0, 0.0
    for m in mats:
        gen = torch.Generator(device="cuda").manual_seed(5200 + m.M + m.N)   # seeded: the stand-in for an output gradient
        dY = torch.randn((m.T, m.M), device="cuda", generator=gen).to(torch.bfloat16)
        padded = int(m.blk_ptr[-1].item())
        D = torch.empty(m.R * padded, dtype=torch.bfloat16, device="cuda")
        ws = torch.empty(bsp.lib().bsp_linear_dvals_workspace_bytes(m.M, m.N, m.R, m.capacity), dtype=torch.uint8,
                         device="cuda")
        def timed(state):
            for _ in range(3):
                bsp.bsp_linear_dvals(m.X, dY, m.packed, D=D, ws=ws, ws_state=bsp.DVALS_BUILD)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                bsp.bsp_linear_dvals(m.X, dY, m.packed, D=D, ws=ws, ws_state=state)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps * 1e3
        us_first = timed(bsp.DVALS_BUILD)
        us = timed(bsp.DVALS_REUSE)
        by = 2.0 * m.T * m.N + 2.0 * m.T * m.M + 2.0 * m.R * padded + 4.0 * padded
        tf = m.useful_flops() / us / 1e6
        hbm_bytes += by
        out[m.name] = {"shape": [m.M, m.N], "us": round(us, 1), "us_first_call": round(us_first, 1),
                       "useful_tflops": round(tf, 2), "frac_mfma_peak": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
                       "hbm_gbs": round(by / us / 1e3, 1), "frac_hbm_peak": round(by / us / 1e3 / HBM_PEAK_GBS, 4)}
        tot_us += us
        tot_flops += m.useful_flops()
        del dY, D, ws
    res = {"kernels": ["dvals_items_kernel", "dvals_partial_kernel", "dvals_reduce_kernel"], "per_matrix": out,
           "us": round(tot_us, 1), "useful_tflops": round(tot_flops / tot_us / 1e6, 2),
           "frac_mfma_peak": round(tot_flops / tot_us / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4),
           "roofline": {"bound": "hbm", "achieved": round(hbm_bytes / tot_us / 1e3, 1), "peak": HBM_PEAK_GBS,
                        "unit": "GB/s", "frac": round(hbm_bytes / tot_us / 1e3 / HBM_PEAK_GBS, 4), "traffic": None}}
    if with_cpu:
        from oracle import bsp_oracle as orc
        m = mats[1]
        cores = min(len(os.sched_getaffinity(0)), 16)
        p = orc.pack(m.W.float().cpu().numpy(), m.R, m.keep.cpu().numpy(), m.k_align, orc.BF16)
        rows = 2048
        rng = np.random.default_rng(2)
        X1 = rng.standard_normal((rows, m.N)).astype(np.float32)
        dY1 = rng.standard_normal((rows, m.M)).astype(np.float32)
        t = time.perf_counter()
        orc.linear_dvals(X1, dY1, p, gdt=orc.BF16, n_threads=cores)
        secs = time.perf_counter() - t
        res["cpu_oracle"] = {"value": round(2.0 * rows * m.R * int(p["blk_cnt"].sum()) / secs / 1e12, 5),
                             "unit": "TFLOP/s", "cores": cores,
                             "sample": f"oracle weight gradient (fp64, OpenMP over row-blocks), {rows} token rows of "
                                       f"the {m.name} matrix, {secs:.2f} s"}
    return res


def prune_path_c5(layers=24, reps=5, with_cpu=True):
    """HBM rate of the pruning pipeline on the 24-layer BERT-large weight set (fp32, 302 M parameters, R = 16):
    group norms + reweighting factors, regulariser gradient, one global percentile over all 18.9 M groups (5x),
    pack with fp32 and with bf16 value panels, and the zeroing of the pruned groups in W.  Matrices that are adjacent in the buffer and share their
    width are stacked along the rows into one launch (row-blocks are independent), which leaves two launches
    per layer.  Every stage is recorded into a HIP graph and replayed `reps` times between two events."""
    c = wl.config5(layers)
    R, eps, lam = c["R"], c["eps"], c["lam"]
    Wbuf = torch.from_numpy(c["W"]).cuda()
    runs = []                                   # (offset, rows, N) of every stacked launch
    for off, m, n in c["desc"]:
        if runs and runs[-1][2] == n and runs[-1][0] + runs[-1][1] * n == off:
            runs[-1] = (runs[-1][0], runs[-1][1] + m, n)
        else:
            runs.append((off, m, n))
    params = Wbuf.numel()
    groups = params // R
    dev = Wbuf.device
    sumsq = torch.empty(groups, dtype=torch.float32, device=dev)
    alpha = torch.empty(groups, dtype=torch.float32, device=dev)
    grad = torch.empty_like(Wbuf)
    keep = torch.empty(groups, dtype=torch.uint8, device=dev)
    n_keep = groups * c["rate"][1] // c["rate"][0]
    Bm, Nm = groups // 1024, 1024               # the global scope: all groups as one [B, N] array
    ws = torch.empty(bsp.lib().bsp_prune_mask_workspace_bytes(Bm, Nm, bsp.SCOPE_MATRIX), dtype=torch.uint8, device=dev)
    views = []
    for off, rows, n in runs:
        g0, ng = off // R, rows // R * n
        views.append(dict(W=Wbuf[off:off + rows * n].view(rows, n), G=grad[off:off + rows * n].view(rows, n),
                          s=sumsq[g0:g0 + ng].view(rows // R, n), a=alpha[g0:g0 + ng].view(rows // R, n),
                          k=keep[g0:g0 + ng].view(rows // R, n),
                          cnt=torch.empty(rows // R, dtype=torch.int32, device=dev),
                          ptr=torch.empty(rows // R + 1, dtype=torch.int32, device=dev)))

    def norms():
        for v in views:
            bsp.bsp_group_norms(v["W"], R, eps=eps, mode=bsp.ALPHA_SQNORM, sumsq=v["s"], alpha=v["a"], want=())

    def gradient():
        for v in views:
            bsp.bsp_penalty_grad(v["W"], R, v["a"], lam, mode=bsp.ALPHA_SQNORM, grad=v["G"])

    def norms_gradient():
        for v in views:
            bsp.bsp_group_norms_grad(v["W"], R, lam, eps=eps, mode=bsp.ALPHA_SQNORM, sumsq=v["s"], alpha=v["a"],
                                     grad=v["G"], want=())

    def mask():
        bsp.bsp_prune_mask(sumsq.view(Bm, Nm), n_keep=n_keep, scope=bsp.SCOPE_MATRIX, keep=keep.view(Bm, Nm), ws=ws)

    def count():
        for v in views:
            bsp.bsp_pack_count(v["k"], 32, blk_cnt=v["cnt"], blk_ptr=v["ptr"])

    def pack(vdt):
        L = bsp.lib()
        for v in views:
            rows, n = v["W"].shape
            st = L.bsp_pack(v["W"].data_ptr(), bsp.F32, rows, n, R, v["k"].data_ptr(), 32, v["cnt"].data_ptr(),
                            v["ptr"].data_ptr(), v["cap"], v["col"].data_ptr(), v["vals"][vdt].data_ptr(), vdt,
                            torch.cuda.current_stream().cuda_stream)
            if st != 0:
                raise bsp.BspError(st, "bsp_pack")

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3   # us

    t = {}
    t["group_norms"] = timed(norms)
    t["penalty_grad"] = timed(gradient)
    t["group_norms_grad"] = timed(norms_gradient)
    t["prune_mask"] = timed(mask)
    t["pack_count"] = timed(count)
    kept = 0
    for v in views:                                 # capacities, read back once
        v["cap"] = int(v["ptr"][-1].item())
        kept += int(v["cnt"].sum().item())
        v["col"] = torch.empty(max(v["cap"], 1), dtype=torch.int32, device=dev)
        v["vals"] = {bsp.F32: torch.empty(max(R * v["cap"], 1), dtype=torch.float32, device=dev),
                     bsp.BF16: torch.empty(max(R * v["cap"], 1), dtype=torch.bfloat16, device=dev)}
    t["pack_fp32"] = timed(lambda: pack(bsp.F32))
    t["pack_bf16"] = timed(lambda: pack(bsp.BF16))

    def mask_weights():                              # last: it overwrites the pruned groups of W (idempotent)
        for v in views:
            bsp.bsp_mask_weights(v["W"], R, v["k"])

    t["mask_weights"] = timed(mask_weights)
    mom1, mom2 = torch.zeros_like(Wbuf), torch.zeros_like(Wbuf)
    grad.normal_(0.0, 1e-3)

    def adam(reg, masked):                           # the weight update of Alg. 2's two loops, whole state in place
        for v in views:
            off = v["W"].data_ptr() - Wbuf.data_ptr()
            sl = slice(off // 4, off // 4 + v["W"].numel())
            bsp.bsp_adam_step(v["W"], v["G"], mom1[sl].view_as(v["W"]), mom2[sl].view_as(v["W"]), R, 3e-5, t=3,
                              alpha=v["a"] if reg else None, lam=lam, keep=v["k"] if masked else None)

    t["adam_mixed_loss"] = timed(lambda: adam(True, False))
    t["adam_masked"] = timed(lambda: adam(False, True))
    padded = sum(v["cap"] for v in views)
    # algorithmic bytes: W fp32 read once per stage that needs it, group arrays fp32, the mask 1 byte per group
    by = {"group_norms": 4.0 * params + 8.0 * groups,
          "penalty_grad": 8.0 * params + 4.0 * groups,
          "group_norms_grad": 8.0 * params + 8.0 * groups,   # both of the above with W read once
          "prune_mask": (4.0 * 4 + 1.0) * groups,
          "pack_count": 1.0 * groups,
          "pack_fp32": 4.0 * params + 1.0 * groups + (4.0 * R + 4.0) * padded,
          "pack_bf16": 4.0 * params + 1.0 * groups + (2.0 * R + 4.0) * padded,
          "mask_weights": 8.0 * params + 1.0 * groups,   # W read and written back, the mask read
          "adam_mixed_loss": 28.0 * params + 4.0 * groups,   # w, g, m, v read; w, m, v written; the factors read
          "adam_masked": 28.0 * params + 1.0 * groups}
    stages = {k: {"us": round(t[k], 1), "gbs": round(by[k] / (t[k] * 1e-6) / 1e9, 1),
                  "frac_hbm_peak": round(by[k] / (t[k] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)} for k in t}
    cpu = None
    if with_cpu:
        from oracle import bsp_oracle as orc
        off, rows, n = runs[0]
        rows1 = min(rows, 8192)                    # one layer's matrices of width 1024: 8.4 M parameters, 524 288 groups
        W1 = c["W"][off:off + rows1 * n].reshape(rows1, n)
        tt = time.perf_counter()
        s1 = orc.sumsq(W1, R)
        _, a1 = orc.norm_alpha(s1, eps, orc.ALPHA_SQNORM)
        t_norm = time.perf_counter() - tt
        tt = time.perf_counter()
        orc.penalty_grad(W1, R, a1, lam, orc.ALPHA_SQNORM)
        t_grad = time.perf_counter() - tt
        tt = time.perf_counter()
        k1, _ = orc.mask_rank(s1.reshape(1, -1), s1.size // 5, orc.SCOPE_MATRIX)
        t_mask = time.perf_counter() - tt
        tt = time.perf_counter()
        orc.pack(W1, R, k1.reshape(s1.shape), 32, orc.F32)
        t_pack = time.perf_counter() - tt
        p1, g1 = W1.size, s1.size
        cpu = {"kind": "oracle", "cores": 1, "sample": "the first layer's matrices of width 1024 (%d parameters)" % p1,
               "group_norms_gbs": round((4.0 * p1 + 8.0 * g1) / t_norm / 1e9, 2),
               "penalty_grad_gbs": round((8.0 * p1 + 4.0 * g1) / t_grad / 1e9, 2),
               "prune_mask_gbs": round(17.0 * g1 / t_mask / 1e9, 3),
               "pack_fp32_gbs": round((4.0 * p1 + g1 + 68.0 * (g1 // 5)) / t_pack / 1e9, 2)}
    return {"workload": "config 5: %d-layer BERT-large weight set, fp32, %d parameters, R = 16, global 5x percentile"
                        % (layers, params),
            "cpu_baseline": cpu,
            "launches_per_stage": len(views), "groups": groups, "kept_groups": kept,
            "rate": round(params / (R * max(kept, 1)), 4), "stages": stages}


def linear_grid(T=8192, R=16, reps=3):
    """The layer alone over (matrix, compression rate): BERT-base and BERT-large shapes at 1.5x, 2x, 3x and 5x.
    Per entry: microseconds per call (10 calls in a HIP graph, `reps` replays between two events), useful
    TFLOP/s, and that rate as a fraction of the lower of the two roofs (MFMA peak, HBM peak x arithmetic
    intensity).  Warm timing: the same layer is launched back to back, so X (12 to 67 MB) can stay in the
    256 MB Infinity Cache between launches."""
    shapes = [("base_qkv", 2304, 768), ("base_out", 768, 768), ("base_up", 3072, 768), ("base_down", 768, 3072),
              ("large_qkv", 3072, 1024), ("large_out", 1024, 1024), ("large_up", 4096, 1024), ("large_down", 1024, 4096)]
    out = {}
    for si, (name, M, N) in enumerate(shapes):
        # for comparison: the unpruned layer as a dense library product (torch.matmul on the same X and W)
        d0 = wl.layer(900 + si, T, M, N, "bf16")
        Xd = torch.from_numpy(d0["X"]).to(torch.bfloat16).cuda()
        Wd = torch.from_numpy(d0["W"]).to(torch.bfloat16).cuda()
        Yd = torch.empty((T, M), dtype=torch.bfloat16, device="cuda")
        for _ in range(3):
            torch.matmul(Xd, Wd.t(), out=Yd)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10 * reps):
            torch.matmul(Xd, Wd.t(), out=Yd)
        e1.record()
        torch.cuda.synchronize()
        dense_us = e0.elapsed_time(e1) * 1e3 / (10 * reps)
        del Xd, Wd, Yd
        for num, den in ((3, 2), (2, 1), (3, 1), (5, 1)):
            d = wl.layer(900 + si, T, M, N, "bf16")
            d.update(name=name, M=M, N=N, R=R, T=T, n_keep=(M // R) * N * den // num)
            m = Matrix(d)
            m.prune_and_pack()
            m.linear()
            torch.cuda.synchronize()
            m.kept_cols = int(m.blk_cnt.sum().item())
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for _ in range(10):
                    m.linear()
            g.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                g.replay()
            e1.record()
            torch.cuda.synchronize()
            sec = e0.elapsed_time(e1) * 1e-3 / (10 * reps)
            tf = m.useful_flops() / sec / 1e12
            roof = min(MFMA_BF16_PEAK_TFLOPS, HBM_PEAK_GBS * 1e-3 * m.useful_flops() / m.linear_bytes())
            out["%s@%.1fx" % (name, num / den)] = {"us": round(sec * 1e6, 1), "useful_tflops": round(tf, 1),
                                                  "dense_library_us": round(dense_us, 1),
                                                  "speedup_over_dense": round(dense_us / (sec * 1e6), 2),
                                                  "frac_mfma_peak": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
                                                  "frac_of_lower_roof": round(tf / roof, 4)}
            del m, g
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--R", type=int, default=16)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--path", choices=["planned", "canonical"], default="planned",
                    help="layer operands: the derived plan buffer (default) or the compact storage itself")
    ap.add_argument("--launch", choices=["overlap", "serial", "eager"], default="overlap",
                    help="overlap: one HIP graph, a branch per matrix; serial: one HIP graph, matrices in turn; "
                         "eager: every kernel launched from Python")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one 256 MiB device-to-device copy (a kernel of known traffic, to scale the "
                         "profiler's memory counters)")
    ap.add_argument("--no-grid", action="store_true",
                    help="skip the layer-only table over BERT-base / BERT-large shapes and compression rates")
    ap.add_argument("--no-transposed", action="store_true",
                    help="skip the timing of the transposed product (input gradient) and of the weight gradient on the same "
                         "storages")
    ap.add_argument("--only", choices=["layer", "transposed", "dvals"], default=None,
                    help="run nothing but the layer launches (or the transposed product's) of the workload, `--steps` "
                         "times in turn: the command the kernel profiles under profiles/ are taken with")
    ap.add_argument("--no-sets", action="store_true",
                    help="skip the layer-only lines of R = 8 and R = 32 and of configs 1 to 3")
    ap.add_argument("--no-c5", action="store_true",
                    help="skip the bandwidth measurement of the pruning pipeline on the 302 M parameter weight set")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the path has no multi-GPU part; run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)

    if args.copy_probe:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    mats = [Matrix(d, path=args.path) for d in wl.config4(R=args.R)]
    for m in mats:   # once, to learn the kept counts (needed only for the FLOP accounting)
        m.prune_and_pack()
        m.linear()
    torch.cuda.synchronize()
    for m in mats:
        m.kept_cols = int(m.blk_cnt.sum().item())
    if args.only == "layer":
        ms = time_layers(mats, args.steps, args.warmup).mean(axis=0)
        print(json.dumps({"only": "layer", "block_rows": args.R, "per_matrix": per_matrix_report(mats, ms)}))
        return
    if args.only == "dvals":
        print(json.dumps({"only": "dvals", "block_rows": args.R,
                          "weight_gradient": weight_gradient(mats, reps=args.steps, with_cpu=False)}))
        return
    if args.only == "transposed":
        print(json.dumps({"only": "transposed", "block_rows": args.R,
                          "transposed_product": transposed_product(mats, reps=args.steps, with_cpu=False)}))
        return

    graphs, side_streams = [], []
    if args.launch == "serial":
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for m in mats:
                m.whole_step()
        graphs = [g]
    elif args.launch == "overlap":
        # one graph per matrix, each replayed on a default-priority stream of its own
        for m in mats:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                m.whole_step()
            graphs.append(g)
        pool, stream_probe = streams_on_different_queues(4)   # default priority

    def step():
        if args.launch == "eager":
            for m in mats:
                m.whole_step()
        elif args.launch == "serial":
            graphs[0].replay()
        else:
            # every matrix keeps to its own stream: its steps follow each other there, and nothing orders
            # one matrix's step k against another matrix's step k (they share no data)
            for g, side in zip(graphs, side_streams):
                with torch.cuda.stream(side):
                    g.replay()

    def run_steps(k):
        main = torch.cuda.current_stream()
        for side in side_streams:
            side.wait_stream(main)
        for _ in range(k):
            step()
        for side in side_streams:
            main.wait_stream(side)
        torch.cuda.synchronize()

    if args.launch == "overlap":
        side_streams = pool[:4]   # chosen by the queue probe above, before anything of the benchmark ran on them

    run_steps(args.warmup)
    t0 = time.perf_counter()
    run_steps(args.steps)
    wall = time.perf_counter() - t0

    # second pass: the layer launches alone, each between two events on the launch stream
    ms_per_step = wall * 1e3 / args.steps
    lin_ms = time_layers(mats, args.steps, args.warmup)                             # [steps, matrices]
    lin_avg = lin_ms.mean(axis=0)
    useful = sum(m.useful_flops() for m in mats)
    dense = sum(m.dense_flops() for m in mats)
    lin_bytes = [m.linear_bytes() for m in mats]
    lin_total_ms = float(lin_avg.sum())

    per_matrix = per_matrix_report(mats, lin_avg)

    # the layer kernel that takes the most time per step: algorithmic bytes of its launches over their durations
    def kernel_of(m):
        if not m.use_plan:
            return "bsp_linear (compact storage)"
        # the kernels of 16-row blocks (pairs of 8-row blocks, slabs of 32-, 48- and 64-row blocks ride them): which
        # one, the plan's chunking decides
        if m.R in (16, 32, 48, 64) or (m.R == 8 and m.M % 16 == 0):
            streams_x = m.N > 1024 or (m.N > 512 and m.M // 16 <= 64)
            return "linear_stream16_kernel" if streams_x else "linear_steploop16_kernel"
        return "linear_tiled_planned_kernel" if m.N <= 1024 else "linear_tiled_chunked_kernel"
    fam = {}
    for m, ms, by in zip(mats, lin_avg, lin_bytes):
        f = fam.setdefault(kernel_of(m), {"ms": 0.0, "bytes": 0.0, "launches": []})
        f["ms"] += float(ms); f["bytes"] += by; f["launches"].append(m.name)
    dom_name, dom = max(fam.items(), key=lambda kv: kv[1]["ms"])
    achieved_gbs = dom["bytes"] / (dom["ms"] * 1e-3) / 1e9
    achieved_tflops = useful / (lin_total_ms * 1e-3) / 1e12
    out = {
        "metric": "block-sparse linear useful TFLOP/s at BERT-large",
        "value": round(useful / (ms_per_step * 1e-3) / 1e12, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "BERT-large linear set (configs[3]): QKV 3072x1024, out 1024x1024, up 4096x1024, "
                               "down 1024x4096; 8192 tokens; 5x compression; matrix-scope percentile mask",
                   "block_rows": args.R, "k_align": 32, "tokens": 8192,
                   "layer_path": args.path,
                   "stream_probe": stream_probe if args.launch == "overlap" else None,
                   "launch": {"overlap": "one HIP graph per matrix, the four replayed side by side on four streams of "
                                         "which no two share a hardware queue (found by a probe of tiny kernels "
                                         "before the timed region)",
                              "serial": "one HIP graph per step, matrices in turn",
                              "eager": "every kernel launched from Python"}[args.launch],
                   "step": "group_norms_grad (norms, factors and regulariser gradient in one pass) + prune_mask_count "
                           "(mask and storage sizes) + pack + linear_plan + linear, 4 matrices"},
        "linear_only": {"cache_state": "cold: the four layers run in turn, so about 250 MB of other X / Y traffic "
                                       "(the size of the Infinity Cache) passes between two launches of one layer",
                        "ms": round(lin_total_ms, 4),
                        "ms_back_to_back": round(time_set_back_to_back(mats, args.steps, 2), 4),
                        "useful_tflops": round(achieved_tflops, 2),
                        "dense_equiv_tflops": round(dense / (lin_total_ms * 1e-3) / 1e12, 2),
                        "frac_mfma_peak": round(achieved_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                        "per_matrix": per_matrix,
                        "on_the_compact_storage": compact_storage_layers(mats, max(3, args.steps // 10))},
        "roofline": {"kernel": dom_name, "launches_per_step": dom["launches"],
                     "avg_launch_us": round(dom["ms"] * 1e3 / len(dom["launches"]), 2), "bound": "hbm",
                     "achieved": round(achieved_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved_gbs / HBM_PEAK_GBS, 4),
                     "traffic": DOMINANT_KERNEL_HBM_BYTES_PER_LAUNCH.get(dom_name) if args.R == 16 else None},
        "roofline_mfma": {"bound": "mfma", "achieved": round(achieved_tflops, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                          "unit": "TFLOP/s", "frac": round(achieved_tflops / MFMA_BF16_PEAK_TFLOPS, 4)},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(mats)
    if not args.no_sets:
        k = max(10, args.steps // 4)
        sets = {}
        for R in (8, 16, 32):
            if R != args.R:
                sets["config4_R%d" % R] = linear_only_set(
                    wl.config4(R=R), k, 5, "config 4 (BERT-large set, 8192 tokens, 5x) with row-blocks of %d rows" % R)
        sets["config3"] = linear_only_set(
            wl.config3(), k, 5, "config 3 (BERT-base set, 8192 tokens, R = 16, per-matrix rate drawn from 1.5x, 2x, "
                                "3x, 5x, matrix-scope percentile), the four layers timed in turn")
        sets["config3"]["rates"] = {d["name"]: "%d/%d" % d["rate"] for d in wl.config3(tokens=16)}
        c2 = wl.config2()
        c2.update(name="ffn_up", T=c2["X"].shape[0])
        sets["config2"] = config2_layer(c2, k)
        sets["config1"] = config1_latency()
        out["linear_only_sets"] = sets
        if args.R == 16:
            out["fused_epilogue"] = fused_epilogue(mats, k)
            out["whole_block_mode"] = whole_block_mode(k)
    if not args.no_grid:
        out["linear_grid"] = linear_grid()
    if not args.no_transposed:
        out["transposed_product"] = transposed_product(mats, with_cpu=not args.no_cpu_baseline)
        out["weight_gradient"] = weight_gradient(mats, with_cpu=not args.no_cpu_baseline)
    if not args.no_c5:
        del mats
        torch.cuda.empty_cache()
        out["prune_path_c5"] = prune_path_c5(with_cpu=not args.no_cpu_baseline)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
