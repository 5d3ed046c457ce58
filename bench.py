#!/usr/bin/env python3
"""Benchmark of the MACKO sparse matrix-vector product on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-sweep] [--no-stack] [--no-spmm]

Workload (default): the Llama2-7B-shaped linear layers at 50 % per-row
unstructured sparsity (4 x 4096x4096, 2 x 11008x4096, 1 x 4096x11008), fp16
N(0, 0.02) weights, fp16 N(0,1) activations, batch 1.  One "step" is one pass
over one decoder layer's seven sparse products on one stream, in the order their
data dependences allow: {q,k,v} -> {o} -> {gate,up} -> {down}, four grouped
launches (macko_spmv_group); the seven-separate-launches timing is reported too.
Steps rotate over several copies of the layer at distinct addresses so that no
step finds its matrices in the 256 MB last-level cache (the paper invalidates
the cache before every run, Section 5.1).

Every timed region is repeated in rounds of K steps (of the smallest multiple of K steps that
lasts 5 ms, when K steps are shorter) until at least 30 ms have been timed, and the median
round is reported per K steps (a region of a millisecond right after set-up work reads up to
8 % slow: the clocks have not settled; the event between two rounds costs 1 % of a 1 ms round).  Outside the headline's timed region the
default run also times the 36864 x 12288 sparsity sweep at its nine levels, the 32-layer
Llama2-13B-shaped stack and the small-batch product, and compares y of every timed
configuration with the CPU oracle's dense product once before timing it.

Prints ONE JSON line.  `value` is algorithmic bytes (format arrays + x + y, the
compute-intensity accounting of Section 3.1) moved per second over the timed
region; the same loop over the dense fp16 GEMV gives the speedup.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0       # MI355X published HBM3E bandwidth
CACHE_BYTES = 256 << 20      # last-level (Infinity Cache) capacity to defeat


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def spmv_bytes(rep) -> int:
    """values + deltas + row pointers + x once + y once."""
    return rep.total_bytes + 2 * rep.cols + 2 * rep.rows


def dense_bytes(rows, cols) -> int:
    return 2 * rows * cols + 2 * cols + 2 * rows


class SparseOp:
    """One matrix bound to the device `copies` times at distinct addresses."""

    def __init__(self, M, torch, case, copies, b_delta=4):
        self.name, self.rows, self.cols = case.name, case.rows, case.cols
        first = M.encode(case.W, b_delta).to_device()     # host encoder, torch-owned device memory
        self.report = first.report
        self.handles = [first]
        if copies > 1:                                   # further copies: GPU encoder (bit-identical output)
            Wd = torch.from_numpy(case.W.view(np.float16)).cuda()
            for _ in range(copies - 1):
                self.handles.append(M.encode_device(Wd, b_delta=b_delta))
            del Wd
        self.x = torch.from_numpy(case.x.view(np.float16)).cuda()
        self.y = torch.empty(case.rows, dtype=torch.float16, device="cuda")
        self.bytes = spmv_bytes(self.report)

    def launch(self, copy, stream_ptr):
        return self.handles[copy].spmv_raw(self.x.data_ptr(), self.y.data_ptr(), stream_ptr)


class DenseOp:
    def __init__(self, M, torch, case, copies):
        self.name, self.rows, self.cols = case.name, case.rows, case.cols
        W = torch.from_numpy(case.W.view(np.float16)).cuda()
        self.W = [W] + [W.clone() for _ in range(copies - 1)]
        self.x = torch.from_numpy(case.x.view(np.float16)).cuda()
        self.y = torch.empty(case.rows, dtype=torch.float16, device="cuda")
        self.bytes = dense_bytes(case.rows, case.cols)
        self._fn = M.load_library().macko_dense_gemv

    def launch(self, copy, stream_ptr):
        W = self.W[copy]
        return self._fn(W.data_ptr(), self.rows, self.cols, W.stride(0), self.x.data_ptr(),
                        self.y.data_ptr(), stream_ptr)


LAST_ROUNDS = 0
LAST_ROUND_STEPS = 0


def time_region(torch, fn, n_warm, n_timed):
    """fn(i) enqueues iteration i on torch's current stream.  Returns seconds for n_timed
    iterations: the median of the rounds time_rounds() runs (HIP events on that stream)."""
    global LAST_ROUNDS, LAST_ROUND_STEPS
    t, LAST_ROUNDS, LAST_ROUND_STEPS = time_rounds(torch, fn, n_warm, n_timed)
    return t


MIN_TIMED_SECONDS = 0.030
MIN_ROUND_SECONDS = 0.005


def time_rounds(torch, fn, n_warm, n_timed, min_seconds=MIN_TIMED_SECONDS, max_rounds=200):
    """Rounds of a whole multiple of n_timed iterations each, after n_warm untimed ones.  A pilot round
    of n_timed iterations sizes the measurement: a round is the smallest multiple of n_timed iterations
    that lasts MIN_ROUND_SECONDS (the event between two rounds costs the launch stream a few
    microseconds, 1 % of a round of 1 ms), and enough rounds for min_seconds in total (at least 3) are
    enqueued back to back with an event between two rounds and no host synchronisation before the last
    one, so that no round starts on an idle device.  Returns (median seconds per n_timed iterations,
    rounds, iterations per round)."""
    it = 0

    def run(k):
        nonlocal it
        for _ in range(k):
            fn(it)
            it += 1

    run(n_warm)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    run(n_timed)
    b.record()
    torch.cuda.synchronize()
    pilot = max(a.elapsed_time(b) * 1e-3, 1e-7)
    mult = int(max(1, -(-MIN_ROUND_SECONDS // pilot)))
    n = int(min(max_rounds, max(3, -(-min_seconds // (pilot * mult)))))
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
    marks[0].record()
    for r in range(n):
        run(n_timed * mult)
        marks[r + 1].record()
    torch.cuda.synchronize()
    rounds = sorted(marks[r].elapsed_time(marks[r + 1]) * 1e-3 for r in range(n))
    return rounds[n // 2] / mult, n, n_timed * mult


def time_multi_stream(torch, launch, n_warm, n_timed, n_streams=3):
    """launch(i, stream_ptr) enqueues the independent item i on the given stream.  Items go to
    n_streams streams in turn, so the tail of one kernel overlaps the start of the next; returns
    seconds per item between two events on torch's current stream that enclose all of them."""
    main = torch.cuda.current_stream()
    streams = [torch.cuda.Stream() for _ in range(n_streams)]     # default priority
    ptrs = [int(st.cuda_stream) for st in streams]

    def burst(first, count):
        start = torch.cuda.Event(enable_timing=True)
        stop = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        start.record(main)
        for st in streams:
            st.wait_stream(main)
        for i in range(first, first + count):
            launch(i, ptrs[i % n_streams])
        for st in streams:
            main.wait_stream(st)
        stop.record(main)
        torch.cuda.synchronize()
        return start.elapsed_time(stop) * 1e-3 / count

    burst(0, n_warm)
    return burst(n_warm, n_timed)


def time_single_op(torch, op, stream_ptr, n_warm, n_timed):
    copies = len(op.handles) if hasattr(op, "handles") else len(op.W)

    def fn(i):
        st = op.launch(i % copies, stream_ptr)
        if st != 0:
            raise RuntimeError(f"launch failed with status {st}")
    return time_region(torch, fn, n_warm, n_timed) / n_timed


# Secondary measurements (sweep, shapes, widths, small batch, stress matrices): the paper's protocol of
# 100 warm-up and 1000 timed launches (Section 5.1).  Short regions read up to 8 % slow: the
# clocks need tens of milliseconds of load to settle after the set-up work in between.
SIDE_WARM, SIDE_TIMED = 100, 1000
STACK_WARM, STACK_TIMED = 10, 40      # passes over the 32-layer stack (2-4 ms each)


def copies_for(nbytes, total=2 << 30):
    """Enough copies that consecutive uses of one copy are separated by more than
    the last-level cache, within a bounded footprint."""
    return max(2, min(64, -(-total // max(nbytes, 1))))


def cpu_baseline(oracle, cases, min_cpu_seconds=10.0):
    """The oracle's SpMV (fp64, from the format buffers) timed on the host."""
    encs = [(oracle.encode(c.W), c.x) for c in cases]
    threads = oracle.max_threads()
    # one thread, smallest matrix only (a bounded sample: about a second)
    e0, x0 = min(encs, key=lambda ex: ex[0].total_bytes)
    oracle.set_threads(1)
    oracle.spmv(e0, x0)
    t1 = float("inf")
    for _ in range(3):
        ta = time.perf_counter()
        oracle.spmv(e0, x0)
        t1 = min(t1, time.perf_counter() - ta)
    oracle.set_threads(threads)
    one_thread = {"GBps": round((e0.total_bytes + 2 * e0.cols + 2 * e0.rows) / t1 / 1e9, 3),
                  "us": round(t1 * 1e6, 1), "matrix": f"{e0.rows}x{e0.cols}"}
    nbytes = sum(e.total_bytes + 2 * e.cols + 2 * e.rows for e, _ in encs)
    for e, x in encs:          # warm-up
        oracle.spmv(e, x)
    passes, t0 = 0, time.perf_counter()
    best = float("inf")
    while True:
        t1 = time.perf_counter()
        for e, x in encs:
            oracle.spmv(e, x)
        best = min(best, time.perf_counter() - t1)
        passes += 1
        if (time.perf_counter() - t0) * threads >= min_cpu_seconds or passes >= 50:
            break
    # the oracle's dense product by definition (fp64, O(rows x cols)): the parity reference, timed once per matrix
    dense_us = {}
    for c in cases:
        td = time.perf_counter()
        oracle.dense_matvec(c.W, c.x)
        dense_us[f"{c.rows}x{c.cols}"] = round((time.perf_counter() - td) * 1e6, 1)
    return {
        "value": nbytes / best / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
        "dense_matvec_by_definition_us": dense_us,
        "sample": f"one pass over the {len(encs)} distinct layer matrices "
                  f"({nbytes / 1e6:.1f} MB of format+x+y), best of {passes} passes, OpenMP over rows",
        "us_per_pass": best * 1e6,
        "one_thread": one_thread,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--no-sweep", action="store_true", help="skip the 36864x12288 sparsity sweep (configs[2])")
    ap.add_argument("--no-stack", action="store_true", help="skip the Llama2-13B-shaped 32-layer stack (configs[4])")
    ap.add_argument("--no-spmm", action="store_true", help="skip the small-batch product macko_spmm")
    ap.add_argument("--no-verify", action="store_true",
                    help="do not compare y of every timed configuration with the CPU oracle before timing it")
    ap.add_argument("--sweep", action="store_true", help=argparse.SUPPRESS)     # on by default now
    ap.add_argument("--stack", action="store_true", help=argparse.SUPPRESS)
    ap.add_argument("--spmm", action="store_true", help=argparse.SUPPRESS)
    ap.add_argument("--shapes", action="store_true",
                    help="also time every shape of the paper's Appendix D (see --shapes-sparsity)")
    ap.add_argument("--shapes-sparsity", default="50", metavar="LIST",
                    help="sparsity levels in per cent for --shapes, comma separated (default 50)")
    ap.add_argument("--adversarial", action="store_true",
                    help="also time the two 8192x8192 padding stress matrices (configs[3])")
    ap.add_argument("--widths", action="store_true",
                    help="also time 2-, 4- and 8-bit codes on the 36864x12288 matrix (Appendix C of the paper)")
    ap.add_argument("--fp8", action="store_true", help="also time the layer step with 8-bit (E4M3) values")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--probe", action="store_true",
                    help="counter probe for rocprofv3 --pmc: a 1 GiB device copy of known size, then a "
                         "few cold launches of every kernel of the step; prints no JSON line")
    ap.add_argument("--probe-sweep", type=int, default=None, metavar="S",
                    help="counter probe: a few cold launches on the 36864x12288 matrix at S %% sparsity; no JSON line")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the path has no multi-GPU part); use --gpus 1")
    args.sweep, args.stack, args.spmm = not args.no_sweep, not args.no_stack, not args.no_spmm

    import torch
    import oracle
    import workloads as wl
    import paper_2511_13061_amd as M

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    M.load_library()
    verified = []

    def verify(y_dev, case, what):
        """y of a configuration that is about to be timed, against the oracle's dense product (fp64, by
        definition), with the acceptance bound |y - y64| <= 1e-2 * sum_j |w_ij x_j| + 1e-3."""
        if args.no_verify:
            return
        torch.cuda.synchronize()
        y64, s64 = oracle.dense_matvec(case.W, case.x)
        y = y_dev.float().cpu().numpy().astype(np.float64)
        bad = ~(np.abs(y - y64) <= 1e-2 * s64 + 1e-3)
        if bad.any():
            raise SystemExit(f"bench.py: {what}: {int(bad.sum())} rows of y are outside the tolerance; not timing it")
        verified.append(what)
    torch.cuda.set_device(0)
    stream_ptr = int(torch.cuda.current_stream().cuda_stream)
    props = torch.cuda.get_device_properties(0)
    log(f"device: {props.name}, {props.multi_processor_count} CUs, {props.total_memory / 2**30:.0f} GiB")

    if args.probe_sweep is not None:
        case = wl.config3(args.probe_sweep)
        nb = int(2.5 * case.rows * case.cols * (1 - args.probe_sweep / 100.0))
        nc = copies_for(nb, 1 << 30)                    # rotate over >= 1 GiB so that no launch finds its matrix cached
        so = SparseOp(M, torch, case, copies=nc)
        do = DenseOp(M, torch, case, copies=2)
        ts = time_single_op(torch, so, stream_ptr, nc, 4 * nc)
        td = time_single_op(torch, do, stream_ptr, 2, 8)
        log(f"probe-sweep {args.probe_sweep}%: spmv {ts * 1e6:.1f} us ({5 * nc} launches over {nc} copies, "
            f"{so.bytes} bytes each), dense gemv {td * 1e6:.1f} us (10 launches)")
        print(json.dumps({"probe_sweep": args.probe_sweep, "spmv_us": round(ts * 1e6, 2), "spmv_bytes": int(so.bytes),
                          "spmv_launches": 5 * nc, "gemv_us": round(td * 1e6, 2), "gemv_bytes": int(do.bytes)}))
        return

    # ---- workload: one Llama2-7B-shaped layer at 50 % ------------------------
    t0 = time.perf_counter()
    cases = list(wl.config2())
    layer_plan = [("qkvo", 4), ("gate_up", 2), ("down", 1)]
    layer_macko_bytes = 0
    n_layers = 8
    sparse_ops, dense_ops = {}, {}
    for case, (tag, mult) in zip(cases, layer_plan):
        sparse_ops[tag] = SparseOp(M, torch, case, copies=mult * n_layers)
        dense_ops[tag] = DenseOp(M, torch, case, copies=mult * n_layers)
        layer_macko_bytes += mult * sparse_ops[tag].bytes
    layer_dense_bytes = sum(mult * dense_ops[tag].bytes for tag, mult in layer_plan)
    for case, (tag, mult) in zip(cases, layer_plan):       # first (host-encoded) and last (GPU-encoded) copy, and the baseline
        for copy in (0, mult * n_layers - 1):
            sparse_ops[tag].launch(copy, stream_ptr)
            verify(sparse_ops[tag].y, case, f"{case.name} copy {copy}")
        dense_ops[tag].launch(0, stream_ptr)
        verify(dense_ops[tag].y, case, f"{case.name} dense gemv")
    log(f"setup {time.perf_counter() - t0:.1f}s: layer = {layer_macko_bytes / 1e6:.1f} MB MACKO, "
        f"{layer_dense_bytes / 1e6:.1f} MB dense, {n_layers} copies")

    def make_step(ops):
        def step(i):
            layer = i % n_layers
            for tag, mult in layer_plan:
                op = ops[tag]
                for k in range(mult):
                    st = op.launch(layer * mult + k, stream_ptr)
                    if st != 0:
                        raise RuntimeError(f"launch failed with status {st}")
        return step

    torch.cuda.synchronize()

    # ---- the same layer with grouped launches in dependency order --------------
    # {q,k,v} -> {o} -> {gate,up} -> {down}: products that do not depend on each other share a launch
    def grouped_steps(kind, ops=None):
        steps = []
        for layer in range(n_layers):
            def pick(tag, ks):
                op = (ops if ops is not None else sparse_ops if kind == "sparse" else dense_ops)[tag]
                mult = dict(layer_plan)[tag]
                if kind == "sparse":
                    return [op.handles[layer * mult + k] for k in ks], [op.x] * len(ks), \
                           [torch.empty_like(op.y) for _ in ks]
                return [op.W[layer * mult + k] for k in ks], [op.x] * len(ks), [torch.empty_like(op.y) for _ in ks]
            Group = M.SpmvGroup if kind == "sparse" else M.GemvGroup
            steps.append([Group(*pick("qkvo", [0, 1, 2])), Group(*pick("qkvo", [3])),
                          Group(*pick("gate_up", [0, 1])), Group(*pick("down", [0]))])
        return steps

    def make_grouped_step(steps):
        def step(i):
            for g in steps[i % n_layers]:
                st = g.launch_raw(stream_ptr)
                if st != 0:
                    raise RuntimeError(f"grouped launch failed with status {st}")
        return step

    gs, gd = grouped_steps("sparse"), grouped_steps("dense")
    if args.probe:
        # known traffic for scaling the counters: 1 GiB read + 1 GiB written per copy
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        for i in range(2 * n_layers):
            make_grouped_step(gs)(i)
            make_grouped_step(gd)(i)
        torch.cuda.synchronize()
        log("probe done: 3 copies of 1 GiB, then", 2 * n_layers, "sparse and dense steps (4 grouped launches each)")
        return

    # the timed region: K steps of 4 grouped launches each
    t_sparse = time_region(torch, make_grouped_step(gs), args.warmup, args.steps)
    t_dense = time_region(torch, make_grouped_step(gd), args.warmup, args.steps)
    launches_per_step = 4
    ms_per_step = t_sparse / args.steps * 1e3
    gbps = layer_macko_bytes / (t_sparse / args.steps) / 1e9
    dense_gbps = layer_dense_bytes / (t_dense / args.steps) / 1e9
    log(f"layer, 4 grouped launches: MACKO {ms_per_step * 1e3:.1f} us/step ({gbps:.0f} GB/s), dense "
        f"{t_dense / args.steps * 1e6:.1f} us/step ({dense_gbps:.0f} GB/s), speedup {t_dense / t_sparse:.3f}")
    headline_rounds, headline_round_steps = LAST_ROUNDS, LAST_ROUND_STEPS
    # every grouped launch of layer 0 must give what the single launches gave (same arithmetic per row)
    if not args.no_verify:
        for g in gs[0]:
            g.launch_raw(stream_ptr)
        torch.cuda.synchronize()
        for g in gs[0]:
            for m, yv in zip(g._keep[0], g._keep[2]):
                tag = next(t for t in sparse_ops if m in sparse_ops[t].handles)
                sparse_ops[tag].launch(0, stream_ptr)
                torch.cuda.synchronize()
                if not torch.equal(yv, sparse_ops[tag].y):
                    raise SystemExit("bench.py: a grouped launch disagrees with the single launch of the same product")
        verified.append("grouped launches of layer 0 == single launches, bit for bit")

    # the same step as ONE launch that honours the dependences (macko_spmv_chain_static: the four phases
    # wait for each other inside the kernel); reported beside `value`, which stays on the four launches
    chain_steps = []
    for layer in range(n_layers):
        phases = [[(m, xv, yv) for m, xv, yv in zip(*g._keep)] for g in gs[layer]]
        chain_steps.append(M.SpmvChain(phases))

    def chain_step(i):
        st = chain_steps[i % n_layers].launch_raw(stream_ptr)
        if st != 0:
            raise RuntimeError(f"chain launch failed with status {st}")
    t_chain = time_region(torch, chain_step, args.warmup, args.steps)
    if M.chain_status(None)[0] != 0:
        raise SystemExit("bench.py: a chain gave up waiting during the timed region")
    chain = {"launches_per_step": 1, "macko_ms_per_step": round(t_chain / args.steps * 1e3, 5),
             "macko_GBps": round(layer_macko_bytes / (t_chain / args.steps) / 1e9, 1),
             "macko_frac_of_hbm_peak": round(layer_macko_bytes / (t_chain / args.steps) / 1e9 / HBM_PEAK_GBPS, 4),
             "speedup_vs_dense_gemv": round(t_dense / t_chain, 3)}
    log(f"layer, one launch with the dependences honoured inside (macko_spmv_chain_static): {chain}")
    del chain_steps
    del gs, gd

    # the same seven products as seven separate launches (macko_spmv / macko_dense_gemv)
    t1_sparse = time_region(torch, make_step(sparse_ops), args.warmup, args.steps)
    t1_dense = time_region(torch, make_step(dense_ops), args.warmup, args.steps)
    single = {
        "launches_per_step": 7,
        "macko_ms_per_step": round(t1_sparse / args.steps * 1e3, 5),
        "dense_ms_per_step": round(t1_dense / args.steps * 1e3, 5),
        "macko_GBps": round(layer_macko_bytes / (t1_sparse / args.steps) / 1e9, 1),
        "dense_GBps": round(layer_dense_bytes / (t1_dense / args.steps) / 1e9, 1),
        "speedup_vs_dense_gemv": round(t1_dense / t1_sparse, 3),
    }
    log(f"layer, 7 separate launches: {single}")

    # and as ONE grouped launch: in this benchmark the seven products share no data, so nothing
    # but the decoder's own dependences (which `value` honours) forbids it
    def one_launch_steps(kind):
        steps = []
        for layer in range(n_layers):
            mats, xs, ys = [], [], []
            for tag, mult in layer_plan:
                op = (sparse_ops if kind == "sparse" else dense_ops)[tag]
                for k in range(mult):
                    mats.append((op.handles if kind == "sparse" else op.W)[layer * mult + k])
                    xs.append(op.x)
                    ys.append(torch.empty_like(op.y))
            steps.append([(M.SpmvGroup if kind == "sparse" else M.GemvGroup)(mats, xs, ys)])
        return steps
    g1s, g1d = one_launch_steps("sparse"), one_launch_steps("dense")
    t7_sparse = time_region(torch, make_grouped_step(g1s), args.warmup, args.steps)
    t7_dense = time_region(torch, make_grouped_step(g1d), args.warmup, args.steps)
    one_launch = {
        "launches_per_step": 1,
        "macko_ms_per_step": round(t7_sparse / args.steps * 1e3, 5),
        "dense_ms_per_step": round(t7_dense / args.steps * 1e3, 5),
        "macko_GBps": round(layer_macko_bytes / (t7_sparse / args.steps) / 1e9, 1),
        "dense_GBps": round(layer_dense_bytes / (t7_dense / args.steps) / 1e9, 1),
        "macko_frac_of_hbm_peak": round(layer_macko_bytes / (t7_sparse / args.steps) / 1e9 / HBM_PEAK_GBPS, 4),
        "speedup_vs_dense_gemv": round(t7_dense / t7_sparse, 3),
    }
    log(f"layer, all 7 products in 1 launch (ignores the decoder's dependences): {one_launch}")
    del g1s, g1d

    # the same four grouped launches with 2-bit codes (Appendix C: the smaller encoding up to
    # about 50 % sparsity); `value` stays on the paper's default of 4 bits
    sparse2 = {tag: SparseOp(M, torch, case, copies=mult * n_layers, b_delta=2)
               for case, (tag, mult) in zip(cases, layer_plan)}
    gs2 = grouped_steps("sparse", sparse2)
    t2 = time_region(torch, make_grouped_step(gs2), args.warmup, args.steps)
    bytes2 = sum(mult * sparse2[tag].bytes for tag, mult in layer_plan)
    two_bit = {
        "ms_per_step": round(t2 / args.steps * 1e3, 5), "bytes_per_step": bytes2,
        "GBps": round(bytes2 / (t2 / args.steps) / 1e9, 1),
        "frac_of_hbm_peak": round(bytes2 / (t2 / args.steps) / 1e9 / HBM_PEAK_GBPS, 4),
        "speedup_vs_dense_gemv": round(t_dense / t2, 3),
        "memory_reduction_vs_dense": round(layer_dense_bytes / bytes2, 3),
        "padding_per_nnz": round(sparse2["qkvo"].report.padding_entries / sparse2["qkvo"].report.nnz, 4),
    }
    log(f"layer, 4 grouped launches, 2-bit codes: {two_bit}")
    del gs2, sparse2
    torch.cuda.empty_cache()

    # the same layer with 8-bit values (OCP E4M3; the paper leaves 8-bit values to future work):
    # 1 byte of value + half a byte of code per stored entry.  Not `value`; no dense 8-bit baseline is built.
    fp8 = None
    if args.fp8:
        class Fp8Op:
            def __init__(self, case, copies):
                W8 = wl.fp8_values_of(case.W)
                W8d = torch.from_numpy(W8).cuda()
                self.handles = [M.encode_fp8(W8).to_device()] + [M.encode_device_fp8(W8d) for _ in range(copies - 1)]
                del W8d
                self.report = self.handles[0].report
                self.x = torch.from_numpy(case.x.view(np.float16)).cuda()
                self.y = torch.empty(case.rows, dtype=torch.float16, device="cuda")
                self.bytes = spmv_bytes(self.report)
        ops8 = {tag: Fp8Op(case, mult * n_layers) for case, (tag, mult) in zip(cases, layer_plan)}
        gs8 = grouped_steps("sparse", ops8)
        t8 = time_region(torch, make_grouped_step(gs8), args.warmup, args.steps)
        bytes8 = sum(mult * ops8[tag].bytes for tag, mult in layer_plan)
        fp8 = {
            "ms_per_step": round(t8 / args.steps * 1e3, 5), "bytes_per_step": bytes8,
            "GBps": round(bytes8 / (t8 / args.steps) / 1e9, 1),
            "frac_of_hbm_peak": round(bytes8 / (t8 / args.steps) / 1e9 / HBM_PEAK_GBPS, 4),
            "speedup_vs_dense_fp16_gemv": round(t_dense / t8, 3),
            "speedup_vs_16_bit_values": round(t_sparse / t8, 3),
            "memory_reduction_vs_dense_fp16": round(layer_dense_bytes / bytes8, 3),
            "effd_vs_dense_8_bit": round(ops8["qkvo"].report.effd, 4),
            "values": "OCP E4M3, the 16-bit layer times 32 rounded by the framework's conversion",
        }
        log(f"layer, 4 grouped launches, 8-bit values: {fp8}")
        del gs8, ops8
        torch.cuda.empty_cache()

    # ---- per-shape numbers (cold rotation over the same copies) ---------------
    per_shape = {}
    n_single = max(50, args.steps // 2)
    for tag, _ in layer_plan:
        so, do = sparse_ops[tag], dense_ops[tag]
        ts = time_single_op(torch, so, stream_ptr, max(10, args.warmup // 2), n_single)
        td = time_single_op(torch, do, stream_ptr, max(10, args.warmup // 2), n_single)
        # the same launch on ONE copy over and over: the matrix stays in the 256 MB last-level cache
        tsw = time_region(torch, lambda i: so.launch(0, stream_ptr), 10, n_single) / n_single
        tdw = time_region(torch, lambda i: do.launch(0, stream_ptr), 10, n_single) / n_single
        # context for the baseline: the vendor library's GEMV on the same dense matrices (torch.mv)
        ncop = len(do.W)
        tlib = time_region(torch, lambda i: torch.mv(do.W[i % ncop], do.x, out=do.y), 10, n_single) / n_single
        per_shape[f"{so.rows}x{so.cols}"] = {
            "macko_us": round(ts * 1e6, 2), "dense_us": round(td * 1e6, 2),
            "warm_cache_macko_us": round(tsw * 1e6, 2), "warm_cache_dense_us": round(tdw * 1e6, 2),
            "library_gemv_us": round(tlib * 1e6, 2),
            "macko_GBps": round(so.bytes / ts / 1e9, 1), "dense_GBps": round(do.bytes / td / 1e9, 1),
            "speedup_vs_dense": round(td / ts, 3),
            "memory_reduction": round(so.report.dense_bytes / so.report.total_bytes, 3),
            "effd": round(so.report.effd, 4), "padding_entries": so.report.padding_entries,
        }
        log(f"  {tag}: {per_shape[f'{so.rows}x{so.cols}']}")

    # dominant kernel of the step: the wave-per-row SpMV kernel (all four grouped launches)
    avg_launch_s = t_sparse / (args.steps * launches_per_step)
    avg_launch_bytes = layer_macko_bytes / launches_per_step
    # HBM traffic per launch is not measured by this run: it comes from two rocprofv3 --pmc runs of this
    # same command (FETCH_SIZE, WRITE_SIZE), whose summary is kept in the file named beside it
    traffic = None
    traffic_file = "profiles/spmv_wave_row_kernel_llama2_7b_layer_hbm_traffic.txt"
    tpath = os.path.join(ROOT, traffic_file)
    if os.path.exists(tpath):
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = int(float(line.split(":")[1]))
    roofline = {
        "bound": "hbm", "kernel": "spmv_wave_row_kernel",
        "achieved": round(avg_launch_bytes / avg_launch_s / 1e9, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": round(avg_launch_bytes / avg_launch_s / 1e9 / HBM_PEAK_GBPS, 4),
        "avg_launch_us": round(avg_launch_s * 1e6, 3), "bytes_per_launch": int(avg_launch_bytes),
        "traffic": traffic,
        "traffic_from_profile": traffic_file if traffic is not None else None,
    }

    extra = {}

    # ---- dense -> MACKO conversion (done once per matrix, outside the timed region) ----
    enc = {}
    for case, (tag, _) in zip(cases, layer_plan):
        Wd = dense_ops[tag].W[0]
        t_h0 = time.perf_counter()
        h = M.encode(case.W)
        t_host = time.perf_counter() - t_h0
        h.destroy()
        M.encode_device(Wd).destroy()
        torch.cuda.synchronize()
        t_g0 = time.perf_counter()
        for _ in range(5):
            M.encode_device(Wd).destroy()
        torch.cuda.synchronize()
        t_gpu = (time.perf_counter() - t_g0) / 5
        # bytes the GPU encoder moves: the dense matrix twice (count, fill), values + one code byte
        # per entry written, the code bytes read again and packed, counts and row pointers
        rep_e = sparse_ops[tag].report
        n_e = rep_e.alloc_nnz
        enc_bytes = 2 * case.W.nbytes + 3 * n_e + n_e + n_e // 2 + 16 * case.rows
        # and back: the dense matrix from the format on the device (rows assembled in LDS, written once);
        # handles and outputs rotate so that neither is found in the last-level cache
        hs = sparse_ops[tag].handles
        backs = [torch.empty_like(Wd) for _ in range(len(hs))]
        hs[0].decode_device(backs[0])
        t_dec = time_region(torch, lambda i: hs[i % len(hs)].decode_device(backs[i % len(hs)]), 20, 200) / 200
        dec_bytes = case.W.nbytes + 2 * n_e + n_e // 2 + 4 * case.rows
        back = backs[0]
        del backs
        del back
        enc[f"{case.rows}x{case.cols}"] = {
            "decode_gpu_ms": round(t_dec * 1e3, 3), "decode_gpu_traffic_GBps": round(dec_bytes / t_dec / 1e9, 1),
            "host_ms": round(t_host * 1e3, 2), "gpu_ms": round(t_gpu * 1e3, 3),
            "gpu_dense_input_GBps": round(case.W.nbytes / t_gpu / 1e9, 1),
            "gpu_traffic_GBps": round(enc_bytes / t_gpu / 1e9, 1),
            "gpu_frac_of_hbm_peak": round(enc_bytes / t_gpu / 1e9 / HBM_PEAK_GBPS, 4),
        }
    extra["encode"] = enc
    log(f"encode: {enc}")
    del dense_ops
    torch.cuda.empty_cache()

    # ---- optional: sparsity sweep on 36864 x 12288 ---------------------------
    if args.sweep:
        sweep = {}
        dense_t = None
        for s in wl.SWEEP_SPARSITIES:
            case = wl.config3(s)
            # rotate over >= 1 GiB of copies: two copies of the 90 % matrix (278 MB) would half fit the 256 MB cache
            nc = copies_for(int(2.5 * case.rows * case.cols * (1 - s / 100.0)), 1 << 30)
            so = SparseOp(M, torch, case, copies=nc)
            for copy in (0, nc - 1):
                so.launch(copy, stream_ptr)
                verify(so.y, case, f"{case.name} copy {copy}")
            ts = time_single_op(torch, so, stream_ptr, max(SIDE_WARM, nc), SIDE_TIMED)
            row = {"bytes": int(so.bytes), "us": round(ts * 1e6, 1), "GBps": round(so.bytes / ts / 1e9, 1),
                   "frac_of_hbm_peak": round(so.bytes / ts / 1e9 / HBM_PEAK_GBPS, 4),
                   "copies_rotated": nc,
                   "memory_reduction": round(so.report.dense_bytes / so.report.total_bytes, 3),
                   "effd": round(so.report.effd, 4), "padding_entries": so.report.padding_entries}
            # the same launches dealt to three streams in turn (independent products overlap at the seams)
            def launch3(i, sp, so=so, nc=nc):
                st = so.handles[i % nc].spmv_raw(so.x.data_ptr(), so.y.data_ptr(), sp)
                if st != 0:
                    raise RuntimeError(f"launch failed with status {st}")
            t3 = time_multi_stream(torch, launch3, max(SIDE_WARM, nc), SIDE_TIMED)
            row["three_streams_us"] = round(t3 * 1e6, 1)
            row["three_streams_frac_of_hbm_peak"] = round(so.bytes / t3 / 1e9 / HBM_PEAK_GBPS, 4)
            if s == 0:
                do = DenseOp(M, torch, case, copies=2)
                do.launch(0, stream_ptr)
                verify(do.y, case, f"{case.name} dense gemv")
                dense_t = time_single_op(torch, do, stream_ptr, SIDE_WARM, SIDE_TIMED)
                row["dense_us"] = round(dense_t * 1e6, 1)
                row["dense_GBps"] = round(do.bytes / dense_t / 1e9, 1)
                del do
            row["speedup_vs_dense"] = round(dense_t / ts, 3)
            sweep[str(s)] = row
            log(f"  sweep {s}%: {row}")
            del so, case
            torch.cuda.empty_cache()
        extra["sweep_36864x12288"] = sweep

    # ---- optional: padding stress (configs[3]) ------------------------------------
    if args.adversarial:
        table = {}
        for case in (wl.config4(), wl.config4b()):
            so = SparseOp(M, torch, case, copies=12)
            do = DenseOp(M, torch, case, copies=8)
            ts = time_single_op(torch, so, stream_ptr, SIDE_WARM, SIDE_TIMED)
            td = time_single_op(torch, do, stream_ptr, SIDE_WARM, SIDE_TIMED)
            rep = so.report
            table[case.name] = {
                "macko_us": round(ts * 1e6, 1), "dense_us": round(td * 1e6, 1),
                "macko_GBps": round(so.bytes / ts / 1e9), "speedup_vs_dense": round(td / ts, 3),
                "sparsity": round(1.0 - rep.density, 4), "effd": round(rep.effd, 4),
                "effd_worst_case_eq9": round(rep.effd_worst, 4),
                "padding_per_nnz": round(rep.padding_entries / max(rep.nnz, 1), 4),
                "max_row_entries": rep.max_row_entries, "empty_rows": rep.empty_rows,
            }
            log(f"  adversarial {case.name}: {table[case.name]}")
            del so, do
            torch.cuda.empty_cache()
        extra["adversarial_8192x8192"] = table

    # ---- optional: other code widths (Appendix C) on the sweep matrix ---------------
    if args.widths:
        table = {}
        for s in (10, 25, 40, 50, 70, 90, 97):
            W = wl.bernoulli(36864, 12288, 1.0 - s / 100.0, 0.02, wl.BASE_SEED, 300 + s)
            Wd = torch.from_numpy(W.view(np.float16)).cuda()
            x = torch.from_numpy(wl.x_vector(12288).view(np.float16)).cuda()
            y = torch.empty(36864, dtype=torch.float16, device="cuda")
            row = {}
            for b in (1, 2, 4, 8):
                if b == 1 and s > 50:
                    continue                      # 1-bit codes pad every gap above 2: pointless on sparse rows
                ms = [M.encode_device(Wd, b_delta=b)]
                rep = ms[0].get_report()
                nc = copies_for(spmv_bytes(rep), 1 << 30)                    # rotate over >= 1 GiB of copies
                ms += [M.encode_device(Wd, b_delta=b) for _ in range(nc - 1)]

                def f(i):
                    st = ms[i % nc].spmv_raw(x.data_ptr(), y.data_ptr(), stream_ptr)
                    if st != 0:
                        raise RuntimeError(f"macko_spmv failed with status {st}")
                t = time_region(torch, f, max(SIDE_WARM, nc), SIDE_TIMED) / SIDE_TIMED
                row[f"b_delta_{b}"] = {"macko_us": round(t * 1e6, 1), "GBps": round(spmv_bytes(rep) / t / 1e9),
                                       "effd": round(rep.effd, 4),
                                       "padding_per_nnz": round(rep.padding_entries / max(rep.nnz, 1), 4)}
                del ms
            table[f"sparsity_{s}"] = row
            log(f"  widths {s}%: {row}")
            del Wd
            torch.cuda.empty_cache()
        extra["code_widths_36864x12288"] = table

    # ---- optional: small-batch products (batch 1..8) on the layer's shapes --------
    if args.spmm:
        lib = M.load_library()
        table = {}
        for case, (tag, _) in zip(cases, layer_plan):
            so = sparse_ops[tag]
            copies = len(so.handles)
            Wd = [torch.from_numpy(case.W.view(np.float16)).cuda() for _ in range(8)]
            row = {}
            for B in (1, 2, 4, 8):
                X = torch.randn(B, case.cols, device="cuda", dtype=torch.float16)
                Y = torch.empty(B, case.rows, device="cuda", dtype=torch.float16)

                def f(i):
                    st = lib.macko_spmm(so.handles[i % copies]._h, B, X.data_ptr(), X.stride(0), Y.data_ptr(),
                                        Y.stride(0), stream_ptr)
                    if st != 0:
                        raise RuntimeError(f"macko_spmm failed with status {st}")

                def g(i):
                    torch.matmul(X, Wd[i % 8].t(), out=Y)          # library GEMM on the dense matrix

                ts = time_region(torch, f, SIDE_WARM, SIDE_TIMED) / SIDE_TIMED
                td = time_region(torch, g, SIDE_WARM, SIDE_TIMED) / SIDE_TIMED
                row[f"batch{B}"] = {"macko_us": round(ts * 1e6, 2), "dense_library_gemm_us": round(td * 1e6, 2),
                                    "format_GBps": round(so.bytes / ts / 1e9)}
            # the same with 8-bit (E4M3) values: 1.5 bytes per stored entry, the same batch kernel
            W8 = wl.fp8_values_of(case.W)
            W8d = torch.from_numpy(W8).cuda()
            h8 = [M.encode_fp8(W8).to_device()] + [M.encode_device_fp8(W8d) for _ in range(7)]
            del W8d
            for B in (1, 8):
                X = torch.randn(B, case.cols, device="cuda", dtype=torch.float16)
                Y = torch.empty(B, case.rows, device="cuda", dtype=torch.float16)

                def f8(i):
                    st = lib.macko_spmm(h8[i % 8]._h, B, X.data_ptr(), X.stride(0), Y.data_ptr(), Y.stride(0), stream_ptr)
                    if st != 0:
                        raise RuntimeError(f"macko_spmm failed with status {st}")
                t8 = time_region(torch, f8, SIDE_WARM, SIDE_TIMED) / SIDE_TIMED
                row[f"batch{B}"]["macko_8_bit_values_us"] = round(t8 * 1e6, 2)
            del h8
            table[f"{case.rows}x{case.cols}"] = row
            log(f"  spmm {case.rows}x{case.cols}: {row}")
            del Wd
        extra["spmm_small_batch"] = table

    # ---- optional: every shape of Appendix D, at 50 % and at the other levels asked for ----
    if args.shapes:
        levels = sorted({int(v) for v in args.shapes_sparsity.split(",") if v.strip()})
        for pct in levels:
            table = {}
            for (r, c) in wl.APPENDIX_D_SHAPES:
                case = wl.appendix_d_case(r, c, pct)
                nb = int(2.5 * r * c * (1 - pct / 100.0))
                so = SparseOp(M, torch, case, copies=copies_for(nb, 1 << 30))
                do = DenseOp(M, torch, case, copies=copies_for(2 * r * c, 1 << 30))
                ts = time_single_op(torch, so, stream_ptr, SIDE_WARM, SIDE_TIMED)
                td = time_single_op(torch, do, stream_ptr, SIDE_WARM, SIDE_TIMED)
                table[f"{r}x{c}"] = {"macko_us": round(ts * 1e6, 1), "dense_us": round(td * 1e6, 1),
                                     "macko_GBps": round(so.bytes / ts / 1e9), "dense_GBps": round(do.bytes / td / 1e9),
                                     "speedup_vs_dense": round(td / ts, 3)}
                log(f"  appendix D {r}x{c} @ {pct} %: {table[f'{r}x{c}']}")
                del so, do, case
                torch.cuda.empty_cache()
            sp = sorted(v["speedup_vs_dense"] for v in table.values())
            extra[f"appendix_d_shapes_s{pct}"] = {"shapes": table, "speedup_min": sp[0],
                                                   "speedup_median": sp[len(sp) // 2], "speedup_max": sp[-1]}
            log(f"  appendix D @ {pct} %: speedup min {sp[0]} median {sp[len(sp) // 2]} max {sp[-1]}")

    # ---- optional: Llama2-13B-shaped 32-layer stack ---------------------------
    if args.stack:
        plan13 = [("qkvo", 4), ("gate_up", 2), ("down", 1)]
        ops13 = {}
        dops13 = {}
        cases13 = list(wl.config5_layer())
        for case, (tag, mult) in zip(cases13, plan13):
            ops13[tag] = SparseOp(M, torch, case, copies=mult * 32)
            dops13[tag] = DenseOp(M, torch, case, copies=mult * 32)
            for copy in (0, mult * 32 - 1):
                ops13[tag].launch(copy, stream_ptr)
                verify(ops13[tag].y, case, f"{case.name} copy {copy}")
            dops13[tag].launch(0, stream_ptr)
            verify(dops13[tag].y, case, f"{case.name} dense gemv")
        def stack_pass(ops):
            def run(_i):
                for layer in range(32):
                    for tag, mult in plan13:
                        for k in range(mult):
                            ops[tag].launch(layer * mult + k, stream_ptr)
            return run

        def grouped_stack(kind):
            groups = []
            for layer in range(32):
                def pick(tag, ks):
                    op = (ops13 if kind == "sparse" else dops13)[tag]
                    mult = dict(plan13)[tag]
                    mats = [(op.handles if kind == "sparse" else op.W)[layer * mult + k] for k in ks]
                    return mats, [op.x] * len(ks), [torch.empty_like(op.y) for _ in ks]
                Group = M.SpmvGroup if kind == "sparse" else M.GemvGroup
                groups += [Group(*pick("qkvo", [0, 1, 2])), Group(*pick("qkvo", [3])),
                           Group(*pick("gate_up", [0, 1])), Group(*pick("down", [0]))]

            def run(_i):
                for g in groups:
                    g.launch_raw(stream_ptr)
            return run

        def layer_groups(kind):
            groups = []
            for layer in range(32):
                mats, xs, ys = [], [], []
                for tag, mult in plan13:
                    op = (ops13 if kind == "sparse" else dops13)[tag]
                    for k in range(mult):
                        mats.append((op.handles if kind == "sparse" else op.W)[layer * mult + k])
                        xs.append(op.x)
                        ys.append(torch.empty_like(op.y))
                groups.append((M.SpmvGroup if kind == "sparse" else M.GemvGroup)(mats, xs, ys))

            def run(_i):
                for g in groups:
                    g.launch_raw(stream_ptr)
            return run

        ts32 = time_region(torch, layer_groups("sparse"), STACK_WARM, STACK_TIMED) / STACK_TIMED
        td32 = time_region(torch, layer_groups("dense"), STACK_WARM, STACK_TIMED) / STACK_TIMED
        ts1 = time_region(torch, stack_pass(ops13), STACK_WARM, STACK_TIMED) / STACK_TIMED
        td1 = time_region(torch, stack_pass(dops13), STACK_WARM, STACK_TIMED) / STACK_TIMED
        ts = time_region(torch, grouped_stack("sparse"), STACK_WARM, STACK_TIMED) / STACK_TIMED
        td = time_region(torch, grouped_stack("dense"), STACK_WARM, STACK_TIMED) / STACK_TIMED
        # the same 128 grouped launches dealt to three streams in turn: the products of this workload are
        # independent, and kernels of different streams overlap (the next one starts on the compute units
        # the previous one has already left)
        def over_streams(kind):
            groups = []
            for layer in range(32):
                def pick(tag, ks):
                    op = (ops13 if kind == "sparse" else dops13)[tag]
                    mult = dict(plan13)[tag]
                    mats = [(op.handles if kind == "sparse" else op.W)[layer * mult + k] for k in ks]
                    return mats, [op.x] * len(ks), [torch.empty_like(op.y) for _ in ks]
                Group = M.SpmvGroup if kind == "sparse" else M.GemvGroup
                groups += [Group(*pick("qkvo", [0, 1, 2])), Group(*pick("qkvo", [3])),
                           Group(*pick("gate_up", [0, 1])), Group(*pick("down", [0]))]

            def launch(i, sp):
                st = groups[i % len(groups)].launch_raw(sp)
                if st != 0:
                    raise RuntimeError(f"grouped launch failed with status {st}")
            return launch
        def separate_over_streams(ops):
            seq = [(tag, layer * mult + k) for layer in range(32) for tag, mult in plan13 for k in range(mult)]

            def launch(i, sp):
                tag, copy = seq[i % len(seq)]
                st = ops[tag].launch(copy, sp)
                if st != 0:
                    raise RuntimeError(f"launch failed with status {st}")
            return launch
        # the whole stack in one library call (macko_spmv_many: groups of 8 over the library's three side streams)
        seq = [(tag, layer * mult + k) for layer in range(32) for tag, mult in plan13 for k in range(mult)]
        many = M.SpmvMany([ops13[t].handles[c] for t, c in seq], [ops13[t].x for t, _ in seq],
                          [torch.empty_like(ops13[t].y) for t, _ in seq])

        def many_pass(_i):
            st = many.launch_raw(stream_ptr)
            if st != 0:
                raise RuntimeError(f"macko_spmv_many failed with status {st}")
        many_pass(0)
        for case, (tag, mult) in zip(cases13, plan13):
            idx = [i for i, (t, _) in enumerate(seq) if t == tag]
            for i in (idx[0], idx[-1]):
                verify(many._keep[2][i], case, f"macko_spmv_many product {i} ({case.name})")
        tsm = time_region(torch, many_pass, STACK_WARM, STACK_TIMED) / STACK_TIMED
        del many
        ts224 = time_multi_stream(torch, separate_over_streams(ops13), STACK_WARM * 224, STACK_TIMED * 224) * 224
        td224 = time_multi_stream(torch, separate_over_streams(dops13), STACK_WARM * 224, STACK_TIMED * 224) * 224
        ts3 = time_multi_stream(torch, over_streams("sparse"), STACK_WARM * 128, STACK_TIMED * 128) * 128
        td3 = time_multi_stream(torch, over_streams("dense"), STACK_WARM * 128, STACK_TIMED * 128) * 128
        sb = 32 * sum(m * ops13[t].bytes for t, m in plan13)
        db = 32 * sum(m * dops13[t].bytes for t, m in plan13)
        stack_key = "stack_llama2_13b_32layers"
        extra[stack_key] = {
            "launches": 128, "macko_us": round(ts * 1e6, 1), "dense_us": round(td * 1e6, 1),
            "separate_launches_224": {"macko_us": round(ts1 * 1e6, 1), "dense_us": round(td1 * 1e6, 1)},
            "one_launch_per_layer_32": {"macko_us": round(ts32 * 1e6, 1), "dense_us": round(td32 * 1e6, 1),
                                        "macko_GBps": round(0 / 1e9, 1), "dense_GBps": round(0 / 1e9, 1)},
            "three_streams_128": {"macko_us": round(ts3 * 1e6, 1), "dense_us": round(td3 * 1e6, 1),
                                  "macko_GBps": round(sb / ts3 / 1e9, 1), "dense_GBps": round(db / td3 / 1e9, 1),
                                  "macko_frac_of_hbm_peak": round(sb / ts3 / 1e9 / HBM_PEAK_GBPS, 4),
                                  "speedup_vs_dense": round(td3 / ts3, 3)},
            "one_call_spmv_many_224": {"macko_us": round(tsm * 1e6, 1), "launches": 28,
                                       "bytes": int(sb), "us": round(tsm * 1e6, 1),
                                       "GBps": round(sb / tsm / 1e9, 1),
                                       "frac_of_hbm_peak": round(sb / tsm / 1e9 / HBM_PEAK_GBPS, 4),
                                       "speedup_vs_dense": round(td3 / tsm, 3),
                                       "dense_is": "the 128 grouped dense launches over three streams"},
            "three_streams_224_separate": {"macko_us": round(ts224 * 1e6, 1), "dense_us": round(td224 * 1e6, 1),
                                           "macko_frac_of_hbm_peak": round(sb / ts224 / 1e9 / HBM_PEAK_GBPS, 4),
                                           "speedup_vs_dense": round(td224 / ts224, 3)},
            "macko_GB": round(sb / 1e9, 3), "dense_GB": round(db / 1e9, 3),
            "bytes": int(sb), "us": round(ts * 1e6, 1), "GBps": round(sb / ts / 1e9, 1),
            "frac_of_hbm_peak": round(sb / ts / 1e9 / HBM_PEAK_GBPS, 4),
            "macko_GBps": round(sb / ts / 1e9, 1), "dense_GBps": round(db / td / 1e9, 1),
            "speedup_vs_dense": round(td / ts, 3),
            "note": "one layer's three distinct matrices, device buffers replicated to 32 layers at distinct addresses",
        }
        one = extra[stack_key]["one_launch_per_layer_32"]
        one["macko_GBps"], one["dense_GBps"] = round(sb / ts32 / 1e9, 1), round(db / td32 / 1e9, 1)
        one["macko_frac_of_hbm_peak"] = round(sb / ts32 / 1e9 / HBM_PEAK_GBPS, 4)
        one["speedup_vs_dense"] = round(td32 / ts32, 3)
        log(f"  stack: {extra[stack_key]}")
        del ops13, dops13
        torch.cuda.empty_cache()

    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(oracle, cases)
        log(f"cpu oracle: {cpu}")

    out = {
        "metric": "achieved HBM GB/s of the MACKO SpMV (format + x + y bytes) at 50% sparsity, Llama2-7B-shaped layers",
        "value": round(gbps, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16 in, f32 accumulate", "data": "synthetic",
        "config": {"workload": "configs[1]: Llama2-7B-shaped layer set, 50% per-row unstructured sparsity, "
                               "one step = 4x(4096x4096) + 2x(11008x4096) + 1x(4096x11008) SpMVs, batch 1, "
                               "issued in dependency order {q,k,v} -> {o} -> {gate,up} -> {down} as 4 grouped launches",
                   "layer_copies_rotated": n_layers, "launches_per_step": launches_per_step,
                   "macko_bytes_per_step": layer_macko_bytes, "dense_bytes_per_step": layer_dense_bytes},
        "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4),
        "us_per_spmv": round(ms_per_step * 1e3 / 7, 3),
        "dense_gemv": {"ms_per_step": round(t_dense / args.steps * 1e3, 5), "GBps": round(dense_gbps, 1),
                       "frac_of_hbm_peak": round(dense_gbps / HBM_PEAK_GBPS, 4)},
        "speedup_vs_dense_gemv": round(t_dense / t_sparse, 3),
        "memory_reduction_vs_dense": round(layer_dense_bytes / layer_macko_bytes, 3),
        "per_shape": per_shape,
        "rounds_of_steps_timed": headline_rounds,
        "steps_per_timed_round": headline_round_steps,
        "separate_launches": single,
        "one_launch_chain_dependences_honoured": chain,
        "one_launch_independent_products": one_launch,
        "two_bit_codes": two_bit,
        **({"eight_bit_values": fp8} if fp8 else {}),
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    out.update(extra)
    out["verified_against_oracle_before_timing"] = len(verified)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
