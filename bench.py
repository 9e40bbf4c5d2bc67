#!/usr/bin/env python3
"""Benchmark of the attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c3|c4|c5] [--no-extra] [--no-cpu] [--no-tune]

A step is one call of the library on one synthetic batch with every input resident in HBM.
The headline line is the Llama-3-8B-shaped paged decode (config 2), reported as algorithmic
HBM GB/s; the same JSON line carries the other configurations (varlen prefill, chunked prefill,
long-context decode) under "extra", each with its own roofline figure, and the fp64 CPU oracle
timed on the host's cores under "cpu_baseline".  Inputs are seeded synthetic stand-ins for the
paper's unpublished length samples (see workloads.py).
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

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published

WORKLOADS = {"c2": 2, "c3": 3, "c4": 4, "c5": 5}
GRAPH_REPLAYS = 3  # timed replays of the K-step graph; the median one is reported

TRAFFIC_JSON = os.path.join(ROOT, "profiles", "hbm_traffic.json")
PROBE_LIB = os.path.join(ROOT, "paper_2505_03780_amd", "libprobe_gfx950.so")


def _traffic(wl_name: str, instance: str):
    """HBM bytes per call of this workload, measured with rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE
    (separate runs), each scaled by what the same counter reads for a 1 GiB device copy; written to
    profiles/hbm_traffic.json by `bench.py --summarize-traffic` (commands and tables in
    profiles/hbm_traffic_all_workloads_pmc.md).  The figure belongs to the instance it was measured
    with: a run that times another instance reports null and says so on stderr."""
    try:
        with open(TRAFFIC_JSON) as f:
            table = json.load(f)
    except (OSError, ValueError) as e:
        print("bench.py: %s unreadable (%r): roofline.traffic is null" % (TRAFFIC_JSON, e), file=sys.stderr)
        return None
    rec = table.get(wl_name)
    if rec is None:
        print("bench.py: no traffic record for %s in %s: roofline.traffic is null" % (wl_name, TRAFFIC_JSON), file=sys.stderr)
        return None
    if rec["instance"] != instance:
        print("bench.py: traffic of %s was measured on '%s', this run timed '%s': roofline.traffic is null" % (
            wl_name, rec["instance"], instance), file=sys.stderr)
        return None
    return int(rec["bytes_per_call"])


def summarize_traffic(directory: str, workload: str):
    """Reads the four rocprofv3 --pmc runs under `directory` (probe_FETCH_SIZE, run_FETCH_SIZE,
    probe_WRITE_SIZE, run_WRITE_SIZE: counter_collection.csv files; the run_* logs hold the bench
    line with the instance that ran) and records the workload's HBM bytes per call in
    profiles/hbm_traffic.json."""
    import csv
    import glob

    def per_dispatch(sub, want):
        agg = {}
        for fn in glob.glob(os.path.join(directory, sub, "**", "*counter_collection.csv"), recursive=True):
            for r in csv.DictReader(open(fn)):
                if want(r["Kernel_Name"]):
                    a = agg.setdefault(r["Kernel_Name"], [0.0, 0])
                    a[0] += float(r["Counter_Value"])
                    a[1] += 1
        return {k: v[0] / v[1] for k, v in agg.items()}

    # the library's kernels, without the probes and the tuner's fill kernels
    ours = lambda n: "attn::" in n and not any(x in n for x in ("hbm_read_kernel", "mfma_bf16_kernel", "fill_bf16_kernel", "fill_f16_kernel"))
    copy = lambda n: "copyBuffer" in n
    out = {}
    for counter in ("FETCH_SIZE", "WRITE_SIZE"):
        probe = per_dispatch("probe_" + counter, copy)
        if not probe:
            raise SystemExit("no copy kernel under %s/probe_%s" % (directory, counter))
        factor = float(1 << 20) / (sum(probe.values()) / len(probe))  # true KiB per counted KiB
        out[counter] = {"factor": factor, "kernels": {k: v for k, v in per_dispatch("run_" + counter, ours).items()}}
    line = None
    for l in open(os.path.join(directory, "run_FETCH_SIZE.log")):
        if l.startswith("{") and '"metric"' in l:
            line = json.loads(l)
    if line is None:
        raise SystemExit("no bench line in run_FETCH_SIZE.log")
    name, instance = line["config"]["workload"], line["config"]["instance"]
    total = sum(out[c]["factor"] * sum(out[c]["kernels"].values()) for c in out) * 1024.0
    try:
        table = json.load(open(TRAFFIC_JSON))
    except (OSError, ValueError):
        table = {}
    table[name] = {"instance": instance, "bytes_per_call": int(round(total)),
                   "fetch_KiB_per_dispatch": out["FETCH_SIZE"]["kernels"], "fetch_factor": out["FETCH_SIZE"]["factor"],
                   "write_KiB_per_dispatch": out["WRITE_SIZE"]["kernels"], "write_factor": out["WRITE_SIZE"]["factor"]}
    with open(TRAFFIC_JSON, "w") as f:
        json.dump(table, f, indent=1, sort_keys=True)
        f.write("\n")
    print(json.dumps({name: table[name]}, indent=1))


def probe_achievable(read_bytes: int = 1 << 31, mfma_iters: int = 1 << 14) -> dict:
    """Times the two probes of libprobe_gfx950.so (a library of its own, outside the attention ABI) on
    the current stream: sustained HBM read bandwidth (GB/s) and sustained bf16 MFMA rate (TFLOP/s)."""
    import ctypes

    import torch

    if not os.path.exists(PROBE_LIB):
        raise ImportError("%s is missing: build it with `python -m paper_2505_03780_amd.build`" % PROBE_LIB)
    lib = ctypes.CDLL(PROBE_LIB)
    lib.probe_hbm_read.restype = ctypes.c_int
    lib.probe_hbm_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
    lib.probe_mfma_bf16.restype = ctypes.c_int64
    lib.probe_mfma_bf16.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    buf = torch.zeros(read_bytes // 4, dtype=torch.int32, device="cuda")
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    sp = int(torch.cuda.current_stream().cuda_stream)
    out = {}
    for name in ("hbm_read_GBps", "mfma_bf16_TFLOPs"):
        best = 0.0
        for rep in range(4):  # the first repetition warms clocks and caches
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            if name == "hbm_read_GBps":
                rc = lib.probe_hbm_read(buf.data_ptr(), read_bytes, sink.data_ptr(), sp)
                work = float(read_bytes) / 1e9
            else:
                rc = lib.probe_mfma_bf16(mfma_iters, sink.data_ptr(), sp)
                work = float(rc) / 1e12
            if rc < 0:
                raise RuntimeError("probe failed: %d" % rc)
            e1.record()
            torch.cuda.synchronize()
            if rep:
                best = max(best, work / (e0.elapsed_time(e1) * 1e-3))
        out[name] = best
    return out


def _dev(a):
    import torch

    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(a).cuda()


class Runner:
    """Holds one workload on the device and enqueues one step per call."""

    def __init__(self, wl, pools: int = 1):
        import torch

        import paper_2505_03780_amd as A

        self.A, self.torch, self.wl = A, torch, wl
        self.is_decode = wl.kind == "decode"
        self.q = _dev(wl.q)
        self.out = torch.zeros_like(self.q)
        k, v = _dev(wl.k), _dev(wl.v)
        # decode streams the KV cache once per step: alternate between distinct copies of the pool so
        # that a step never finds its keys in the last-level cache left over from the previous step
        self.kv = [(k, v)] + [(k.clone(), v.clone()) for _ in range(pools - 1)]
        self.qsl = torch.from_numpy(wl.query_start_loc).cuda()
        self.sl = torch.from_numpy(wl.seq_lens).cuda()
        self.bt = None if wl.block_table is None else torch.from_numpy(wl.block_table).cuda()
        self.kvsl = None if wl.kv_start_loc is None else torch.from_numpy(wl.kv_start_loc).cuda()
        self.max_q = 1 if self.is_decode else int(wl.q_lens().max())
        self.max_kv = int(wl.seq_lens.max())
        self.args = []
        self.ws = None
        for (kk, vv) in self.kv:
            a = A.make_args(self.q, kk, vv, self.out, self.sl, wl.scale, max_q_len=self.max_q, max_kv_len=self.max_kv,
                            query_start_loc=None if self.is_decode else self.qsl, kv_start_loc=self.kvsl,
                            block_table=self.bt, causal=wl.causal, is_decode=self.is_decode)
            if self.is_decode:
                if self.ws is None:
                    self.ws = torch.empty(max(A.attn_workspace_bytes(a, True) // 4, 4), dtype=torch.float32, device="cuda")
                a.workspace = self.ws.data_ptr()
                a.workspace_bytes = self.ws.numel() * 4
            self.args.append(a)
        self.lib = A.load_library()
        self.fn = self.lib.attn_decode_paged if self.is_decode else self.lib.attn_prefill_varlen
        self.i = 0
        self.instance = A.attn_instance_name(self.is_decode, A.attn_selected_instance(self.args[0], self.is_decode))

    def step(self, stream_ptr):
        a = self.args[self.i % len(self.args)]
        self.i += 1
        rc = self.fn(a, stream_ptr)
        if rc != 0:
            raise RuntimeError("library call failed: %s" % self.A.attn_status_string(rc))


def time_steps(run: Runner, steps: int, warmup: int):
    """Returns (ms per step of the timed region, HIP-event ms per step of the same region, median ms of
    per-step event pairs in eager mode, eager wall ms per step, eager event mean, whether the timed
    region was a graph replay)."""
    torch = run.torch
    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream
    for _ in range(warmup):
        run.step(sp)
    torch.cuda.synchronize()
    # per-step event pairs on the launch stream: the duration of one step's kernels
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in ev:
        a.record(stream)
        run.step(sp)
        b.record(stream)
    torch.cuda.synchronize()
    eager_ms = (time.perf_counter() - t0) * 1e3 / steps
    per = np.array([a.elapsed_time(b) for a, b in ev])
    # The same K steps as one HIP graph (the paper times its kernels under CUDA/HIP graphs, section
    # "Method and Investigated Kernels"): the hot calls only enqueue kernels, so they can be captured,
    # and a replay is free of the host's launch cost.  The graph is replayed once untimed, then timed.
    graph_ms = None
    try:
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.graph(g, stream=side):
            for _ in range(steps):
                run.step(side.cuda_stream)
        g.replay()
        torch.cuda.synchronize()
        # three timed replays of the same K steps; the median replay is reported (one replay of 20
        # steps moves by a few percent from run to run)
        reps = []
        for _ in range(GRAPH_REPLAYS):
            g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t0 = time.perf_counter()
            g0.record(stream)
            g.replay()
            g1.record(stream)
            torch.cuda.synchronize()
            reps.append(((time.perf_counter() - t0) * 1e3 / steps, g0.elapsed_time(g1) / steps))
        reps.sort(key=lambda r: r[1])
        graph_ms, graph_ev_ms = reps[len(reps) // 2]
        del g
    except Exception as e:  # keep the eager figure if capture is unavailable
        print("bench.py: graph timing skipped: %r" % (e,), file=sys.stderr)
    if graph_ms is None:
        return eager_ms, float(per.mean()), float(np.median(per)), eager_ms, float(per.mean()), False
    # under the graph the HIP events bracket all K steps: kernels of a step plus the gap to the next
    return graph_ms, graph_ev_ms, float(np.median(per)), eager_ms, float(per.mean()), True


def _figures(wl, run, wall_ms, ev_mean_ms, ev_med_ms, eager_ms, eager_ev_ms, graphed):
    res = {"workload": wl.name, "instance": run.instance, "ms_per_step": wall_ms, "kernel_ms_mean": ev_mean_ms,
           "kernel_ms_median_eager": ev_med_ms, "kernel_ms_mean_eager": eager_ev_ms, "ms_per_step_eager": eager_ms,
           "timed_as": ("one HIP graph of all steps, median of %d replays" % GRAPH_REPLAYS) if graphed else "eager launches"}
    if wl.kind == "decode":
        nbytes = wl.algorithmic_bytes()
        ach = nbytes / (ev_mean_ms * 1e-3) / 1e9
        res.update(metric="decode_hbm_GBps", unit="GB/s", value=nbytes / (wall_ms * 1e-3) / 1e9, algorithmic_bytes=nbytes,
                   roofline={"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                             "frac": ach / HBM_PEAK_GBPS, "traffic": _traffic(wl.name, run.instance)})
    else:
        fl = wl.flops()
        ach = fl / (ev_mean_ms * 1e-3) / 1e12
        res.update(metric="prefill_TFLOPs", unit="TFLOP/s", value=fl / (wall_ms * 1e-3) / 1e12, algorithmic_flops=fl,
                   roofline={"bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                             "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": _traffic(wl.name, run.instance)})
    return res


def check_output(wl, run: "Runner"):
    """After timing, outside the timed region: what the timed instance left in the output buffer,
    against the fp64 oracle.  Decode: every output row.  Prefill: one row per query head and run of
    32 tokens of every sequence (workloads.stratified_rows), so no workgroup of any tile size escapes."""
    import oracle
    import workloads as W

    torch = run.torch
    torch.cuda.synchronize()
    f16 = wl.dtype == "f16"
    wide = (lambda a: a.astype(np.float32)) if f16 else (lambda a: a)
    prob = oracle.OracleProblem(wide(wl.q), wide(wl.k), wide(wl.v), wl.query_start_loc, wl.seq_lens, wl.scale, wl.causal,
                                block_table=wl.block_table, kv_start_loc=wl.kv_start_loc)
    if wl.kind == "decode":
        B, H = wl.num_seqs, wl.num_q_heads
        seqs = np.repeat(np.arange(B, dtype=np.int32), H)
        toks = np.zeros(B * H, np.int32)
        heads = np.tile(np.arange(H, dtype=np.int32), B)
    else:
        seqs, toks, heads = W.stratified_rows(wl, 32)
    ref = oracle.attention_rows(prob, seqs, toks, heads)
    rows = torch.from_numpy(wl.query_start_loc[seqs].astype(np.int64) + toks).cuda()
    got = run.out[rows, torch.from_numpy(heads.astype(np.int64)).cuda()].float().cpu().numpy().astype(np.float64)
    d = got - ref
    max_abs = float(np.max(np.abs(d)))
    rel_rms = float(np.sqrt(np.sum(d * d) / np.sum(ref * ref)))
    ok = bool(np.isfinite(got).all() and max_abs <= 2e-2 and rel_rms <= 5e-3)
    if not ok:
        print("bench.py: %s: the timed instance '%s' is outside the tolerance: max-abs %.3e rel-RMS %.3e" % (
            wl.name, run.instance, max_abs, rel_rms), file=sys.stderr)
    return {"rows": int(len(seqs)), "of_rows": int(wl.q.shape[0] * wl.num_q_heads), "max_abs": max_abs, "rel_rms": rel_rms,
            "tol": [2e-2, 5e-3], "ok": ok, "against": "fp64 oracle, after timing"}


def measure(wl_id: int, steps: int, warmup: int, tune: bool, check: bool = True):
    """Times the workload with the instance a user gets after attn_tune on this batch's lengths (the
    paper's thesis: tune ahead of time, then only look up).  The untuned figure (built-in heuristic)
    is measured first, with fewer steps, and reported next to it."""
    import workloads as W

    wl = W.CONFIGS[wl_id]()
    run = Runner(wl, pools=2 if wl.kind == "decode" else 1)
    # bring the clocks up before anything is timed: about a third of a second of steps
    import torch
    sp = torch.cuda.current_stream().cuda_stream
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < 0.3:
        for _ in range(20):
            run.step(sp)
        torch.cuda.synchronize()
    untuned = None
    if tune:
        u = _figures(wl, run, *time_steps(run, max(5, steps // 3), warmup))
        untuned = {"instance": u["instance"], "value": u["value"], "kernel_ms_mean": u["kernel_ms_mean"]}
        run.A.attn_tune(run.args[0], run.is_decode, os.environ.get("ATTN_TUNE_CACHE"), 20, 0)
        run.instance = run.A.attn_instance_name(run.is_decode, run.A.attn_selected_instance(run.args[0], run.is_decode))
        # the tuner has just allocated and freed gigabytes and left the chip idle while it did: bring the
        # clocks up again exactly as before the first leg (the W warm-up steps alone are too short for
        # that: without it the same instance measured 3 % slower after tuning than before)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < 0.3:
            for _ in range(20):
                run.step(sp)
            torch.cuda.synchronize()
    res = _figures(wl, run, *time_steps(run, steps, warmup))
    res["untuned"] = untuned
    res["check"] = check_output(wl, run) if check else None
    if wl.kind == "decode":
        # a note next to the headline: the same steps always on ONE copy of the KV pool, which the
        # 256 MB last-level cache may partly hold from the step before (the headline rotates two copies)
        hot = Runner(wl, pools=1)
        h = _figures(wl, hot, *time_steps(hot, max(5, steps // 3), warmup))
        res["hot_cache_note"] = {"value": h["value"], "kernel_ms_mean": h["kernel_ms_mean"], "pools": 1}
        del hot
    return wl, res


def measure_rmsnorm(steps: int, warmup: int, tune: bool, hidden: int = 4096):
    """The paper's second kernel, fused residual add + RMS norm at the 8B (hidden 4096) or 70B (8192)
    model's hidden size over a prefill-sized batch of tokens: HBM-bound, reported as algorithmic GB/s."""
    import torch

    import paper_2505_03780_amd as A
    import workloads as W

    wl = W.rmsnorm_8b_prefill() if hidden == 4096 else W.rmsnorm_70b_prefill()
    x, res, w = _dev(wl.x), _dev(wl.residual), _dev(wl.weight)
    # two sets of buffers take turns, so that a step never finds its rows in the last-level cache
    sets = [(x, res, torch.empty_like(x)), (x.clone(), res.clone(), torch.empty_like(x))]
    args = [A.make_rmsnorm_args(a, w, o, wl.eps, r) for a, r, o in sets]
    lib = A.load_library()
    stream = torch.cuda.current_stream()
    import ctypes

    def loop(n, sp):
        for i in range(n):
            rc = lib.rmsnorm_fused_add(ctypes.byref(args[i % 2]), sp)
            if rc != 0:
                raise RuntimeError("rmsnorm_fused_add failed: %d" % rc)

    untuned = A.rmsnorm_instance_name(A.rmsnorm_selected_instance(args[0]))
    if tune:
        A.rmsnorm_tune(args[0], os.environ.get("ATTN_TUNE_CACHE"), 10, 0)
    inst = A.rmsnorm_instance_name(A.rmsnorm_selected_instance(args[0]))
    loop(warmup, stream.cuda_stream)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(stream)
    with torch.cuda.graph(g, stream=side):
        loop(steps, side.cuda_stream)
    g.replay()
    torch.cuda.synchronize()
    reps = []
    for _ in range(GRAPH_REPLAYS):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        g.replay()
        e1.record(stream)
        torch.cuda.synchronize()
        reps.append(((time.perf_counter() - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps))
    reps.sort(key=lambda r: r[1])
    wall_ms, ev_ms = reps[len(reps) // 2]
    nbytes = wl.algorithmic_bytes()
    ach = nbytes / (ev_ms * 1e-3) / 1e9
    return {"workload": wl.name, "instance": inst, "untuned_instance": untuned, "metric": "rmsnorm_hbm_GBps", "unit": "GB/s",
            "value": nbytes / (wall_ms * 1e-3) / 1e9, "ms_per_step": wall_ms, "kernel_ms_mean": ev_ms, "algorithmic_bytes": nbytes,
            "timed_as": "one HIP graph of all steps, median of %d replays" % GRAPH_REPLAYS,
            "roofline": {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBPS,
                         "traffic": _traffic(wl.name, inst)}}


def cpu_baseline(wl, unit: str):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload (about 10-30 s of CPU)."""
    import oracle

    prob = oracle.OracleProblem(wl.q, wl.k, wl.v, wl.query_start_loc, wl.seq_lens, wl.scale, wl.causal,
                                block_table=wl.block_table, kv_start_loc=wl.kv_start_loc)
    nq = wl.q_lens()
    # sample: whole (sequence, head) rows until about 4 GFLOP of oracle work is collected
    budget = 4e9
    seqs, toks, heads = [], [], []
    flops = 0.0
    nbytes = 0.0
    rng = np.random.default_rng(0)
    order = rng.permutation(wl.num_seqs)
    for s in order:
        for h in range(wl.num_q_heads):
            if flops >= budget:
                break
            off = int(wl.seq_lens[s] - nq[s])
            t = np.arange(nq[s])
            seqs.append(np.full(nq[s], s)); toks.append(t); heads.append(np.full(nq[s], h))
            pairs = float(np.sum(off + t + 1)) if wl.causal else float(nq[s] * wl.seq_lens[s])
            flops += 4.0 * wl.head_dim * pairs
            nbytes += float(wl.seq_lens[s]) * wl.head_dim * 2 * 2 / (wl.num_q_heads // wl.num_kv_heads)
    seqs, toks, heads = (np.concatenate(x).astype(np.int32) for x in (seqs, toks, heads))
    oracle.attention_rows(prob, seqs[:8], toks[:8], heads[:8])  # load the library, touch the data
    # a small workload is over in a fraction of a second: repeat the pass until about 10 s have gone by
    reps, t0 = 0, time.perf_counter()
    while True:
        oracle.attention_rows(prob, seqs, toks, heads)
        reps += 1
        if time.perf_counter() - t0 >= 10.0 or reps >= 200:
            break
    dt = (time.perf_counter() - t0) / reps
    val = (nbytes / dt / 1e9) if unit == "GB/s" else (flops / dt / 1e12)
    return {"value": val, "unit": unit, "cores": oracle.num_threads(), "kind": "oracle", "seconds": dt, "passes": reps,
            "sample": "%d output rows (%d whole (sequence, head) pairs, %.2f GFLOP of the workload's %.2f) of %s" % (
                len(seqs), len(np.unique(seqs * 1000 + heads)), flops / 1e9, wl.flops() / 1e9, wl.name)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", choices=sorted(WORKLOADS) + ["rmsnorm", "rmsnorm_h8192"], default="c2",
                    help="c2..c5: attention configurations (c2 is the headline); rmsnorm, rmsnorm_h8192: only the fused RMS norm "
                         "leg at hidden 4096 or 8192")
    ap.add_argument("--no-extra", action="store_true", help="skip the other configurations")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-tune", action="store_true", help="keep the built-in heuristic (default: attn_tune runs first, untimed)")
    ap.add_argument("--no-check", action="store_true", help="skip the oracle check of the timed outputs")
    ap.add_argument("--summarize-traffic", metavar="DIR",
                    help="no GPU work: read the rocprofv3 --pmc runs under DIR (see profiles/hbm_traffic_all_workloads_pmc.md) "
                         "and record the workload's HBM bytes per call in profiles/hbm_traffic.json")
    ap.add_argument("--copy-probe", action="store_true",
                    help="only run a 1 GiB device-to-device copy three times (calibrates the FETCH_SIZE / WRITE_SIZE counters)")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU only (one MI355X, no collectives); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if a.summarize_traffic:
        summarize_traffic(a.summarize_traffic, a.workload)
        return
    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    if a.copy_probe:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_read": 1 << 30, "copy_probe_bytes_written": 1 << 30, "copies": 3}))
        return

    if a.workload.startswith("rmsnorm"):
        r = measure_rmsnorm(a.steps, a.warmup, not a.no_tune, 8192 if a.workload.endswith("8192") else 4096)
        print(json.dumps({"metric": r["metric"], "value": r["value"], "unit": r["unit"], "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
                          "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
                          "dtype": "bf16", "data": "synthetic", "config": {"workload": r["workload"], "instance": r["instance"]},
                          "kernel_ms_mean": r["kernel_ms_mean"], "roofline": r["roofline"]}), flush=True)
        return
    wl, main_res = measure(WORKLOADS[a.workload], a.steps, a.warmup, not a.no_tune, not a.no_check)
    # what this machine sustains for the two bounding resources (the benchmark's own probes), next to
    # the published peaks the roofline fractions are quoted against
    achievable = probe_achievable()

    def _with_achievable(roof):
        ref = achievable["hbm_read_GBps"] if roof["bound"] == "hbm" else achievable["mfma_bf16_TFLOPs"]
        roof = dict(roof)
        roof["frac_of_achievable"] = roof["achieved"] / ref if ref > 0 else None
        return roof

    main_res["roofline"] = _with_achievable(main_res["roofline"])
    line = {
        "metric": main_res["metric"], "value": main_res["value"], "unit": main_res["unit"], "n_gpus": 1,
        "steps": a.steps, "warmup": a.warmup, "ms_per_step": main_res["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "instance": main_res["instance"], "num_seqs": wl.num_seqs,
                   "num_q_heads": wl.num_q_heads, "num_kv_heads": wl.num_kv_heads, "head_dim": wl.head_dim,
                   "kv_block_size": wl.block_size, "kv_tokens": int(wl.seq_lens.sum()), "tuned": not a.no_tune},
        "kernel_ms_mean": main_res["kernel_ms_mean"], "kernel_ms_mean_eager": main_res["kernel_ms_mean_eager"],
        "ms_per_step_eager": main_res["ms_per_step_eager"], "timed_as": main_res["timed_as"],
        "roofline": main_res["roofline"], "untuned": main_res["untuned"], "achievable": achievable,
        "check": main_res["check"],
    }
    if "hot_cache_note" in main_res:
        line["hot_cache_note"] = main_res["hot_cache_note"]
    if not a.no_cpu:
        line["cpu_baseline"] = cpu_baseline(wl, main_res["unit"])
    del wl
    if not a.no_extra:
        extra = {}
        for name, wid in sorted(WORKLOADS.items()):
            if name == a.workload:
                continue
            torch.cuda.empty_cache()
            _, r = measure(wid, max(5, a.steps // 2), max(2, a.warmup // 2), not a.no_tune, not a.no_check)
            extra[name] = {k: r[k] for k in ("workload", "instance", "metric", "value", "unit", "ms_per_step", "ms_per_step_eager", "timed_as",
                                             "kernel_ms_mean", "roofline", "untuned", "check")}
            extra[name]["roofline"] = _with_achievable(extra[name]["roofline"])
        torch.cuda.empty_cache()
        for key, hidden in (("rmsnorm", 4096), ("rmsnorm_h8192", 8192)):
            extra[key] = measure_rmsnorm(a.steps, a.warmup, not a.no_tune, hidden)
            extra[key]["roofline"] = _with_achievable(extra[key]["roofline"])
            torch.cuda.empty_cache()
        line["extra"] = extra
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
