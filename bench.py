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

# HBM bytes per call measured with rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE (separate runs, KiB
# per dispatch summed over the kernels of one call), each scaled by what the same counter reads for a
# 1 GiB device copy (FETCH_SIZE reads 0.5 KiB per KiB fetched, WRITE_SIZE 1.0); the summary and the
# commands are in profiles/hbm_traffic_all_workloads_pmc.md.  Keyed by workload and kernel family:
# a run that selects another family reports null.
MEASURED_TRAFFIC_BYTES = {
    ("c2_decode_8b", "decode_bf16_balanced"): (2 * (311630 + 2690) + 5152 + 512) * 1024,
    ("c5_decode_70b_long", "decode_bf16_balanced"): (2 * (756726 + 4546) + 8809 + 256) * 1024,
    ("c3_prefill_8b", "prefill_bf16_ring"): (2 * 78890 + 70104) * 1024,
    ("c4_chunked_prefill", "prefill_bf16_ring seqmajor"): (2 * 212289 + 65536) * 1024,
    ("rmsnorm_8b_t8192_h4096", "rmsnorm"): (2 * 65585 + 131131) * 1024,
}


def _traffic(wl_name: str, instance: str):
    family = instance.split(" ")[0] + (" seqmajor" if instance.endswith("seqmajor") else "")
    return MEASURED_TRAFFIC_BYTES.get((wl_name, family))


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
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        g0.record(stream)
        g.replay()
        g1.record(stream)
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / steps
        graph_ev_ms = g0.elapsed_time(g1) / steps
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
           "timed_as": "one HIP graph of all steps" if graphed else "eager launches"}
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


def measure(wl_id: int, steps: int, warmup: int, tune: bool):
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
        run.A.attn_tune(run.args[0], run.is_decode, os.environ.get("ATTN_TUNE_CACHE"), 10, 0)
        run.instance = run.A.attn_instance_name(run.is_decode, run.A.attn_selected_instance(run.args[0], run.is_decode))
    res = _figures(wl, run, *time_steps(run, steps, warmup))
    res["untuned"] = untuned
    if wl.kind == "decode":
        # a note next to the headline: the same steps always on ONE copy of the KV pool, which the
        # 256 MB last-level cache may partly hold from the step before (the headline rotates two copies)
        hot = Runner(wl, pools=1)
        h = _figures(wl, hot, *time_steps(hot, max(5, steps // 3), warmup))
        res["hot_cache_note"] = {"value": h["value"], "kernel_ms_mean": h["kernel_ms_mean"], "pools": 1}
        del hot
    return wl, res


def measure_rmsnorm(steps: int, warmup: int, tune: bool):
    """The paper's second kernel, fused residual add + RMS norm at the 8B model's hidden size over a
    prefill-sized batch of tokens: HBM-bound, reported as algorithmic GB/s."""
    import torch

    import paper_2505_03780_amd as A
    import workloads as W

    wl = W.rmsnorm_8b_prefill()
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
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    g.replay()
    e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    ev_ms = e0.elapsed_time(e1) / steps
    nbytes = wl.algorithmic_bytes()
    ach = nbytes / (ev_ms * 1e-3) / 1e9
    return {"workload": wl.name, "instance": inst, "untuned_instance": untuned, "metric": "rmsnorm_hbm_GBps", "unit": "GB/s",
            "value": nbytes / (wall_ms * 1e-3) / 1e9, "ms_per_step": wall_ms, "kernel_ms_mean": ev_ms, "algorithmic_bytes": nbytes,
            "timed_as": "one HIP graph of all steps",
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
    ap.add_argument("--workload", choices=sorted(WORKLOADS) + ["rmsnorm"], default="c2",
                    help="c2..c5: attention configurations (c2 is the headline); rmsnorm: only the fused RMS norm leg")
    ap.add_argument("--no-extra", action="store_true", help="skip the other configurations")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-tune", action="store_true", help="keep the built-in heuristic (default: attn_tune runs first, untimed)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="only run a 1 GiB device-to-device copy three times (calibrates the FETCH_SIZE / WRITE_SIZE counters)")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU only (one MI355X, no collectives); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
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

    if a.workload == "rmsnorm":
        r = measure_rmsnorm(a.steps, a.warmup, not a.no_tune)
        print(json.dumps({"metric": r["metric"], "value": r["value"], "unit": r["unit"], "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
                          "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
                          "dtype": "bf16", "data": "synthetic", "config": {"workload": r["workload"], "instance": r["instance"]},
                          "kernel_ms_mean": r["kernel_ms_mean"], "roofline": r["roofline"]}), flush=True)
        return
    wl, main_res = measure(WORKLOADS[a.workload], a.steps, a.warmup, not a.no_tune)
    # what this machine sustains for the two bounding resources (the library's own probes), next to
    # the published peaks the roofline fractions are quoted against
    import paper_2505_03780_amd as A
    achievable = A.probe_achievable()

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
            _, r = measure(wid, max(5, a.steps // 2), max(2, a.warmup // 2), not a.no_tune)
            extra[name] = {k: r[k] for k in ("workload", "instance", "metric", "value", "unit", "ms_per_step", "ms_per_step_eager", "timed_as",
                                             "kernel_ms_mean", "roofline", "untuned")}
            extra[name]["roofline"] = _with_achievable(extra[name]["roofline"])
        torch.cuda.empty_cache()
        extra["rmsnorm"] = measure_rmsnorm(a.steps, a.warmup, not a.no_tune)
        extra["rmsnorm"]["roofline"] = _with_achievable(extra["rmsnorm"]["roofline"])
        line["extra"] = extra
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
