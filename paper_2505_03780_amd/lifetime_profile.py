"""Where the workgroups of the ring prefill kernel spend their time, and where they run.

    python -m paper_2505_03780_amd.build --profile          # builds libattn_gfx950_profile.so
    python -m paper_2505_03780_amd.lifetime_profile c3|c4 [--instance NAME] [--out FILE.md]

The profiling build of the library stamps every wavefront of `prefill_ring_kernel` with the 100 MHz
wall clock at entry, at the start and the end of its unit loop and at exit, and records the block
index and the hardware ids (XCD, shader engine, compute unit) it ran on.  This tool runs one call of
a benchmark workload (run from the repository root: the input generators live in workloads.py),
reads the stamps back and prints: prologue / loop / epilogue times, a least-squares fit of the loop
time against the number of 32-key units, and per XCD and shader engine the sum of wave lifetimes,
the block indices served and the time of the last exit.  It is how the dispatch order of workgroups
(round-robin over XCDs, then over the shader engines of an XCD, by block index) was found.
"""
from __future__ import annotations

import argparse
import ctypes
import os
import sys

import numpy as np

TICK_US = 0.01  # one wall_clock64 tick


def collect(which: str, instance: str | None):
    import torch

    from . import binding as B
    from .build import PROFILE_LIB

    if not os.path.exists(PROFILE_LIB):
        raise ImportError("%s is missing: build it with `python -m paper_2505_03780_amd.build --profile`" % PROFILE_LIB)
    B.use_library(PROFILE_LIB)
    import workloads as W

    wl = W.CONFIGS[{"c3": 3, "c4": 4}[which]]()
    dev = lambda a: None if a is None else torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda()
    as16 = lambda t: t.view(torch.bfloat16) if t.dtype == torch.int16 else t
    q, k, v = as16(dev(wl.q)), as16(dev(wl.k)), as16(dev(wl.v))
    out = torch.zeros_like(q)
    sl, qsl, bt, kvsl = dev(wl.seq_lens), dev(wl.query_start_loc), dev(wl.block_table), dev(wl.kv_start_loc)
    a = B.make_args(q, k, v, out, sl, wl.scale, max_q_len=int(wl.q_lens().max()), max_kv_len=int(wl.seq_lens.max()),
                    query_start_loc=qsl, kv_start_loc=kvsl, block_table=bt, causal=wl.causal, is_decode=False)
    names = [B.attn_instance_name(False, i) for i in range(B.attn_num_instances(False))]
    if instance is not None:
        B.attn_force_instance(False, names.index(instance))
    chosen = names[B.attn_selected_instance(a, False)]
    if "ring" not in chosen:
        raise RuntimeError("only the ring prefill kernel carries the stamps; selected: " + chosen)
    stamps = torch.zeros((1 << 16) * 8 * 16, dtype=torch.int64, device="cuda")  # 16 words per wave, up to 65536 workgroups of 8 waves
    a.workspace, a.workspace_bytes = stamps.data_ptr(), stamps.numel() * 8
    lib = B.load_library()
    sp = torch.cuda.current_stream().cuda_stream
    for _ in range(3):
        assert lib.attn_prefill_varlen(ctypes.byref(a), sp) == 0
    torch.cuda.synchronize()
    stamps.zero_()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    assert lib.attn_prefill_varlen(ctypes.byref(a), sp) == 0
    e1.record()
    torch.cuda.synchronize()
    t = stamps.cpu().numpy().reshape(-1, 16)
    return wl.name, chosen, e0.elapsed_time(e1) * 1e3, t[t[:, 5] > 0]


def report(name, chosen, kernel_us, t) -> str:
    t0 = t[:, 8].min()
    ent, l0, l1, ex = [(t[:, i] - t0) * TICK_US for i in (8, 9, 7, 10)]
    units, bid, hw, xcc = t[:, 5].astype(float), t[:, 11], t[:, 12], t[:, 13] & 15
    pro, loop, epi, life = l0 - ent, l1 - l0, ex - l1, ex - ent
    coef = np.linalg.lstsq(np.vstack([np.ones_like(units), units]).T, loop, rcond=None)[0]
    se = (hw >> 13) & 7
    cu = ((hw >> 8) & 15) | (se << 4) | (xcc << 8)
    L = ["# Workgroup lifetimes of the ring prefill kernel: %s" % name, "",
         "Instance `%s`; one call, %.1f us between HIP events (profiling build: its per-phase cycle counters slow the unit loop by 10-30 %%)." % (chosen, kernel_us), "",
         "| per wavefront | mean us | median | 90th percentile | max |", "|---|---|---|---|---|"]
    for lab, x in (("prologue (entry to first loop iteration)", pro), ("unit loop", loop), ("epilogue (last iteration to exit, stores drained)", epi), ("lifetime", life)):
        L.append("| %s | %.2f | %.2f | %.2f | %.2f |" % (lab, x.mean(), np.median(x), np.percentile(x, 90), x.max()))
    L += ["", "Waves: %d; units per wave: mean %.1f, max %d; loop time = %.2f us + %.3f us per 32-key unit (least squares)." % (len(t), units.mean(), units.max(), coef[0], coef[1]),
          "Share of the summed wave lifetimes: prologue %.1f %%, loop %.1f %%, epilogue %.1f %%." % (100 * pro.sum() / life.sum(), 100 * loop.sum() / life.sum(), 100 * epi.sum() / life.sum()), ""]
    cus = np.unique(cu)
    first = np.array([ent[cu == c].min() for c in cus])
    last = np.array([ex[cu == c].max() for c in cus])
    L += ["Compute units seen: %d.  First workgroup on a compute unit: %.1f / %.1f / %.1f us (min / mean / max after the first entry); last exit per compute unit: %.1f / %.1f / %.1f us." % (
        len(cus), first.min(), first.mean(), first.max(), last.min(), last.mean(), last.max()), "",
          "| XCD | shader engine | compute units | waves | sum of wave lifetimes us | last exit us | (block index / 8) mod 4 | block index mod 8 |", "|---|---|---|---|---|---|---|---|"]
    for x in np.unique(xcc):
        for s in np.unique(se):
            m = (xcc == x) & (se == s)
            if m.any():
                L.append("| %d | %d | %d | %d | %.0f | %.1f | %s | %s |" % (x, s, len(np.unique(cu[m])), m.sum(), life[m].sum(), ex[m].max(),
                                                                     sorted(set(((bid[m] // 8) % 4).tolist())), sorted(set((bid[m] % 8).tolist()))))
    return "\n".join(L) + "\n"


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("workload", choices=["c3", "c4"])
    ap.add_argument("--instance", default=None)
    ap.add_argument("--out", default=None)
    a = ap.parse_args(argv)
    text = report(*collect(a.workload, a.instance))
    if a.out:
        with open(a.out, "w") as f:
            f.write(text)
    sys.stdout.write(text)
    return 0


if __name__ == "__main__":
    sys.exit(main())
