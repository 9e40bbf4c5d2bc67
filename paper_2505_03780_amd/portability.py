"""Configuration-portability study on one GPU.

    python -m paper_2505_03780_amd.portability --kind decode|prefill [--iters 10] [--out FILE.md]
                                               [--cache FILE] [--batches 1,16] [--lengths 1024,4096]

The paper's second research question is how far a configuration tuned for one setting carries over
to another (section "Evaluation": reusing the other platform's configurations costs between 20 % and
14x).  With one GPU the settings that vary are the shape buckets: this tool tunes every bucket of a
batch x sequence-length grid (Llama-3-8B head shapes; the grid includes the batch-64 points the
paper plots), then runs every bucket's winner on every other bucket and prints the slowdown matrix,
next to the built-in heuristic's slowdown.  Inputs are random device tensors: only time is measured.
"""
from __future__ import annotations

import argparse
import sys

import numpy as np


def _bucket_inputs(kind, batch, seqlen, rng_seed=0):
    import torch

    from . import binding as B

    g = torch.Generator(device="cuda").manual_seed(rng_seed)
    Hq, Hkv, D, bs = 32, 8, 128, 16
    # lengths spread between half of and the full nominal length, one sequence at the full length
    lens = np.linspace(seqlen // 2, seqlen, batch).astype(np.int32)
    lens[-1] = seqlen
    np.random.default_rng(rng_seed).shuffle(lens)
    seq_lens = torch.from_numpy(lens).cuda()
    if kind == "decode":
        nblk = int(np.sum((lens + bs - 1) // bs))
        width = (seqlen + bs - 1) // bs
        table = np.full((batch, width), 0, np.int32)
        perm = np.random.default_rng(rng_seed + 1).permutation(nblk).astype(np.int32)
        pos = 0
        for s, n in enumerate(lens):
            nb = (int(n) + bs - 1) // bs
            table[s, :nb] = perm[pos:pos + nb]
            pos += nb
        k = torch.randn(nblk, bs, Hkv, D, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        v = torch.randn(nblk, bs, Hkv, D, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        q = torch.randn(batch, Hq, D, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        out = torch.empty_like(q)
        bt = torch.from_numpy(table).cuda()
        a = B.make_args(q, k, v, out, seq_lens, D ** -0.5, max_q_len=1, max_kv_len=seqlen, block_table=bt, is_decode=True)
        ws = torch.empty(max(B.attn_workspace_bytes(a, True) // 4, 4), dtype=torch.float32, device="cuda")
        a.workspace, a.workspace_bytes = ws.data_ptr(), ws.numel() * 4
        keep = (q, k, v, out, bt, seq_lens, ws)
    else:
        qsl = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).cuda()
        total = int(lens.sum())
        q = torch.randn(total, Hq, D, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        k = torch.randn(total, Hkv, D, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        v = torch.randn(total, Hkv, D, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        out = torch.empty_like(q)
        a = B.make_args(q, k, v, out, seq_lens, D ** -0.5, max_q_len=seqlen, max_kv_len=seqlen, query_start_loc=qsl, causal=True)
        keep = (q, k, v, out, qsl, seq_lens)
    return a, keep


def _time(lib_fn, args, iters):
    import ctypes

    import torch

    sp = torch.cuda.current_stream().cuda_stream
    for _ in range(2):
        if lib_fn(ctypes.byref(args), sp) != 0:
            return None
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for e0, e1 in ev:
        e0.record()
        if lib_fn(ctypes.byref(args), sp) != 0:
            return None
        e1.record()
    torch.cuda.synchronize()
    return float(np.median([e0.elapsed_time(e1) for e0, e1 in ev])) * 1e3  # microseconds


def study(kind: str, iters: int, batches, seqlens, cache_path=None):
    import torch

    from . import binding as B

    is_decode = kind == "decode"
    lib = B.load_library()
    fn = lib.attn_decode_paged if is_decode else lib.attn_prefill_varlen
    names = [B.attn_instance_name(is_decode, i) for i in range(B.attn_num_instances(is_decode))]
    buckets = [(b, s) for b in batches for s in seqlens]
    winner, t_heur, t_self = {}, {}, {}
    B.attn_clear_cache()
    for bk in buckets:
        print("tuning", kind, "batch %d x len %d" % bk, file=sys.stderr, flush=True)
        a, keep = _bucket_inputs(kind, *bk)
        B.attn_force_instance(is_decode, -1)
        t_heur[bk] = (_time(fn, a, iters), names[B.attn_selected_instance(a, is_decode)])
        B.attn_tune(a, is_decode, cache_path, iters, 0)
        winner[bk] = B.attn_selected_instance(a, is_decode)
        del a, keep
        torch.cuda.empty_cache()
    cross = {}
    for tgt in buckets:
        a, keep = _bucket_inputs(kind, *tgt)
        for src in buckets:
            B.attn_force_instance(is_decode, winner[src])
            cross[(src, tgt)] = _time(fn, a, iters) if B.attn_selected_instance(a, is_decode) == winner[src] else None
        t_self[tgt] = cross[(tgt, tgt)]
        del a, keep
        torch.cuda.empty_cache()
    B.attn_force_instance(is_decode, -1)
    B.attn_clear_cache()

    lab = lambda bk: "B%d x %d" % bk
    lines = ["## %s: winners" % kind, "", "| bucket (batch x length) | tuned instance | tuned us | built-in choice | built-in us | built-in / tuned |", "|---|---|---|---|---|---|"]
    for bk in buckets:
        th, nh = t_heur[bk]
        lines.append("| %s | %s | %.1f | %s | %.1f | %.2f |" % (lab(bk), names[winner[bk]], t_self[bk], nh, th, th / t_self[bk]))
    lines += ["", "## %s: slowdown of the row bucket's winner when it runs the column bucket (1.00 = that bucket's own winner)" % kind, "",
              "| tuned for \\\\ run on | " + " | ".join(lab(b) for b in buckets) + " |", "|---|" + "---|" * len(buckets)]
    worst, allv = 0.0, []
    for src in buckets:
        row = []
        for tgt in buckets:
            t = cross[(src, tgt)]
            if t is None:
                row.append("n/a")
            else:
                r = t / t_self[tgt]
                row.append("%.2f" % r)
                if src != tgt:
                    allv.append(r)
                    worst = max(worst, r)
        lines.append("| %s | " % lab(src) + " | ".join(row) + " |")
    lines += ["", "Off-diagonal slowdown: worst %.2fx, mean %.2fx, %d of %d pairs above 1.10x." % (
        worst, float(np.mean(allv)), int(np.sum(np.array(allv) > 1.10)), len(allv))]
    return "\n".join(lines) + "\n"


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--kind", choices=["decode", "prefill"], required=True)
    ap.add_argument("--iters", type=int, default=10)
    ap.add_argument("--out", default=None)
    ap.add_argument("--cache", default=None, help="also record every bucket's winner in this cache file (ahead-of-time tuning: "
                                                   "point ATTN_TUNE_CACHE at it later)")
    ap.add_argument("--batches", default=None, help="comma-separated batch sizes instead of the default grid")
    ap.add_argument("--lengths", default=None, help="comma-separated sequence lengths instead of the default grid")
    a = ap.parse_args()
    ints = lambda s, d: d if s is None else [int(x) for x in s.split(",")]
    if a.kind == "decode":
        text = study("decode", a.iters, ints(a.batches, [1, 16, 64, 256]), ints(a.lengths, [1024, 4096, 16384]), a.cache)
    else:
        text = study("prefill", a.iters, ints(a.batches, [1, 8, 64]), ints(a.lengths, [512, 1024, 2048, 8192]), a.cache)
    print(text)
    if a.out:
        open(a.out, "w").write(text)


if __name__ == "__main__":
    main()
