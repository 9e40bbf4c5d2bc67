"""Static statistics of the compiled kernel instances: instruction counts, distinct opcodes, registers, LDS.

The single-GPU analogue of the paper's code-diversity analysis (section "Evaluation": unique opcodes and
instruction counts of the binaries an autotuner generates, against a template library).  Every
translation unit is compiled to gfx950 assembly with the library's own flags (no GPU needed) and the
text of each kernel is counted.

    python -m paper_2505_03780_amd.isa_stats [--out FILE.md]
"""
from __future__ import annotations

import argparse
import collections
import concurrent.futures as cf
import os
import re
import subprocess
import sys
import tempfile

from .build import CSRC, EXTRA, FLAGS, SOURCES

_INSTR = re.compile(r"^\t([a-z][a-z0-9_]+)\b")
_FAMILIES = (("prefill_ring_kernel", "prefill ring"), ("prefill_bf16_kernel", "prefill staged"), ("prefill_f32_kernel", "prefill fp32"),
             ("decode_bf16_kernel", "decode fixed split"), ("decode_seq_kernel", "decode wave per head"),
             ("decode_balanced_kernel", "decode token-balanced"), ("combine_kernel", "decode merge"),
             ("rmsnorm_kernel", "rms norm"), ("kv_cache_write_kernel", "kv write"))


def _asm(src: str, tmp: str) -> str:
    out = os.path.join(tmp, src.replace(".hip", ".s"))
    flags = [f for f in FLAGS if f != "-fPIC"]
    cmd = ["hipcc", *flags, *EXTRA.get(src, []), "-S", "--cuda-device-only", os.path.join(CSRC, src), "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc -S failed for %s:\n%s" % (src, r.stderr[-2000:]))
    return out


def _demangle(names):
    try:
        r = subprocess.run(["c++filt"], input="\n".join(names), capture_output=True, text=True)
    except OSError:
        return list(names)
    return r.stdout.splitlines() if r.returncode == 0 else list(names)


def _parse(path: str):
    """Yield (mangled name, opcode counter, {vgpr, agpr, sgpr, lds, scratch}) per kernel of one .s file."""
    text = open(path).read()
    meta = {}
    for m in re.finditer(r"\.amdhsa_kernel (\S+)\n(.*?)\.end_amdhsa_kernel", text, re.S):
        body = m.group(2)
        get = lambda k: int(re.search(r"\.amdhsa_%s (\d+)" % k, body).group(1)) if re.search(r"\.amdhsa_%s (\d+)" % k, body) else 0
        meta[m.group(1)] = {"lds": get("group_segment_fixed_size"), "scratch": get("private_segment_fixed_size"),
                            "vgpr_total": get("next_free_vgpr"), "accum_offset": get("accum_offset"), "sgpr": get("next_free_sgpr")}
    for name in meta:
        m = re.search(r"^%s:[^\n]*\n(.*?)\n\.Lfunc_end\d+:" % re.escape(name), text, re.S | re.M)
        if not m:
            continue
        ops = collections.Counter()
        for line in m.group(1).splitlines():
            im = _INSTR.match(line)
            if im and not im.group(1).startswith("amdhsa"):
                ops[im.group(1)] += 1
        yield name, ops, meta[name]


def collect():
    rows = []
    with tempfile.TemporaryDirectory() as tmp:
        with cf.ThreadPoolExecutor(max_workers=8) as ex:
            paths = list(ex.map(lambda s: _asm(s, tmp), [s for s in SOURCES if s != "attn_api.hip"]))
        for path in paths:
            parsed = list(_parse(path))
            for (name, ops, meta), nice in zip(parsed, _demangle([p[0] for p in parsed])):
                nice = nice.replace("void attn::(anonymous namespace)::", "").replace("attn::(anonymous namespace)::", "")
                nice = re.sub(r"\((attn::)?(KParams|RmsParams|KvWriteParams)\)$", "", nice)
                rows.append({"tu": os.path.basename(path)[:-2], "kernel": nice, "ops": ops, **meta})
    return rows


def family(kernel: str) -> str:
    for key, fam in _FAMILIES:
        if key in kernel:
            return fam
    return "other"


def render(rows) -> str:
    L = ["# Static instruction statistics of every compiled kernel instance", "",
         "Command (no GPU needed; compiles every translation unit to gfx950 assembly with the library's flags):",
         "`python -m paper_2505_03780_amd.isa_stats --out profiles/instance_isa_stats.md`", "",
         "## Per kernel", "", "| translation unit | kernel | instructions | distinct opcodes | MFMA | LDS ops | global/buffer loads | VGPRs (of which AGPRs) | SGPRs | static LDS B | scratch B |",
         "|---|---|---|---|---|---|---|---|---|---|---|"]
    for r in sorted(rows, key=lambda r: (r["tu"], r["kernel"])):
        ops = r["ops"]
        n = sum(ops.values())
        mfma = sum(c for o, c in ops.items() if o.startswith("v_mfma"))
        lds = sum(c for o, c in ops.items() if o.startswith("ds_"))
        gl = sum(c for o, c in ops.items() if o.startswith(("global_load", "buffer_load")))
        agpr = max(r["vgpr_total"] - r["accum_offset"], 0) if r["accum_offset"] else 0
        L.append("| %s | %s | %d | %d | %d | %d | %d | %d (%d) | %d | %d | %d |" % (r["tu"], r["kernel"], n, len(ops), mfma, lds, gl, r["vgpr_total"], agpr, r["sgpr"], r["lds"], r["scratch"]))
    fam = collections.defaultdict(list)
    for r in rows:
        fam[family(r["kernel"])].append(r)
    L += ["", "## Per kernel family (all instances the autotuner can choose from)", "",
          "| family | instances | instructions min / median / max | distinct opcodes per instance min / max | distinct opcodes over the family |", "|---|---|---|---|---|"]
    allops = set()
    for f, rs in sorted(fam.items()):
        counts = sorted(sum(r["ops"].values()) for r in rs)
        uniq = sorted(len(r["ops"]) for r in rs)
        union = set().union(*[set(r["ops"]) for r in rs])
        allops |= union
        L.append("| %s | %d | %d / %d / %d | %d / %d | %d |" % (f, len(rs), counts[0], counts[len(counts) // 2], counts[-1], uniq[0], uniq[-1], len(union)))
    L += ["", "Kernels: %d; distinct opcodes over the whole library: %d." % (len(rows), len(allops))]
    return "\n".join(L) + "\n"


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--out", default=None)
    a = ap.parse_args(argv)
    text = render(collect())
    if a.out:
        with open(a.out, "w") as f:
            f.write(text)
    else:
        sys.stdout.write(text)
    return 0


if __name__ == "__main__":
    sys.exit(main())
