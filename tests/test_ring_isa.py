"""Static hazard check of the ring prefill kernels (see ring_isa_lint.py): no instruction may touch a
register while one of the loop's untracked LDS reads, or its untracked scalar load, may still be in
flight into it.  Runs on the CPU: hipcc cross-compiles the two translation units to assembly."""
import concurrent.futures as cf
import os
import subprocess

import ring_isa_lint as L

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2505_03780_amd", "csrc")


def _asm(src, out):
    from paper_2505_03780_amd import build as B

    cmd = ["hipcc", *B.FLAGS, *B.EXTRA.get(src, []), "-S", "--cuda-device-only", os.path.join(CSRC, src), "-o", out]
    subprocess.check_call(cmd, stderr=subprocess.DEVNULL)
    return open(out).read()


def test_no_register_is_touched_while_an_untracked_load_may_land_in_it(tmp_path):
    srcs = ["prefill_bf16_ring.hip", "prefill_f16_ring.hip"]
    with cf.ThreadPoolExecutor(max_workers=2) as ex:
        texts = list(ex.map(lambda s: _asm(s, str(tmp_path / s.replace(".hip", ".s"))), srcs))
    seen = 0
    for text in texts:
        for name, body in L.kernels(text):
            if "prefill_ring_kernel" not in name:
                continue
            seen += 1
            assert any(l.startswith("ds_read_b64_tr_b16") for l in body), name  # the kernel the check is about
            problems = L.lint(body)
            assert not problems, (name, problems[:5])
    assert seen >= 20


def test_the_check_sees_a_planted_hazard():
    body = ["s_waitcnt lgkmcnt(0)", ";;#ASMSTART", "ds_read_b128 v[4:7], v1 offset:0", ";;#ASMEND", "ds_read_b128 v[8:11], v1 offset:16",
            "s_waitcnt lgkmcnt(1)", "v_add_f32_e32 v0, v4, v5", "v_mov_b32_e32 v9, 0", "s_waitcnt lgkmcnt(0)", "v_add_f32_e32 v0, v8, v9"]
    problems = L.lint(body)
    assert [p[0] for p in problems] == [7]  # only the write into v9 while the second read is in flight
    loop = [".LBB0_1:", "v_add_f32_e32 v0, v4, v4", "ds_read_b128 v[4:7], v1 offset:0", "s_cbranch_scc1 .LBB0_1", "s_waitcnt lgkmcnt(0)", "s_endpgm"]
    problems = L.lint(loop)
    # seen on the second trip: the read of the previous trip is still in flight when v4 is used and when it is loaded again
    assert [p[0] for p in problems] == [1, 2]
