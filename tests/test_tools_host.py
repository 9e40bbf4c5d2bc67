"""Host test of the assembly statistics parser, on a hand-made sample."""
import os

from paper_2505_03780_amd import isa_stats

SAMPLE = """\t.text
\t.globl\t_ZN4attn12_GLOBAL__N_114rmsnorm_kernelILb0ELi64ELi2ELi4EEEvNS0_9RmsParamsE
_ZN4attn12_GLOBAL__N_114rmsnorm_kernelILb0ELi64ELi2ELi4EEEvNS0_9RmsParamsE: ; @kernel
; %bb.0:
\ts_load_dwordx2 s[0:1], s[4:5], 0x0
\ts_waitcnt lgkmcnt(0)
\tglobal_load_dwordx4 v[0:3], v[4:5], off nt
\tv_mfma_f32_32x32x16_bf16 a[0:15], v[0:3], v[4:7], a[0:15]
\tds_read_b128 v[8:11], v12
\tv_add_f32_e32 v0, v1, v2
\tv_add_f32_e32 v0, v0, v3
\ts_endpgm
\t.section\t.rodata,"a",@progbits
\t.amdhsa_kernel _ZN4attn12_GLOBAL__N_114rmsnorm_kernelILb0ELi64ELi2ELi4EEEvNS0_9RmsParamsE
\t\t.amdhsa_group_segment_fixed_size 4096
\t\t.amdhsa_private_segment_fixed_size 0
\t\t.amdhsa_next_free_vgpr 48
\t\t.amdhsa_next_free_sgpr 20
\t\t.amdhsa_accum_offset 32
\t.end_amdhsa_kernel
\t.text
.Lfunc_end0:
\t.size\tfoo, .Lfunc_end0-foo
"""


def test_parse_counts_instructions_and_reads_the_kernel_descriptor(tmp_path):
    path = os.path.join(tmp_path, "sample.s")
    with open(path, "w") as f:
        f.write(SAMPLE)
    parsed = list(isa_stats._parse(path))
    assert len(parsed) == 1
    name, ops, meta = parsed[0]
    assert name.endswith("RmsParamsE")
    assert sum(ops.values()) == 8 and len(ops) == 7          # v_add_f32_e32 twice; directives are not counted
    assert ops["v_add_f32_e32"] == 2 and ops["v_mfma_f32_32x32x16_bf16"] == 1
    assert meta == {"lds": 4096, "scratch": 0, "vgpr_total": 48, "accum_offset": 32, "sgpr": 20}
    row = {"tu": "sample", "kernel": "rmsnorm_kernel<false, 64, 2, 4>", "ops": ops, **meta}
    text = isa_stats.render([row])
    assert "| sample | rmsnorm_kernel<false, 64, 2, 4> | 8 | 7 | 1 | 1 | 1 | 48 (16) | 20 | 4096 | 0 |" in text
    assert "| rms norm | 1 | 8 / 8 / 8 | 7 / 7 | 7 |" in text
    assert isa_stats.family("decode_balanced_kernel<128, 8>") == "decode token-balanced"
