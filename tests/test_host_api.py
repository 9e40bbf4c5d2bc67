"""Host-side logic of the library, exercised without a GPU: exports, validation, buckets, cache."""
import ctypes
import os
import re

import pytest

import paper_2505_03780_amd as A

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _args(**kw):
    a = A.AttnArgs()
    a.struct_bytes = ctypes.sizeof(A.AttnArgs)
    a.dtype = A.ATTN_BF16
    a.num_seqs, a.num_q_heads, a.num_kv_heads, a.head_dim = 4, 32, 8, 128
    a.total_q, a.max_q_len, a.max_kv_len = 400, 100, 100
    a.q = a.out = a.k = a.v = 0x1000
    a.q_stride_tok = a.o_stride_tok = 32 * 128
    a.q_stride_head = a.o_stride_head = 128
    a.kv_stride_tok, a.kv_stride_head, a.kv_stride_block = 8 * 128, 128, 16 * 8 * 128
    a.query_start_loc = a.seq_lens = 0x2000
    a.scale, a.causal = 0.088, 1
    for k, v in kw.items():
        setattr(a, k, v)
    return a


def _paged(**kw):
    base = dict(block_table=0x3000, block_table_stride=64, block_size=16, num_blocks=1024)
    base.update(kw)
    return _args(**base)


def test_library_exports_every_declared_symbol():
    names = set()
    for h in sorted(os.listdir(os.path.join(ROOT, "include"))):
        header = open(os.path.join(ROOT, "include", h)).read()
        header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        names |= set(re.findall(r"\b((?:attn|rmsnorm)_[a-z_]+)\s*\(", header))
    assert {"attn_prefill_varlen", "attn_decode_paged", "attn_tune", "attn_workspace_bytes", "rmsnorm_fused_add", "rmsnorm_tune"} <= names
    lib = A.load_library()
    for n in sorted(names):
        assert hasattr(lib, n), "missing export " + n


def test_struct_layout_matches_and_workspace_bytes():
    a = _paged(total_q=4, max_q_len=1, max_kv_len=4096)
    # The largest need of any instance that may run (256 compute units assumed without a device).
    # Fixed splits: at most 64 parts per context and two parts per compute unit over the batch, here
    # 4 seqs * 32 heads * ceil(4096/128) parts * (128 + 2) floats.  Token-balanced: at most two
    # workgroups per compute unit, (512 workgroups + 4 seqs) * 32 heads * 130 floats + 5 chunk prefix sums.
    fixed = 4 * 32 * 32 * 130 * 4
    balanced = (512 + 4) * 32 * 130 * 4 + 5 * 4
    assert A.attn_workspace_bytes(a, True) == max(fixed, balanced)
    # 64 long contexts: no fixed split with at most 512 parts in all is finer than 4096 keys (8 parts each)
    long = _paged(num_seqs=64, total_q=64, max_q_len=1, max_kv_len=32768, block_table_stride=2048)
    assert A.attn_workspace_bytes(long, True) == max(64 * 32 * 8 * 130 * 4, (512 + 64) * 32 * 130 * 4 + 65 * 4)
    # the two decode configurations of the benchmark: what the caller must provide stays near what runs
    c2 = _paged(num_seqs=64, total_q=64, max_q_len=1, max_kv_len=4071, block_table_stride=256)
    assert A.attn_workspace_bytes(c2, True) <= 10 * 1000 * 1000
    c5 = _paged(num_seqs=16, total_q=16, max_q_len=1, max_kv_len=32672, block_table_stride=2048, num_q_heads=64)
    assert A.attn_workspace_bytes(c5, True) <= 20 * 1000 * 1000
    # pointer fields are ignored
    assert A.attn_workspace_bytes(_paged(total_q=4, max_q_len=1, max_kv_len=4096, block_table=None), True) == max(fixed, balanced)
    assert A.attn_workspace_bytes(a, False) == 0
    a.struct_bytes += 8
    assert A.attn_workspace_bytes(a, True) == 0


def test_status_strings():
    assert A.attn_status_string(0) == "ok"
    for code in range(-7, 0):
        assert A.attn_status_string(code) not in ("ok", "unknown status")
    assert A.attn_status_string(-99) == "unknown status"


@pytest.mark.parametrize("mutate,decode,code", [
    (dict(struct_bytes=8), False, -2),
    (dict(dtype=7), False, -3),
    (dict(dtype=A.ATTN_F32), True, -3),
    (dict(num_kv_heads=5), False, -2),
    (dict(head_dim=96), False, -4),
    (dict(q=None), False, -1),
    (dict(seq_lens=None), False, -1),
    (dict(query_start_loc=None), False, -1),
    (dict(q_stride_tok=32 * 128 + 4), False, -2),
    (dict(q=0x1008), False, -2),
    (dict(q_stride_head=64), False, -2),
])
def test_validation_errors_without_touching_the_device(mutate, decode, code):
    lib = A.load_library()
    a = _args(**mutate)
    fn = lib.attn_decode_paged if decode else lib.attn_prefill_varlen
    assert fn(a, None) == code


def test_validation_of_paged_arguments():
    lib = A.load_library()
    assert lib.attn_decode_paged(_args(total_q=4, max_q_len=1), None) == -1  # decode needs a block table
    assert lib.attn_decode_paged(_paged(total_q=5, max_q_len=1), None) == -2  # one token per sequence
    assert lib.attn_prefill_varlen(_paged(block_size=24), None) == -4
    assert lib.attn_prefill_varlen(_paged(block_size=8), None) == -4
    assert lib.attn_prefill_varlen(_paged(max_kv_len=64 * 16 + 1), None) == -2  # table too narrow
    assert lib.attn_prefill_varlen(None, None) == -1
    # empty batches are fine and enqueue nothing
    assert lib.attn_prefill_varlen(_args(num_seqs=0, total_q=0, q=None, out=None), None) == 0


def test_instance_tables_and_heuristic_selection():
    names_p = [A.attn_instance_name(False, i) for i in range(A.attn_num_instances(False))]
    names_d = [A.attn_instance_name(True, i) for i in range(A.attn_num_instances(True))]
    assert len(set(names_p)) == len(names_p) and len(set(names_d)) == len(names_d)
    with pytest.raises(A.AttnError):
        A.attn_instance_name(False, len(names_p))
    A.attn_clear_cache()
    A.attn_force_instance(False, -1)
    A.attn_force_instance(True, -1)
    # GQA 32/8 prefill packs the 4 heads of a KV head into one workgroup; short sequences take the
    # small workgroups (two per compute unit), long ones the large ring and the sequence-major grid
    i = A.attn_selected_instance(_args(), False)
    assert "hpw4" in names_p[i] and "d128" in names_p[i] and "w4" in names_p[i] and "seqmajor" not in names_p[i]
    i = A.attn_selected_instance(_args(max_kv_len=8192, max_q_len=8192), False)
    assert "hpw4" in names_p[i] and "w8" in names_p[i] and "seqmajor" in names_p[i]
    i = A.attn_selected_instance(_paged(max_kv_len=1536, max_q_len=512), False)  # a cached prefix twice the chunk
    assert "seqmajor" in names_p[i]
    # a long paged context: the large ring with the deepest prefetch (the table entry lengthens the address chain)
    i = A.attn_selected_instance(_paged(max_kv_len=8704, max_q_len=512, block_table_stride=544), False)
    assert names_p[i] == "prefill_bf16_ring d128 qb1 w8 hpw4 slots8 pf8 seqmajor"
    i = A.attn_selected_instance(_args(max_kv_len=8192, max_q_len=8192), False)
    assert names_p[i] == "prefill_bf16_ring d128 qb1 w8 hpw4 slots8 pf5 seqmajor"
    # a cache whose blocks lie 4 GiB or more apart: the ring kernel's transfers do their block arithmetic
    # in 32 bits, so the choice falls to the register-staged kernel
    i = A.attn_selected_instance(_paged(max_kv_len=8704, max_q_len=512, block_table_stride=544, kv_stride_block=1 << 31, num_blocks=4), False)
    assert "ring" not in names_p[i] and "d128" in names_p[i]
    # MHA cannot
    i = A.attn_selected_instance(_args(num_kv_heads=32), False)
    assert "hpw1" in names_p[i]
    # head_dim 64 picks a d64 instance
    i = A.attn_selected_instance(_args(head_dim=64), False)
    assert "d64" in names_p[i]
    # long-context decode with few sequences takes split-K; short contexts do not split
    long = _paged(num_seqs=16, total_q=16, max_q_len=1, max_kv_len=32768, block_table_stride=2048, num_q_heads=64)
    assert "split0" not in names_d[A.attn_selected_instance(long, True)]
    # with eight KV heads the default is the token-balanced kernel (one workgroup per compute unit)
    assert "balanced" in names_d[A.attn_selected_instance(long, True)]
    short = _paged(num_seqs=512, total_q=512, max_q_len=1, max_kv_len=200)
    assert "balanced" in names_d[A.attn_selected_instance(short, True)]
    # a small batch of short contexts: one KV head per workgroup, fixed parts
    small = _paged(num_seqs=4, total_q=4, max_q_len=1, max_kv_len=4096, block_table_stride=256)
    assert names_d[A.attn_selected_instance(small, True)].startswith("decode_bf16 d128 w4 split")
    # one long context: parts long enough that the merge takes them in one round trip (32), eight waves
    one_long = _paged(num_seqs=1, total_q=1, max_q_len=1, max_kv_len=16384, block_table_stride=1024)
    assert names_d[A.attn_selected_instance(one_long, True)] == "decode_bf16 d128 w8 split512"
    one_mid = _paged(num_seqs=1, total_q=1, max_q_len=1, max_kv_len=4096, block_table_stride=256)
    assert names_d[A.attn_selected_instance(one_mid, True)] == "decode_bf16 d128 w4 split256"
    few_heads = _paged(num_seqs=512, total_q=512, max_q_len=1, max_kv_len=200, num_q_heads=4, num_kv_heads=1)
    assert "split0" in names_d[A.attn_selected_instance(few_heads, True)]
    # a forced instance that does not fit the shape is refused, not silently replaced
    d64 = next(i for i, n in enumerate(names_p) if "d64" in n)
    A.attn_force_instance(False, d64)
    assert A.attn_selected_instance(_args(), False) == -4
    A.attn_force_instance(False, -1)


def test_cache_file_round_trip_stale_and_corrupt(tmp_path):
    names_p = [A.attn_instance_name(False, i) for i in range(A.attn_num_instances(False))]
    A.attn_clear_cache()
    default = A.attn_selected_instance(_args(), False)
    other = next(i for i, n in enumerate(names_p) if "d128" in n and "hpw1" in n and i != default)
    key = "prefill|bf16|d128|hq32|hkv8|contig|bs0|c1|B2|q7|kv7"
    env_here = A.attn_environment_key()
    import torch
    if not torch.cuda.is_available():  # what the library reports in a process without a GPU
        assert re.fullmatch(r"nodevice\|cu0\|k[0-9a-f]{16}", env_here), env_here
    good = tmp_path / "cache.txt"
    good.write_text("attn-tune-cache-v1\n%s\t%s\t%s\t12.5\n" % (env_here, key, names_p[other]))
    assert A.attn_load_cache(str(good)) == 0
    assert A.attn_selected_instance(_args(), False) == other
    # another bucket is untouched: it keeps the built-in choice for its own shape
    far = _args(max_kv_len=5000, max_q_len=5000)
    assert A.attn_selected_instance(far, False) != other
    assert "seqmajor" in names_p[A.attn_selected_instance(far, False)] and "w8" in names_p[A.attn_selected_instance(far, False)]
    A.attn_clear_cache()
    assert A.attn_selected_instance(_args(), False) == default
    # stale environment (another device / build): entry ignored
    stale = tmp_path / "stale.txt"
    stale.write_text("attn-tune-cache-v1\ngfx942|cu304|hip0|k0\t%s\t%s\t12.5\n" % (key, names_p[other]))
    assert A.attn_load_cache(str(stale)) == 0
    assert A.attn_selected_instance(_args(), False) == default
    # unknown instance name: ignored
    unk = tmp_path / "unk.txt"
    unk.write_text("attn-tune-cache-v1\n%s\t%s\tno such kernel\t1\n" % (env_here, key))
    assert A.attn_load_cache(str(unk)) == 0
    assert A.attn_selected_instance(_args(), False) == default
    # corrupt and missing files report an error and change nothing
    bad = tmp_path / "bad.txt"
    bad.write_text("garbage\n")
    assert A.attn_load_cache(str(bad)) == -7
    bad.write_text("attn-tune-cache-v1\nonly\ttwo\n")
    assert A.attn_load_cache(str(bad)) == -7  # nothing but damage
    # one damaged line in the middle: the lines around it still count
    mixed = tmp_path / "mixed.txt"
    key2 = "prefill|bf16|d128|hq32|hkv8|contig|bs0|c1|B2|q13|kv13"
    mixed.write_text("attn-tune-cache-v1\n%s\t%s\t%s\t12.5\n\x00\x01garbage without tabs\n%s\t%s\t%s\t7\n" % (
        env_here, key, names_p[other], env_here, key2, names_p[other]))
    assert A.attn_load_cache(str(mixed)) == 0
    assert A.attn_selected_instance(_args(), False) == other
    assert A.attn_selected_instance(_args(max_kv_len=5000, max_q_len=5000), False) == other
    A.attn_clear_cache()
    assert A.attn_load_cache(str(tmp_path / "missing.txt")) == -7
    assert A.attn_selected_instance(_args(), False) == default


def test_tune_rejects_bad_requests_before_touching_the_device():
    lib = A.load_library()
    assert lib.attn_tune(None, 0, None, 1, 0) == -1
    assert lib.attn_tune(_args(dtype=A.ATTN_F32), 0, None, 1, 0) == -3
    assert lib.attn_tune(_args(head_dim=80), 0, None, 1, 0) == -4
    assert lib.attn_tune(_args(num_kv_heads=5), 0, None, 1, 0) == -2


def _rms(**kw):
    a = A.RmsNormArgs()
    a.struct_bytes = ctypes.sizeof(A.RmsNormArgs)
    a.dtype, a.num_tokens, a.hidden = A.ATTN_BF16, 128, 4096
    a.x, a.weight, a.out, a.residual = 0x10000, 0x20000, 0x30000, 0x40000
    a.x_stride = a.out_stride = a.residual_stride = 4096
    a.eps = 1e-5
    for k, v in kw.items():
        setattr(a, k, v)
    return a


def test_rmsnorm_validation_and_selection_on_the_host():
    lib = A.load_library()
    assert ctypes.sizeof(A.RmsNormArgs) == 80
    assert lib.rmsnorm_fused_add(None, None) == -1
    assert lib.rmsnorm_fused_add(_rms(struct_bytes=8), None) == -2
    assert lib.rmsnorm_fused_add(_rms(dtype=A.ATTN_F32), None) == -3
    assert lib.rmsnorm_fused_add(_rms(hidden=4100), None) == -4
    assert lib.rmsnorm_fused_add(_rms(hidden=32768, x_stride=32768, out_stride=32768, residual_stride=32768), None) == -4
    assert lib.rmsnorm_fused_add(_rms(x=None), None) == -1
    assert lib.rmsnorm_fused_add(_rms(x_stride=4000), None) == -2
    assert lib.rmsnorm_fused_add(_rms(out=0x30008), None) == -2  # not 16-byte aligned
    assert lib.rmsnorm_fused_add(_rms(num_tokens=0, x=None, out=None), None) == 0  # nothing to do
    names = [A.rmsnorm_instance_name(i) for i in range(A.rmsnorm_num_instances())]
    assert len(set(names)) == len(names) >= 10
    # the row is spread over as many lanes as it has 16-byte vectors (one vector per lane), up to 1024
    assert names[A.rmsnorm_selected_instance(_rms(num_tokens=8192))] == "rmsnorm tpr512 vpt1 rows1"
    assert names[A.rmsnorm_selected_instance(_rms(hidden=8192, x_stride=8192, out_stride=8192, residual_stride=8192))] == "rmsnorm tpr1024 vpt1 rows1"
    assert names[A.rmsnorm_selected_instance(_rms(hidden=1024))] == "rmsnorm tpr256 vpt1 rows1"
    # mid-size calls (tens of MB of traffic, rows of at most 4096): four vectors per lane, 256-lane workgroups
    assert names[A.rmsnorm_selected_instance(_rms(num_tokens=2048))] == "rmsnorm tpr128 vpt4 rows2"
    assert names[A.rmsnorm_selected_instance(_rms(num_tokens=8192, hidden=1024))] == "rmsnorm tpr32 vpt4 rows8"
    assert names[A.rmsnorm_selected_instance(_rms(hidden=16384, x_stride=16384, out_stride=16384, residual_stride=16384))] == "rmsnorm tpr1024 vpt2 rows1"
    # every supported hidden size has at least one instance; a forced one that does not fit is refused
    for h in range(8, 16385, 8):
        assert A.rmsnorm_selected_instance(_rms(hidden=h, x_stride=h, out_stride=h, residual_stride=h)) >= 0, h
    A.rmsnorm_force_instance(names.index("rmsnorm tpr64 vpt2 rows4"))
    assert A.rmsnorm_selected_instance(_rms()) == -4
    A.rmsnorm_force_instance(-1)
    assert lib.rmsnorm_tune(None, None, 1, 0) == -1
    assert lib.rmsnorm_tune(_rms(hidden=12), None, 1, 0) == -4


def test_kv_cache_write_validation_on_the_host():
    lib = A.load_library()
    a = A.KvWriteArgs()
    a.struct_bytes = ctypes.sizeof(A.KvWriteArgs)
    assert a.struct_bytes == 112
    a.dtype, a.num_tokens, a.num_kv_heads, a.head_dim, a.block_size, a.num_blocks = A.ATTN_BF16, 4, 8, 128, 16, 10
    a.k_new = a.v_new = 0x1000
    a.k_cache = a.v_cache = 0x2000
    a.slot_mapping = 0x3000
    a.new_stride_tok, a.new_stride_head = 1024, 128
    a.kv_stride_block, a.kv_stride_tok, a.kv_stride_head = 16 * 1024, 1024, 128
    assert lib.attn_kv_cache_write(None, None) == -1
    bad = A.KvWriteArgs.from_buffer_copy(a); bad.struct_bytes = 8
    assert lib.attn_kv_cache_write(bad, None) == -2
    bad = A.KvWriteArgs.from_buffer_copy(a); bad.dtype = 7
    assert lib.attn_kv_cache_write(bad, None) == -3
    bad = A.KvWriteArgs.from_buffer_copy(a); bad.head_dim = 100  # 200 bytes per head row
    assert lib.attn_kv_cache_write(bad, None) == -4
    bad = A.KvWriteArgs.from_buffer_copy(a); bad.slot_mapping = None
    assert lib.attn_kv_cache_write(bad, None) == -1
    bad = A.KvWriteArgs.from_buffer_copy(a); bad.kv_stride_tok = 100
    assert lib.attn_kv_cache_write(bad, None) == -2
    bad = A.KvWriteArgs.from_buffer_copy(a); bad.num_tokens = 0; bad.k_new = None
    assert lib.attn_kv_cache_write(bad, None) == 0


def test_selection_memo_follows_cache_changes(tmp_path):
    """The per-thread memo of the last selection must not outlive a change of the winner table."""
    names_p = [A.attn_instance_name(False, i) for i in range(A.attn_num_instances(False))]
    A.attn_clear_cache()
    default = A.attn_selected_instance(_args(), False)
    assert A.attn_selected_instance(_args(), False) == default  # memoised answer
    other = next(i for i, n in enumerate(names_p) if "bf16_ring" in n and "hpw1" in n and i != default)
    f = tmp_path / "c.txt"
    f.write_text("attn-tune-cache-v1\n%s\tprefill|bf16|d128|hq32|hkv8|contig|bs0|c1|B2|q7|kv7\t%s\t1.0\n" % (A.attn_environment_key(), names_p[other]))
    assert A.attn_load_cache(str(f)) == 0
    assert A.attn_selected_instance(_args(), False) == other
    A.attn_clear_cache()
    assert A.attn_selected_instance(_args(), False) == default
    A.attn_force_instance(False, other)
    assert A.attn_selected_instance(_args(), False) == other
    A.attn_force_instance(False, -1)
    assert A.attn_selected_instance(_args(), False) == default
    # a different shape is not answered from the memo of the previous one
    assert "w8" in names_p[A.attn_selected_instance(_args(max_kv_len=8192, max_q_len=8192), False)]
    assert A.attn_selected_instance(_args(), False) == default


def test_environment_knobs_force_and_log_in_a_fresh_process():
    """ATTN_FORCE_INSTANCE and ATTN_LOG are read once per process, so they are checked in a child."""
    import subprocess
    import sys

    code = (
        "import sys; sys.path.insert(0, %r); sys.path.insert(0, %r)\n"
        "import test_host_api as T, paper_2505_03780_amd as A\n"
        "d = A.attn_selected_instance(T._paged(total_q=4, max_q_len=1, max_kv_len=4096), True)\n"
        "p = A.attn_selected_instance(T._args(), False)\n"
        "s = A.attn_selected_instance(T._paged(total_q=4, max_q_len=1, max_kv_len=4096, head_dim=64, q_stride_head=64, "
        "o_stride_head=64, kv_stride_head=64), True)\n"
        "print(A.attn_instance_name(True, d)); print(A.attn_instance_name(False, p)); print(A.attn_instance_name(True, s))\n"
    ) % (ROOT, os.path.join(ROOT, "tests"))
    env = dict(os.environ, ATTN_FORCE_INSTANCE="decode_bf16_seq d128 w8 split512", ATTN_LOG="1")
    env.pop("ATTN_TUNE_CACHE", None)
    r = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr
    out = r.stdout.strip().splitlines()
    assert out[0] == "decode_bf16_seq d128 w8 split512"          # forced where valid
    assert out[1].startswith("prefill_bf16_ring")                 # the other kind is untouched
    assert out[2].startswith("decode_bf16") and "d64" in out[2]   # not valid for D = 64: the usual choice
    log = [l for l in r.stderr.splitlines() if l.startswith("[attn] ")]
    assert len(log) == 3 and "ATTN_FORCE_INSTANCE" in log[0] and "(heuristic)" in log[1] and "decode|" in log[0].replace(" ", "|")
