"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle, element by element."""
import numpy as np
import pytest
import torch

import paper_2505_03780_amd as A
import workloads as W
from attn_testlib import DeviceWorkload, assert_close, check_full, oracle_problem, to_host_f64

import oracle

pytestmark = pytest.mark.gpu

RAGGED = [1, 31, 32, 33, 63, 64, 65, 127, 129, 200, 257]


@pytest.fixture(autouse=True)
def _auto_instance():
    A.attn_force_instance(False, -1)
    A.attn_force_instance(True, -1)
    yield
    A.attn_force_instance(False, -1)
    A.attn_force_instance(True, -1)


def _valid_instances(dw, is_decode):
    ids = []
    a = dw.args(is_decode)
    for i in range(A.attn_num_instances(is_decode)):
        A.attn_force_instance(is_decode, i)
        if A.attn_selected_instance(a, is_decode) == i:
            ids.append(i)
    A.attn_force_instance(is_decode, -1)
    return ids


def test_config1_tiny_fp32_full():
    print("config 1: fp32, L=128, 4 heads, D=64", flush=True)
    check_full(W.config1())


def _paged_f32(seed, q_lens, kv_lens, Hq, Hkv, D, bs):
    """A paged fp32 workload: packed fp32 K/V scattered into a pool by a random block table (a pure
    copy); blocks and slots that no sequence owns hold NaN, so a read of them would show."""
    rng = np.random.default_rng(seed)
    kv_lens = np.asarray(kv_lens, np.int32)
    q_lens = np.asarray(q_lens, np.int32)
    qsl = np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int32)
    kvsl = np.concatenate([[0], np.cumsum(kv_lens)]).astype(np.int32)
    q = rng.standard_normal((int(qsl[-1]), Hq, D), dtype=np.float32)
    k = rng.standard_normal((int(kvsl[-1]), Hkv, D), dtype=np.float32)
    v = rng.standard_normal((int(kvsl[-1]), Hkv, D), dtype=np.float32)
    nb = int(np.sum((kv_lens + bs - 1) // bs)) + 3
    table = W._block_table(rng, kv_lens, bs, nb, int((kv_lens.max() + bs - 1) // bs) + 1)
    kp, vp = W.scatter_to_pool(k, v, kvsl, kv_lens, table, bs, nb, fill=np.float32("nan"))
    scale = float(np.float32(1.0 / np.sqrt(np.float32(D))))
    paged = W.Workload("paged_f32", "prefill", "f32", q, kp, vp, qsl, kv_lens.copy(), scale, True, block_table=table, block_size=bs)
    contig = W.Workload("contig_f32", "prefill", "f32", q, k, v, qsl, kv_lens.copy(), scale, True, kv_start_loc=kvsl)
    return paged, contig


@pytest.mark.parametrize("D", [64, 128])
def test_fp32_varlen_gqa_and_paged(D):
    wl = W.make_prefill_contiguous(11, [1, 5, 64, 65, 130], 4, 2, D, dtype="f32")
    check_full(wl)
    wl = W.make_prefill_contiguous(12, [7, 70], 2, 2, D, dtype="f32", causal=False)
    check_full(wl)
    # the fp32 kernel's block-table branch: chunked prefill over a paged prefix, block sizes 16 and 32;
    # the same tokens in the contiguous layout give the same bits (same kernel, same summation order)
    for bs in (16, 32):
        paged, contig = _paged_f32(13 + bs, [1, 40, 17, 33], [1, 100, 17, 65], 4, 2, D, bs)
        check_full(paged, what="paged fp32 bs %d" % bs)
        a = to_host_f64(DeviceWorkload(paged).run(False))
        b = to_host_f64(DeviceWorkload(contig).run(False))
        assert np.array_equal(a, b), "paged and contiguous fp32 outputs differ"


@pytest.mark.parametrize("Hq,Hkv,D", [(8, 2, 128), (4, 4, 128), (4, 2, 128), (6, 2, 128), (8, 2, 64), (2, 2, 64)])
def test_prefill_contiguous_ragged_every_instance(Hq, Hkv, D):
    wl = W.make_prefill_contiguous(21, RAGGED, Hq, Hkv, D)
    dw = DeviceWorkload(wl)
    ref = oracle.attention(oracle_problem(wl))
    ids = _valid_instances(dw, False)
    assert ids, "no instance for this shape"
    for i in ids:
        print("prefill instance", i, A.attn_instance_name(False, i), "Hq", Hq, "Hkv", Hkv, "D", D, flush=True)
        A.attn_force_instance(False, i)
        got = to_host_f64(dw.run(False))
        assert_close(got, ref, "bf16", A.attn_instance_name(False, i))


def test_prefill_non_causal_and_peaked():
    wl = W.make_prefill_contiguous(22, [50, 129, 300], 8, 2, 128, causal=False)
    check_full(wl)
    # peaked softmax (scores ~ N(0, 36)): max-abs becomes a meaningful bound
    wl = W.make_prefill_contiguous(23, [200, 333], 8, 2, 128, scale=6.0 / np.sqrt(128.0))
    check_full(wl)


def test_prefill_with_empty_sequences_in_batch():
    wl = W.make_prefill_contiguous(24, [0, 70, 0, 5, 0], 8, 2, 128)
    check_full(wl)


def _chunked(seed, q_lens, kv_lens, Hq=8, Hkv=2, D=128, bs=16, nb=None):
    nb = nb or int(sum((n + bs - 1) // bs for n in kv_lens)) + 5
    return W.make_paged(seed, "prefill", q_lens, kv_lens, Hq, Hkv, D, bs, nb)


def test_chunked_prefill_over_paged_prefix_every_instance():
    wl = _chunked(31, [64, 1, 33, 100, 17, 128], [64, 90, 33, 500, 270, 1000])
    dw = DeviceWorkload(wl)
    ref = oracle.attention(oracle_problem(wl))
    for i in _valid_instances(dw, False):
        print("chunked prefill instance", i, A.attn_instance_name(False, i), flush=True)
        A.attn_force_instance(False, i)
        assert_close(to_host_f64(dw.run(False)), ref, "bf16", A.attn_instance_name(False, i))


@pytest.mark.parametrize("bs", [16, 32, 128])
def test_paged_block_sizes(bs):
    wl = _chunked(32, [40, 70], [100, 333], bs=bs)
    check_full(wl)
    wl = W.make_paged(33, "decode", [1, 1, 1], [1, 77, 600], 8, 2, 128, bs, 64)
    check_full(wl)
    # every decode and prefill instance, with eight KV heads so that all kernel families apply
    wl = W.make_paged(34, "decode", [1, 1, 1, 1], [1, 77, 600, 129], 32, 8, 128, bs, 64)
    dw = DeviceWorkload(wl)
    ref = oracle.attention(oracle_problem(wl))
    for i in _valid_instances(dw, True):
        A.attn_force_instance(True, i)
        assert_close(to_host_f64(dw.run(True)), ref, "bf16", "bs %d %s" % (bs, A.attn_instance_name(True, i)))
    A.attn_force_instance(True, -1)
    wl = _chunked(35, [40, 70, 1], [100, 333, 65], Hq=32, Hkv=8, bs=bs)
    dw = DeviceWorkload(wl)
    ref = oracle.attention(oracle_problem(wl))
    for i in _valid_instances(dw, False):
        A.attn_force_instance(False, i)
        assert_close(to_host_f64(dw.run(False)), ref, "bf16", "bs %d %s" % (bs, A.attn_instance_name(False, i)))


DECODE_LENS = [1, 15, 16, 17, 31, 32, 33, 100, 255, 256, 257, 700, 1500]


@pytest.mark.parametrize("Hq,Hkv,D", [(32, 8, 128), (16, 2, 128), (4, 4, 128), (8, 2, 64)])
def test_decode_every_instance(Hq, Hkv, D):
    wl = W.make_paged(41, "decode", np.ones(len(DECODE_LENS), np.int32), DECODE_LENS, Hq, Hkv, D, 16, 400)
    dw = DeviceWorkload(wl)
    ref = oracle.attention(oracle_problem(wl))
    ids = _valid_instances(dw, True)
    assert ids
    for i in ids:
        print("decode instance", i, A.attn_instance_name(True, i), "Hq", Hq, "Hkv", Hkv, "D", D, flush=True)
        A.attn_force_instance(True, i)
        assert_close(to_host_f64(dw.run(True)), ref, "bf16", A.attn_instance_name(True, i))


def test_decode_peaked_and_one_short_sequence_with_many_splits():
    lens = [1] + [3000] * 3
    wl = W.make_paged(42, "decode", np.ones(4, np.int32), lens, 32, 8, 128, 16, 600, scale=5.0 / np.sqrt(128.0))
    dw = DeviceWorkload(wl)
    ref = oracle.attention(oracle_problem(wl))
    for i in _valid_instances(dw, True):
        A.attn_force_instance(True, i)
        assert_close(to_host_f64(dw.run(True)), ref, "bf16", A.attn_instance_name(True, i))


def test_decode_two_batches_take_turns_on_one_workspace():
    """Nothing a decode call leaves in the workspace may matter to the next one, whatever its shape."""
    big = W.make_paged(43, "decode", np.ones(6, np.int32), [3000, 1, 2500, 40, 1777, 900], 32, 8, 128, 16, 700)
    small = W.make_paged(44, "decode", np.ones(3, np.int32), [513, 64, 1200], 32, 8, 128, 16, 200)
    dwb, dws = DeviceWorkload(big), DeviceWorkload(small)
    refb, refs = oracle.attention(oracle_problem(big)), oracle.attention(oracle_problem(small))
    dwb.args(True)
    dws.ws = dwb.ws  # large enough for the smaller batch: args() keeps it
    for i in _valid_instances(dwb, True):
        A.attn_force_instance(True, i)
        for rep in range(2):
            assert_close(to_host_f64(dwb.run(True)), refb, "bf16", "big %d rep %d" % (i, rep))
            assert_close(to_host_f64(dws.run(True)), refs, "bf16", "small %d rep %d" % (i, rep))
    assert dws.ws is dwb.ws


def test_decode_writes_zeros_for_contexts_without_keys():
    lens = [1, 700, 1, 1500, 33]
    wl = W.make_paged(45, "decode", np.ones(5, np.int32), lens, 32, 8, 128, 16, 300)
    dw = DeviceWorkload(wl)
    ref = oracle.attention(oracle_problem(wl))
    dw.seq_lens[0] = 0
    dw.seq_lens[2] = 0
    for i in _valid_instances(dw, True):
        name = A.attn_instance_name(True, i)
        A.attn_force_instance(True, i)
        got = to_host_f64(dw.run(True))
        assert np.all(got[0] == 0) and np.all(got[2] == 0), name
        assert_close(got[[1, 3, 4]], ref[[1, 3, 4]], "bf16", name)


# ---- the benchmark configurations at full size ------------------------------------------------

def _tuned(dw, is_decode):
    """Tunes the workload's bucket the way bench.py does (its own lengths, few iterations) and returns
    the name of the instance hot calls now take."""
    a = dw.args(is_decode)
    A.attn_tune(a, is_decode, None, 5, 0)
    return A.attn_instance_name(is_decode, A.attn_selected_instance(a, is_decode))


def _check_rows(wl, dw, seqs, toks, heads, what):
    out = dw.run()
    assert bool(torch.isfinite(out.float()).all()), "%s: unwritten or non-finite output rows" % what
    ref = oracle.attention_rows(oracle_problem(wl), seqs, toks, heads)
    rows = torch.from_numpy(wl.query_start_loc[seqs].astype(np.int64) + toks).cuda()
    got = to_host_f64(out[rows, torch.from_numpy(heads.astype(np.int64)).cuda()])
    return assert_close(got, ref, wl.dtype, what)


def _full_then_tuned(wl, is_decode):
    """Every output element of the built-in choice against the oracle, then the tuner's winner (the
    instance bench.py times) the same way."""
    dw = DeviceWorkload(wl)
    ref = oracle.attention(oracle_problem(wl))
    qsl = wl.query_start_loc

    def compare(what):
        got = to_host_f64(dw.run(is_decode))
        for s in range(wl.num_seqs):
            assert_close(got[qsl[s]:qsl[s + 1]], ref[qsl[s]:qsl[s + 1]], wl.dtype, "%s seq %d" % (what, s))
        print(what, "max-abs %.3e rel-RMS %.3e" % assert_close(got, ref, wl.dtype, what), flush=True)

    a = dw.args(is_decode)
    builtin = A.attn_instance_name(is_decode, A.attn_selected_instance(a, is_decode))
    compare("%s built-in %s" % (wl.name, builtin))
    try:
        winner = _tuned(dw, is_decode)
        compare("%s tuned %s" % (wl.name, winner))
    finally:
        A.attn_clear_cache()
    return builtin


def test_config2_decode_8b_full_size():
    print("config 2: paged decode, batch 64, ctx U[512,4096], every output element", flush=True)
    _full_then_tuned(W.config2(), True)


def test_config3_prefill_8b_full_size():
    print("config 3: varlen prefill, 8 sequences U[256,2048], every output element", flush=True)
    _full_then_tuned(W.config3(), False)


def test_config4_chunked_prefill_full_size():
    """Config 4 is 717 GFLOP (about a minute of fp64 oracle time): every sequence is covered, with one
    row per query head and run of 32 tokens (no query tile of any kernel escapes) plus the first and
    last token of every sequence for every head; built-in choice and tuner's winner."""
    print("config 4: chunked prefill over paged prefix, stratified rows of every sequence", flush=True)
    wl = W.config4()
    dw = DeviceWorkload(wl)
    seqs, toks, heads = W.stratified_rows(wl, 32)
    assert len(seqs) == 16 * (16 + 2) * 32 and set(seqs.tolist()) == set(range(16))
    a = dw.args(False)
    builtin = A.attn_instance_name(False, A.attn_selected_instance(a, False))
    print("built-in", builtin, _check_rows(wl, dw, seqs, toks, heads, "config 4 built-in " + builtin), flush=True)
    try:
        winner = _tuned(dw, False)
        print("tuned", winner, _check_rows(wl, dw, seqs, toks, heads, "config 4 tuned " + winner), flush=True)
    finally:
        A.attn_clear_cache()


def test_config5_decode_70b_long_full_size():
    print("config 5: long-context paged decode, split-K, every output element", flush=True)
    name = _full_then_tuned(W.config5(), True)
    assert "split0" not in name, "long contexts must take the split-K path, got " + name


@pytest.mark.parametrize("B", [333, 4200])
def test_decode_large_batches_of_short_contexts(B):
    """Many sequences per workgroup run: both ways of taking the chunk prefix sums (up to 4096
    sequences one block per lane, beyond that a loop over the batch), a few empty contexts' worth of
    one-key sequences, every token-balanced instance."""
    rng = np.random.default_rng(B)
    lens = rng.integers(1, 70, size=B).astype(np.int32)
    lens[::17] = 1
    wl = W.make_paged(50 + B, "decode", np.ones(B, np.int32), lens, 8, 4, 128, 16, int(np.sum((lens + 15) // 16)) + 3)
    dw = DeviceWorkload(wl)
    ref = oracle.attention(oracle_problem(wl))
    ids = [i for i in _valid_instances(dw, True) if "balanced" in A.attn_instance_name(True, i)]
    assert ids
    for i in ids:
        A.attn_force_instance(True, i)
        assert_close(to_host_f64(dw.run(True)), ref, "bf16", "B %d %s" % (B, A.attn_instance_name(True, i)))
