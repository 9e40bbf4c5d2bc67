"""GPU invariants: properties that hold at any size and catch indexing and synchronisation slips."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_03780_amd as A
import workloads as W
from attn_testlib import DeviceWorkload, assert_close, oracle_problem, to_host_f64

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _auto_instance():
    A.attn_force_instance(False, -1)
    A.attn_force_instance(True, -1)
    yield
    A.attn_force_instance(False, -1)
    A.attn_force_instance(True, -1)


def _bits(t):
    return t.view(torch.int16).cpu().numpy().copy()


def test_paged_equals_contiguous_bit_exact_and_poison_is_ignored():
    lens = [1, 40, 64, 130, 300]
    wl = W.make_prefill_contiguous(51, lens, 8, 2, 128)
    base = _bits(DeviceWorkload(wl).run(False))
    # same tokens scattered into a pool through a random table
    rng = np.random.default_rng(52)
    bs, nb = 16, 64
    need = [(n + bs - 1) // bs for n in lens]
    perm = rng.permutation(nb).astype(np.int32)
    table = np.full((len(lens), max(need)), -1, np.int32)
    pos = 0
    for s, n in enumerate(need):
        table[s, :n] = perm[pos:pos + n]
        pos += n
    for fill in (None, np.uint16(0x7FC0)):  # ordinary values, then NaN in every unused slot and block
        kp, vp = W.scatter_to_pool(wl.k, wl.v, wl.kv_start_loc, wl.seq_lens, table, bs, nb, fill=fill, seed=53)
        t = table.copy()
        if fill is not None:
            t[t < 0] = 2**31 - 1  # unused table entries must never be read
        pw = W.Workload("paged", "prefill", "bf16", wl.q, kp, vp, wl.query_start_loc, wl.seq_lens, wl.scale, True,
                        block_table=t, block_size=bs)
        got = _bits(DeviceWorkload(pw).run(False))
        assert np.array_equal(base, got), "paged result differs from contiguous (fill=%r)" % (fill,)


def test_decode_poisoned_pool_and_table():
    lens = [1, 17, 250, 1000]
    wl = W.make_paged(54, "decode", np.ones(4, np.int32), lens, 32, 8, 128, 16, 100)
    base = _bits(DeviceWorkload(wl).run(True))
    k, v, bt = wl.k.copy(), wl.v.copy(), wl.block_table.copy()
    used = np.zeros(k.shape[:2], bool)
    for s, n in enumerate(lens):
        for j in range(n):
            used[bt[s, j // 16], j % 16] = True
    k[~used] = np.uint16(0x7FC0)
    v[~used] = np.uint16(0x7FC0)
    bt[bt < 0] = 2**31 - 1
    pw = W.Workload("poison", "decode", "bf16", wl.q, k, v, wl.query_start_loc, wl.seq_lens, wl.scale, True,
                    block_table=bt, block_size=16)
    assert np.array_equal(base, _bits(DeviceWorkload(pw).run(True)))


def test_repeated_runs_are_bit_identical():
    # a race in the LDS double buffering or the split-K merge would show up as run-to-run differences
    wl = W.make_prefill_contiguous(55, [500, 77, 260], 8, 2, 128)
    dw = DeviceWorkload(wl)
    first = _bits(dw.run(False))
    for _ in range(3):
        assert np.array_equal(first, _bits(dw.run(False)))
    wl = W.make_paged(56, "decode", np.ones(3, np.int32), [2000, 130, 999], 32, 8, 128, 16, 300)
    dw = DeviceWorkload(wl)
    first = _bits(dw.run(True))
    for _ in range(3):
        assert np.array_equal(first, _bits(dw.run(True)))


def test_decode_equals_last_prefill_row_and_split_count_invariance():
    lens = [300, 1000, 33]
    wl = W.make_paged(57, "decode", np.ones(3, np.int32), lens, 32, 8, 128, 16, 120)
    dw = DeviceWorkload(wl)
    ref = oracle.attention(oracle_problem(wl))
    outs = []
    for i in range(A.attn_num_instances(True)):
        A.attn_force_instance(True, i)
        if A.attn_selected_instance(dw.args(True), True) != i:
            continue
        outs.append(to_host_f64(dw.run(True)))
        assert_close(outs[-1], ref, "bf16", A.attn_instance_name(True, i))
    A.attn_force_instance(True, -1)
    spread = max(float(np.max(np.abs(o - outs[0]))) for o in outs)
    assert spread <= 2e-3, "split counts disagree by %.3e" % spread  # one bf16 ulp of values ~0.25
    # the same problem as a 1-token chunked prefill through the prefill entry point
    pw = W.Workload("as_prefill", "prefill", "bf16", wl.q, wl.k, wl.v, wl.query_start_loc, wl.seq_lens, wl.scale, True,
                    block_table=wl.block_table, block_size=16)
    assert_close(to_host_f64(DeviceWorkload(pw).run(False)), ref, "bf16", "decode via prefill entry point")


def test_strided_views_and_gqa_equals_repeated_mha():
    wl = W.make_prefill_contiguous(58, [90, 200], 8, 2, 128)
    dw = DeviceWorkload(wl)
    base = _bits(dw.run(False))
    # q and out as column slices of a wider buffer (e.g. a fused QKV projection output)
    wide = torch.zeros(wl.q.shape[0], 8 + 3, 128, dtype=torch.bfloat16, device="cuda")
    wide[:, 2:10] = dw.q
    dw2 = DeviceWorkload(wl)
    dw2.q = wide[:, 2:10]
    dw2.out = torch.zeros_like(wide)[:, 1:9]
    assert np.array_equal(base, _bits(dw2.run(False, poison_out=False).contiguous()))
    # GQA == MHA over K/V heads repeated G times (same instance family is not required: tolerance)
    rep = W.Workload("mha", "prefill", "bf16", wl.q, np.repeat(wl.k, 4, axis=1), np.repeat(wl.v, 4, axis=1),
                     wl.query_start_loc, wl.seq_lens, wl.scale, True, kv_start_loc=wl.kv_start_loc)
    a = to_host_f64(dw.out)
    b = to_host_f64(DeviceWorkload(rep).run(False))
    assert float(np.max(np.abs(a - b))) <= 4e-3


def test_empty_batch_and_error_codes_on_device():
    wl = W.make_prefill_contiguous(59, [5], 8, 2, 128)
    dw = DeviceWorkload(wl)
    a = dw.args(False)
    a.num_seqs = 0
    a.total_q = 0
    assert A.load_library().attn_prefill_varlen(a, None) == 0
    a = dw.args(False)
    a.head_dim = 96
    assert A.load_library().attn_prefill_varlen(a, None) == -4
    wl = W.make_paged(60, "decode", np.ones(2, np.int32), [3000, 10], 32, 8, 128, 16, 200)
    dw = DeviceWorkload(wl)
    a = dw.args(True)
    a.workspace_bytes = 16
    names = [A.attn_instance_name(True, i) for i in range(A.attn_num_instances(True))]
    A.attn_force_instance(True, names.index("decode_bf16 d128 w4 split256"))
    assert A.load_library().attn_decode_paged(a, None) == -5
    A.attn_force_instance(True, -1)


def test_graph_capture_and_replay_matches_eager():
    # hot calls neither allocate nor synchronise, so they can be captured (the paper measures under graphs)
    wl = W.make_paged(61, "decode", np.ones(3, np.int32), [1500, 700, 64], 32, 8, 128, 16, 200)
    dw = DeviceWorkload(wl)
    eager = _bits(dw.run(True))
    a = dw.args(True)
    lib = A.load_library()
    stream = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(g, stream=stream):
            rc = lib.attn_decode_paged(a, torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    for _ in range(3):
        dw.out.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(eager, _bits(dw.out))


def test_a_serving_step_of_four_calls_captured_in_one_graph_replays_like_eager():
    """KV-cache write -> chunked prefill over the written cache -> paged decode -> fused add + RMS norm,
    recorded into one graph and replayed with eager work and synchronisations between the replays."""
    rng = np.random.default_rng(63)
    lens = [700, 130, 64, 1500]
    wl = W.make_paged(63, "decode", np.ones(4, np.int32), lens, 32, 8, 128, 16, 200)
    dw = DeviceWorkload(wl)
    pw = W.make_paged(64, "prefill", [64, 1, 33, 100], lens, 32, 8, 128, 16, 200)
    pw = W.Workload("chunk", "prefill", "bf16", pw.q, wl.k, wl.v, pw.query_start_loc, wl.seq_lens, wl.scale, True, block_table=wl.block_table,
                    block_size=16)
    dp = DeviceWorkload(pw)
    dp.k, dp.v = dw.k, dw.v  # both attend to the cache that the first call writes into
    # new keys and values for the last token of every sequence
    slots = np.array([wl.block_table[s, (n - 1) // 16] * 16 + (n - 1) % 16 for s, n in enumerate(lens)], np.int32)
    k_new = torch.from_numpy(rng.standard_normal((4, 8, 128)).astype(np.float32)).cuda().to(torch.bfloat16)
    v_new = torch.from_numpy(rng.standard_normal((4, 8, 128)).astype(np.float32)).cuda().to(torch.bfloat16)
    d_slots = torch.from_numpy(slots).cuda()
    weight = torch.from_numpy(rng.standard_normal(32 * 128).astype(np.float32)).cuda().to(torch.bfloat16)
    res0 = torch.from_numpy(rng.standard_normal((4, 32 * 128)).astype(np.float32)).cuda().to(torch.bfloat16)
    residual = res0.clone()
    normed = torch.empty_like(residual)
    lib = A.load_library()
    a_dec, a_pre = dw.args(True), dp.args(False)

    def step(stream):
        A.attn_kv_cache_write(k_new, v_new, dw.k, dw.v, d_slots, stream=stream)
        assert lib.attn_prefill_varlen(a_pre, stream.cuda_stream) == 0
        assert lib.attn_decode_paged(a_dec, stream.cuda_stream) == 0
        A.rmsnorm_fused_add(dw.out.view(4, 32 * 128), weight, normed, 1e-5, residual=residual, stream=stream)

    step(torch.cuda.current_stream())
    torch.cuda.synchronize()
    want = [_bits(dp.out), _bits(dw.out), _bits(normed), _bits(residual)]
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            step(torch.cuda.current_stream())
    for _ in range(3):
        dp.out.fill_(float("nan"))
        dw.out.fill_(float("nan"))
        normed.fill_(float("nan"))
        residual.copy_(res0)  # the norm updates the residual stream in place
        (dw.k[0, 0, 0, :4] + 1).sum().item()  # eager work and a synchronisation between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = [_bits(dp.out), _bits(dw.out), _bits(normed), _bits(residual)]
        for name, x, y in zip(("prefill", "decode", "norm", "residual"), want, got):
            assert np.array_equal(x, y), name


def test_debug_validate_catches_bad_device_side_integers():
    """ATTN_DEBUG_VALIDATE is read once per process, so the checks run in a child that has it set."""
    import os
    import subprocess
    import sys

    here = os.path.dirname(os.path.abspath(__file__))
    code = "import sys; sys.path[:0] = [%r, %r]; import test_gpu_invariants as T; T._debug_validate_body(); print('child ok')" % (
        os.path.dirname(here), here)
    r = subprocess.run([sys.executable, "-c", code], env=dict(os.environ, ATTN_DEBUG_VALIDATE="1"), capture_output=True, text=True, timeout=280)
    assert r.returncode == 0 and "child ok" in r.stdout, (r.stdout[-1500:], r.stderr[-3000:])


def _debug_validate_body():
    wl = W.make_paged(61, "decode", np.ones(3, np.int32), [100, 40, 257], 32, 8, 128, 16, 64)
    dw = DeviceWorkload(wl)
    lib = A.load_library()
    a = dw.args(True)
    assert lib.attn_decode_paged(a, None) == 0  # consistent inputs pass
    good = int(dw.bt[1, 0])
    dw.bt[1, 0] = 64  # one past the pool
    assert lib.attn_decode_paged(a, None) == -2
    dw.bt[1, 0] = -1
    assert lib.attn_decode_paged(a, None) == -2
    dw.bt[1, 0] = good
    dw.bt[1, 5] = 10 ** 6  # past ceil(40 / 16) entries: never read, never checked
    assert lib.attn_decode_paged(a, None) == 0
    keep = int(dw.seq_lens[2])
    dw.seq_lens[2] = dw.max_kv + 1  # longer than the host was told
    assert lib.attn_decode_paged(a, None) == -2
    dw.seq_lens[2] = keep
    # prefill: query_start_loc that disagrees with total_q, and a chunk longer than max_q_len
    pw = W.make_prefill_contiguous(62, [33, 70], 8, 2, 128)
    dp = DeviceWorkload(pw)
    b = dp.args(False)
    assert lib.attn_prefill_varlen(b, None) == 0
    b.total_q -= 1
    assert lib.attn_prefill_varlen(b, None) == -2
    b.total_q += 1
    b.max_q_len = 64
    assert lib.attn_prefill_varlen(b, None) == -2
    torch.cuda.synchronize()


def test_probes_report_plausible_sustained_rates():
    import bench

    r = bench.probe_achievable(read_bytes=1 << 29, mfma_iters=1 << 12)
    # an MI355X sustains several TB/s and more than a PFLOP/s; far looser bounds catch a broken probe
    assert 1000.0 < r["hbm_read_GBps"] < 8000.0, r
    assert 300.0 < r["mfma_bf16_TFLOPs"] < 2600.0, r
    import ctypes

    lib = ctypes.CDLL(bench.PROBE_LIB)
    assert lib.probe_hbm_read(None, ctypes.c_size_t(64), None, None) == -1
    lib.probe_mfma_bf16.restype = ctypes.c_int64
    assert lib.probe_mfma_bf16(0, ctypes.c_void_p(0x1000), None) == -2
    # the measurement aids are not part of the attention ABI
    assert not hasattr(A.load_library(), "probe_hbm_read") and not hasattr(A.load_library(), "attn_probe_hbm_read")
