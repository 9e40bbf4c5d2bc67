"""Buffers beyond 4 GiB: a KV-cache pool whose block offsets, and a packed batch whose row offsets, do not fit in 32 bits.

The cache of a long-context server on a 288 GB device is far larger than any pool the parity tests
build on the host, so the 64-bit part of the kernels' address arithmetic (block index x block stride)
is exercised here: the pool lives only on the device, the blocks a sequence owns are scattered over
its whole index range (most of them past the 4 GiB mark), and the oracle sees the same tokens through
a compact pool with a compact table.  The result does not depend on how the blocks are numbered."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_03780_amd as A
import workloads as W
from attn_testlib import DeviceWorkload, assert_close, oracle_problem, to_device, to_host_f64

pytestmark = pytest.mark.gpu

BS, HKV, D = 16, 8, 128
BLOCK_BYTES = BS * HKV * D * 2          # 32 KiB
NB_BIG = (5 << 30) // BLOCK_BYTES        # a 5 GiB pool for K and another for V


@pytest.fixture(scope="module")
def big_pools():
    k = torch.full((NB_BIG, BS, HKV, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    v = torch.full((NB_BIG, BS, HKV, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    yield k, v
    del k, v
    torch.cuda.empty_cache()


def _spread(rng, n_compact):
    """An injective map compact block -> big block with three quarters of the blocks past 4 GiB."""
    first_high = (4 << 30) // BLOCK_BYTES
    high = first_high + rng.permutation(NB_BIG - first_high)[: (3 * n_compact) // 4]
    low = rng.permutation(first_high)[: n_compact - len(high)]
    m = np.concatenate([high, low]).astype(np.int64)
    m[0] = NB_BIG - 1  # the very last block of the pool is in use
    rng.shuffle(m)
    return m


def _on_big_pool(wl, big_pools, rng):
    """DeviceWorkload of `wl` whose blocks have been moved into the big device pools."""
    big_k, big_v = big_pools
    n_compact = wl.k.shape[0]
    m = _spread(rng, n_compact)
    idx = torch.from_numpy(m).cuda()
    big_k.index_copy_(0, idx, to_device(wl.k))
    big_v.index_copy_(0, idx, to_device(wl.v))
    table = wl.block_table.copy()
    table[table >= 0] = m[table[table >= 0]]
    dw = DeviceWorkload(wl)
    dw.k, dw.v = big_k, big_v
    dw.bt = torch.from_numpy(table.astype(np.int32)).cuda()
    return dw, m


def test_decode_and_chunked_prefill_read_blocks_past_4_gib(big_pools):
    rng = np.random.default_rng(71)
    lens = [1000, 300, 2049, 17]
    wl = W.make_paged(71, "decode", np.ones(4, np.int32), lens, 32, HKV, D, BS, 260)
    dw, _ = _on_big_pool(wl, big_pools, rng)
    assert int(dw.bt.max()) * BLOCK_BYTES > (1 << 32)
    ref = oracle.attention(oracle_problem(wl))
    names = [A.attn_instance_name(True, i) for i in range(A.attn_num_instances(True))]
    try:
        for name in ("decode_bf16_balanced d128 w4 percu1", "decode_bf16_seq d128 w8 split512", "decode_bf16 d128 w4 split512"):
            A.attn_force_instance(True, names.index(name))
            assert A.attn_selected_instance(dw.args(True), True) == names.index(name)
            assert_close(to_host_f64(dw.run(True)), ref, "bf16", name)
    finally:
        A.attn_force_instance(True, -1)
    # chunked prefill over the same kind of pool (the ring kernel's table path, both workgroup sizes)
    pw = W.make_paged(72, "prefill", [64, 1, 33, 100], [500, 90, 1033, 270], 32, HKV, D, BS, 140)
    dp, _ = _on_big_pool(pw, big_pools, rng)
    ref = oracle.attention(oracle_problem(pw))
    pnames = [A.attn_instance_name(False, i) for i in range(A.attn_num_instances(False))]
    try:
        for name in ("prefill_bf16_ring d128 qb1 w8 hpw4 slots8 pf8 seqmajor", "prefill_bf16_ring d128 qb1 w4 hpw4 slots4 pf4"):
            A.attn_force_instance(False, pnames.index(name))
            assert A.attn_selected_instance(dp.args(False), False) == pnames.index(name)
            assert_close(to_host_f64(dp.run(False)), ref, "bf16", name)
    finally:
        A.attn_force_instance(False, -1)


def test_kv_cache_write_reaches_slots_past_4_gib(big_pools):
    big_k, big_v = big_pools
    rng = np.random.default_rng(73)
    T = 300
    blocks = _spread(rng, 40)
    slots = (blocks[rng.integers(0, 40, T)] * BS + rng.integers(0, BS, T)).astype(np.int64)
    slots = np.unique(slots)[:T]
    rng.shuffle(slots)
    T = len(slots)
    assert slots.max() * (BLOCK_BYTES // BS) > (1 << 32) and slots.max() < 2 ** 31
    kn = rng.integers(0, 1 << 16, size=(T, HKV, D), dtype=np.uint16)
    vn = rng.integers(0, 1 << 16, size=(T, HKV, D), dtype=np.uint16)
    A.attn_kv_cache_write(to_device(kn), to_device(vn), big_k, big_v, torch.from_numpy(slots.astype(np.int32)).cuda())
    torch.cuda.synchronize()
    idx = torch.from_numpy(slots).cuda()
    got_k = big_k.reshape(-1, HKV, D)[idx].view(torch.int16).cpu().numpy().view(np.uint16)
    got_v = big_v.reshape(-1, HKV, D)[idx].view(torch.int16).cpu().numpy().view(np.uint16)
    # the oracle scatters into a compact cache: slot i of the compact cache stands for slots[i]
    kc = np.zeros((T, 1, HKV, D), np.uint16)
    vc = np.zeros((T, 1, HKV, D), np.uint16)
    oracle.kv_cache_write(kc, vc, kn, vn, np.arange(T, dtype=np.int32))
    np.testing.assert_array_equal(got_k, kc[:, 0])
    np.testing.assert_array_equal(got_v, vc[:, 0])


def test_packed_prefill_whose_rows_lie_past_4_gib():
    """9000 packed sequences of 30-90 tokens: 540 000 query rows x 32 heads x 128 = 4.4 GB of Q and of
    output, so the row offsets of most sequences need more than 32 bits.  The data is made on the
    device; the oracle gets a sample of whole sequences (the first, the last, the ones around the
    4 GiB mark and 60 drawn at random), each an independent problem."""
    rng = np.random.default_rng(75)
    lens = rng.integers(30, 91, 9000).astype(np.int32)
    qsl = np.zeros(len(lens) + 1, np.int32)
    qsl[1:] = np.cumsum(lens)
    total = int(qsl[-1])
    Hq = 32
    assert total * Hq * D * 2 > (1 << 32)
    g = torch.Generator(device="cuda")
    g.manual_seed(76)
    q = torch.empty(total, Hq, D, dtype=torch.bfloat16, device="cuda").normal_(generator=g)
    k = torch.empty(total, HKV, D, dtype=torch.bfloat16, device="cuda").normal_(generator=g)
    v = torch.empty(total, HKV, D, dtype=torch.bfloat16, device="cuda").normal_(generator=g)
    out = torch.full_like(q, float("nan"))
    d_qsl, d_lens = torch.from_numpy(qsl).cuda(), torch.from_numpy(lens).cuda()
    scale = float(np.float32(1.0 / np.sqrt(np.float32(D))))
    A.attn_prefill_varlen(q, k, v, out, d_qsl, d_lens, scale, max_q_len=int(lens.max()), max_kv_len=int(lens.max()), kv_start_loc=d_qsl)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(out).any()), "a row was not written"
    mark = int(np.searchsorted(qsl, (1 << 32) // (Hq * D * 2)))
    seqs = np.unique(np.concatenate([[0, 1, mark - 1, mark, mark + 1, len(lens) - 2, len(lens) - 1], rng.integers(0, len(lens), 60)]))
    seqs = seqs[(seqs >= 0) & (seqs < len(lens))]
    rows = np.concatenate([np.arange(qsl[s], qsl[s + 1]) for s in seqs])
    idx = torch.from_numpy(rows).cuda()

    def bits(t):
        return t[idx].view(torch.int16).cpu().numpy().view(np.uint16)

    sub_lens = lens[seqs]
    sub_qsl = np.zeros(len(seqs) + 1, np.int32)
    sub_qsl[1:] = np.cumsum(sub_lens)
    sub = W.Workload("sample", "prefill", "bf16", bits(q), bits(k), bits(v), sub_qsl, sub_lens.copy(), scale, True, kv_start_loc=sub_qsl.copy())
    ref = oracle.attention(oracle_problem(sub))
    assert_close(to_host_f64(out[idx]), ref, "bf16", "sampled sequences of a 4.4 GB packed batch")
