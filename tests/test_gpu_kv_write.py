"""GPU parity (bit-exact) of the KV-cache write step, and the write -> paged attention chain."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_03780_amd as A
import workloads as W
from attn_testlib import DeviceWorkload, to_host_f64

pytestmark = pytest.mark.gpu


def _bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def _dev(bits, dtype=torch.bfloat16):
    return torch.from_numpy(bits.view(np.int16)).view(dtype).cuda()


@pytest.mark.parametrize("T,Hkv,D,bs,nb", [(1, 8, 128, 16, 4), (777, 8, 128, 16, 64), (300, 2, 64, 32, 16), (5000, 8, 128, 16, 400), (64, 1, 8, 128, 2)])
def test_scatter_matches_the_oracle_bit_for_bit(T, Hkv, D, bs, nb):
    rng = np.random.default_rng(T)
    kc = rng.integers(0, 1 << 16, size=(nb, bs, Hkv, D), dtype=np.uint16)
    vc = rng.integers(0, 1 << 16, size=(nb, bs, Hkv, D), dtype=np.uint16)
    kn = rng.integers(0, 1 << 16, size=(T, Hkv, D), dtype=np.uint16)
    vn = rng.integers(0, 1 << 16, size=(T, Hkv, D), dtype=np.uint16)
    slots = rng.permutation(nb * bs)[:T].astype(np.int32)
    slots[rng.random(T) < 0.1] = -1  # padding tokens
    dk, dv = _dev(kc), _dev(vc)
    A.attn_kv_cache_write(_dev(kn), _dev(vn), dk, dv, torch.from_numpy(slots).cuda())
    torch.cuda.synchronize()
    oracle.kv_cache_write(kc, vc, kn, vn, slots)
    np.testing.assert_array_equal(_bits(dk), kc)
    np.testing.assert_array_equal(_bits(dv), vc)
    # fp16 caches: the same bytes under the other 16-bit element type
    kc2 = rng.integers(0, 1 << 16, size=(nb, bs, Hkv, D), dtype=np.uint16)
    vc2 = rng.integers(0, 1 << 16, size=(nb, bs, Hkv, D), dtype=np.uint16)
    hk, hv = _dev(kc2, torch.float16), _dev(vc2, torch.float16)
    A.attn_kv_cache_write(_dev(kn, torch.float16), _dev(vn, torch.float16), hk, hv, torch.from_numpy(slots).cuda())
    torch.cuda.synchronize()
    oracle.kv_cache_write(kc2, vc2, kn, vn, slots)
    np.testing.assert_array_equal(_bits(hk), kc2)
    np.testing.assert_array_equal(_bits(hv), vc2)


def test_fp32_elements_strided_sources_and_errors():
    rng = np.random.default_rng(0)
    T, H, D, bs, nb = 40, 2, 64, 16, 8
    kc = torch.from_numpy(rng.standard_normal((nb, bs, H, D), dtype=np.float32)).cuda()
    vc = torch.from_numpy(rng.standard_normal((nb, bs, H, D), dtype=np.float32)).cuda()
    wide = torch.from_numpy(rng.standard_normal((T, 3 * H, D), dtype=np.float32)).cuda()  # a fused q|k|v projection
    kn, vn = wide[:, H:2 * H], wide[:, 2 * H:]
    slots = rng.permutation(nb * bs)[:T].astype(np.int32)
    rk, rv = kc.cpu().numpy().copy(), vc.cpu().numpy().copy()
    A.attn_kv_cache_write(kn, vn, kc, vc, torch.from_numpy(slots).cuda())
    torch.cuda.synchronize()
    oracle.kv_cache_write(rk, rv, kn.cpu().numpy(), vn.cpu().numpy(), slots)
    np.testing.assert_array_equal(kc.cpu().numpy(), rk)
    np.testing.assert_array_equal(vc.cpu().numpy(), rv)
    with pytest.raises(A.AttnError) as e:  # 6 fp32 = 24 bytes per head row
        A.attn_kv_cache_write(torch.zeros(2, 1, 6, device="cuda"), torch.zeros(2, 1, 6, device="cuda"), torch.zeros(1, 16, 1, 6, device="cuda"),
                              torch.zeros(1, 16, 1, 6, device="cuda"), torch.zeros(2, dtype=torch.int32, device="cuda"))
    assert e.value.status == -4
    empty = torch.zeros(0, H, D, device="cuda")
    A.attn_kv_cache_write(empty, empty, kc, vc, torch.zeros(0, dtype=torch.int32, device="cuda"))


def test_written_cache_feeds_paged_decode_like_a_prefilled_one():
    """Tokens scattered by the kernel, then decode through the same table: equal to decode over a pool
    that the host filled (bit-identical: same kernel, same data)."""
    wl = W.make_paged(91, "decode", np.ones(3, np.int32), [100, 257, 33], 32, 8, 128, 16, 64)
    dw = DeviceWorkload(wl)
    want = to_host_f64(dw.run(True)).copy()
    # gather every sequence's tokens out of the pool, wipe the pool, scatter them back with the kernel
    bs = 16
    slots, toks = [], []
    for s, n in enumerate(wl.seq_lens):
        for j in range(int(n)):
            slots.append(int(wl.block_table[s, j // bs]) * bs + j % bs)
    slots = np.array(slots, np.int32)
    flat_k, flat_v = dw.k.reshape(-1, 8, 128), dw.v.reshape(-1, 8, 128)
    idx = torch.from_numpy(slots.astype(np.int64)).cuda()
    k_new, v_new = flat_k[idx].contiguous(), flat_v[idx].contiguous()
    dw.k.fill_(float("nan")); dw.v.fill_(float("nan"))
    A.attn_kv_cache_write(k_new, v_new, dw.k, dw.v, torch.from_numpy(slots).cuda())
    got = to_host_f64(dw.run(True))
    np.testing.assert_array_equal(got, want)
