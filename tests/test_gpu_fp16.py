"""GPU parity of the fp16 instances (prefill ring and register-staged kernels, paged decode) against the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_03780_amd as A
import workloads as W
from attn_testlib import DeviceWorkload, assert_close, check_full, check_sampled, oracle_problem, to_host_f64

pytestmark = pytest.mark.gpu

RAGGED = [1, 31, 32, 33, 63, 64, 65, 127, 129, 200, 257]


@pytest.fixture(autouse=True)
def _auto_instance():
    A.attn_force_instance(False, -1)
    A.attn_force_instance(True, -1)
    A.attn_clear_cache()
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


@pytest.mark.parametrize("Hq,Hkv,D", [(8, 2, 128), (4, 4, 128), (4, 2, 128), (32, 8, 128), (8, 2, 64), (4, 4, 64)])
def test_prefill_contiguous_ragged_every_f16_instance(Hq, Hkv, D):
    wl = W.as_f16(W.make_prefill_contiguous(121, RAGGED, Hq, Hkv, D))
    dw = DeviceWorkload(wl)
    assert dw.q.dtype == torch.float16
    ref = oracle.attention(oracle_problem(wl))
    ids = _valid_instances(dw, False)
    assert ids and all("f16" in A.attn_instance_name(False, i) for i in ids)
    for i in ids:
        print("f16 prefill instance", A.attn_instance_name(False, i), flush=True)
        A.attn_force_instance(False, i)
        assert_close(to_host_f64(dw.run(False)), ref, "f16", A.attn_instance_name(False, i))


def test_chunked_prefill_over_a_paged_prefix_peaked_and_non_causal():
    q_lens, kv_lens = [64, 1, 200, 33], [64, 300, 777, 33 + 512]
    wl = W.as_f16(W.make_paged(122, "prefill", q_lens, kv_lens, 8, 2, 128, 16, 200))
    dw = DeviceWorkload(wl)
    ref = oracle.attention(oracle_problem(wl))
    for i in _valid_instances(dw, False):
        A.attn_force_instance(False, i)
        assert_close(to_host_f64(dw.run(False)), ref, "f16", A.attn_instance_name(False, i))
    A.attn_force_instance(False, -1)
    peaked = W.as_f16(W.make_prefill_contiguous(123, [257, 64, 130], 8, 2, 128, scale=5.0 / np.sqrt(128.0)))
    check_full(peaked, what="peaked f16")
    flat = W.as_f16(W.make_prefill_contiguous(124, [100, 257], 4, 4, 128, causal=False))
    check_full(flat, what="non-causal f16")


@pytest.mark.parametrize("Hq,Hkv,D", [(32, 8, 128), (16, 2, 128), (4, 4, 128), (8, 2, 64)])
def test_decode_every_f16_instance(Hq, Hkv, D):
    lens = [1, 15, 16, 17, 31, 32, 33, 100, 255, 256, 257, 700, 1500]
    wl = W.as_f16(W.make_paged(141, "decode", np.ones(len(lens), np.int32), lens, Hq, Hkv, D, 16, 400))
    dw = DeviceWorkload(wl)
    ref = oracle.attention(oracle_problem(wl))
    ids = _valid_instances(dw, True)
    assert ids and all("f16" in A.attn_instance_name(True, i) for i in ids)
    for i in ids:
        print("f16 decode instance", A.attn_instance_name(True, i), flush=True)
        A.attn_force_instance(True, i)
        assert_close(to_host_f64(dw.run(True)), ref, "f16", A.attn_instance_name(True, i))


def test_full_size_configs_in_f16_and_what_is_refused():
    print("config 2 in fp16", flush=True)
    check_full(W.as_f16(W.config2()))
    print("config 3 in fp16 (sampled)", flush=True)
    check_sampled(W.as_f16(W.config3()), 400, seed=33)
    # a head size without instances is refused, nothing silently converted
    small = W.as_f16(W.make_prefill_contiguous(125, [64, 64], 8, 2, 32))
    dw = DeviceWorkload(small)
    with pytest.raises(A.AttnError) as e:
        dw.run(False)
    assert e.value.status in (-2, -4)
    # head size 64 over a paged prefix in fp16 (register-staged kernel)
    paged64 = W.as_f16(W.make_paged(127, "prefill", [64, 1, 130], [64, 300, 130 + 256], 8, 2, 64, 16, 100))
    check_full(paged64, what="fp16 d64 chunked prefill")
    # the autotuner works on fp16 buckets too
    wl = W.as_f16(W.make_prefill_contiguous(126, [300, 200], 32, 8, 128))
    dw = DeviceWorkload(wl)
    a = dw.args(False)
    A.attn_tune(a, False, None, 2, 0)
    assert "f16" in A.attn_instance_name(False, A.attn_selected_instance(a, False))
    assert_close(to_host_f64(dw.run(False)), oracle.attention(oracle_problem(wl)), "f16", "tuned f16")
