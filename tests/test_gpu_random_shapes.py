"""Seeded sweep over random shapes: every call kind, both 16-bit types, random head counts, block
sizes and lengths, the built-in instance and one random valid instance each, against the oracle."""
import numpy as np
import pytest

import oracle
import paper_2505_03780_amd as A
import workloads as W
from attn_testlib import DeviceWorkload, assert_close, oracle_problem, to_host_f64

pytestmark = pytest.mark.gpu

HEADS = [(32, 8), (8, 8), (16, 2), (4, 1), (12, 3), (64, 8), (8, 2), (2, 2)]


@pytest.fixture(autouse=True)
def _auto_instance():
    A.attn_force_instance(False, -1)
    A.attn_force_instance(True, -1)
    A.attn_clear_cache()
    yield
    A.attn_force_instance(False, -1)
    A.attn_force_instance(True, -1)


def _lens(rng, n, hi):
    # a mix of tiny, tile-edge and long lengths
    pool = [1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257]
    out = [int(rng.choice(pool)) if rng.random() < 0.5 else int(rng.integers(1, hi)) for _ in range(n)]
    return [min(x, hi) for x in out]


@pytest.mark.parametrize("seed", range(60))
def test_random_shape(seed):
    rng = np.random.default_rng(1000 + seed)
    kind = ["prefill", "chunked", "decode"][seed % 3]
    Hq, Hkv = HEADS[int(rng.integers(len(HEADS)))]
    f16 = bool(rng.integers(2))
    D = int(rng.choice([64, 128]))
    B = int(rng.integers(1, 9)) if seed < 40 else int(rng.integers(9, 41))  # the last third: batches that wrap the grid's sequence rotation
    causal = True
    if kind == "prefill":
        causal = bool(rng.random() < 0.8)
        wl = W.make_prefill_contiguous(seed, _lens(rng, B, 700), Hq, Hkv, D, causal=causal)
    else:
        bs = int(rng.choice([16, 32, 64]))
        kv = _lens(rng, B, 1500)
        q = [1] * B if kind == "decode" else [int(rng.integers(1, n + 1)) for n in kv]
        nb = int(sum((n + bs - 1) // bs for n in kv)) + int(rng.integers(1, 9))
        wl = W.make_paged(seed, "decode" if kind == "decode" else "prefill", q, kv, Hq, Hkv, D, bs, nb)
    if f16:
        wl = W.as_f16(wl)
    is_decode = kind == "decode"
    dw = DeviceWorkload(wl)
    a = dw.args(is_decode)
    valid = []
    for i in range(A.attn_num_instances(is_decode)):
        A.attn_force_instance(is_decode, i)
        if A.attn_selected_instance(a, is_decode) == i:
            valid.append(i)
    A.attn_force_instance(is_decode, -1)
    what = "seed %d %s Hq %d Hkv %d D %d %s B %d causal %s" % (seed, kind, Hq, Hkv, D, wl.dtype, B, causal)
    print(what, "lens", wl.seq_lens.tolist(), flush=True)
    assert valid, what
    ref = oracle.attention(oracle_problem(wl))
    assert_close(to_host_f64(dw.run(is_decode)), ref, wl.dtype, what + " built-in")
    pick = valid[int(rng.integers(len(valid)))]
    A.attn_force_instance(is_decode, pick)
    assert_close(to_host_f64(dw.run(is_decode)), ref, wl.dtype, what + " " + A.attn_instance_name(is_decode, pick))
