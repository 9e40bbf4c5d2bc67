"""GPU test of the in-library autotuner and its persistent cache."""
import numpy as np
import pytest

import paper_2505_03780_amd as A
import workloads as W
from attn_testlib import DeviceWorkload, assert_close, oracle_problem, to_host_f64

import oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _clean():
    A.attn_force_instance(False, -1)
    A.attn_force_instance(True, -1)
    A.attn_clear_cache()
    yield
    A.attn_clear_cache()


def _cache_lines(path):
    lines = open(path).read().splitlines()
    assert lines[0] == "attn-tune-cache-v1"
    return [l.split("\t") for l in lines[1:] if l and not l.startswith("#")]


@pytest.mark.parametrize("kind", ["prefill", "decode"])
def test_tune_writes_cache_and_hot_calls_use_the_winner(tmp_path, kind):
    is_decode = kind == "decode"
    if is_decode:
        wl = W.make_paged(71, "decode", np.ones(8, np.int32), [900, 1024, 700, 33, 512, 1000, 64, 800], 32, 8, 128, 16, 600)
    else:
        wl = W.make_prefill_contiguous(72, [300, 512, 129, 400], 32, 8, 128)
    dw = DeviceWorkload(wl)
    args = dw.args(is_decode)
    names = [A.attn_instance_name(is_decode, i) for i in range(A.attn_num_instances(is_decode))]
    default = A.attn_selected_instance(args, is_decode)
    cache = str(tmp_path / "tune.txt")
    print("tuning", kind, "over", len(names), "instances", flush=True)
    A.attn_tune(args, is_decode, cache, iters=3, flags=0)
    rows = _cache_lines(cache)
    assert len(rows) == 1
    env, key, winner, us = rows[0]
    assert env.startswith("gfx950") and "|cu" in env and key.startswith(kind) and winner in names and float(us) > 0
    win_id = names.index(winner)
    assert A.attn_selected_instance(args, is_decode) == win_id
    # hot call with the tuned instance is still correct
    ref = oracle.attention(oracle_problem(wl))
    assert_close(to_host_f64(dw.run(is_decode)), ref, "bf16", "tuned " + winner)
    # a fresh state falls back to the heuristic, loading the file brings the winner back
    A.attn_clear_cache()
    assert A.attn_selected_instance(args, is_decode) == default
    assert A.attn_load_cache(cache) == 0
    assert A.attn_selected_instance(args, is_decode) == win_id
    # a second bucket is merged into the same file, the first entry survives
    other = A.make_args(dw.q, dw.k, dw.v, dw.out, dw.seq_lens, wl.scale, max_q_len=1 if is_decode else 4 * dw.max_q,
                        max_kv_len=4 * dw.max_kv, query_start_loc=None if is_decode else dw.qsl, kv_start_loc=dw.kvsl,
                        block_table=dw.bt, is_decode=is_decode)
    if is_decode:
        other.block_table_stride = 4 * dw.bt.shape[1]  # only the shape fields matter to attn_tune
    A.attn_tune(other, is_decode, cache, iters=2, flags=0)
    rows = _cache_lines(cache)
    assert len(rows) == 2 and rows[0][1] == key and rows[1][1] != key
    # an entry written for another environment is ignored
    stale = tmp_path / "stale.txt"
    stale.write_text("attn-tune-cache-v1\ngfx942|cu304|hip0|k0\t%s\t%s\t1.0\n" % (key, names[(win_id + 1) % len(names)]))
    A.attn_clear_cache()
    assert A.attn_load_cache(str(stale)) == 0
    assert A.attn_selected_instance(args, is_decode) == default


def test_exhaustive_sweep_flag_and_environment_key(tmp_path):
    wl = W.make_paged(73, "decode", np.ones(4, np.int32), [700, 333, 1024, 90], 32, 8, 128, 16, 300)
    dw = DeviceWorkload(wl)
    args = dw.args(True)
    cache = str(tmp_path / "tune.txt")
    A.attn_tune(args, True, cache, iters=2, flags=2)  # every valid instance, two launches each
    rows = _cache_lines(cache)
    assert len(rows) == 1 and rows[0][0] == A.attn_environment_key()
    assert rows[0][0].startswith("gfx950") and "|hip" in rows[0][0] and "|drv" in rows[0][0]
    ref = oracle.attention(oracle_problem(wl))
    assert_close(to_host_f64(dw.run(True)), ref, "bf16", "after exhaustive tune: " + rows[0][2])
    # the halving search seeded by this winner (a neighbouring bucket) still ends on a valid instance
    wider = A.make_args(dw.q, dw.k, dw.v, dw.out, dw.seq_lens, wl.scale, max_q_len=1, max_kv_len=2 * dw.max_kv,
                        block_table=dw.bt, is_decode=True)
    A.attn_tune(wider, True, cache, iters=4, flags=0)
    assert len(_cache_lines(cache)) == 2
    assert_close(to_host_f64(dw.run(True)), ref, "bf16", "after seeded tune")
