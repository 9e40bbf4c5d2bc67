"""The configuration-portability tool (the single-GPU analogue of the paper's second research question,
section "Evaluation": how far does a configuration tuned for one setting carry over to another) on a
small grid: it must run, tune every bucket, time every winner on every bucket and leave a cache file
that a later process can load."""
import re

import pytest

import paper_2505_03780_amd as A
from paper_2505_03780_amd import portability

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _clean():
    A.attn_force_instance(False, -1)
    A.attn_force_instance(True, -1)
    A.attn_clear_cache()
    yield
    A.attn_force_instance(False, -1)
    A.attn_force_instance(True, -1)
    A.attn_clear_cache()


def _matrix(text):
    rows = []
    grab = False
    for line in text.splitlines():
        if line.startswith("| tuned for"):
            grab = True
            continue
        if grab and line.startswith("|---"):
            continue
        if grab and line.startswith("| B"):
            rows.append([c.strip() for c in line.strip().strip("|").split("|")][1:])
        elif grab and not line.startswith("|"):
            break
    return rows


@pytest.mark.parametrize("kind,batches,lengths", [("decode", [2, 16], [512, 2048]), ("prefill", [1, 4], [256, 1024])])
def test_portability_study_on_a_two_by_two_grid(tmp_path, kind, batches, lengths):
    cache = str(tmp_path / ("%s_cache.txt" % kind))
    print("portability study", kind, batches, lengths, flush=True)
    text = portability.study(kind, 2, batches, lengths, cache)
    m = _matrix(text)
    assert len(m) == 4 and all(len(r) == 4 for r in m), text
    for i, row in enumerate(m):
        assert row[i] == "1.00", text  # a bucket's own winner on its own bucket
        for cell in row:
            assert cell == "n/a" or (re.fullmatch(r"[0-9]+\.[0-9]{2}", cell) and 0.2 < float(cell) < 1000.0), text
    assert "Off-diagonal slowdown" in text
    # four winners, each with its environment, in a file that loads back
    lines = open(cache).read().splitlines()
    assert lines[0] == "attn-tune-cache-v1" and len(lines) == 5
    names = {A.attn_instance_name(kind == "decode", i) for i in range(A.attn_num_instances(kind == "decode"))}
    for l in lines[1:]:
        env, key, inst, us = l.split("\t")
        assert env == A.attn_environment_key() and key.startswith(kind) and inst in names and float(us) > 0
    assert A.attn_load_cache(cache) == 0
