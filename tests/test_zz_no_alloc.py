"""The decode entry point that allocates nothing (attn_decode_paged_static: split-K records in the
library's own static device array) against attn_decode_paged with a caller workspace: same kernels,
same instance, so the outputs must be bit-identical, and both within the bf16 tolerance of the fp64
oracle.  Two calls in a row share the array; the second is smaller and must not see the first's
records.  Collected last on purpose (file name), so that a failure here hides no other test."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2505_03780_amd as A
import workloads as W
from attn_testlib import DeviceWorkload, assert_close, oracle_problem, to_host_f64

import oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _auto_instance():
    A.attn_force_instance(True, -1)
    A.attn_clear_cache()
    yield
    A.attn_force_instance(True, -1)


def _both(wl, what):
    dw = DeviceWorkload(wl)
    a = dw.args(True)
    name = A.attn_instance_name(True, A.attn_selected_instance(a, True))
    want = to_host_f64(dw.run(True)).copy()
    # the same arguments without any workspace
    a.workspace, a.workspace_bytes = None, 0
    dw.out.fill_(float("nan"))
    rc = A.load_library().attn_decode_paged_static(ctypes.byref(a), torch.cuda.current_stream().cuda_stream)
    assert rc == 0, A.attn_status_string(rc)
    torch.cuda.synchronize()
    got = to_host_f64(dw.out)
    print(what, name, "records", A.attn_workspace_bytes(a, True), "of", A.attn_static_scratch_bytes(), flush=True)
    assert np.array_equal(got, want), "%s (%s): outputs of the two entry points differ" % (what, name)
    assert_close(got, oracle.attention(oracle_problem(wl)), "bf16", what)
    return name


def test_static_scratch_decode_matches_workspace_decode_twice_in_a_row():
    assert A.attn_static_scratch_bytes() == 16 << 20
    big = W.make_paged(91, "decode", np.ones(24, np.int32), [4000, 1, 3500, 40, 2777, 900, 4096, 17] * 3, 32, 8, 128, 16, 4200)
    small = W.make_paged(92, "decode", np.ones(3, np.int32), [513, 64, 1200], 32, 8, 128, 16, 200)
    n1 = _both(big, "first call (24 sequences up to 4096 keys)")
    n2 = _both(small, "second call (3 short sequences)")
    assert "split0" not in n1, "the first call was meant to use split-K records, got " + n1
    # every family that keeps records in the workspace, forced, big then small on the shared array
    dw = DeviceWorkload(big)
    a = dw.args(True)
    tried = 0
    for i in range(A.attn_num_instances(True)):
        A.attn_force_instance(True, i)
        if A.attn_selected_instance(a, True) != i or "split0" in A.attn_instance_name(True, i):
            continue
        if tried % 4 == 0:  # a sample of the table keeps the test short
            _both(big, "forced big")
            _both(small, "forced small")
        tried += 1
    assert tried > 0


def test_static_scratch_decode_rejects_what_does_not_fit_and_bad_arguments():
    lib = A.load_library()
    assert lib.attn_decode_paged_static(None, None) == -1
    # 2000 sequences of one key: one record per sequence and query head alone is 2000 * 32 * 130 * 4 bytes = 33 MB
    B = 2000
    wl = W.make_paged(93, "decode", np.ones(B, np.int32), np.ones(B, np.int32), 32, 8, 128, 16, B + 1)
    dw = DeviceWorkload(wl)
    a = dw.args(True)
    bal = next(i for i in range(A.attn_num_instances(True)) if "balanced d128" in A.attn_instance_name(True, i))
    A.attn_force_instance(True, bal)
    assert A.attn_selected_instance(a, True) == bal
    a.workspace, a.workspace_bytes = None, 0
    dw.out.zero_()
    assert lib.attn_decode_paged_static(ctypes.byref(a), None) == -5  # ATTN_ERR_WORKSPACE, nothing enqueued
    torch.cuda.synchronize()
    assert float(dw.out.float().abs().sum()) == 0.0
