"""GPU parity of the fused RMS layer norm against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_03780_amd as A
import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _auto():
    A.rmsnorm_force_instance(-1)
    A.attn_clear_cache()
    yield
    A.rmsnorm_force_instance(-1)
    A.attn_clear_cache()


def _dev(bits):
    return None if bits is None else torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()


def _f64(t):
    return t.float().cpu().numpy().astype(np.float64)


def _ref(wl):
    res = None if wl.residual is None else W.bf16_bits_to_f32(wl.residual).astype(np.float64)
    return oracle.rms_norm(W.bf16_bits_to_f32(wl.x).astype(np.float64), W.bf16_bits_to_f32(wl.weight).astype(np.float64), wl.eps, res)


def _check(got, ref, what):
    # One rounding to bf16 (8 significant bits: half an ulp is at most 2^-8 relative) on top of fp32
    # arithmetic (a few 2^-24 relative, which may also push a value across a rounding boundary).
    assert np.all(np.isfinite(got)), what
    err = np.abs(got - ref)
    bound = (2.0 ** -8 + 2.0 ** -20) * np.abs(ref) + 1e-30
    assert np.all(err <= bound), "%s: worst error %.3e of bound at %s" % (what, float(np.max(err / bound)), np.unravel_index(np.argmax(err / bound), err.shape))
    # and in the mean the error is that of a correctly rounded result
    rel_rms = float(np.sqrt(np.sum(err ** 2) / max(np.sum(ref ** 2), 1e-300)))
    assert rel_rms <= 2.5e-3, "%s: relative RMS %.3e" % (what, rel_rms)


def _run(wl, instance=None, poison=True):
    x, res, w = _dev(wl.x), _dev(wl.residual), _dev(wl.weight)
    out = torch.full_like(x, float("nan")) if poison else torch.empty_like(x)
    if instance is not None:
        A.rmsnorm_force_instance(instance)
    A.rmsnorm_fused_add(x, w, out, wl.eps, residual=res)
    torch.cuda.synchronize()
    return _f64(out), (None if res is None else _f64(res))


@pytest.mark.parametrize("hidden", [64, 1000, 1024, 4096, 5120, 8192, 16384])
@pytest.mark.parametrize("with_residual", [True, False])
def test_every_instance_matches_the_oracle(hidden, with_residual):
    wl = W.make_rmsnorm(100 + hidden, 37, hidden, with_residual)  # 37 rows: ragged against every rows-per-workgroup
    y_ref, r_ref = _ref(wl)
    args = A.make_rmsnorm_args(_dev(wl.x), _dev(wl.weight), _dev(wl.x), wl.eps, _dev(wl.residual))
    ids = []
    for i in range(A.rmsnorm_num_instances()):
        A.rmsnorm_force_instance(i)
        if A.rmsnorm_selected_instance(args) == i:
            ids.append(i)
    A.rmsnorm_force_instance(-1)
    assert ids, "no instance for hidden %d" % hidden
    for i in ids:
        print("rmsnorm instance", A.rmsnorm_instance_name(i), "hidden", hidden, "residual", with_residual, flush=True)
        y, r = _run(wl, i)
        _check(y, y_ref, A.rmsnorm_instance_name(i))
        if with_residual:
            _check(r, r_ref, "residual of " + A.rmsnorm_instance_name(i))


def test_benchmark_shape_sampled_rows_and_strided_views():
    wl = W.rmsnorm_8b_prefill()
    y_ref, r_ref = _ref(wl)
    y, r = _run(wl)
    _check(y, y_ref, "8192 x 4096")
    _check(r, r_ref, "8192 x 4096 residual")
    # row-strided views: every second row of a wider buffer
    T, H = 64, 4096
    small = W.make_rmsnorm(5, T, H, True)
    big_x = torch.zeros(2 * T, H + 64, dtype=torch.bfloat16, device="cuda")
    big_r = torch.zeros(2 * T, H + 64, dtype=torch.bfloat16, device="cuda")
    big_o = torch.full((2 * T, H + 64), float("nan"), dtype=torch.bfloat16, device="cuda")
    xv, rv, ov = big_x[::2, :H], big_r[::2, :H], big_o[::2, :H]
    xv.copy_(_dev(small.x)); rv.copy_(_dev(small.residual))
    A.rmsnorm_fused_add(xv, _dev(small.weight), ov, small.eps, residual=rv)
    torch.cuda.synchronize()
    ys, rs = _ref(small)
    _check(_f64(ov), ys, "strided out")
    _check(_f64(rv), rs, "strided residual")
    assert torch.isnan(big_o[1::2]).all() and torch.isnan(big_o[::2, H:]).all(), "wrote outside the view"
    assert (big_r[1::2] == 0).all() and (big_r[::2, H:] == 0).all()


def test_rows_past_4_gib_in_every_buffer():
    """300 000 rows of 8192 elements: 4.9 GB per buffer, so the byte offset of most rows needs more than
    32 bits.  The data is made on the device; the oracle takes a sample of rows (each row is an
    independent problem), among them the first and the last."""
    T, H = 300_000, 8192
    assert T * H * 2 > (1 << 32)
    g = torch.Generator(device="cuda")
    g.manual_seed(77)
    x = torch.empty(T, H, dtype=torch.bfloat16, device="cuda").normal_(generator=g)
    res = torch.empty(T, H, dtype=torch.bfloat16, device="cuda").normal_(generator=g)
    w = torch.empty(H, dtype=torch.bfloat16, device="cuda").normal_(generator=g)
    out = torch.full((T, H), float("nan"), dtype=torch.bfloat16, device="cuda")
    rows = np.unique(np.concatenate([[0, 1, T - 2, T - 1, (1 << 32) // (2 * H), (1 << 32) // (2 * H) + 1],
                                     np.random.default_rng(78).integers(0, T, 250)]))
    idx = torch.from_numpy(rows).cuda()
    x_s, r_s = _f64(x[idx]), _f64(res[idx])
    A.rmsnorm_fused_add(x, w, out, 1e-5, residual=res)
    torch.cuda.synchronize()
    y_ref, r_ref = oracle.rms_norm(x_s, _f64(w), 1e-5, r_s)
    _check(_f64(out[idx]), y_ref, "rows past 4 GiB")
    _check(_f64(res[idx]), r_ref, "rows past 4 GiB, residual")
    # every row was written: no NaN left anywhere (one pass over the 4.9 GB on the device)
    assert not bool(torch.isnan(out).any())
    del x, res, out
    torch.cuda.empty_cache()


def test_in_place_output_zero_rows_large_values_and_errors():
    wl = W.make_rmsnorm(6, 5, 4096, False)
    y_ref, _ = _ref(wl)
    x = _dev(wl.x)
    A.rmsnorm_fused_add(x, _dev(wl.weight), x, wl.eps)  # out aliases x
    torch.cuda.synchronize()
    _check(_f64(x), y_ref, "in place")
    # an all-zero row stays zero; a row of huge values does not overflow the square sum (bf16 max ~3e38
    # would, 1e17 must not)
    z = torch.zeros(2, 1024, dtype=torch.bfloat16, device="cuda")
    z[1] = 1e17
    o = torch.empty_like(z)
    w = torch.ones(1024, dtype=torch.bfloat16, device="cuda")
    A.rmsnorm_fused_add(z, w, o, 1e-6)
    torch.cuda.synchronize()
    assert (o[0] == 0).all() and torch.allclose(o[1].float(), torch.ones(1024, device="cuda"), atol=2 ** -8)
    # nothing to do / refused requests
    empty = torch.empty(0, 1024, dtype=torch.bfloat16, device="cuda")
    A.rmsnorm_fused_add(empty, w, empty, 1e-6)
    with pytest.raises(A.AttnError) as e:
        A.rmsnorm_fused_add(torch.zeros(2, 1001, dtype=torch.bfloat16, device="cuda"), w, torch.zeros(2, 1001, dtype=torch.bfloat16, device="cuda"), 1e-6)
    assert e.value.status == -4
    with pytest.raises(A.AttnError) as e:  # bf16 or fp16 rows only
        A.rmsnorm_fused_add(torch.zeros(2, 1024, dtype=torch.float32, device="cuda"), w, o, 1e-6)
    assert e.value.status == -3


@pytest.mark.parametrize("hidden", [64, 1000, 4096, 16384])
def test_fp16_rows_every_instance(hidden):
    """fp16 inputs, the same oracle; one rounding to fp16 (11 significant bits) instead of bf16."""
    wl = W.make_rmsnorm(300 + hidden, 37, hidden, True)
    # the bf16 workload's values rounded to fp16 (exact but for values below fp16's subnormal range), then
    # widened exactly for the oracle
    x64, r64, w64 = (W.bf16_bits_to_f32(b).astype(np.float16).astype(np.float64) for b in (wl.x, wl.residual, wl.weight))
    h = lambda a: torch.from_numpy(a.astype(np.float16)).cuda()
    y_ref, z_ref = oracle.rms_norm(x64, w64, wl.eps, r64)
    ran = 0
    for i in range(A.rmsnorm_num_instances()):
        x, r, w = h(x64), h(r64), h(w64)
        out = torch.full_like(x, float("nan"))
        A.rmsnorm_force_instance(i)
        if A.rmsnorm_selected_instance(A.make_rmsnorm_args(x, w, out, wl.eps, r)) != i:
            continue
        A.rmsnorm_fused_add(x, w, out, wl.eps, residual=r)
        torch.cuda.synchronize()
        for got, ref, what in ((_f64(out), y_ref, "out"), (_f64(r), z_ref, "residual")):
            assert np.all(np.isfinite(got))
            err = np.abs(got - ref)
            bound = (2.0 ** -11 + 2.0 ** -20) * np.abs(ref) + 2.0 ** -25  # half an fp16 ulp; subnormal floor
            assert np.all(err <= bound), "fp16 %s %s: %.3e of bound" % (what, A.rmsnorm_instance_name(i), float(np.max(err / bound)))
        ran += 1
    assert ran >= 1


def test_tune_records_a_winner_in_the_shared_cache_file(tmp_path):
    wl = W.make_rmsnorm(7, 512, 4096, True)
    x, res, w = _dev(wl.x), _dev(wl.residual), _dev(wl.weight)
    out = torch.empty_like(x)
    args = A.make_rmsnorm_args(x, w, out, wl.eps, res)
    cache = str(tmp_path / "tune.txt")
    A.rmsnorm_tune(args, cache, iters=3)
    lines = [l.split("\t") for l in open(cache).read().splitlines()[1:]]
    assert len(lines) == 1 and lines[0][0] == A.attn_environment_key() and lines[0][1] == "rmsnorm|bf16|h4096|res1|T9"
    names = [A.rmsnorm_instance_name(i) for i in range(A.rmsnorm_num_instances())]
    win = names.index(lines[0][2])
    assert A.rmsnorm_selected_instance(args) == win
    A.attn_clear_cache()
    heuristic = A.rmsnorm_selected_instance(args)
    assert A.attn_load_cache(cache) == 0
    assert A.rmsnorm_selected_instance(args) == win
    y_ref, _ = _ref(wl)
    A.rmsnorm_fused_add(x, w, out, wl.eps, residual=res)
    torch.cuda.synchronize()
    _check(_f64(out), y_ref, "tuned")
    assert 0 <= heuristic < len(names)
