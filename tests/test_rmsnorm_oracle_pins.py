"""Pins of the fp64 RMS-norm oracle against things other than itself (CPU only)."""
import os

import numpy as np
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "rmsnorm_three_four.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            name, *vals = line.split()
            out[name] = np.array([float(v) for v in vals])
    return out


def test_hand_computed_rows():
    g = _golden()
    x = np.array([[3.0, 4.0]])
    w = np.array([1.0, 2.0])
    y, r = oracle.rms_norm(x, w, 0.0)
    assert r is None
    np.testing.assert_allclose(y[0], g["plain"], rtol=0, atol=1e-15)
    y, r = oracle.rms_norm(x, w, 0.0, residual=np.array([[-1.0, 1.0]]))
    np.testing.assert_allclose(y[0], g["residual"], rtol=0, atol=1e-15)
    np.testing.assert_array_equal(r, [[2.0, 5.0]])
    y, _ = oracle.rms_norm(x, w, 3.5)
    np.testing.assert_allclose(y[0], g["eps"], rtol=0, atol=1e-15)


def test_constant_row_gives_the_signed_weight():
    w = np.linspace(-2, 2, 16)
    for c in (0.25, -7.0):
        y, _ = oracle.rms_norm(np.full((3, 16), c), w, 0.0)
        np.testing.assert_allclose(y, np.sign(c) * np.tile(w, (3, 1)), atol=1e-15)


def test_scale_invariance_and_unit_mean_square_without_eps():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 96))
    w = rng.standard_normal(96)
    y1, _ = oracle.rms_norm(x, w, 0.0)
    y2, _ = oracle.rms_norm(37.5 * x, w, 0.0)
    np.testing.assert_allclose(y1, y2, rtol=1e-13, atol=1e-14)
    ones, _ = oracle.rms_norm(x, np.ones(96), 0.0)
    np.testing.assert_allclose(np.mean(ones ** 2, axis=1), 1.0, rtol=1e-13)
    # rows do not mix: normalising a row alone gives the same row
    alone, _ = oracle.rms_norm(x[2:3], w, 0.0)
    np.testing.assert_array_equal(alone[0], y1[2])


def test_eps_is_added_to_the_mean_square_not_to_the_rms():
    x = np.array([[1.0, 1.0, 1.0, 1.0]])
    y, _ = oracle.rms_norm(x, np.ones(4), 3.0)  # mean square 1 + eps 3 -> divide by 2
    np.testing.assert_allclose(y, 0.5, atol=1e-15)
    y, _ = oracle.rms_norm(np.zeros((1, 4)), np.ones(4), 1e-6)  # an all-zero row stays zero
    np.testing.assert_array_equal(y, 0.0)


def test_library_special_case_torch_rms_norm_fp64():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((7, 128))
    w = rng.standard_normal(128)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (128,), torch.from_numpy(w), eps=1e-5).numpy()
    y, _ = oracle.rms_norm(x, w, 1e-5)
    np.testing.assert_allclose(y, ref, rtol=1e-13, atol=1e-14)


def test_fused_residual_equals_norm_of_the_sum():
    rng = np.random.default_rng(2)
    x, r = rng.standard_normal((4, 64)), rng.standard_normal((4, 64))
    w = rng.standard_normal(64)
    fused, r_out = oracle.rms_norm(x, w, 1e-6, residual=r)
    plain, _ = oracle.rms_norm(x + r, w, 1e-6)
    np.testing.assert_array_equal(fused, plain)
    np.testing.assert_array_equal(r_out, x + r)


def test_brute_force_loops_on_a_tiny_case():
    rng = np.random.default_rng(3)
    x, r, w = rng.standard_normal((2, 5)), rng.standard_normal((2, 5)), rng.standard_normal(5)
    y, _ = oracle.rms_norm(x, w, 0.125, residual=r)
    for t in range(2):
        acc = 0.0
        for i in range(5):
            acc += (x[t, i] + r[t, i]) ** 2
        denom = (acc / 5 + 0.125) ** 0.5
        for i in range(5):
            assert abs(y[t, i] - (x[t, i] + r[t, i]) / denom * w[i]) < 1e-14
