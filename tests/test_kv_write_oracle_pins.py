"""Pins of the KV-cache write oracle (CPU only): a copy has a closed form for every mapping."""
import numpy as np

import oracle


def _pool(nb, bs, H, D, seed):
    rng = np.random.default_rng(seed)
    return rng.integers(0, 1 << 16, size=(nb, bs, H, D), dtype=np.uint16), rng.integers(0, 1 << 16, size=(nb, bs, H, D), dtype=np.uint16)


def test_identity_mapping_is_a_reshape():
    kc, vc = _pool(4, 16, 2, 8, 0)
    rng = np.random.default_rng(1)
    kn = rng.integers(0, 1 << 16, size=(64, 2, 8), dtype=np.uint16)
    vn = rng.integers(0, 1 << 16, size=(64, 2, 8), dtype=np.uint16)
    oracle.kv_cache_write(kc, vc, kn, vn, np.arange(64))
    np.testing.assert_array_equal(kc, kn.reshape(4, 16, 2, 8))
    np.testing.assert_array_equal(vc, vn.reshape(4, 16, 2, 8))


def test_permutation_gather_back_and_untouched_slots():
    kc, vc = _pool(8, 16, 3, 4, 2)
    k0, v0 = kc.copy(), vc.copy()
    rng = np.random.default_rng(3)
    slots = rng.permutation(8 * 16)[:50]
    kn = rng.integers(0, 1 << 16, size=(50, 3, 4), dtype=np.uint16)
    vn = rng.integers(0, 1 << 16, size=(50, 3, 4), dtype=np.uint16)
    oracle.kv_cache_write(kc, vc, kn, vn, slots)
    flat_k, flat_v = kc.reshape(128, 3, 4), vc.reshape(128, 3, 4)
    np.testing.assert_array_equal(flat_k[slots], kn)  # reading the slots back returns the tokens
    np.testing.assert_array_equal(flat_v[slots], vn)
    rest = np.setdiff1d(np.arange(128), slots)
    np.testing.assert_array_equal(flat_k[rest], k0.reshape(128, 3, 4)[rest])  # nothing else moved
    np.testing.assert_array_equal(flat_v[rest], v0.reshape(128, 3, 4)[rest])


def test_negative_slots_store_nothing_and_k_v_do_not_cross():
    kc, vc = _pool(2, 16, 1, 4, 4)
    k0, v0 = kc.copy(), vc.copy()
    kn = np.full((3, 1, 4), 7, np.uint16)
    vn = np.full((3, 1, 4), 9, np.uint16)
    oracle.kv_cache_write(kc, vc, kn, vn, [-1, 17, -5])
    assert (kc[1, 1] == 7).all() and (vc[1, 1] == 9).all()
    kc[1, 1], vc[1, 1] = k0[1, 1], v0[1, 1]
    np.testing.assert_array_equal(kc, k0)
    np.testing.assert_array_equal(vc, v0)
