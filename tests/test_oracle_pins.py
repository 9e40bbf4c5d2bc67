"""Pins for the fp64 oracle: things the mathematics fixes, none of them the oracle itself.

Each test is chosen so that one plausible mistake (dropped scale, wrong mask
alignment, wrong GQA mapping, transposed operand, wrong block/slot arithmetic,
missing normalisation) fails it.
"""
import os

import numpy as np
import pytest
import torch

import oracle
import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "two_by_two.txt")


def _prob(q, k, v, lens_q, lens_kv, scale, causal=True, **kw):
    qsl = np.concatenate([[0], np.cumsum(lens_q)]).astype(np.int32)
    return oracle.OracleProblem(np.asarray(q, np.float32), np.asarray(k, np.float32), np.asarray(v, np.float32),
                                qsl, np.asarray(lens_kv, np.int32), scale, causal, **kw)


def _contig(q, k, v, lens_q, lens_kv, scale, causal=True):
    kvsl = np.concatenate([[0], np.cumsum(lens_kv)]).astype(np.int32)
    return _prob(q, k, v, lens_q, lens_kv, scale, causal, kv_start_loc=kvsl)


def test_hand_computed_two_by_two():
    rows = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        case, r, a, b = line.split()
        rows[(case, int(r))] = (float(a), float(b))
    q = np.eye(2, dtype=np.float32).reshape(2, 1, 2)
    v = np.array([[1, 2], [3, 4]], np.float32).reshape(2, 1, 2)
    for case, scale, causal in [("causal_scale1", 1.0, True), ("full_scale1", 1.0, False),
                                ("causal_scale0", 0.0, True), ("full_scale0", 0.0, False)]:
        out = oracle.attention(_contig(q, q.copy(), v, [2], [2], scale, causal))
        for r in range(2):
            np.testing.assert_allclose(out[r, 0], rows[(case, r)], rtol=0, atol=1e-15)


def test_transposed_operand_would_fail():
    # Q != K and D != n so that swapping q/k or contracting over the wrong axis changes the result:
    # scores q0.k = [2, 0], q1.k = [0, 3] with distinct values; non-causal.
    q = np.array([[[1, 0, 0]], [[0, 1, 0]]], np.float32)
    k = np.array([[[2, 0, 5]], [[0, 3, 7]]], np.float32)
    v = np.array([[[1, 0, 0]], [[0, 1, 0]]], np.float32)
    out = oracle.attention(_contig(q, k, v, [2], [2], 1.0, False))
    w0 = np.exp([2.0, 0.0]); w0 /= w0.sum()
    w1 = np.exp([0.0, 3.0]); w1 /= w1.sum()
    np.testing.assert_allclose(out[0, 0], [w0[0], w0[1], 0], atol=1e-15)
    np.testing.assert_allclose(out[1, 0], [w1[0], w1[1], 0], atol=1e-15)


@pytest.mark.parametrize("mode", ["equal_keys", "zero_q", "zero_scale"])
def test_uniform_softmax_gives_running_mean(mode):
    rng = np.random.default_rng(10)
    L, Hq, Hkv, D = 37, 4, 2, 8
    q = rng.standard_normal((L, Hq, D)).astype(np.float32)
    k = rng.standard_normal((L, Hkv, D)).astype(np.float32)
    v = rng.standard_normal((L, Hkv, D)).astype(np.float32)
    scale = 0.37
    if mode == "equal_keys":
        k[:] = k[0:1]
    elif mode == "zero_q":
        q[:] = 0
    else:
        scale = 0.0
    out = oracle.attention(_contig(q, k, v, [L], [L], scale, True))
    vv = v.astype(np.float64)
    run = np.cumsum(vv, axis=0) / np.arange(1, L + 1)[:, None, None]  # [L, Hkv, D]
    for h in range(Hq):
        np.testing.assert_allclose(out[:, h], run[:, h // (Hq // Hkv)], rtol=0, atol=1e-13)
    full = oracle.attention(_contig(q, k, v, [L], [L], scale, False))
    for h in range(Hq):
        np.testing.assert_allclose(full[:, h], np.broadcast_to(vv.mean(axis=0)[h // 2], (L, D)), atol=1e-13)


def test_one_hot_selects_value_through_block_table():
    # Orthogonal keys, Q = 60 * K[target]: softmax is one-hot to ~e^-60, so out == V[target]
    # and any slip in block/slot arithmetic picks a different row.
    L, D, bs, nb = 48, 64, 16, 7
    k = np.zeros((L, 1, D), np.float32)
    k[np.arange(L), 0, np.arange(L)] = 1.0
    v = np.random.default_rng(3).standard_normal((L, 1, D)).astype(np.float32)
    targets = np.array([(5 * i + 3) % (i + 1) for i in range(L)])
    q = 60.0 * k[targets]
    table = np.array([[4, 1, 6]], np.int32)
    kp, vp = W.scatter_to_pool(k, v, [0, L], [L], table, bs, nb, fill=np.float32(9.0))
    p = _prob(q, kp, vp, [L], [L], 1.0, True, block_table=table)
    out = oracle.attention(p)
    np.testing.assert_allclose(out[:, 0], v[targets, 0].astype(np.float64), atol=1e-12)


def _dense_reference(q, k, v, scale, off, causal):
    """Second formulation: dense score matrix with an explicit boolean mask, numpy fp64."""
    nq, nkv = q.shape[0], k.shape[0]
    s = (q.astype(np.float64) @ k.astype(np.float64).T) * float(np.float32(scale))
    if causal:
        mask = np.arange(nkv)[None, :] <= (off + np.arange(nq))[:, None]
        s = np.where(mask, s, -np.inf)
    s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    return (p / p.sum(axis=1, keepdims=True)) @ v.astype(np.float64)


@pytest.mark.parametrize("causal", [True, False])
def test_brute_force_dense_mask_varlen_gqa_chunked(causal):
    rng = np.random.default_rng(20)
    Hq, Hkv, D = 6, 2, 16
    lens_kv = [1, 7, 64, 33]
    lens_q = [1, 3, 64, 10]  # mixes full prefill, chunk over a prefix, single token
    q = rng.standard_normal((sum(lens_q), Hq, D)).astype(np.float32)
    k = rng.standard_normal((sum(lens_kv), Hkv, D)).astype(np.float32)
    v = rng.standard_normal((sum(lens_kv), Hkv, D)).astype(np.float32)
    scale = 0.3
    out = oracle.attention(_contig(q, k, v, lens_q, lens_kv, scale, causal))
    q0 = k0 = 0
    for nq, nkv in zip(lens_q, lens_kv):
        for h in range(Hq):
            ref = _dense_reference(q[q0:q0 + nq, h], k[k0:k0 + nkv, h // 3], v[k0:k0 + nkv, h // 3], scale, nkv - nq, causal)
            np.testing.assert_allclose(out[q0:q0 + nq, h], ref, rtol=0, atol=1e-13)
        q0 += nq
        k0 += nkv


def test_matches_torch_fp64_sdpa():
    # Library special case: equal lengths, MHA, contiguous -> torch's own fp64 attention.
    rng = np.random.default_rng(30)
    B, L, H, D = 3, 40, 4, 32
    q = rng.standard_normal((B * L, H, D)).astype(np.float32)
    k = rng.standard_normal((B * L, H, D)).astype(np.float32)
    v = rng.standard_normal((B * L, H, D)).astype(np.float32)
    scale = float(np.float32(1 / np.sqrt(D)))
    out = oracle.attention(_contig(q, k, v, [L] * B, [L] * B, scale, True)).reshape(B, L, H, D)
    tq, tk, tv = (torch.from_numpy(x.reshape(B, L, H, D)).double().permute(0, 2, 1, 3) for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
    np.testing.assert_allclose(out, ref.permute(0, 2, 1, 3).numpy(), rtol=0, atol=1e-13)


def _small_paged(seed=40):
    return W.make_paged(seed, "prefill", [5, 16, 1, 20], [37, 16, 50, 20], 8, 2, 32, 16, 24, table_width=6)


def test_paged_equals_contiguous_bit_identical():
    wl = _small_paged()
    paged = oracle.attention(oracle.OracleProblem(wl.q, wl.k, wl.v, wl.query_start_loc, wl.seq_lens, wl.scale, True,
                                                  block_table=wl.block_table))
    # gather the same tokens into a packed array (pure copy) and run contiguous mode
    ks, vs = [], []
    for s, n in enumerate(wl.seq_lens):
        for j in range(n):
            ks.append(wl.k[wl.block_table[s, j // 16], j % 16])
            vs.append(wl.v[wl.block_table[s, j // 16], j % 16])
    kvsl = np.concatenate([[0], np.cumsum(wl.seq_lens)]).astype(np.int32)
    cont = oracle.attention(oracle.OracleProblem(wl.q, np.stack(ks), np.stack(vs), wl.query_start_loc, wl.seq_lens,
                                                 wl.scale, True, kv_start_loc=kvsl))
    assert np.array_equal(paged, cont)


def test_poisoned_unused_slots_and_blocks_do_not_matter():
    wl = _small_paged(41)
    base = oracle.attention(oracle.OracleProblem(wl.q, wl.k, wl.v, wl.query_start_loc, wl.seq_lens, wl.scale, True,
                                                 block_table=wl.block_table))
    k, v, bt = wl.k.copy(), wl.v.copy(), wl.block_table.copy()
    nan_bits = np.uint16(0x7FC0)
    used = np.zeros(k.shape[:2], bool)
    for s, n in enumerate(wl.seq_lens):
        for j in range(n):
            used[bt[s, j // 16], j % 16] = True
    k[~used] = nan_bits
    v[~used] = nan_bits
    bt[bt < 0] = 2**31 - 1
    out = oracle.attention(oracle.OracleProblem(wl.q, k, v, wl.query_start_loc, wl.seq_lens, wl.scale, True, block_table=bt))
    assert np.array_equal(base, out)


def test_gqa_equals_repeated_mha():
    rng = np.random.default_rng(50)
    L, Hq, Hkv, D = 29, 8, 2, 16
    q = rng.standard_normal((L, Hq, D)).astype(np.float32)
    k = rng.standard_normal((L, Hkv, D)).astype(np.float32)
    v = rng.standard_normal((L, Hkv, D)).astype(np.float32)
    a = oracle.attention(_contig(q, k, v, [L], [L], 0.25))
    b = oracle.attention(_contig(q, np.repeat(k, 4, axis=1), np.repeat(v, 4, axis=1), [L], [L], 0.25))
    assert np.array_equal(a, b)
    # and the mapping is "consecutive q heads share", not interleaved: head 3 uses kv head 0
    c = oracle.attention(_contig(q[:, 3:4], k[:, 0:1], v[:, 0:1], [L], [L], 0.25))
    assert np.array_equal(a[:, 3:4], c)


def test_chunked_equals_slice_of_full_prefill_and_decode_equals_last_row():
    rng = np.random.default_rng(60)
    L, Hq, Hkv, D, nq = 45, 4, 2, 16, 9
    q = rng.standard_normal((L, Hq, D)).astype(np.float32)
    k = rng.standard_normal((L, Hkv, D)).astype(np.float32)
    v = rng.standard_normal((L, Hkv, D)).astype(np.float32)
    full = oracle.attention(_contig(q, k, v, [L], [L], 0.25))
    chunk = oracle.attention(_contig(q[L - nq:], k, v, [nq], [L], 0.25))
    assert np.array_equal(full[L - nq:], chunk)
    dec = oracle.attention(_contig(q[L - 1:], k, v, [1], [L], 0.25))
    assert np.array_equal(full[L - 1:], dec)
    # decode ignores the causal flag (one query at the last position sees everything)
    dec_nc = oracle.attention(_contig(q[L - 1:], k, v, [1], [L], 0.25, causal=False))
    assert np.array_equal(dec, dec_nc)


def test_scale_folding_linearity_convexity_and_batch_permutation():
    rng = np.random.default_rng(70)
    lens = [12, 30, 7]
    Hq, Hkv, D = 4, 4, 8
    T = sum(lens)
    q = rng.standard_normal((T, Hq, D)).astype(np.float32)
    k = rng.standard_normal((T, Hkv, D)).astype(np.float32)
    v = rng.standard_normal((T, Hkv, D)).astype(np.float32)
    a = oracle.attention(_contig(q, k, v, lens, lens, 0.5))
    # scale folded into q exactly (power of two): same function
    b = oracle.attention(_contig(q * np.float32(0.5), k, v, lens, lens, 1.0))
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-14)
    # linear in V
    c = oracle.attention(_contig(q, k, np.float32(2.0) * v, lens, lens, 0.5))
    np.testing.assert_allclose(c, 2 * a, rtol=0, atol=1e-14)
    # convexity: outputs lie inside the range of visible values
    st = np.concatenate([[0], np.cumsum(lens)])
    for s, n in enumerate(lens):
        for i in range(n):
            vis = v[st[s]: st[s] + i + 1].astype(np.float64)
            row = a[st[s] + i]
            assert np.all(row <= vis.max(axis=0) + 1e-12) and np.all(row >= vis.min(axis=0) - 1e-12)
    # permuting the sequences of the batch permutes the output blocks
    order = [2, 0, 1]
    idx = np.concatenate([np.arange(st[s], st[s + 1]) for s in order])
    lens_p = [lens[s] for s in order]
    d = oracle.attention(_contig(q[idx], k[idx], v[idx], lens_p, lens_p, 0.5))
    assert np.array_equal(d, a[idx])


def test_rows_api_matches_full_and_bf16_widening_is_exact():
    wl = _small_paged(42)
    p = oracle.OracleProblem(wl.q, wl.k, wl.v, wl.query_start_loc, wl.seq_lens, wl.scale, True, block_table=wl.block_table)
    full = oracle.attention(p)
    seqs = np.array([0, 1, 1, 3, 2]); toks = np.array([4, 0, 15, 19, 0]); heads = np.array([0, 7, 3, 5, 2])
    rows = oracle.attention_rows(p, seqs, toks, heads)
    for r in range(5):
        assert np.array_equal(rows[r], full[wl.query_start_loc[seqs[r]] + toks[r], heads[r]])
    # bf16 bit patterns and the same values as fp32 give the same result
    pf = oracle.OracleProblem(W.bf16_bits_to_f32(wl.q), W.bf16_bits_to_f32(wl.k), W.bf16_bits_to_f32(wl.v),
                              wl.query_start_loc, wl.seq_lens, wl.scale, True, block_table=wl.block_table)
    assert np.array_equal(full, oracle.attention(pf))


def test_bf16_rounding_helper_is_rne():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.3895314e38], np.float32)  # ties: 1+2^-8 -> even
    bits = W.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    big = np.random.default_rng(0).standard_normal(100000).astype(np.float32)
    ref = torch.from_numpy(big).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(W.f32_to_bf16_bits(big), ref)


def test_generator_draws_match_documented_totals():
    w3 = W.config3()
    assert w3.meta["lens"] == [1711, 409, 577, 680, 581, 1692, 1814, 1299]
    assert w3.visible_pairs_per_head() == 6038658 and w3.flops() == 98937372672
    w1 = W.config1()
    assert w1.q.dtype == np.float32 and w1.flops() == 8454144
