"""Seeded synthetic attention workloads (inputs only; none of the method's arithmetic).

The paper takes its kernel parameters from Llama3-8B (head size 128, 32 query
heads, 8 KV heads) and batches sequences of different lengths drawn from
real-world samples that it does not publish (section "Method and Investigated
Kernels").  These generators stand in for those samples: lengths are uniform in
a stated range, Q/K/V are N(0,1) rounded to bf16 (fp32 for the tiny case), and
the paged KV cache is addressed through a random permutation of a block pool.

Both the fp64 oracle and the HIP library are fed from here; this module calls
neither of them.  Draw order for a seed: lengths, block permutation, Q, K, V.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_bf16(rng: np.random.Generator, shape, chunk: int = 1 << 24) -> np.ndarray:
    """N(0,1) samples rounded to bf16 bits, drawn in chunks to bound host memory."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        out[lo:hi] = f32_to_bf16_bits(rng.standard_normal(hi - lo, dtype=np.float32))
    return out.reshape(shape)


@dataclass
class Workload:
    """One attention call's inputs on the host.

    q [total_q, Hq, D]; contiguous k, v [total_kv, Hkv, D] or paged
    [num_blocks, block_size, Hkv, D].  bf16 data are uint16 bit patterns.
    """

    name: str
    kind: str  # "prefill" or "decode"
    dtype: str  # "f32" or "bf16"
    q: np.ndarray
    k: np.ndarray
    v: np.ndarray
    query_start_loc: np.ndarray
    seq_lens: np.ndarray
    scale: float
    causal: bool
    block_table: Optional[np.ndarray] = None
    kv_start_loc: Optional[np.ndarray] = None
    block_size: int = 0
    meta: dict = field(default_factory=dict)

    @property
    def num_seqs(self) -> int:
        return int(self.seq_lens.shape[0])

    @property
    def num_q_heads(self) -> int:
        return int(self.q.shape[1])

    @property
    def num_kv_heads(self) -> int:
        return int(self.k.shape[-2])

    @property
    def head_dim(self) -> int:
        return int(self.q.shape[2])

    def q_lens(self) -> np.ndarray:
        return np.diff(self.query_start_loc).astype(np.int64)

    def visible_pairs_per_head(self) -> int:
        """Unmasked (query, key) pairs of one query head, summed over the batch."""
        nq = self.q_lens()
        nkv = self.seq_lens.astype(np.int64)
        if self.causal:
            off = nkv - nq
            return int(np.sum(nq * off + nq * (nq + 1) // 2))
        return int(np.sum(nq * nkv))

    def flops(self) -> int:
        """QK^T plus PV multiply-adds over unmasked pairs only: 4*D per pair and head."""
        return 4 * self.head_dim * self.num_q_heads * self.visible_pairs_per_head()

    def kv_bytes(self) -> int:
        """K and V bytes of every key any query can see, each counted once."""
        return int(self.seq_lens.astype(np.int64).sum()) * self.num_kv_heads * self.head_dim * 2 * self.k.itemsize

    def algorithmic_bytes(self) -> int:
        """K+V once, Q read, O written, and the block-table entries that are referenced."""
        qo = 2 * int(self.q.size) * self.q.itemsize
        bt = 0
        if self.block_table is not None:
            bt = 4 * int(np.sum((self.seq_lens.astype(np.int64) + self.block_size - 1) // self.block_size))
        return self.kv_bytes() + qo + bt


def _block_table(rng, seq_lens, block_size, num_blocks, width):
    """Sequence s takes the next ceil(len/block_size) entries of one pool permutation; rest -1."""
    perm = rng.permutation(num_blocks).astype(np.int32)
    need = (np.asarray(seq_lens, dtype=np.int64) + block_size - 1) // block_size
    if int(need.sum()) > num_blocks or (need.size and int(need.max()) > width):
        raise ValueError("pool or table too small for these lengths")
    table = np.full((len(seq_lens), width), -1, dtype=np.int32)
    pos = 0
    for s, n in enumerate(need):
        table[s, :n] = perm[pos : pos + n]
        pos += int(n)
    used = table[table >= 0]
    assert used.size == np.unique(used).size, "a physical block is referenced twice"
    return table


def make_prefill_contiguous(seed, lens, Hq, Hkv, D, dtype="bf16", scale=None, causal=True, name="prefill"):
    """Packed causal varlen prefill: n_q == n_kv per sequence, K/V packed like Q."""
    rng = np.random.default_rng(seed)
    return _prefill_contiguous(rng, np.asarray(lens, dtype=np.int32), Hq, Hkv, D, dtype, scale, causal, name)


def _prefill_contiguous(rng, lens, Hq, Hkv, D, dtype, scale, causal, name):
    qsl = np.zeros(len(lens) + 1, dtype=np.int32)
    qsl[1:] = np.cumsum(lens)
    total = int(qsl[-1])
    if dtype == "f32":
        q = rng.standard_normal((total, Hq, D), dtype=np.float32)
        k = rng.standard_normal((total, Hkv, D), dtype=np.float32)
        v = rng.standard_normal((total, Hkv, D), dtype=np.float32)
    else:
        q = _normal_bf16(rng, (total, Hq, D))
        k = _normal_bf16(rng, (total, Hkv, D))
        v = _normal_bf16(rng, (total, Hkv, D))
    if scale is None:
        scale = float(np.float32(1.0 / np.sqrt(np.float32(D))))
    return Workload(name, "prefill", dtype, q, k, v, qsl, lens.astype(np.int32).copy(), scale, causal,
                    kv_start_loc=qsl.copy(), meta={"lens": lens.tolist()})


def make_paged(seed, kind, q_lens, kv_lens, Hq, Hkv, D, block_size, num_blocks, table_width=None, scale=None,
               causal=True, name="paged", rng=None):
    """Paged-KV workload: the whole pool is filled with N(0,1) bf16, so blocks and
    slots no sequence owns hold ordinary finite values (poison tests overwrite them)."""
    if rng is None:
        rng = np.random.default_rng(seed)
    q_lens = np.asarray(q_lens, dtype=np.int32)
    kv_lens = np.asarray(kv_lens, dtype=np.int32)
    if table_width is None:
        table_width = int((int(kv_lens.max()) + block_size - 1) // block_size) if kv_lens.size else 1
    table = _block_table(rng, kv_lens, block_size, num_blocks, table_width)
    qsl = np.zeros(len(q_lens) + 1, dtype=np.int32)
    qsl[1:] = np.cumsum(q_lens)
    q = _normal_bf16(rng, (int(qsl[-1]), Hq, D))
    k = _normal_bf16(rng, (num_blocks, block_size, Hkv, D))
    v = _normal_bf16(rng, (num_blocks, block_size, Hkv, D))
    if scale is None:
        scale = float(np.float32(1.0 / np.sqrt(np.float32(D))))
    return Workload(name, kind, "bf16", q, k, v, qsl, kv_lens.copy(), scale, causal, block_table=table,
                    block_size=block_size, meta={"kv_lens": kv_lens.tolist(), "num_blocks": num_blocks})


def as_f16(wl: "Workload") -> "Workload":
    """The same workload with q, k, v stored as IEEE fp16 (the bf16 values rounded to nearest even)."""
    import copy

    out = copy.copy(wl)
    conv = lambda a: (bf16_bits_to_f32(a) if a.dtype == np.uint16 else a).astype(np.float16)
    out.q, out.k, out.v = conv(wl.q), conv(wl.k), conv(wl.v)
    out.dtype = "f16"
    out.name = wl.name + "_f16"
    return out


# --- the five benchmark configurations ------------------------------------------------

def config1(seed=1):
    """Tiny causal attention: 1 sequence of 128, 4 = 4 heads, D 64, fp32, scale 1/8."""
    rng = np.random.default_rng(seed)
    lens = np.array([128], dtype=np.int32)
    return _prefill_contiguous(rng, lens, 4, 4, 64, "f32", 0.125, True, "c1_tiny_f32")


def config2(seed=2, batch=64, lo=512, hi=4096, num_blocks=16384):
    """Llama-3-8B-shaped paged decode: batch 64, 32/8 heads, D 128, ctx U[512,4096], block 16."""
    rng = np.random.default_rng(seed)
    ctx = rng.integers(lo, hi, size=batch, endpoint=True).astype(np.int32)
    return make_paged(seed, "decode", np.ones(batch, np.int32), ctx, 32, 8, 128, 16, num_blocks,
                      table_width=(hi + 15) // 16, causal=True, name="c2_decode_8b", rng=rng)


def config3(seed=3, batch=8, lo=256, hi=2048):
    """Llama-3-8B-shaped causal varlen prefill: 8 sequences, lengths U[256,2048], packed."""
    rng = np.random.default_rng(seed)
    lens = rng.integers(lo, hi, size=batch, endpoint=True).astype(np.int32)
    return _prefill_contiguous(rng, lens, 32, 8, 128, "bf16", None, True, "c3_prefill_8b")


def config4(seed=4, batch=16, chunk=512, max_prefix=8192, num_blocks=16384):
    """Chunked prefill over a paged prefix: 16 sequences, prefix U[0,8192] + 512 new causal tokens.
    seq_lens counts prefix plus chunk, and the chunk's K/V already sit in the paged cache."""
    rng = np.random.default_rng(seed)
    prefix = rng.integers(0, max_prefix, size=batch, endpoint=True).astype(np.int32)
    wl = make_paged(seed, "prefill", np.full(batch, chunk, np.int32), prefix + chunk, 32, 8, 128, 16, num_blocks,
                    table_width=(max_prefix + chunk + 15) // 16, causal=True, name="c4_chunked_prefill", rng=rng)
    wl.meta["prefix"] = prefix.tolist()
    return wl


def config5(seed=5, batch=16, lo=16384, hi=32768, num_blocks=32768):
    """Llama-3-70B-shaped long-context paged decode: batch 16, 64/8 heads, ctx U[16384,32768]."""
    rng = np.random.default_rng(seed)
    ctx = rng.integers(lo, hi, size=batch, endpoint=True).astype(np.int32)
    return make_paged(seed, "decode", np.ones(batch, np.int32), ctx, 64, 8, 128, 16, num_blocks,
                      table_width=(hi + 15) // 16, causal=True, name="c5_decode_70b_long", rng=rng)


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}


def stratified_rows(wl: "Workload", tile: int = 32):
    """A deterministic sample of output rows that no query tile can escape: one (sequence, token, head)
    triple for every query head and every run of `tile` consecutive tokens of every sequence (the
    token inside the run varies with run and head; `tile` at most the smallest query tile any kernel
    uses), plus each sequence's first and last token for every head.  Returns int32 arrays
    (seqs, toks, heads)."""
    nq = wl.q_lens()
    H = wl.num_q_heads
    seqs, toks, heads = [], [], []
    hh = np.arange(H, dtype=np.int64)
    for s in range(wl.num_seqs):
        n = int(nq[s])
        if n == 0:
            continue
        for r in range((n + tile - 1) // tile):
            t = np.minimum(r * tile + (7 * r + 3 * hh) % tile, n - 1)
            seqs.append(np.full(H, s)); toks.append(t); heads.append(hh)
        for t in (0, n - 1):
            seqs.append(np.full(H, s)); toks.append(np.full(H, t)); heads.append(hh)
    if not seqs:
        z = np.zeros(0, np.int32)
        return z, z.copy(), z.copy()
    return tuple(np.concatenate(x).astype(np.int32) for x in (seqs, toks, heads))


def scatter_to_pool(k_contig, v_contig, kv_start_loc, seq_lens, block_table, block_size, num_blocks, fill=None, seed=0):
    """Copy packed [total_kv, Hkv, D] K/V into a paged pool following block_table (a pure copy)."""
    Hkv, D = k_contig.shape[1], k_contig.shape[2]
    if fill is None:
        rng = np.random.default_rng(seed)
        kp = _normal_bf16(rng, (num_blocks, block_size, Hkv, D)) if k_contig.dtype == np.uint16 else \
            rng.standard_normal((num_blocks, block_size, Hkv, D), dtype=np.float32)
        vp = kp.copy()
    else:
        kp = np.full((num_blocks, block_size, Hkv, D), fill, dtype=k_contig.dtype)
        vp = kp.copy()
    for s, n in enumerate(np.asarray(seq_lens)):
        base = int(kv_start_loc[s])
        for j0 in range(0, int(n), block_size):
            cnt = min(block_size, int(n) - j0)
            blk = int(block_table[s, j0 // block_size])
            kp[blk, :cnt] = k_contig[base + j0 : base + j0 + cnt]
            vp[blk, :cnt] = v_contig[base + j0 : base + j0 + cnt]
    return kp, vp


# --- fused RMS layer norm (the paper's second kernel) ----------------------------------------------

@dataclass
class RmsNormWorkload:
    """Seeded inputs of one fused (residual add +) RMS norm call; arrays are bf16 bit patterns."""
    name: str
    x: np.ndarray                  # [T, H] uint16
    residual: Optional[np.ndarray]  # [T, H] uint16 or None
    weight: np.ndarray             # [H] uint16
    eps: float

    @property
    def num_tokens(self) -> int:
        return int(self.x.shape[0])

    @property
    def hidden(self) -> int:
        return int(self.x.shape[1])

    def algorithmic_bytes(self) -> int:
        """Every row read once and written once per tensor, plus the weight once."""
        rows = 2 * self.x.size * 2 + (2 * self.x.size * 2 if self.residual is not None else 0)
        return int(rows + self.weight.size * 2)


def make_rmsnorm(seed: int, num_tokens: int, hidden: int, with_residual: bool = True, eps: float = 1e-5,
                 name: str = "rmsnorm") -> RmsNormWorkload:
    """Activations N(0,1), a residual stream of larger spread N(0, 2^2), weights 1 + 0.1 N(0,1), all
    rounded to bf16: the shape of a transformer layer's input norm (hidden 4096 for the 8B model of
    the paper's study, 8192 for the 70B one)."""
    rng = np.random.default_rng(seed)
    x = _normal_bf16(rng, (num_tokens, hidden))
    res = None
    if with_residual:
        res = f32_to_bf16_bits(2.0 * rng.standard_normal((num_tokens, hidden), dtype=np.float32))
    w = f32_to_bf16_bits(1.0 + 0.1 * rng.standard_normal(hidden, dtype=np.float32))
    return RmsNormWorkload(name, x, res, w, eps)


def rmsnorm_8b_prefill(seed: int = 11) -> RmsNormWorkload:
    """8192 tokens (a prefill batch like configuration 3) x hidden 4096."""
    return make_rmsnorm(seed, 8192, 4096, True, 1e-5, "rmsnorm_8b_t8192_h4096")


def rmsnorm_70b_prefill(seed: int = 12) -> RmsNormWorkload:
    """8192 tokens x hidden 8192 (the 70B model's hidden size)."""
    return make_rmsnorm(seed, 8192, 8192, True, 1e-5, "rmsnorm_70b_t8192_h8192")
