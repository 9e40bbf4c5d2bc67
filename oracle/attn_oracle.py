"""ctypes loader for the plain-C fp64 attention oracle (test infrastructure).

Marshals numpy arrays into ``attn_oracle.c``; holds no arithmetic of its own.
The operation is the plain attention definition the paper uses as its
"PyTorch native" baseline (Table I), at the Llama3-8B shapes of the section
"Method and Investigated Kernels".
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attn_oracle.c")
_LIB = os.path.join(_HERE, "libattn_oracle.so")
_lib = None

F32, BF16 = 0, 1


class _CProblem(ctypes.Structure):
    _fields_ = [
        ("dtype", ctypes.c_int),
        ("num_seqs", ctypes.c_int),
        ("num_q_heads", ctypes.c_int),
        ("num_kv_heads", ctypes.c_int),
        ("head_dim", ctypes.c_int),
        ("q", ctypes.c_void_p),
        ("q_stride_tok", ctypes.c_int64),
        ("q_stride_head", ctypes.c_int64),
        ("k", ctypes.c_void_p),
        ("v", ctypes.c_void_p),
        ("kv_stride_block", ctypes.c_int64),
        ("kv_stride_tok", ctypes.c_int64),
        ("kv_stride_head", ctypes.c_int64),
        ("block_table", ctypes.c_void_p),
        ("block_table_stride", ctypes.c_int),
        ("block_size", ctypes.c_int),
        ("query_start_loc", ctypes.c_void_p),
        ("kv_start_loc", ctypes.c_void_p),
        ("seq_lens", ctypes.c_void_p),
        ("scale", ctypes.c_float),
        ("causal", ctypes.c_int),
    ]


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc: strict IEEE arithmetic, no FMA contraction, baseline x86-64
    (the library may be built on one host and run on another), OpenMP over rows."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.oracle_attention.restype = ctypes.c_int
        lib.oracle_attention.argtypes = [ctypes.POINTER(_CProblem), ctypes.c_void_p]
        lib.oracle_attention_rows.restype = ctypes.c_int
        lib.oracle_attention_rows.argtypes = [
            ctypes.POINTER(_CProblem),
            ctypes.c_int,
            ctypes.c_void_p,
            ctypes.c_void_p,
            ctypes.c_void_p,
            ctypes.c_void_p,
        ]
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


@dataclass
class OracleProblem:
    """Inputs of one attention call, as host numpy arrays.

    q: [total_q, Hq, D]; k, v: [total_kv, Hkv, D] (contiguous) or
    [num_blocks, block_size, Hkv, D] (paged, with ``block_table`` int32
    [num_seqs, max_blocks]).  dtype float32, or uint16 holding bf16 bit patterns.
    """

    q: np.ndarray
    k: np.ndarray
    v: np.ndarray
    query_start_loc: np.ndarray
    seq_lens: np.ndarray
    scale: float
    causal: bool = True
    block_table: Optional[np.ndarray] = None
    kv_start_loc: Optional[np.ndarray] = None


def _as_c(p: OracleProblem):
    keep = []

    def arr(a, dt):
        a = np.ascontiguousarray(a, dtype=dt)
        keep.append(a)
        return a

    if p.q.dtype == np.float32:
        dtype, dt = F32, np.float32
    elif p.q.dtype == np.uint16:
        dtype, dt = BF16, np.uint16
    else:
        raise TypeError("q must be float32 or uint16 (bf16 bits)")
    if p.k.dtype != p.q.dtype or p.v.dtype != p.q.dtype:
        raise TypeError("q, k, v must share a dtype")
    q, k, v = arr(p.q, dt), arr(p.k, dt), arr(p.v, dt)
    total_q, Hq, D = q.shape
    qsl = arr(p.query_start_loc, np.int32)
    sl = arr(p.seq_lens, np.int32)
    num_seqs = sl.shape[0]
    if qsl.shape[0] != num_seqs + 1 or int(qsl[-1]) != total_q:
        raise ValueError("query_start_loc does not match q / seq_lens")
    c = _CProblem()
    c.dtype = dtype
    c.num_seqs, c.num_q_heads, c.head_dim = num_seqs, Hq, D
    c.q = q.ctypes.data
    c.q_stride_tok, c.q_stride_head = Hq * D, D
    c.k, c.v = k.ctypes.data, v.ctypes.data
    if p.block_table is not None:
        if k.ndim != 4:
            raise ValueError("paged k/v must be [num_blocks, block_size, Hkv, D]")
        nb, bs, Hkv, Dk = k.shape
        bt = arr(p.block_table, np.int32)
        need = (sl.astype(np.int64) + bs - 1) // bs
        for s in range(num_seqs):
            row = bt[s, : need[s]]
            if row.size and (row.min() < 0 or row.max() >= nb):
                raise ValueError("block_table entry out of range")
        c.block_table = bt.ctypes.data
        c.block_table_stride = bt.shape[1]
        c.block_size = bs
        c.kv_stride_block, c.kv_stride_tok, c.kv_stride_head = bs * Hkv * Dk, Hkv * Dk, Dk
        c.kv_start_loc = None
    else:
        if k.ndim != 3:
            raise ValueError("contiguous k/v must be [total_kv, Hkv, D]")
        _, Hkv, Dk = k.shape
        kvsl = arr(p.kv_start_loc if p.kv_start_loc is not None else qsl, np.int32)
        if kvsl.shape[0] != num_seqs + 1:
            raise ValueError("kv_start_loc must have num_seqs+1 entries")
        if np.any(kvsl[:-1].astype(np.int64) + sl > k.shape[0]):
            raise ValueError("kv rows out of range")
        c.block_table = None
        c.block_table_stride, c.block_size = 0, 0
        c.kv_stride_block, c.kv_stride_tok, c.kv_stride_head = 0, Hkv * Dk, Dk
        c.kv_start_loc = kvsl.ctypes.data
    if Dk != D or v.shape != k.shape or Hq % Hkv:
        raise ValueError("inconsistent head shapes")
    nq = np.diff(qsl)
    if np.any(nq < 0) or np.any(nq > sl):
        raise ValueError("each sequence needs 0 <= n_q <= seq_len")
    c.num_kv_heads = Hkv
    c.query_start_loc = qsl.ctypes.data
    c.seq_lens = sl.ctypes.data
    c.scale = float(np.float32(p.scale))
    c.causal = 1 if p.causal else 0
    return c, keep, (total_q, Hq, D, qsl)


def attention(p: OracleProblem) -> np.ndarray:
    """Full fp64 output [total_q, Hq, D]."""
    c, keep, (total_q, Hq, D, _) = _as_c(p)
    out = np.zeros((total_q, Hq, D), dtype=np.float64)
    if _load().oracle_attention(ctypes.byref(c), out.ctypes.data) != 0:
        raise MemoryError("oracle_attention failed")
    del keep
    return out


def attention_rows(p: OracleProblem, sel_seq, sel_tok, sel_head) -> np.ndarray:
    """fp64 output rows for (sequence, new-token index, query head) triples -> [n, D]."""
    c, keep, (total_q, Hq, D, qsl) = _as_c(p)
    ss = np.ascontiguousarray(sel_seq, dtype=np.int32)
    st = np.ascontiguousarray(sel_tok, dtype=np.int32)
    sh = np.ascontiguousarray(sel_head, dtype=np.int32)
    if not (ss.shape == st.shape == sh.shape):
        raise ValueError("selection arrays differ in length")
    nq = np.diff(qsl)
    if ss.size and (ss.min() < 0 or ss.max() >= nq.size or np.any(st < 0) or np.any(st >= nq[ss]) or sh.min() < 0 or sh.max() >= Hq):
        raise ValueError("selection out of range")
    out = np.zeros((ss.size, D), dtype=np.float64)
    if _load().oracle_attention_rows(ctypes.byref(c), ss.size, ss.ctypes.data, st.ctypes.data, sh.ctypes.data, out.ctypes.data) != 0:
        raise MemoryError("oracle_attention_rows failed")
    del keep
    return out


def num_threads() -> int:
    return int(_load().oracle_num_threads())
