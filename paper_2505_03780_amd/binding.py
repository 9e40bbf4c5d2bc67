"""Argument marshalling for the C ABI declared in ``include/attn.h`` (same names, no arithmetic).

The operation is the fused attention kernel the paper studies (section "Method and
Investigated Kernels"): causal variable-length prefill and paged-KV decode with grouped-query
heads.  If the shared library has not been built this module raises; there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

ATTN_F32, ATTN_BF16, ATTN_F16 = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libattn_gfx950.so")
_lib = None


class AttnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, attn_status_string(status), status))


class AttnArgs(ctypes.Structure):
    """Mirror of ``struct attn_args``."""

    _fields_ = [
        ("struct_bytes", ctypes.c_uint32),
        ("dtype", ctypes.c_int32),
        ("num_seqs", ctypes.c_int32),
        ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("total_q", ctypes.c_int32),
        ("max_q_len", ctypes.c_int32),
        ("max_kv_len", ctypes.c_int32),
        ("q", ctypes.c_void_p),
        ("q_stride_tok", ctypes.c_int64),
        ("q_stride_head", ctypes.c_int64),
        ("out", ctypes.c_void_p),
        ("o_stride_tok", ctypes.c_int64),
        ("o_stride_head", ctypes.c_int64),
        ("k", ctypes.c_void_p),
        ("v", ctypes.c_void_p),
        ("kv_stride_block", ctypes.c_int64),
        ("kv_stride_tok", ctypes.c_int64),
        ("kv_stride_head", ctypes.c_int64),
        ("block_table", ctypes.c_void_p),
        ("block_table_stride", ctypes.c_int32),
        ("block_size", ctypes.c_int32),
        ("num_blocks", ctypes.c_int32),
        ("query_start_loc", ctypes.c_void_p),
        ("kv_start_loc", ctypes.c_void_p),
        ("seq_lens", ctypes.c_void_p),
        ("scale", ctypes.c_float),
        ("causal", ctypes.c_int32),
        ("workspace", ctypes.c_void_p),
        ("workspace_bytes", ctypes.c_uint64),
    ]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the HIP library.  Raises if it has not been built (python -m paper_2505_03780_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("%s is missing: build it with `python -m paper_2505_03780_amd.build`" % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    P = ctypes.POINTER(AttnArgs)
    lib.attn_prefill_varlen.restype = ctypes.c_int
    lib.attn_prefill_varlen.argtypes = [P, ctypes.c_void_p]
    lib.attn_decode_paged.restype = ctypes.c_int
    lib.attn_decode_paged.argtypes = [P, ctypes.c_void_p]
    lib.attn_decode_paged_static.restype = ctypes.c_int
    lib.attn_decode_paged_static.argtypes = [P, ctypes.c_void_p]
    lib.attn_static_scratch_bytes.restype = ctypes.c_size_t
    lib.attn_static_scratch_bytes.argtypes = []
    lib.attn_workspace_bytes.restype = ctypes.c_size_t
    lib.attn_workspace_bytes.argtypes = [P, ctypes.c_int]
    lib.attn_tune.restype = ctypes.c_int
    lib.attn_tune.argtypes = [P, ctypes.c_int, ctypes.c_char_p, ctypes.c_int, ctypes.c_int]
    lib.attn_environment_key.restype = ctypes.c_int
    lib.attn_environment_key.argtypes = [ctypes.c_char_p, ctypes.c_size_t]
    lib.attn_load_cache.restype = ctypes.c_int
    lib.attn_load_cache.argtypes = [ctypes.c_char_p]
    lib.attn_clear_cache.restype = None
    lib.attn_clear_cache.argtypes = []
    lib.attn_num_instances.restype = ctypes.c_int
    lib.attn_num_instances.argtypes = [ctypes.c_int]
    lib.attn_instance_name.restype = ctypes.c_int
    lib.attn_instance_name.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_char_p, ctypes.c_size_t]
    lib.attn_selected_instance.restype = ctypes.c_int
    lib.attn_selected_instance.argtypes = [P, ctypes.c_int]
    lib.attn_force_instance.restype = None
    lib.attn_force_instance.argtypes = [ctypes.c_int, ctypes.c_int]
    lib.attn_status_string.restype = ctypes.c_char_p
    lib.attn_status_string.argtypes = [ctypes.c_int]
    lib.attn_kv_cache_write.restype = ctypes.c_int
    lib.attn_kv_cache_write.argtypes = [ctypes.POINTER(KvWriteArgs), ctypes.c_void_p]
    R = ctypes.POINTER(RmsNormArgs)
    lib.rmsnorm_fused_add.restype = ctypes.c_int
    lib.rmsnorm_fused_add.argtypes = [R, ctypes.c_void_p]
    lib.rmsnorm_tune.restype = ctypes.c_int
    lib.rmsnorm_tune.argtypes = [R, ctypes.c_char_p, ctypes.c_int, ctypes.c_int]
    lib.rmsnorm_num_instances.restype = ctypes.c_int
    lib.rmsnorm_num_instances.argtypes = []
    lib.rmsnorm_instance_name.restype = ctypes.c_int
    lib.rmsnorm_instance_name.argtypes = [ctypes.c_int, ctypes.c_char_p, ctypes.c_size_t]
    lib.rmsnorm_selected_instance.restype = ctypes.c_int
    lib.rmsnorm_selected_instance.argtypes = [R]
    lib.rmsnorm_force_instance.restype = None
    lib.rmsnorm_force_instance.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


class KvWriteArgs(ctypes.Structure):
    """Mirror of ``attn_kv_write_args`` in include/attn.h."""
    _fields_ = [
        ("struct_bytes", ctypes.c_uint32),
        ("dtype", ctypes.c_int32),
        ("num_tokens", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("block_size", ctypes.c_int32),
        ("num_blocks", ctypes.c_int32),
        ("reserved", ctypes.c_int32),
        ("k_new", ctypes.c_void_p),
        ("v_new", ctypes.c_void_p),
        ("new_stride_tok", ctypes.c_int64),
        ("new_stride_head", ctypes.c_int64),
        ("k_cache", ctypes.c_void_p),
        ("v_cache", ctypes.c_void_p),
        ("kv_stride_block", ctypes.c_int64),
        ("kv_stride_tok", ctypes.c_int64),
        ("kv_stride_head", ctypes.c_int64),
        ("slot_mapping", ctypes.c_void_p),
    ]


class RmsNormArgs(ctypes.Structure):
    """Mirror of ``rmsnorm_args`` in include/rmsnorm.h."""
    _fields_ = [
        ("struct_bytes", ctypes.c_uint32),
        ("dtype", ctypes.c_int32),
        ("num_tokens", ctypes.c_int32),
        ("hidden", ctypes.c_int32),
        ("x", ctypes.c_void_p),
        ("x_stride", ctypes.c_int64),
        ("residual", ctypes.c_void_p),
        ("residual_stride", ctypes.c_int64),
        ("weight", ctypes.c_void_p),
        ("out", ctypes.c_void_p),
        ("out_stride", ctypes.c_int64),
        ("eps", ctypes.c_float),
    ]


def attn_status_string(status: int) -> str:
    return load_library().attn_status_string(int(status)).decode()


def _dtype_code(t) -> int:
    import torch

    if t.dtype == torch.bfloat16:
        return ATTN_BF16
    if t.dtype == torch.float32:
        return ATTN_F32
    if t.dtype == torch.float16:
        return ATTN_F16
    raise TypeError("tensors must be bfloat16, float16 or float32")


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def make_args(q, k, v, out, seq_lens, scale, *, max_q_len, max_kv_len, query_start_loc=None, kv_start_loc=None,
              block_table=None, causal=True, workspace=None, is_decode=False) -> AttnArgs:
    """Fill an AttnArgs from device tensors.  q/out: [total_q, Hq, D]; k/v: [total_kv, Hkv, D] or,
    with block_table, [num_blocks, block_size, Hkv, D].  Only strides and pointers are read."""
    import torch

    for name, t in (("q", q), ("k", k), ("v", v), ("out", out)):
        if t.stride(-1) != 1:
            raise ValueError("%s: head_dim must be contiguous" % name)
    for name, t in (("seq_lens", seq_lens), ("query_start_loc", query_start_loc), ("kv_start_loc", kv_start_loc),
                    ("block_table", block_table)):
        if t is not None and (t.dtype != torch.int32 or not t.is_contiguous()):
            raise TypeError("%s must be a contiguous int32 tensor" % name)
    if k.dtype != q.dtype or v.dtype != q.dtype or out.dtype != q.dtype:
        raise TypeError("q, k, v, out must share a dtype")
    if k.stride() != v.stride() or k.shape != v.shape:
        raise ValueError("k and v must have the same shape and strides")
    a = AttnArgs()
    a.struct_bytes = ctypes.sizeof(AttnArgs)
    a.dtype = _dtype_code(q)
    a.num_seqs = int(seq_lens.shape[0])
    a.num_q_heads, a.head_dim = int(q.shape[1]), int(q.shape[2])
    a.num_kv_heads = int(k.shape[-2])
    a.total_q = int(q.shape[0])
    a.max_q_len, a.max_kv_len = int(max_q_len), int(max_kv_len)
    a.q, a.q_stride_tok, a.q_stride_head = _ptr(q), q.stride(0), q.stride(1)
    a.out, a.o_stride_tok, a.o_stride_head = _ptr(out), out.stride(0), out.stride(1)
    a.k, a.v = _ptr(k), _ptr(v)
    if block_table is not None:
        if k.dim() != 4:
            raise ValueError("paged k/v must be [num_blocks, block_size, Hkv, D]")
        a.kv_stride_block, a.kv_stride_tok, a.kv_stride_head = k.stride(0), k.stride(1), k.stride(2)
        a.block_table = _ptr(block_table)
        a.block_table_stride = int(block_table.stride(0))
        a.block_size, a.num_blocks = int(k.shape[1]), int(k.shape[0])
    else:
        if k.dim() != 3:
            raise ValueError("contiguous k/v must be [total_kv, Hkv, D]")
        a.kv_stride_block, a.kv_stride_tok, a.kv_stride_head = 0, k.stride(0), k.stride(1)
        a.block_table, a.block_table_stride, a.block_size, a.num_blocks = None, 0, 0, 0
    a.query_start_loc = _ptr(query_start_loc)
    a.kv_start_loc = _ptr(kv_start_loc)
    a.seq_lens = _ptr(seq_lens)
    a.scale = float(scale)
    a.causal = 1 if causal else 0
    a.workspace = _ptr(workspace)
    a.workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    return a


def _stream_ptr(stream) -> int:
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def attn_prefill_varlen(q, k, v, out, query_start_loc, seq_lens, scale, *, max_q_len, max_kv_len, causal=True,
                        block_table=None, kv_start_loc=None, stream=None, args: Optional[AttnArgs] = None) -> None:
    """Enqueue causal variable-length (or chunked, over a paged prefix) prefill on ``stream``."""
    a = args or make_args(q, k, v, out, seq_lens, scale, max_q_len=max_q_len, max_kv_len=max_kv_len,
                          query_start_loc=query_start_loc, kv_start_loc=kv_start_loc, block_table=block_table, causal=causal)
    rc = load_library().attn_prefill_varlen(ctypes.byref(a), _stream_ptr(stream))
    if rc != 0:
        raise AttnError(rc, "attn_prefill_varlen")


def attn_decode_paged(q, k_cache, v_cache, out, block_table, seq_lens, scale, *, max_kv_len, workspace=None, stream=None,
                      args: Optional[AttnArgs] = None) -> None:
    """Enqueue paged-KV decode (one query token per sequence) on ``stream``."""
    a = args or make_args(q, k_cache, v_cache, out, seq_lens, scale, max_q_len=1, max_kv_len=max_kv_len,
                          block_table=block_table, causal=True, workspace=workspace, is_decode=True)
    rc = load_library().attn_decode_paged(ctypes.byref(a), _stream_ptr(stream))
    if rc != 0:
        raise AttnError(rc, "attn_decode_paged")


def attn_decode_paged_static(q, k_cache, v_cache, out, block_table, seq_lens, scale, *, max_kv_len, stream=None,
                             args: Optional[AttnArgs] = None) -> None:
    """attn_decode_paged with the split-K records in the library's own static device array: no workspace
    argument, nothing allocated."""
    a = args or make_args(q, k_cache, v_cache, out, seq_lens, scale, max_q_len=1, max_kv_len=max_kv_len,
                          block_table=block_table, causal=True, is_decode=True)
    rc = load_library().attn_decode_paged_static(ctypes.byref(a), _stream_ptr(stream))
    if rc != 0:
        raise AttnError(rc, "attn_decode_paged_static")


def attn_static_scratch_bytes() -> int:
    return int(load_library().attn_static_scratch_bytes())


def attn_workspace_bytes(args: AttnArgs, is_decode: bool) -> int:
    return int(load_library().attn_workspace_bytes(ctypes.byref(args), 1 if is_decode else 0))


def attn_tune(args: AttnArgs, is_decode: bool, cache_path: Optional[str] = None, iters: int = 20, flags: int = 0) -> None:
    path = None if cache_path is None else os.fsencode(cache_path)
    rc = load_library().attn_tune(ctypes.byref(args), 1 if is_decode else 0, path, int(iters), int(flags))
    if rc != 0:
        raise AttnError(rc, "attn_tune")


def attn_environment_key() -> str:
    buf = ctypes.create_string_buffer(256)
    load_library().attn_environment_key(buf, len(buf))
    return buf.value.decode()


def attn_load_cache(cache_path: str) -> int:
    return int(load_library().attn_load_cache(os.fsencode(cache_path)))


def attn_clear_cache() -> None:
    load_library().attn_clear_cache()


def attn_num_instances(is_decode: bool) -> int:
    return int(load_library().attn_num_instances(1 if is_decode else 0))


def attn_instance_name(is_decode: bool, idx: int) -> str:
    buf = ctypes.create_string_buffer(128)
    rc = load_library().attn_instance_name(1 if is_decode else 0, int(idx), buf, 128)
    if rc < 0:
        raise AttnError(rc, "attn_instance_name")
    return buf.value.decode()


def attn_selected_instance(args: AttnArgs, is_decode: bool) -> int:
    return int(load_library().attn_selected_instance(ctypes.byref(args), 1 if is_decode else 0))


def attn_force_instance(is_decode: bool, idx: int) -> None:
    load_library().attn_force_instance(1 if is_decode else 0, int(idx))


# ---- fused RMS layer norm (include/rmsnorm.h) ------------------------------------------------------

def make_rmsnorm_args(x, weight, out, eps, residual=None) -> RmsNormArgs:
    """x, out, residual: [T, H] device tensors with a contiguous last dimension; weight: [H]."""
    for name, t in (("x", x), ("out", out), ("residual", residual), ("weight", weight)):
        if t is not None and t.stride(-1) != 1:
            raise ValueError("%s: the hidden dimension must be contiguous" % name)
    a = RmsNormArgs()
    a.struct_bytes = ctypes.sizeof(RmsNormArgs)
    a.dtype = _dtype_code(x)
    a.num_tokens, a.hidden = int(x.shape[0]), int(x.shape[1])
    a.x, a.x_stride = _ptr(x), x.stride(0)
    a.residual, a.residual_stride = _ptr(residual), (0 if residual is None else residual.stride(0))
    a.weight = _ptr(weight)
    a.out, a.out_stride = _ptr(out), out.stride(0)
    a.eps = float(eps)
    return a


def rmsnorm_fused_add(x, weight, out, eps, residual=None, stream=None, args: Optional[RmsNormArgs] = None) -> None:
    """Enqueue out = rmsnorm(x + residual) * weight and residual <- x + residual (residual optional)."""
    a = args or make_rmsnorm_args(x, weight, out, eps, residual)
    rc = load_library().rmsnorm_fused_add(ctypes.byref(a), _stream_ptr(stream))
    if rc != 0:
        raise AttnError(rc, "rmsnorm_fused_add")


def rmsnorm_tune(args: RmsNormArgs, cache_path: Optional[str] = None, iters: int = 20, flags: int = 0) -> None:
    path = None if cache_path is None else os.fsencode(cache_path)
    rc = load_library().rmsnorm_tune(ctypes.byref(args), path, int(iters), int(flags))
    if rc != 0:
        raise AttnError(rc, "rmsnorm_tune")


def rmsnorm_num_instances() -> int:
    return int(load_library().rmsnorm_num_instances())


def rmsnorm_instance_name(idx: int) -> str:
    buf = ctypes.create_string_buffer(128)
    n = load_library().rmsnorm_instance_name(int(idx), buf, len(buf))
    if n < 0:
        raise AttnError(n, "rmsnorm_instance_name")
    return buf.value.decode()


def rmsnorm_selected_instance(args: RmsNormArgs) -> int:
    return int(load_library().rmsnorm_selected_instance(ctypes.byref(args)))


def rmsnorm_force_instance(idx: int) -> None:
    load_library().rmsnorm_force_instance(int(idx))


# ---- KV-cache write ----------------------------------------------------------------------------------

def make_kv_write_args(k_new, v_new, k_cache, v_cache, slot_mapping) -> KvWriteArgs:
    """k_new, v_new: [T, Hkv, D]; caches: [num_blocks, block_size, Hkv, D]; slot_mapping: int32 [T]."""
    import torch

    if slot_mapping.dtype != torch.int32 or not slot_mapping.is_contiguous():
        raise TypeError("slot_mapping must be a contiguous int32 tensor")
    for name, t in (("k_new", k_new), ("v_new", v_new), ("k_cache", k_cache), ("v_cache", v_cache)):
        if t.stride(-1) != 1:
            raise ValueError("%s: head_dim must be contiguous" % name)
    if k_new.stride() != v_new.stride() or k_cache.stride() != v_cache.stride():
        raise ValueError("K and V must share their strides")
    a = KvWriteArgs()
    a.struct_bytes = ctypes.sizeof(KvWriteArgs)
    a.dtype = _dtype_code(k_new)
    a.num_tokens, a.num_kv_heads, a.head_dim = int(k_new.shape[0]), int(k_new.shape[1]), int(k_new.shape[2])
    a.block_size, a.num_blocks = int(k_cache.shape[1]), int(k_cache.shape[0])
    a.k_new, a.v_new = _ptr(k_new), _ptr(v_new)
    a.new_stride_tok, a.new_stride_head = k_new.stride(0), k_new.stride(1)
    a.k_cache, a.v_cache = _ptr(k_cache), _ptr(v_cache)
    a.kv_stride_block, a.kv_stride_tok, a.kv_stride_head = k_cache.stride(0), k_cache.stride(1), k_cache.stride(2)
    a.slot_mapping = _ptr(slot_mapping)
    return a


def attn_kv_cache_write(k_new, v_new, k_cache, v_cache, slot_mapping, stream=None, args: Optional[KvWriteArgs] = None) -> None:
    """Enqueue the scatter of new keys/values into the paged caches."""
    a = args or make_kv_write_args(k_new, v_new, k_cache, v_cache, slot_mapping)
    rc = load_library().attn_kv_cache_write(ctypes.byref(a), _stream_ptr(stream))
    if rc != 0:
        raise AttnError(rc, "attn_kv_cache_write")
