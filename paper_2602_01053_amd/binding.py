"""Thin ctypes binding over liblra_attn.so: argument marshalling only.

Every step of the attention path runs inside the library's HIP kernels.  There is
no CPU or PyTorch fallback: if the shared library is missing the first call
raises.  torch is used for device memory and streams, nothing else.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

from .build import LIB_PATH

LRA_OK = 0
LRA_BF16, LRA_F32 = 0, 1

STATIC_WORKSPACE_BYTES = 64 << 20   # LRA_STATIC_WORKSPACE_BYTES of the header

EXPORTS = ("lra_workspace_bytes", "lra_attn_decode", "lra_attn_decode_static", "lra_attn_prefill", "lra_status_string",
           "lra_cache_append", "lra_append_workspace_bytes", "lra_probe_stream_read", "lra_probe_mfma_bf16")


class LraShape(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("rank", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("scale", ctypes.c_float), ("key_rope_theta", ctypes.c_float)]


class LraCache(ctypes.Structure):
    _fields_ = [("k_base", ctypes.c_void_p), ("v_base", ctypes.c_void_p), ("l", ctypes.c_void_p),
                ("kv_token_stride", ctypes.c_int64), ("kv_head_stride", ctypes.c_int64),
                ("kv_block_stride", ctypes.c_int64),
                ("block_size", ctypes.c_int32), ("max_blocks_per_seq", ctypes.c_int32),
                ("num_blocks", ctypes.c_int32), ("n_seqs", ctypes.c_int32),
                ("l_row_stride", ctypes.c_int64), ("l_adapter_stride", ctypes.c_int64),
                ("block_table", ctypes.c_void_p), ("seq_lens", ctypes.c_void_p),
                ("max_seq_len", ctypes.c_int32), ("seq_lens_host", ctypes.c_void_p)]


class LraAdapters(ctypes.Structure):
    _fields_ = [("b_k", ctypes.c_void_p), ("b_v", ctypes.c_void_p), ("n_adapters", ctypes.c_int32)]


class LraProjection(ctypes.Structure):
    _fields_ = [("w", ctypes.c_void_p), ("d_model", ctypes.c_int32), ("rope_theta", ctypes.c_float)]


class LraTuning(ctypes.Structure):
    """lra_tuning of the header: all zero = automatic everywhere."""
    _fields_ = [("kernel_variant", ctypes.c_int32), ("decode_split_keys", ctypes.c_int32),
                ("short_prefill", ctypes.c_int32), ("prefill_splits", ctypes.c_int32),
                ("rope_key_prepass", ctypes.c_int32), ("append_skinny", ctypes.c_int32), ("append_stages", ctypes.c_int32),
                ("append_tile", ctypes.c_int32), ("append_k_splits", ctypes.c_int32),
                ("measure_main_kernel_only", ctypes.c_int32)]


# The tuning struct this binding hands to every call.  The C library keeps no tuning state; the
# lra_set_* helpers below are conveniences for tests and benchmarks that edit this one struct
# (process-wide on the Python side only) and return the previous value.
_tuning = LraTuning()


class LraError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"lra_attn status {status}: {message}")
        self.status = status


_lib = None


def load_library() -> ctypes.CDLL:
    """dlopen the in-tree library.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2602_01053_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    sp, cp, ap = ctypes.POINTER(LraShape), ctypes.POINTER(LraCache), ctypes.POINTER(LraAdapters)
    vp, i32 = ctypes.c_void_p, ctypes.c_int32
    lib.lra_workspace_bytes.restype = ctypes.c_size_t
    tp = ctypes.POINTER(LraTuning)
    lib.lra_workspace_bytes.argtypes = [sp, cp, i32, i32, i32, tp]
    lib.lra_attn_decode.restype = ctypes.c_int
    lib.lra_attn_decode.argtypes = [sp, cp, ap, vp, vp, vp, i32, i32, vp, vp, ctypes.c_size_t, tp, vp]
    lib.lra_attn_decode_static.restype = ctypes.c_int
    lib.lra_attn_decode_static.argtypes = [sp, cp, ap, vp, vp, vp, i32, i32, vp, tp, vp]
    lib.lra_attn_prefill.restype = ctypes.c_int
    lib.lra_attn_prefill.argtypes = [sp, cp, ap, vp, i32, i32, i32, vp, vp, ctypes.c_size_t, tp, vp]
    lib.lra_cache_append.restype = ctypes.c_int
    lib.lra_cache_append.argtypes = [sp, cp, ctypes.POINTER(LraProjection), vp, i32, i32, vp, ctypes.c_size_t, tp, vp]
    lib.lra_append_workspace_bytes.restype = ctypes.c_size_t
    lib.lra_append_workspace_bytes.argtypes = [sp, cp, ctypes.POINTER(LraProjection), i32, tp]
    lib.lra_status_string.restype = ctypes.c_char_p
    lib.lra_status_string.argtypes = [ctypes.c_int]
    lib.lra_probe_stream_read.restype = ctypes.c_int
    lib.lra_probe_stream_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
    lib.lra_probe_mfma_bf16.restype = ctypes.c_int
    lib.lra_probe_mfma_bf16.argtypes = [i32, i32, ctypes.POINTER(ctypes.c_int64), vp, vp]
    _lib = lib
    return lib


def lra_status_string(status: int) -> str:
    return load_library().lra_status_string(int(status)).decode()


def lra_cache_append(shape: LraShape, cache: LraCache, w: torch.Tensor, rope_theta: float, x: torch.Tensor,
                     seq_index: int, stream=None, workspace: Optional[torch.Tensor] = None) -> None:
    """Project the new tokens x [n_new][d_model] with w [2*Hkv*d + r][d_model] and write their
    K_base / V_base / L rows into the cache (the last n_new rows of sequence seq_index).  `workspace`
    (optional, lra_append_workspace_bytes bytes) lets mid-sized chunks split d_model over the chip."""
    if not (x.is_contiguous() and w.is_contiguous()) or x.shape[1] != w.shape[1]:
        raise LraError(2, "x and w must be dense and share d_model")
    proj = LraProjection(_ptr(w), int(w.shape[1]), float(rope_theta))
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().lra_cache_append(ctypes.byref(shape), ctypes.byref(cache), ctypes.byref(proj), _ptr(x),
                                           int(seq_index), int(x.shape[0]), _ptr(workspace), ws_bytes,
                                           ctypes.byref(_tuning), _stream_ptr(stream)))


def lra_append_workspace_bytes(shape: LraShape, cache: LraCache, w: torch.Tensor, rope_theta: float, n_new: int) -> int:
    proj = LraProjection(_ptr(w), int(w.shape[1]), float(rope_theta))
    n = load_library().lra_append_workspace_bytes(ctypes.byref(shape), ctypes.byref(cache), ctypes.byref(proj),
                                                  int(n_new), ctypes.byref(_tuning))
    if n == ctypes.c_size_t(-1).value:
        raise LraError(2, "lra_append_workspace_bytes: arguments rejected")
    return int(n)


def lra_set_append_k_splits(parts: int) -> int:
    """Parts of d_model in lra_cache_append when it has a workspace: 0 automatic, 1 never, 2..16 forced."""
    return _swap("append_k_splits", parts)


def _swap(field: str, value: int) -> int:
    old = getattr(_tuning, field)
    setattr(_tuning, field, int(value))
    return int(old)


def lra_set_kernel_variant(variant: int) -> int:
    """0 automatic, 1 vector-ALU kernels, 2 MFMA kernels without the streaming form of the split-KV kernel."""
    return _swap("kernel_variant", variant)


def lra_set_decode_split_keys(keys: int) -> int:
    return _swap("decode_split_keys", keys)


def lra_set_append_tile(tile: int) -> int:
    return _swap("append_tile", tile)


def lra_set_append_stages(stages: int) -> int:
    return _swap("append_stages", stages)


def _swap_default(field: str, tokens: int, default: int) -> int:
    """Fields where 0 means "automatic" in the struct but callers say 0 for "off": stored as -1."""
    raw = getattr(_tuning, field)
    old = default if raw == 0 else max(raw, 0)
    setattr(_tuning, field, -1 if tokens <= 0 else int(tokens))
    return int(old)


def lra_set_append_skinny(tokens: int) -> int:
    """New tokens up to which lra_cache_append streams the weights; 0 switches that off (default 64)."""
    return _swap_default("append_skinny", tokens, 64)


def lra_set_short_prefill(tokens: int) -> int:
    """New tokens up to which a prefill takes the split-KV path; 0 switches that off (default 32)."""
    return _swap_default("short_prefill", tokens, 32)


def lra_set_prefill_splits(splits: int) -> int:
    return _swap("prefill_splits", splits)


def lra_set_rope_key_prepass(on: bool) -> bool:
    """Rotary prefill on contiguous caches: completed keys by a pre-pass into the workspace (default on)."""
    old = _tuning.rope_key_prepass >= 0
    _tuning.rope_key_prepass = 0 if on else -1
    return old


def lra_set_profile_mode(mode: int) -> int:
    """1: later calls enqueue only their dominant kernel (measurement; `out` is not produced)."""
    return _swap("measure_main_kernel_only", 1 if mode == 1 else 0)


def lra_probe_stream_read(src: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    """One streaming read of the whole of src (a machine probe for the benchmark)."""
    _check(load_library().lra_probe_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink),
                                                _stream_ptr(stream)))


def lra_probe_mfma_bf16(iters: int, sink: torch.Tensor, random_operands: bool = False, stream=None) -> int:
    """One launch of the register-resident bf16 MFMA loop; returns its floating-point operations."""
    flops = ctypes.c_int64(0)
    _check(load_library().lra_probe_mfma_bf16(int(iters), int(bool(random_operands)), ctypes.byref(flops), _ptr(sink),
                                              _stream_ptr(stream)))
    return int(flops.value)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return LRA_BF16
    if t.dtype == torch.float32:
        return LRA_F32
    raise LraError(3, f"unsupported torch dtype {t.dtype}")


def make_shape(q: torch.Tensor, n_kv_heads: int, rank: int, scale: float = 0.0,
               key_rope_theta: float = 0.0) -> LraShape:
    return LraShape(int(q.shape[-2]), int(n_kv_heads), int(q.shape[-1]), int(rank), _dtype_code(q),
                    float(scale), float(key_rope_theta))


def make_cache(k_base: torch.Tensor, v_base: torch.Tensor, l: torch.Tensor, seq_lens: torch.Tensor,
               max_seq_len: int, block_table: Optional[torch.Tensor] = None, l_per_adapter: bool = False,
               seq_lens_host=None) -> LraCache:
    """Describe a cache held in torch tensors.
    seq_lens_host: optional host copy of the lengths (a sequence of ints) for launch planning.

    contiguous: k_base/v_base any strided view indexed [token][kv head][d] with a
    unit stride on d; paged: k_base/v_base [num_blocks][Hkv][16][d] (strided view
    allowed), block_table int32 [n_seqs][max_blocks].
    l: one low-rank cache for all adapters, [tokens][r] / [num_blocks][16][r] (rows may be strided);
    with l_per_adapter (BaseShared) a view indexed [adapter][tokens][r] / [adapter][num_blocks][16][r]
    in any storage order with a unit stride on r, e.g. [n][A][r] storage permuted."""
    if k_base.stride() != v_base.stride() or k_base.stride(-1) != 1:
        raise LraError(2, "k_base and v_base must share strides, innermost stride 1")
    l_adapter_stride = 0
    if l_per_adapter:
        l_adapter_stride, l = l.stride(0), l[0]
    if l.stride(-1) != 1:
        raise LraError(2, "l must have a unit stride on the rank")
    mirror = None
    if seq_lens_host is not None:
        vals = [int(x) for x in seq_lens_host]
        mirror = (ctypes.c_int32 * len(vals))(*vals)
    mirror_ptr = None if mirror is None else ctypes.cast(mirror, ctypes.c_void_p)
    if block_table is None:
        if l.dim() != 2:
            raise LraError(2, "contiguous l must be [tokens][r]")
        cache = LraCache(_ptr(k_base), _ptr(v_base), _ptr(l), k_base.stride(0), k_base.stride(1), 0,
                         0, 0, 0, 1, l.stride(0), l_adapter_stride, None, _ptr(seq_lens), int(max_seq_len), mirror_ptr)
    else:
        if l.dim() != 3 or l.stride(0) != 16 * l.stride(1):
            raise LraError(2, "paged l must be [num_blocks][16][r] with the 16 rows of a block one row stride apart")
        cache = LraCache(_ptr(k_base), _ptr(v_base), _ptr(l), k_base.stride(2), k_base.stride(1),
                         k_base.stride(0), int(k_base.shape[2]), int(block_table.shape[1]),
                         int(k_base.shape[0]), int(block_table.shape[0]), l.stride(1), l_adapter_stride, _ptr(block_table),
                         _ptr(seq_lens), int(max_seq_len), mirror_ptr)
    cache._host_mirror = mirror  # the struct holds a raw pointer into it
    return cache


def lra_workspace_bytes(shape: LraShape, cache: LraCache, n_queries: int,
                        max_queries_per_seq: int = 1, n_new: int = 0) -> int:
    """n_new = 0: workspace of a decode call; n_new >= 1: of a prefill call."""
    n = load_library().lra_workspace_bytes(ctypes.byref(shape), ctypes.byref(cache), int(n_queries),
                                           int(max_queries_per_seq), int(n_new), ctypes.byref(_tuning))
    if n == ctypes.c_size_t(-1).value:
        raise LraError(2, "lra_workspace_bytes rejected the arguments")
    return int(n)


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def _check(status: int) -> None:
    if status != LRA_OK:
        raise LraError(status, lra_status_string(status))


def lra_attn_decode(shape: LraShape, cache: LraCache, b_k: Optional[torch.Tensor],
                    b_v: Optional[torch.Tensor], n_adapters: int, q: torch.Tensor,
                    query_adapter: torch.Tensor, seq_query_start: torch.Tensor,
                    max_queries_per_seq: int, out: torch.Tensor, workspace: Optional[torch.Tensor],
                    stream=None) -> None:
    ad = LraAdapters(_ptr(b_k), _ptr(b_v), int(n_adapters))
    ws_ptr = _ptr(workspace)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().lra_attn_decode(
        ctypes.byref(shape), ctypes.byref(cache), ctypes.byref(ad), _ptr(q), _ptr(query_adapter),
        _ptr(seq_query_start), int(q.shape[0]), int(max_queries_per_seq), _ptr(out), ws_ptr,
        ws_bytes, ctypes.byref(_tuning), _stream_ptr(stream)))


def lra_attn_decode_static(shape: LraShape, cache: LraCache, b_k: Optional[torch.Tensor],
                           b_v: Optional[torch.Tensor], n_adapters: int, q: torch.Tensor,
                           query_adapter: torch.Tensor, seq_query_start: torch.Tensor,
                           max_queries_per_seq: int, out: torch.Tensor, stream=None) -> None:
    """lra_attn_decode with the library's own per-device workspace (no allocation anywhere)."""
    ad = LraAdapters(_ptr(b_k), _ptr(b_v), int(n_adapters))
    _check(load_library().lra_attn_decode_static(
        ctypes.byref(shape), ctypes.byref(cache), ctypes.byref(ad), _ptr(q), _ptr(query_adapter),
        _ptr(seq_query_start), int(q.shape[0]), int(max_queries_per_seq), _ptr(out), ctypes.byref(_tuning),
        _stream_ptr(stream)))


def lra_attn_prefill(shape: LraShape, cache: LraCache, b_k: Optional[torch.Tensor],
                     b_v: Optional[torch.Tensor], n_adapters: int, q: torch.Tensor, seq_index: int,
                     adapter_index: int, out: torch.Tensor, workspace: Optional[torch.Tensor],
                     stream=None) -> None:
    ad = LraAdapters(_ptr(b_k), _ptr(b_v), int(n_adapters))
    ws_ptr = _ptr(workspace)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load_library().lra_attn_prefill(
        ctypes.byref(shape), ctypes.byref(cache), ctypes.byref(ad), _ptr(q), int(seq_index),
        int(adapter_index), int(q.shape[0]), _ptr(out), ws_ptr, ws_bytes, ctypes.byref(_tuning), _stream_ptr(stream)))
