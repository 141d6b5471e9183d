"""Thin ctypes binding over libpkv.so: argument marshalling only.

Function names mirror the C ABI (``include/pkv.h``).  Tensors are torch tensors
(used purely as device-memory handles); every step of the computation runs in
the library's HIP kernels.  If the library has not been built the first call
raises — there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libpkv.so")

PKV_OK = 0
PKV_ERR_NULL = -1
PKV_ERR_SHAPE = -2
PKV_ERR_ALIGN = -3
PKV_ERR_WORKSPACE = -4
PKV_ERR_LAUNCH = -5
PKV_ERR_HOST = -6

EXPORTS = (
    "pkv_attn_partition_size", "pkv_attn_workspace_bytes", "paged_decode_attn",
    "paged_decode_attn_layers", "paged_decode_attn_static", "paged_decode_attn_fp8kv",
    "kv_blocks_gather", "kv_blocks_scatter", "kv_blocks_move", "kv_blocks_offload", "kv_blocks_reload",
    "kv_append", "kv_append_fp8", "pkv_set_id_fault_counter", "pkv_status_string",
    "pkv_last_launch_error", "pkv_version", "pkv_probe_stream_read",
)


class AttnShape(ctypes.Structure):
    """Mirror of ``pkv_attn_shape``."""
    _fields_ = [
        ("num_seqs", ctypes.c_int32),
        ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("block_size", ctypes.c_int32),
        ("max_blocks_per_seq", ctypes.c_int32),
        ("partition_size", ctypes.c_int32),
        ("max_context_len", ctypes.c_int32),
        ("num_pool_blocks", ctypes.c_int64),
    ]


class PkvError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"pkv status {status}: {text}")
        self.status = status


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library; raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is not built; run `python -m paper_2602_11530_amd.build` "
                "(there is no fallback path)")
        # PyTorch owns the device memory and the streams this library is handed,
        # so both must sit on one HIP runtime: load torch (and with it the
        # runtime it ships) before libpkv.so resolves its own dependency.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, i32p = ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p
        shp = ctypes.POINTER(AttnShape)
        L.pkv_version.restype = ctypes.c_int
        L.pkv_status_string.argtypes = [ctypes.c_int]
        L.pkv_status_string.restype = ctypes.c_char_p
        L.pkv_last_launch_error.restype = ctypes.c_char_p
        L.pkv_attn_partition_size.argtypes = [shp]
        L.pkv_attn_partition_size.restype = ctypes.c_int
        L.pkv_attn_workspace_bytes.argtypes = [shp, ctypes.POINTER(ctypes.c_size_t)]
        L.pkv_attn_workspace_bytes.restype = ctypes.c_int
        L.paged_decode_attn.argtypes = [vp, vp, vp, i32p, i32p, ctypes.c_float, vp, shp, vp,
                                        ctypes.c_size_t, vp]
        L.paged_decode_attn.restype = ctypes.c_int
        L.paged_decode_attn_fp8kv.argtypes = [vp, vp, vp, i32p, i32p, ctypes.c_float, ctypes.c_float,
                                              ctypes.c_float, vp, shp, vp, ctypes.c_size_t, vp]
        L.paged_decode_attn_fp8kv.restype = ctypes.c_int
        L.paged_decode_attn_static.argtypes = [vp, vp, vp, i32p, i32p, ctypes.c_float, vp, shp, vp]
        L.paged_decode_attn_static.restype = ctypes.c_int
        L.paged_decode_attn_layers.argtypes = [vp, vp, vp, i32p, i32p, ctypes.c_float, vp,
                                               ctypes.c_int32, shp, vp, ctypes.c_size_t, vp]
        L.paged_decode_attn_layers.restype = ctypes.c_int
        L.kv_blocks_gather.argtypes = [vp, i32p, vp, i64, i64, i64, vp]
        L.kv_blocks_gather.restype = ctypes.c_int
        L.kv_blocks_scatter.argtypes = [vp, vp, i32p, i64, i64, i64, vp]
        L.kv_blocks_scatter.restype = ctypes.c_int
        L.kv_blocks_move.argtypes = [vp, i32p, vp, i32p, i64, i64, i64, i64, vp]
        L.kv_blocks_move.restype = ctypes.c_int
        L.kv_blocks_offload.argtypes = [vp, i32p, vp, vp, i64, i64, i64, vp]
        L.kv_blocks_offload.restype = ctypes.c_int
        L.kv_blocks_reload.argtypes = [vp, vp, vp, i32p, i64, i64, i64, vp]
        L.kv_blocks_reload.restype = ctypes.c_int
        L.pkv_probe_stream_read.argtypes = [vp, vp, i64, i64, vp, vp]
        L.pkv_probe_stream_read.restype = ctypes.c_int
        L.pkv_set_id_fault_counter.argtypes = [vp]
        L.pkv_set_id_fault_counter.restype = ctypes.c_int
        L.kv_append_fp8.argtypes = [vp, vp, vp, vp, i32p, i32p, ctypes.c_float, ctypes.c_float, shp, vp]
        L.kv_append_fp8.restype = ctypes.c_int
        L.kv_append.argtypes = [vp, vp, vp, vp, i32p, i32p, shp, vp]
        L.kv_append.restype = ctypes.c_int
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != PKV_OK:
        L = lib()
        text = L.pkv_status_string(status).decode()
        if status == PKV_ERR_LAUNCH:
            text += ": " + L.pkv_last_launch_error().decode()
        raise PkvError(status, text)


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    h = int(getattr(stream, "cuda_stream", stream))
    return h or None


def pkv_set_id_fault_counter(counter) -> None:
    """``counter``: a one-element int32 device tensor that later calls of this thread add the
    number of refused block ids to, or None to switch the report off."""
    _check(lib().pkv_set_id_fault_counter(_ptr(counter)))


def pkv_probe_stream_read(k_buf, v_buf, num_slabs: int, total_blocks: int, sink=None, stream=None) -> None:
    """Measurement aid: the stream pass's loads over ``total_blocks`` hashed slab pairs, no arithmetic."""
    _check(lib().pkv_probe_stream_read(_ptr(k_buf), _ptr(v_buf), num_slabs, total_blocks, _ptr(sink),
                                       _stream(stream)))


def pkv_version() -> int:
    return int(lib().pkv_version())


def make_shape(num_seqs, num_q_heads, num_kv_heads, max_blocks_per_seq, num_pool_blocks,
               head_dim=128, block_size=16, partition_size=0, max_context_len=0) -> AttnShape:
    return AttnShape(num_seqs, num_q_heads, num_kv_heads, head_dim, block_size,
                     max_blocks_per_seq, partition_size, max_context_len, num_pool_blocks)


def pkv_attn_partition_size(shape: AttnShape) -> int:
    p = lib().pkv_attn_partition_size(ctypes.byref(shape))
    if p < 0:
        _check(p)
    return int(p)


def pkv_attn_workspace_bytes(shape: AttnShape) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().pkv_attn_workspace_bytes(ctypes.byref(shape), ctypes.byref(n)))
    return int(n.value)


def paged_decode_attn(q, k_pool, v_pool, block_tables, context_lens, scale, out,
                      shape: AttnShape, workspace=None, stream=None) -> None:
    """Enqueue one batched decode-attention call; see ``include/pkv.h``."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().paged_decode_attn(_ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(block_tables),
                                   _ptr(context_lens), ctypes.c_float(scale), _ptr(out),
                                   ctypes.byref(shape), _ptr(workspace), ws_bytes,
                                   _stream(stream)))


def paged_decode_attn_fp8kv(q, k_pool, v_pool, block_tables, context_lens, scale, k_scale, v_scale,
                            out, shape: AttnShape, workspace=None, stream=None) -> None:
    """Attention over e4m3 KV pools (one byte per element, one fp32 scale per pool)."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().paged_decode_attn_fp8kv(_ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(block_tables),
                                         _ptr(context_lens), ctypes.c_float(scale),
                                         ctypes.c_float(k_scale), ctypes.c_float(v_scale), _ptr(out),
                                         ctypes.byref(shape), _ptr(workspace), ws_bytes,
                                         _stream(stream)))


STATIC_WORKSPACE_BYTES = 32 << 20


def paged_decode_attn_static(q, k_pool, v_pool, block_tables, context_lens, scale, out,
                             shape: AttnShape, stream=None) -> None:
    """The same call on the library's own fixed workspace: allocates nothing."""
    _check(lib().paged_decode_attn_static(_ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(block_tables),
                                          _ptr(context_lens), ctypes.c_float(scale), _ptr(out),
                                          ctypes.byref(shape), _stream(stream)))


def pointer_array(tensors):
    """Host array of the tensors' device pointers, as the multi-layer call takes it.
    Build it once per model: the pools do not move between decode steps."""
    return (ctypes.c_void_p * len(tensors))(*[int(t.data_ptr()) for t in tensors])


def paged_decode_attn_layers(q, k_pools, v_pools, block_tables, context_lens, scale, out,
                             shape: AttnShape, workspace=None, stream=None) -> None:
    """All layers' attention of one decode step in one call.  ``q``, ``k_pools``,
    ``v_pools`` and ``out`` are equally long lists of tensors or ``pointer_array``s."""
    arrs = [a if isinstance(a, ctypes.Array) else pointer_array(a) for a in (q, k_pools, v_pools, out)]
    n = len(arrs[0])
    if any(len(a) != n for a in arrs):
        raise ValueError("q, k_pools, v_pools and out must list the same number of layers")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().paged_decode_attn_layers(arrs[0], arrs[1], arrs[2], _ptr(block_tables),
                                          _ptr(context_lens), ctypes.c_float(scale), arrs[3], n,
                                          ctypes.byref(shape), _ptr(workspace), ws_bytes,
                                          _stream(stream)))


def kv_blocks_gather(pool, block_ids, staging, n_blocks: int, block_bytes: int,
                     num_pool_blocks: int, stream=None) -> None:
    _check(lib().kv_blocks_gather(_ptr(pool), _ptr(block_ids), _ptr(staging), n_blocks,
                                  block_bytes, num_pool_blocks, _stream(stream)))


def kv_blocks_scatter(staging, pool, block_ids, n_blocks: int, block_bytes: int,
                      num_pool_blocks: int, stream=None) -> None:
    _check(lib().kv_blocks_scatter(_ptr(staging), _ptr(pool), _ptr(block_ids), n_blocks,
                                   block_bytes, num_pool_blocks, _stream(stream)))


def kv_blocks_move(src_pool, src_ids, dst_pool, dst_ids, n_blocks: int, block_bytes: int,
                   src_pool_blocks: int, dst_pool_blocks: int, stream=None) -> None:
    """dst_pool[dst_ids[i]] = src_pool[src_ids[i]] in one pass (pools on the same GPU)."""
    _check(lib().kv_blocks_move(_ptr(src_pool), _ptr(src_ids), _ptr(dst_pool), _ptr(dst_ids),
                                n_blocks, block_bytes, src_pool_blocks, dst_pool_blocks,
                                _stream(stream)))


def kv_blocks_offload(pool, block_ids, staging, host_dst, n_blocks: int, block_bytes: int,
                      num_pool_blocks: int, stream=None) -> None:
    """Gather the listed blocks and copy the image to the pinned host tensor ``host_dst``."""
    _check(lib().kv_blocks_offload(_ptr(pool), _ptr(block_ids), _ptr(staging), _ptr(host_dst),
                                   n_blocks, block_bytes, num_pool_blocks, _stream(stream)))


def kv_blocks_reload(host_src, staging, pool, block_ids, n_blocks: int, block_bytes: int,
                     num_pool_blocks: int, stream=None) -> None:
    """Copy a saved image from the pinned host tensor and scatter it into the listed blocks."""
    _check(lib().kv_blocks_reload(_ptr(host_src), _ptr(staging), _ptr(pool), _ptr(block_ids),
                                  n_blocks, block_bytes, num_pool_blocks, _stream(stream)))


def kv_append(k_new, v_new, k_pool, v_pool, block_tables, context_lens, shape: AttnShape,
              stream=None) -> None:
    """Write each request's newest K and V rows into slot context_lens[s] - 1."""
    _check(lib().kv_append(_ptr(k_new), _ptr(v_new), _ptr(k_pool), _ptr(v_pool),
                           _ptr(block_tables), _ptr(context_lens), ctypes.byref(shape),
                           _stream(stream)))


def kv_append_fp8(k_new, v_new, k_pool, v_pool, block_tables, context_lens, k_scale, v_scale,
                  shape: AttnShape, stream=None) -> None:
    """Quantise each request's newest K and V rows to E4M3 and write them into slot context_lens[s] - 1."""
    _check(lib().kv_append_fp8(_ptr(k_new), _ptr(v_new), _ptr(k_pool), _ptr(v_pool),
                               _ptr(block_tables), _ptr(context_lens), ctypes.c_float(k_scale),
                               ctypes.c_float(v_scale), ctypes.byref(shape), _stream(stream)))
