"""fp64 CPU checker for paged decode attention and KV page copies.

TEST INFRASTRUCTURE ONLY.  Imported by ``tests/``, by the smoke check and by the
benchmark's ``cpu_baseline`` leg; the product package never imports it and it
never imports the product's binding.  The arithmetic lives in
``pkv_oracle.c`` (plain C, fp64, the textbook definition restated in that
file's header); this module compiles it with gcc and marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import time
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pkv_oracle.c")
_SO = os.path.join(_HERE, "libpkv_oracle.so")
_lib: Optional[ctypes.CDLL] = None


def build(force: bool = False) -> str:
    """Compile the checker with gcc (OpenMP) if missing or stale."""
    stale = (not os.path.exists(_SO)) or os.path.getmtime(_SO) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _SO + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _SO)
    return _SO


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, p = ctypes.c_int64, ctypes.c_void_p
        lib.pkv_oracle_paged_decode_attn.argtypes = [p, p, p, p, p, ctypes.c_float, p,
                                                     i64, i64, i64, i64, i64, i64, i64,
                                                     ctypes.c_int]
        lib.pkv_oracle_paged_decode_attn.restype = ctypes.c_int
        lib.pkv_oracle_paged_decode_attn_fp8kv.argtypes = [p, p, p, p, p, ctypes.c_float,
                                                           ctypes.c_float, ctypes.c_float, p,
                                                           i64, i64, i64, i64, i64, i64, i64,
                                                           ctypes.c_int]
        lib.pkv_oracle_paged_decode_attn_fp8kv.restype = ctypes.c_int
        lib.pkv_oracle_to_e4m3.argtypes = [ctypes.c_float]
        lib.pkv_oracle_to_e4m3.restype = ctypes.c_uint8
        lib.pkv_oracle_kv_append_fp8.argtypes = [p, p, p, p, p, p, ctypes.c_float, ctypes.c_float,
                                                 i64, i64, i64, i64, i64, i64]
        lib.pkv_oracle_kv_append_fp8.restype = ctypes.c_int
        lib.pkv_oracle_e4m3.argtypes = [ctypes.c_uint8]
        lib.pkv_oracle_e4m3.restype = ctypes.c_double
        lib.pkv_oracle_kv_blocks_gather.argtypes = [p, p, p, i64, i64, i64]
        lib.pkv_oracle_kv_blocks_gather.restype = ctypes.c_int
        lib.pkv_oracle_kv_blocks_scatter.argtypes = [p, p, p, i64, i64, i64]
        lib.pkv_oracle_kv_blocks_scatter.restype = ctypes.c_int
        lib.pkv_oracle_kv_blocks_move.argtypes = [p, p, p, p, i64, i64, i64, i64]
        lib.pkv_oracle_kv_blocks_move.restype = ctypes.c_int
        lib.pkv_oracle_max_threads.restype = ctypes.c_int
        lib.pkv_oracle_kv_append.argtypes = [p, p, p, p, p, p, i64, i64, i64, i64, i64, i64]
        lib.pkv_oracle_kv_append.restype = ctypes.c_int
        _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().pkv_oracle_max_threads())


def _c(a: np.ndarray, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.dtype(dtype):
        raise TypeError(f"expected {np.dtype(dtype)}, got {a.dtype}")
    return a


def paged_decode_attn(q, k_pool, v_pool, block_tables, context_lens, scale,
                      threads: int = 0) -> np.ndarray:
    """fp64 reference [S, Hq, D] from bf16 bit patterns (uint16 arrays).

    q [S,Hq,D]; k_pool, v_pool [NB,Hkv,B,D]; block_tables int32 [S,MAXB];
    context_lens int32 [S]; scale is cast to fp32 first, as the library's is.
    """
    q = _c(q, np.uint16)
    k_pool = _c(k_pool, np.uint16)
    v_pool = _c(v_pool, np.uint16)
    block_tables = _c(block_tables, np.int32)
    context_lens = _c(context_lens, np.int32)
    S, Hq, D = q.shape
    NB, Hkv, B, D2 = k_pool.shape
    if v_pool.shape != k_pool.shape or D2 != D or block_tables.shape[0] != S \
            or context_lens.shape != (S,):
        raise ValueError("inconsistent shapes")
    ref = np.empty((S, Hq, D), dtype=np.float64)
    rc = _load().pkv_oracle_paged_decode_attn(
        q.ctypes.data, k_pool.ctypes.data, v_pool.ctypes.data, block_tables.ctypes.data,
        context_lens.ctypes.data, ctypes.c_float(np.float32(scale)), ref.ctypes.data,
        S, Hq, Hkv, D, B, block_tables.shape[1], NB, int(threads))
    if rc != 0:
        raise ValueError(f"oracle rejected its input (code {rc})")
    return ref


def e4m3(byte: int) -> float:
    """Value of one OCP FP8 E4M3 byte (NaN for 0x7F and 0xFF)."""
    return float(_load().pkv_oracle_e4m3(int(byte) & 0xFF))


def to_e4m3(y) -> int:
    """E4M3 byte of one fp32 value: nearest, ties to even, saturating at +-448."""
    return int(_load().pkv_oracle_to_e4m3(ctypes.c_float(np.float32(y))))


def kv_append_fp8(k_new, v_new, k_pool, v_pool, block_tables, context_lens, k_scale, v_scale):
    """Copies of the E4M3 pools with every request's newest K,V row (bf16 bits [S,Hkv,D]), divided
    by the pool's scale and rounded to E4M3, at position L_s - 1."""
    k_new, v_new = _c(k_new, np.uint16), _c(v_new, np.uint16)
    k_out = np.array(_c(k_pool, np.uint8), copy=True, order="C")
    v_out = np.array(_c(v_pool, np.uint8), copy=True, order="C")
    block_tables, context_lens = _c(block_tables, np.int32), _c(context_lens, np.int32)
    S, Hkv, D = k_new.shape
    NB, Hkv2, B, D2 = k_out.shape
    if (Hkv2, D2) != (Hkv, D) or v_new.shape != k_new.shape or v_out.shape != k_out.shape:
        raise ValueError("inconsistent shapes")
    rc = _load().pkv_oracle_kv_append_fp8(k_new.ctypes.data, v_new.ctypes.data, k_out.ctypes.data,
                                          v_out.ctypes.data, block_tables.ctypes.data,
                                          context_lens.ctypes.data, ctypes.c_float(np.float32(k_scale)),
                                          ctypes.c_float(np.float32(v_scale)), S, Hkv, D, B,
                                          block_tables.shape[1], NB)
    if rc != 0:
        raise ValueError(f"oracle rejected its input (code {rc})")
    return k_out, v_out


def paged_decode_attn_fp8kv(q, k_pool, v_pool, block_tables, context_lens, scale, k_scale, v_scale,
                            threads: int = 0) -> np.ndarray:
    """fp64 reference [S, Hq, D] for E4M3 pools: q bf16 bits [S,Hq,D]; k_pool, v_pool uint8
    [NB,Hkv,B,D]; K = k_scale * e4m3(byte), V = v_scale * e4m3(byte) (scales cast to fp32)."""
    q = _c(q, np.uint16)
    k_pool, v_pool = _c(k_pool, np.uint8), _c(v_pool, np.uint8)
    block_tables, context_lens = _c(block_tables, np.int32), _c(context_lens, np.int32)
    S, Hq, D = q.shape
    NB, Hkv, B, D2 = k_pool.shape
    if v_pool.shape != k_pool.shape or D2 != D or block_tables.shape[0] != S \
            or context_lens.shape != (S,):
        raise ValueError("inconsistent shapes")
    ref = np.empty((S, Hq, D), dtype=np.float64)
    rc = _load().pkv_oracle_paged_decode_attn_fp8kv(
        q.ctypes.data, k_pool.ctypes.data, v_pool.ctypes.data, block_tables.ctypes.data,
        context_lens.ctypes.data, ctypes.c_float(np.float32(scale)),
        ctypes.c_float(np.float32(k_scale)), ctypes.c_float(np.float32(v_scale)), ref.ctypes.data,
        S, Hq, Hkv, D, B, block_tables.shape[1], NB, int(threads))
    if rc != 0:
        raise ValueError(f"oracle rejected its input (code {rc})")
    return ref


def kv_blocks_gather(pool: np.ndarray, block_ids) -> np.ndarray:
    """Contiguous image [n, ...block shape] of the listed pages of ``pool``."""
    pool = np.ascontiguousarray(pool)
    ids = _c(np.asarray(block_ids), np.int32)
    NB = pool.shape[0]
    bb = pool.nbytes // NB if NB else 0
    staging = np.empty((len(ids),) + pool.shape[1:], dtype=pool.dtype)
    if len(ids) == 0:
        return staging
    rc = _load().pkv_oracle_kv_blocks_gather(pool.ctypes.data, ids.ctypes.data,
                                             staging.ctypes.data, len(ids), bb, NB)
    if rc != 0:
        raise ValueError(f"oracle rejected its input (code {rc})")
    return staging


def kv_blocks_scatter(staging: np.ndarray, pool: np.ndarray, block_ids) -> np.ndarray:
    """A copy of ``pool`` with page ids[i] replaced by staging[i]."""
    staging = np.ascontiguousarray(staging)
    out = np.array(pool, copy=True, order="C")
    ids = _c(np.asarray(block_ids), np.int32)
    NB = out.shape[0]
    if len(ids) == 0:
        return out
    bb = out.nbytes // NB
    if staging.nbytes != bb * len(ids):
        raise ValueError("staging size does not match the id list")
    rc = _load().pkv_oracle_kv_blocks_scatter(staging.ctypes.data, out.ctypes.data,
                                              ids.ctypes.data, len(ids), bb, NB)
    if rc != 0:
        raise ValueError(f"oracle rejected its input (code {rc})")
    return out


def kv_blocks_move(src_pool: np.ndarray, src_ids, dst_pool: np.ndarray, dst_ids) -> np.ndarray:
    """A copy of ``dst_pool`` with page dst_ids[i] replaced by page src_ids[i] of ``src_pool``."""
    src = np.ascontiguousarray(src_pool)
    out = np.array(dst_pool, copy=True, order="C")
    a, b = _c(np.asarray(src_ids), np.int32), _c(np.asarray(dst_ids), np.int32)
    if len(a) != len(b):
        raise ValueError("the two id lists differ in length")
    if len(a) == 0:
        return out
    bb = src.nbytes // src.shape[0]
    if out.nbytes // out.shape[0] != bb:
        raise ValueError("the pools' block sizes differ")
    rc = _load().pkv_oracle_kv_blocks_move(src.ctypes.data, a.ctypes.data, out.ctypes.data,
                                           b.ctypes.data, len(a), bb, src.shape[0], out.shape[0])
    if rc != 0:
        raise ValueError(f"oracle rejected its input (code {rc})")
    return out


def kv_append(k_new, v_new, k_pool, v_pool, block_tables, context_lens):
    """Copies of the pools with every request's newest K,V row at position L_s - 1."""
    k_new, v_new = _c(k_new, np.uint16), _c(v_new, np.uint16)
    k_out = np.array(_c(k_pool, np.uint16), copy=True, order="C")
    v_out = np.array(_c(v_pool, np.uint16), copy=True, order="C")
    block_tables, context_lens = _c(block_tables, np.int32), _c(context_lens, np.int32)
    S, Hkv, D = k_new.shape
    NB, Hkv2, B, D2 = k_out.shape
    if (Hkv2, D2) != (Hkv, D) or v_new.shape != k_new.shape or v_out.shape != k_out.shape:
        raise ValueError("inconsistent shapes")
    rc = _load().pkv_oracle_kv_append(k_new.ctypes.data, v_new.ctypes.data, k_out.ctypes.data,
                                      v_out.ctypes.data, block_tables.ctypes.data,
                                      context_lens.ctypes.data, S, Hkv, D, B,
                                      block_tables.shape[1], NB)
    if rc != 0:
        raise ValueError(f"oracle rejected its input (code {rc})")
    return k_out, v_out


def timed_attn(q, k_pool, v_pool, block_tables, context_lens, scale, threads: int = 0):
    """(reference, seconds, threads used) for the benchmark's baseline leg."""
    t0 = time.perf_counter()
    ref = paged_decode_attn(q, k_pool, v_pool, block_tables, context_lens, scale, threads)
    dt = time.perf_counter() - t0
    return ref, dt, (threads if threads > 0 else max_threads())


def compare(gpu_bf16_bits: np.ndarray, ref: np.ndarray) -> dict:
    """max-abs, relative L2 over the whole tensor, worst per-sequence rel-L2."""
    got = (np.ascontiguousarray(gpu_bf16_bits, dtype=np.uint16).astype(np.uint32)
           << np.uint32(16)).view(np.float32).astype(np.float64).reshape(ref.shape)
    diff = got - ref
    den = float(np.sqrt((ref * ref).sum()))
    out = {
        "max_abs": float(np.abs(diff).max()) if diff.size else 0.0,
        "rel_l2": float(np.sqrt((diff * diff).sum()) / den) if den > 0 else
        float(np.sqrt((diff * diff).sum())),
        "worst_seq_rel_l2": 0.0,
    }
    if ref.ndim == 3 and ref.shape[0]:
        num = np.sqrt((diff * diff).reshape(ref.shape[0], -1).sum(1))
        dn = np.sqrt((ref * ref).reshape(ref.shape[0], -1).sum(1))
        ok = dn > 0
        if ok.any():
            out["worst_seq_rel_l2"] = float((num[ok] / dn[ok]).max())
    return out
