"""ctypes binding of the host-side scheduler library (``include/pascal_sched.h``).

Argument marshalling only.  ``Scheduler`` mirrors the C entry points; ``plan``
returns numpy arrays already laid out for ``paged_decode_attn``."""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Tuple

import numpy as np

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libpascal_sched.so")

TOKEN, END_OF_REASONING, END_OF_SEQUENCE = 0, 1, 2
OP_OFFLOAD, OP_RELOAD, OP_PREFILL, OP_GROW, OP_MIGRATE, OP_MIGRATE_HOST, OP_FREE = 1, 2, 3, 4, 5, 6, 7
REASONING, ANSWERING = 0, 1
FLAG_NO_MIGRATION, FLAG_NOT_ADAPTIVE = 1, 2
QUEUED, RESIDENT, OFFLOADED, FINISHED = 0, 1, 2, 3

EXPORTS = (
    "pascal_create", "pascal_destroy", "pascal_submit", "pascal_plan", "pascal_plan_batch",
    "pascal_plan_block_tables", "pascal_ops", "pascal_commit", "pascal_instance_signals",
    "pascal_request", "pascal_request_blocks", "pascal_request_visible_tokens", "pascal_status_string",
)


class Config(ctypes.Structure):
    """Mirror of ``pascal_config``."""
    _fields_ = [("num_instances", ctypes.c_int32), ("gpu_blocks", ctypes.c_int32),
                ("block_tokens", ctypes.c_int32), ("quantum_tokens", ctypes.c_int32),
                ("demote_tokens", ctypes.c_int32), ("headroom_blocks", ctypes.c_int32),
                ("max_batch", ctypes.c_int32), ("flags", ctypes.c_int32),
                ("target_tpot_s", ctypes.c_double)]


class Op(ctypes.Structure):
    """Mirror of ``pascal_op``."""
    _fields_ = [("kind", ctypes.c_int32), ("instance", ctypes.c_int32), ("request", ctypes.c_int32),
                ("other_instance", ctypes.c_int32), ("first_block", ctypes.c_int32),
                ("n_blocks", ctypes.c_int32), ("n_other_blocks", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


class RequestInfo(ctypes.Structure):
    """Mirror of ``pascal_request_info``."""
    _fields_ = [(n, ctypes.c_int32) for n in (
        "instance", "phase", "state", "level", "prompt_tokens", "kv_tokens", "reasoning_tokens",
        "answering_tokens", "n_blocks", "preemptions", "migrations", "reserved")] + \
        [(n, ctypes.c_double) for n in ("arrival", "finish", "ttft", "qoe")]


class SchedError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"pascal_sched status {status}: {text}")
        self.status = status


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is not built; run `python -m paper_2602_11530_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_double
        pi32 = ctypes.POINTER(ctypes.c_int32)
        L.pascal_create.argtypes = [ctypes.POINTER(Config), ctypes.POINTER(vp)]
        L.pascal_destroy.argtypes = [vp]
        L.pascal_destroy.restype = None
        L.pascal_submit.argtypes = [vp, i32, dbl, pi32, pi32]
        L.pascal_plan.argtypes = [vp, i32, pi32, pi32, pi32]
        L.pascal_plan_batch.argtypes = [vp, i32, vp, vp, i32]
        L.pascal_plan_block_tables.argtypes = [vp, i32, vp, i32, i32]
        L.pascal_ops.argtypes = [vp, i32, vp, i32, vp, i32]
        L.pascal_commit.argtypes = [vp, i32, dbl, vp, i32, pi32, pi32]
        L.pascal_instance_signals.argtypes = [vp, i32, dbl, pi32, ctypes.POINTER(ctypes.c_int64),
                                              pi32, pi32, pi32]
        L.pascal_request.argtypes = [vp, i32, ctypes.POINTER(RequestInfo)]
        L.pascal_request_blocks.argtypes = [vp, i32, vp, i32]
        L.pascal_request_visible_tokens.argtypes = [vp, i32, dbl, pi32]
        L.pascal_status_string.argtypes = [ctypes.c_int]
        L.pascal_status_string.restype = ctypes.c_char_p
        for name in EXPORTS:
            if name not in ("pascal_destroy", "pascal_status_string"):
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _check(status: int) -> int:
    if status < 0:
        raise SchedError(status, lib().pascal_status_string(status).decode())
    return status


# (kind, instance, request, blocks, other instance, blocks there)
OpTuple = Tuple[int, int, int, Tuple[int, ...], int, Tuple[int, ...]]


class Scheduler:
    def __init__(self, num_instances=8, gpu_blocks=1024, block_tokens=16, quantum=500,
                 demote_tokens=5000, headroom_blocks=1, tpot=0.1, max_batch=0, migration=True,
                 adaptive=True):
        flags = (0 if migration else FLAG_NO_MIGRATION) | (0 if adaptive else FLAG_NOT_ADAPTIVE)
        self.cfg = Config(num_instances, gpu_blocks, block_tokens, quantum, demote_tokens,
                          headroom_blocks, max_batch, flags, tpot)
        self._h = ctypes.c_void_p()
        _check(lib().pascal_create(ctypes.byref(self.cfg), ctypes.byref(self._h)))

    def __del__(self):
        if getattr(self, "_h", None):
            lib().pascal_destroy(self._h)
            self._h = None

    def submit(self, prompt_tokens: int, now: float) -> Tuple[int, int]:
        rid, inst = ctypes.c_int32(), ctypes.c_int32()
        _check(lib().pascal_submit(self._h, prompt_tokens, now, ctypes.byref(rid), ctypes.byref(inst)))
        return rid.value, inst.value

    def _ops(self, instance: int, n_ops: int, n_blocks: int) -> List[OpTuple]:
        ops = (Op * max(n_ops, 1))()
        blocks = np.empty(max(n_blocks, 1), np.int32)
        _check(lib().pascal_ops(self._h, instance, ctypes.addressof(ops), n_ops,
                                blocks.ctypes.data, n_blocks))
        out = []
        for k in range(n_ops):
            o = ops[k]
            a = blocks[o.first_block:o.first_block + o.n_blocks]
            b = blocks[o.first_block + o.n_blocks:o.first_block + o.n_blocks + o.n_other_blocks]
            out.append((o.kind, o.instance, o.request, tuple(int(x) for x in a), o.other_instance,
                        tuple(int(x) for x in b)))
        return out

    def plan(self, instance: int):
        """(request ids, context lengths after the iteration, ordered data-movement ops)."""
        n_sel, n_ops, n_blk = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
        _check(lib().pascal_plan(self._h, instance, ctypes.byref(n_sel), ctypes.byref(n_ops),
                                 ctypes.byref(n_blk)))
        rids = np.empty(n_sel.value, np.int32)
        lens = np.empty(n_sel.value, np.int32)
        _check(lib().pascal_plan_batch(self._h, instance, rids.ctypes.data, lens.ctypes.data,
                                       n_sel.value))
        return rids.tolist(), lens.tolist(), self._ops(instance, n_ops.value, n_blk.value)

    def block_tables(self, instance: int, n_selected: int, max_blocks_per_seq: int,
                     fill: int = -1) -> np.ndarray:
        """int32 [n_selected, max_blocks_per_seq] for the batch planned last."""
        t = np.empty((n_selected, max_blocks_per_seq), np.int32)
        _check(lib().pascal_plan_block_tables(self._h, instance, t.ctypes.data, max_blocks_per_seq, fill))
        return t

    def commit(self, instance: int, now: float, kinds) -> List[OpTuple]:
        k = np.ascontiguousarray(kinds, dtype=np.int32)
        n_ops, n_blk = ctypes.c_int32(), ctypes.c_int32()
        _check(lib().pascal_commit(self._h, instance, now, k.ctypes.data, len(k),
                                   ctypes.byref(n_ops), ctypes.byref(n_blk)))
        return self._ops(instance, n_ops.value, n_blk.value)

    def signals(self, instance: int, now: float):
        """(t, m, r, a, free blocks) of Algorithms 1 and 2 for one instance."""
        t, r, a, f = (ctypes.c_int32() for _ in range(4))
        m = ctypes.c_int64()
        _check(lib().pascal_instance_signals(self._h, instance, now, ctypes.byref(t), ctypes.byref(m),
                                             ctypes.byref(r), ctypes.byref(a), ctypes.byref(f)))
        return bool(t.value), m.value, r.value, a.value, f.value

    def request(self, rid: int) -> RequestInfo:
        info = RequestInfo()
        _check(lib().pascal_request(self._h, rid, ctypes.byref(info)))
        return info

    def visible_tokens(self, rid: int, now: float) -> int:
        """Answering tokens the pacer has released to the user by ``now``."""
        n = ctypes.c_int32()
        _check(lib().pascal_request_visible_tokens(self._h, rid, now, ctypes.byref(n)))
        return n.value

    def request_blocks(self, rid: int) -> List[int]:
        info = self.request(rid)
        b = np.empty(max(info.n_blocks, 1), np.int32)
        n = _check(lib().pascal_request_blocks(self._h, rid, b.ctypes.data, info.n_blocks))
        return b[:n].tolist()
