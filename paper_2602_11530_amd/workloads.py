"""Seeded synthetic inputs for the paged-decode hot path.

This module only *makes inputs*: context lengths, block tables, block-id lists
and bf16 bit patterns.  It holds none of the attention or copy arithmetic, so it
may serve both the HIP path and the CPU checker without coupling them.

The shapes follow the served model named in the paper's evaluation set-up
(Section V-A: a 32B distilled reasoning model, i.e. 40 query heads, 8 KV heads,
head_dim 128, 64 layers) and the regime the paper studies: long reasoning
contexts next to shorter answering ones (Section III), a KV pool that is full
(Section II-B), and requests whose whole KV cache is evicted or migrated
(Sections II-B, IV-B).  The paper's own traces are not available; these
generators stand in for them.

All tensors are numpy arrays; bf16 tensors are ``uint16`` bit patterns.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

BASE_SEED = 20260211
HEAD_DIM = 128
BLOCK_SIZE = 16


# --------------------------------------------------------------------------
# bf16 bit-pattern helpers (marshalling only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest, ties to even); returns uint16 bits.

    Inputs here are finite; NaN payloads are not treated specially.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns exactly to float64."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def normal_bf16(rng: np.random.Generator, shape) -> np.ndarray:
    """bf16 bit patterns of N(0,1) draws (drawn in fp32, rounded once)."""
    return f32_to_bf16_bits(rng.standard_normal(size=shape, dtype=np.float32))


def normal_e4m3(rng: np.random.Generator, shape, pool_scale: float) -> np.ndarray:
    """E4M3 bytes (uint8) of N(0,1) draws divided by ``pool_scale``: the 8-bit image of a pool
    whose values are ``pool_scale * e4m3(byte)``.  The rounding is the library routine's
    (torch's float8_e4m3fn conversion); draws are clipped to the format's range first."""
    import torch
    x = rng.standard_normal(size=shape, dtype=np.float32) / np.float32(pool_scale)
    x = np.clip(x, -448.0, 448.0)
    return torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()


E4M3_NAN = np.uint8(0x7F)
E4M3_NAN_NEG = np.uint8(0xFF)
BF16_NAN = np.uint16(0x7FC0)
BF16_INF = np.uint16(0x7F80)


# --------------------------------------------------------------------------
# Workload descriptions
# --------------------------------------------------------------------------
@dataclass
class Workload:
    """One batch of decode requests over one or more layers' KV pools."""

    name: str
    num_q_heads: int
    num_kv_heads: int
    context_lens: np.ndarray          # int32 [S]
    block_tables: np.ndarray          # int32 [S, MAXB], unused entries = -1
    num_pool_blocks: int              # NB (per pool)
    num_layers: int = 1
    partition_size: int = 0           # split-K partition in tokens; 0 = library picks
    head_dim: int = HEAD_DIM
    block_size: int = BLOCK_SIZE
    seed: int = BASE_SEED
    phase: Optional[np.ndarray] = None  # per request: 1 = reasoning, 0 = answering
    notes: str = ""

    @property
    def num_seqs(self) -> int:
        return int(self.context_lens.shape[0])

    @property
    def max_blocks_per_seq(self) -> int:
        return int(self.block_tables.shape[1])

    @property
    def scale(self) -> np.float32:
        return np.float32(1.0 / math.sqrt(self.head_dim))

    @property
    def total_tokens(self) -> int:
        return int(self.context_lens.astype(np.int64).sum())

    @property
    def block_elems(self) -> int:
        """bf16 elements in one physical block of one pool (all KV heads)."""
        return self.num_kv_heads * self.block_size * self.head_dim

    @property
    def block_bytes(self) -> int:
        return 2 * self.block_elems

    def pool_shape(self) -> Tuple[int, int, int, int]:
        return (self.num_pool_blocks, self.num_kv_heads, self.block_size, self.head_dim)

    def q_shape(self) -> Tuple[int, int, int]:
        return (self.num_seqs, self.num_q_heads, self.head_dim)

    def used_blocks(self) -> np.ndarray:
        """Blocks per request actually dereferenced: ceil(L/B)."""
        return (self.context_lens.astype(np.int64) + self.block_size - 1) // self.block_size

    def attn_algorithmic_bytes(self) -> int:
        """Bytes one attention call must move: every valid K and V row once
        (shared by the GQA group), q in, out out, the used table entries and
        the lengths.  Workspace traffic and partial-block over-fetch are
        overhead and are not counted."""
        kv = 2 * self.total_tokens * self.num_kv_heads * self.head_dim * 2
        qo = 2 * self.num_seqs * self.num_q_heads * self.head_dim * 2
        tbl = int(self.used_blocks().sum()) * 4 + 4 * self.num_seqs
        return kv + qo + tbl


def _tables_from_perm(lens: np.ndarray, perm: np.ndarray, block_size: int,
                      maxb: Optional[int] = None, fill: int = -1) -> np.ndarray:
    nblk = (lens.astype(np.int64) + block_size - 1) // block_size
    if maxb is None:
        maxb = int(nblk.max()) if len(nblk) else 1
        maxb = max(maxb, 1)
    assert int(nblk.sum()) <= len(perm), "pool too small for the batch"
    assert int(nblk.max(initial=0)) <= maxb
    tables = np.full((len(lens), maxb), fill, dtype=np.int32)
    off = 0
    for s, n in enumerate(nblk):
        n = int(n)
        tables[s, :n] = perm[off:off + n]
        off += n
    return tables


def make_tables(lens, num_pool_blocks: int, rng: np.random.Generator,
                block_size: int = BLOCK_SIZE, maxb: Optional[int] = None,
                fill: int = -1) -> np.ndarray:
    """Cut a seeded permutation of range(NB) consecutively into table rows."""
    lens = np.asarray(lens, dtype=np.int32)
    perm = rng.permutation(num_pool_blocks).astype(np.int32)
    return _tables_from_perm(lens, perm, block_size, maxb, fill)


def custom(lens, num_q_heads: int, num_kv_heads: int, seed: int,
           num_pool_blocks: Optional[int] = None, maxb: Optional[int] = None,
           partition_size: int = 0, name: str = "custom", fill: int = -1,
           block_size: int = BLOCK_SIZE, head_dim: int = HEAD_DIM) -> Workload:
    """Arbitrary lengths (edge-case sweeps), any block size and head dimension."""
    lens = np.asarray(lens, dtype=np.int32)
    need = int(((lens.astype(np.int64) + block_size - 1) // block_size).sum())
    nb = max(need, 1) if num_pool_blocks is None else num_pool_blocks
    rng = np.random.default_rng(seed)
    tables = make_tables(lens, nb, rng, block_size=block_size, maxb=maxb, fill=fill)
    return Workload(name, num_q_heads, num_kv_heads, lens, tables, nb,
                    partition_size=partition_size, head_dim=head_dim, block_size=block_size,
                    seed=seed)


def cfg1_tiny(seed: int = BASE_SEED + 1) -> Workload:
    """Batch 4, 8 query / 2 KV heads, lengths U{17..300}, 128-block pool."""
    rng = np.random.default_rng(seed)
    lens = rng.integers(17, 301, size=4).astype(np.int32)
    tables = make_tables(lens, 128, rng, maxb=19)
    return Workload("cfg1_tiny", 8, 2, lens, tables, 128, seed=seed)


def cfg2_qwen32b(seed: int = BASE_SEED + 2, batch: int = 64,
                 lo: int = 1024, hi: int = 8192, head_dim: int = HEAD_DIM) -> Workload:
    """Batch 64, 40 query / 8 KV heads, lengths U{1024..8192}; the pool holds
    exactly the batch and the tables are a shuffle of it.  (``head_dim`` other
    than 128 gives the same batch for the head-dimension variants.)"""
    rng = np.random.default_rng(seed)
    lens = rng.integers(lo, hi + 1, size=batch).astype(np.int32)
    nb = int(((lens.astype(np.int64) + BLOCK_SIZE - 1) // BLOCK_SIZE).sum())
    tables = make_tables(lens, nb, rng, maxb=(hi + BLOCK_SIZE - 1) // BLOCK_SIZE)
    name = f"cfg2_qwen32b_b{batch}_u{lo}_{hi}" + ("" if head_dim == HEAD_DIM else f"_d{head_dim}")
    return Workload(name, 40, 8, lens, tables, nb, head_dim=head_dim, seed=seed)


def cfg3_long_cot(seed: int = BASE_SEED + 3, batch: int = 128) -> Workload:
    """Batch 128, lognormal lengths (median 6000, sigma 0.8 in natural-log
    units) clipped to [512, 32768], split-K partitions of 512 tokens."""
    rng = np.random.default_rng(seed)
    raw = np.exp(rng.normal(math.log(6000.0), 0.8, size=batch))
    lens = np.clip(np.rint(raw), 512, 32768).astype(np.int32)
    nb = int(((lens.astype(np.int64) + BLOCK_SIZE - 1) // BLOCK_SIZE).sum())
    tables = make_tables(lens, nb, rng, maxb=32768 // BLOCK_SIZE)
    return Workload("cfg3_longcot_b128_lognormal", 40, 8, lens, tables, nb,
                    partition_size=512, seed=seed)


def cfg4_phase_mixed(seed: int = BASE_SEED + 4, batch: int = 96, num_layers: int = 64,
                     spare_blocks: int = 0) -> Workload:
    """Batch 96: 70 % reasoning requests (U{4096..16384}) and 30 % answering
    requests (U{1024..4096}), order shuffled; the same lengths and tables in
    every layer, one K and one V pool per layer."""
    rng = np.random.default_rng(seed)
    n_reason = int(round(0.7 * batch))
    n_answer = batch - n_reason
    lens = np.concatenate([
        rng.integers(4096, 16385, size=n_reason),
        rng.integers(1024, 4097, size=n_answer),
    ]).astype(np.int32)
    phase = np.concatenate([np.ones(n_reason, np.int8), np.zeros(n_answer, np.int8)])
    order = rng.permutation(batch)
    lens, phase = lens[order], phase[order]
    nb = int(((lens.astype(np.int64) + BLOCK_SIZE - 1) // BLOCK_SIZE).sum()) + spare_blocks
    tables = make_tables(lens, nb, rng, maxb=16384 // BLOCK_SIZE)
    return Workload("cfg4_phase_mixed_b96", 40, 8, lens, tables, nb,
                    num_layers=num_layers, seed=seed, phase=phase)


@dataclass
class Migration:
    """One preemption / phase-boundary migration step over a workload."""

    victims: np.ndarray        # int32 request indices being moved
    survivors: np.ndarray      # int32 request indices that keep decoding
    old_ids: np.ndarray        # int32 [n] physical blocks gathered, request-major
    new_ids: np.ndarray        # int32 [n] blocks the staging image is scattered into
    tables_after: np.ndarray   # int32 [S, MAXB] block tables after the move


def make_migration(w: Workload, frac: float = 0.25, seed: Optional[int] = None) -> Migration:
    """Pick a seeded fraction of requests as victims.  Their blocks are gathered
    in request order; the destination ids are a seeded reshuffle of a free list
    made of the pool's spare blocks plus the victims' own just-vacated blocks
    (legal because the gather of a pool completes before its scatter)."""
    seed = w.seed + 5 if seed is None else seed
    rng = np.random.default_rng(seed)
    S = w.num_seqs
    n_v = max(1, int(round(frac * S)))
    perm = rng.permutation(S)
    victims = np.sort(perm[:n_v]).astype(np.int32)
    survivors = np.sort(perm[n_v:]).astype(np.int32)
    used = w.used_blocks()
    old = [w.block_tables[s, :int(used[s])] for s in victims]
    old_ids = np.concatenate(old).astype(np.int32) if old else np.zeros(0, np.int32)
    in_use = np.zeros(w.num_pool_blocks, dtype=bool)
    for s in range(S):
        in_use[w.block_tables[s, :int(used[s])]] = True
    spare = np.nonzero(~in_use)[0].astype(np.int32)
    free = np.concatenate([spare, old_ids])
    new_ids = rng.permutation(free)[:len(old_ids)].astype(np.int32)
    tables_after = w.block_tables.copy()
    off = 0
    for s in victims:
        n = int(used[s])
        tables_after[s, :n] = new_ids[off:off + n]
        off += n
    return Migration(victims, survivors, old_ids, new_ids, tables_after)


def subset(w: Workload, idx) -> Workload:
    """The same pools seen by a sub-batch (continuous batching changes the
    batch every step; the pool and the other requests' blocks stay put)."""
    idx = np.asarray(idx, dtype=np.int64)
    return Workload(w.name + "_subset", w.num_q_heads, w.num_kv_heads,
                    np.ascontiguousarray(w.context_lens[idx]),
                    np.ascontiguousarray(w.block_tables[idx]),
                    w.num_pool_blocks, num_layers=w.num_layers,
                    partition_size=w.partition_size, block_size=w.block_size, seed=w.seed,
                    phase=None if w.phase is None else w.phase[idx])


def make_host_tensors(w: Workload, layer: int = 0, poison_unused: bool = False):
    """q, K pool, V pool as bf16 bit patterns (uint16), N(0,1).

    ``poison_unused`` overwrites every slot no request may read (whole unused
    blocks and the tail slots of each last block) with NaN / Inf patterns."""
    rng = np.random.default_rng(w.seed + 1000 * layer + 17)
    q = normal_bf16(rng, w.q_shape())
    k = normal_bf16(rng, w.pool_shape())
    v = normal_bf16(rng, w.pool_shape())
    if poison_unused:
        valid = np.zeros((w.num_pool_blocks, w.block_size), dtype=bool)
        used = w.used_blocks()
        for s in range(w.num_seqs):
            L = int(w.context_lens[s])
            for j in range(int(used[s])):
                n = min(w.block_size, L - j * w.block_size)
                valid[w.block_tables[s, j], :n] = True
        mask = ~valid
        k[mask[:, None, :, None].repeat(w.num_kv_heads, 1).repeat(w.head_dim, 3)] = BF16_NAN
        v[mask[:, None, :, None].repeat(w.num_kv_heads, 1).repeat(w.head_dim, 3)] = BF16_INF
    return q, k, v


def make_host_tensors_fp8(w: Workload, k_scale: float, v_scale: float, layer: int = 0,
                          poison_unused: bool = False):
    """q as bf16 bit patterns, K pool and V pool as E4M3 bytes (uint8) such that
    scale * e4m3(byte) ~ N(0,1).  ``poison_unused`` fills every slot no request may read with
    the format's two NaN bytes."""
    rng = np.random.default_rng(w.seed + 1000 * layer + 19)
    q = normal_bf16(rng, w.q_shape())
    k = normal_e4m3(rng, w.pool_shape(), k_scale)
    v = normal_e4m3(rng, w.pool_shape(), v_scale)
    if poison_unused:
        valid = np.zeros((w.num_pool_blocks, w.block_size), dtype=bool)
        used = w.used_blocks()
        for s in range(w.num_seqs):
            L = int(w.context_lens[s])
            for j in range(int(used[s])):
                n = min(w.block_size, L - j * w.block_size)
                valid[w.block_tables[s, j], :n] = True
        mask = (~valid)[:, None, :, None].repeat(w.num_kv_heads, 1).repeat(w.head_dim, 3)
        k[mask] = E4M3_NAN
        v[mask] = E4M3_NAN_NEG
    return q, k, v


@dataclass
class ServingTrace:
    """Synthetic request trace for the scheduler: arrival times (seconds,
    ascending) and, per request, the prompt length and the number of reasoning
    and answering tokens the model will emit (the last reasoning token is the
    end-of-reasoning marker, the last answering token ends the sequence)."""
    arrival: np.ndarray
    prompt: np.ndarray
    reasoning: np.ndarray
    answering: np.ndarray
    seed: int

    def __len__(self) -> int:
        return len(self.arrival)


def serving_trace(n_requests: int = 300, rate_per_s: float = 4.0, prompt: int = 128,
                  lo: int = 128, hi: int = 2048, seed: int = BASE_SEED + 6) -> ServingTrace:
    """Poisson arrivals; fixed prompt length; reasoning and answering lengths
    uniform in [lo, hi] — the shape of the paper's synthetic characterization
    workload (Section III-A: 300 requests, prompt 128, 128..2048 tokens per phase)."""
    rng = np.random.default_rng(seed)
    arrival = np.cumsum(rng.exponential(1.0 / rate_per_s, size=n_requests))
    return ServingTrace(arrival, np.full(n_requests, prompt, np.int32),
                        rng.integers(lo, hi + 1, size=n_requests).astype(np.int32),
                        rng.integers(lo, hi + 1, size=n_requests).astype(np.int32), seed)
