"""The scheduler library driving the kernels: a seeded trace is served on two instances
(two sets of per-layer KV pools on the one GPU).  Every order the scheduler issues is
executed through the C ABI — prefill installs, kv_append + paged_decode_attn per
iteration, preemption through kv_blocks_offload / kv_blocks_reload, phase-transition
migration through kv_blocks_move between the instances' pools.

A host mirror keeps what each request's K and V rows must be, independent of where
they live; attention is compared with the oracle run on the mirror, and a request's
blocks are compared with the mirror whenever they move and when it finishes.  Freed
blocks are overwritten with NaN patterns so that a stale table entry cannot pass."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_11530_amd import binding as pkv
from paper_2602_11530_amd import sched_binding as sb
from paper_2602_11530_amd import workloads as wl

from gpu_util import MAX_ABS, REL_L2, to_bits, to_dev
from serving_driver import replay

pytestmark = pytest.mark.gpu

HQ, HKV, D, B = 40, 8, 128, 16
POISON = 0x7FC1     # a bf16 NaN


class Engine:
    """Executes the scheduler's orders and batches on the GPU and checks them."""

    def __init__(self, sched, n_inst, gpu_blocks, n_layers, maxb, device, seed):
        self.s, self.L, self.NB, self.maxb, self.dev = sched, n_layers, gpu_blocks, maxb, device
        self.rng = np.random.default_rng(seed)
        mk = lambda: torch.full((gpu_blocks, HKV, B, D), POISON, dtype=torch.int16, device=device)
        self.k = [[mk() for _ in range(n_layers)] for _ in range(n_inst)]
        self.v = [[mk() for _ in range(n_layers)] for _ in range(n_inst)]
        self.bb = HKV * B * D * 2
        self.staging = torch.empty((maxb, HKV, B, D), dtype=torch.int16, device=device)
        self.host = {}      # request -> per layer (pinned K image, pinned V image)
        self.mirror = {}    # request -> per layer [K rows, V rows] as uint16 [T, HKV, D]
        self.scale = np.float32(1.0 / np.sqrt(D))
        self.checked_attn = self.checked_blocks = self.iterations = 0
        self.ops_seen = {}

    # ---- helpers ----------------------------------------------------------------------
    def rows(self, n):
        return wl.normal_bf16(self.rng, (n, HKV, D))

    def block_image(self, rows):
        """uint16 [ceil(T/16), HKV, 16, D] holding the rows, unused slots poisoned."""
        T = rows.shape[0]
        nb = -(-T // B)
        img = np.full((nb * B, HKV, D), POISON, np.uint16)
        img[:T] = rows
        return np.ascontiguousarray(img.reshape(nb, B, HKV, D).transpose(0, 2, 1, 3))

    def ids(self, blocks):
        assert all(0 <= b < self.NB for b in blocks)
        return to_dev(np.asarray(blocks, np.int32), self.dev)

    def check_blocks(self, inst, rid, blocks):
        """The request's rows on the GPU equal the mirror (valid slots only)."""
        idx = torch.as_tensor(blocks, dtype=torch.long, device=self.dev)
        for l in range(self.L):
            for pool, rows in ((self.k[inst][l], self.mirror[rid][l][0]), (self.v[inst][l], self.mirror[rid][l][1])):
                T = rows.shape[0]
                got = to_bits(pool.index_select(0, idx[: -(-T // B)]))
                got = got.transpose(0, 2, 1, 3).reshape(-1, HKV, D)[:T]
                assert np.array_equal(got, rows), f"request {rid} layer {l}: KV differs from the mirror"
        self.checked_blocks += 1

    def poison(self, inst, blocks):
        idx = torch.as_tensor(blocks, dtype=torch.long, device=self.dev)
        for l in range(self.L):
            self.k[inst][l][idx] = POISON
            self.v[inst][l][idx] = POISON

    # ---- the scheduler's orders ------------------------------------------------------
    def execute(self, ops):
        for kind, inst, rid, blocks, other, other_blocks in ops:
            self.ops_seen[kind] = self.ops_seen.get(kind, 0) + 1
            n = len(blocks)
            if kind == sb.OP_PREFILL:
                prompt = self.s.request(rid).prompt_tokens
                self.mirror[rid] = [[self.rows(prompt), self.rows(prompt)] for _ in range(self.L)]
                assert n == -(-prompt // B) <= self.maxb
                ids = self.ids(blocks)
                for l in range(self.L):
                    for pool, rows in ((self.k[inst][l], self.mirror[rid][l][0]), (self.v[inst][l], self.mirror[rid][l][1])):
                        self.staging[:n].copy_(to_dev(self.block_image(rows), self.dev))
                        pkv.kv_blocks_scatter(self.staging, pool, ids, n, self.bb, self.NB)
            elif kind in (sb.OP_OFFLOAD, sb.OP_MIGRATE_HOST):
                self.check_blocks(inst, rid, blocks)
                ids = self.ids(blocks)
                images = []
                for l in range(self.L):
                    pair = []
                    for pool in (self.k[inst][l], self.v[inst][l]):
                        h = torch.empty((n, HKV, B, D), dtype=torch.int16, pin_memory=True)
                        pkv.kv_blocks_offload(pool, ids, self.staging, h, n, self.bb, self.NB)
                        pair.append(h)
                    images.append(pair)
                torch.cuda.synchronize()
                self.host[rid] = images
                self.poison(inst, blocks)
            elif kind == sb.OP_RELOAD:
                images = self.host.pop(rid)
                assert n == images[0][0].shape[0]
                ids = self.ids(blocks)
                for l in range(self.L):
                    for pool, h in zip((self.k[inst][l], self.v[inst][l]), images[l]):
                        pkv.kv_blocks_reload(h, self.staging, pool, ids, n, self.bb, self.NB)
                torch.cuda.synchronize()
                self.check_blocks(inst, rid, blocks)
            elif kind == sb.OP_MIGRATE:
                assert len(other_blocks) == n and other != inst
                src, dst = self.ids(blocks), self.ids(other_blocks)
                for l in range(self.L):
                    for a, b in ((self.k[inst][l], self.k[other][l]), (self.v[inst][l], self.v[other][l])):
                        pkv.kv_blocks_move(a, src, b, dst, n, self.bb, self.NB, self.NB)
                self.check_blocks(other, rid, other_blocks)
                self.poison(inst, blocks)
            elif kind == sb.OP_FREE:
                info = self.s.request(rid)
                assert info.state == sb.FINISHED
                self.check_blocks(inst, rid, blocks)
                self.poison(inst, blocks)
                del self.mirror[rid]
            else:
                assert kind == sb.OP_GROW and n >= 1

    # ---- one decode iteration of an instance ----------------------------------------
    def run_batch(self, inst, rids, lens):
        S = len(rids)
        tables = self.s.block_tables(inst, S, self.maxb)
        for s, (rid, L) in enumerate(zip(rids, lens)):
            assert list(tables[s, : -(-L // B)]) == self.s.request_blocks(rid)
        t_d, l_d = to_dev(tables, self.dev), to_dev(np.asarray(lens, np.int32), self.dev)
        shape = pkv.make_shape(S, HQ, HKV, self.maxb, self.NB)
        ws = torch.empty(pkv.pkv_attn_workspace_bytes(shape), dtype=torch.uint8, device=self.dev)
        check_layer = self.iterations % self.L
        for l in range(self.L):
            k_new, v_new = np.empty((S, HKV, D), np.uint16), np.empty((S, HKV, D), np.uint16)
            for s, (rid, L) in enumerate(zip(rids, lens)):
                kr, vr = self.mirror[rid][l]
                if kr.shape[0] == L:            # first run: the prompt is installed already
                    k_new[s], v_new[s] = kr[-1], vr[-1]
                else:                           # a decode step appends this token's rows
                    assert kr.shape[0] == L - 1
                    k_new[s], v_new[s] = self.rows(1)[0], self.rows(1)[0]
                    self.mirror[rid][l] = [np.concatenate([kr, k_new[s:s + 1]]),
                                           np.concatenate([vr, v_new[s:s + 1]])]
            q = wl.normal_bf16(self.rng, (S, HQ, D))
            out = torch.full((S, HQ, D), POISON, dtype=torch.int16, device=self.dev)
            pkv.kv_append(to_dev(k_new, self.dev), to_dev(v_new, self.dev), self.k[inst][l],
                          self.v[inst][l], t_d, l_d, shape)
            pkv.paged_decode_attn(to_dev(q, self.dev), self.k[inst][l], self.v[inst][l], t_d, l_d,
                                  float(self.scale), out, shape, ws)
            if l == check_layer:
                torch.cuda.synchronize()
                self.check_attention(to_bits(out), q, rids, lens, l)
        self.iterations += 1

    def check_attention(self, got, q, rids, lens, layer):
        """Oracle on the mirror, laid out in blocks of its own."""
        imgs_k = [self.block_image(self.mirror[r][layer][0]) for r in rids]
        imgs_v = [self.block_image(self.mirror[r][layer][1]) for r in rids]
        tables = np.full((len(rids), self.maxb), -1, np.int32)
        off = 0
        for s, img in enumerate(imgs_k):
            tables[s, : img.shape[0]] = np.arange(off, off + img.shape[0])
            off += img.shape[0]
        ref = oracle.paged_decode_attn(q, np.concatenate(imgs_k), np.concatenate(imgs_v), tables,
                                       np.asarray(lens, np.int32), self.scale)
        c = oracle.compare(got, ref)
        assert c["max_abs"] <= MAX_ABS and c["rel_l2"] <= REL_L2 and c["worst_seq_rel_l2"] <= 2 * REL_L2, \
            (self.iterations, rids, lens, c)
        self.checked_attn += 1


def test_trace_served_through_the_kernels(device):
    n_inst, gpu_blocks, n_layers, maxb = 2, 72, 2, 20
    trace = wl.serving_trace(n_requests=24, rate_per_s=12.0, prompt=40, lo=24, hi=120,
                             seed=wl.BASE_SEED + 62)
    sched = sb.Scheduler(num_instances=n_inst, gpu_blocks=gpu_blocks, quantum=32, demote_tokens=220,
                         headroom_blocks=1, tpot=0.05)
    eng = Engine(sched, n_inst, gpu_blocks, n_layers, maxb, device, seed=62)
    log = replay(sched, trace, n_inst, on_ops=eng.execute, on_batch=eng.run_batch)
    print(f"{eng.iterations} iterations, {eng.checked_attn} attention checks, {eng.checked_blocks} block "
          f"checks, orders by kind {dict(sorted(eng.ops_seen.items()))}", flush=True)
    assert not eng.mirror and not eng.host, "a request never finished or an image was left behind"
    for kind in (sb.OP_PREFILL, sb.OP_OFFLOAD, sb.OP_RELOAD, sb.OP_GROW, sb.OP_MIGRATE,
                 sb.OP_MIGRATE_HOST, sb.OP_FREE):
        assert eng.ops_seen.get(kind, 0) > 0, f"the trace never exercised order kind {kind}"
    assert eng.ops_seen[sb.OP_PREFILL] == eng.ops_seen[sb.OP_FREE] == len(trace)
    stats = [sched.request(r) for r in range(len(trace))]
    assert all(s.state == sb.FINISHED and s.ttft > 0 and 0 < s.qoe <= 1 + 1e-12 for s in stats)
    assert all(s.kv_tokens == trace.prompt[r] + trace.reasoning[r] + trace.answering[r] - 1
               for r, s in enumerate(stats))
    # every pool is back to all-poison: nothing leaked, every freed block was released
    for i in range(n_inst):
        assert sched.signals(i, 1e9)[4] == gpu_blocks
