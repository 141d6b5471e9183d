"""CPU-only checks of the C-ABI layer: the library loads, exports every symbol
the header declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

from paper_2602_11530_amd import binding as pkv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "pkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b([a-z_][a-z0-9_]*)\s*\(", text)) - {"defined"}


def test_exports_match_header():
    L = pkv.lib()
    syms = declared_symbols()
    assert syms == set(pkv.EXPORTS)
    for s in syms:
        assert getattr(L, s) is not None
    assert pkv.pkv_version() >= 1000


def test_shape_struct_layout():
    assert ctypes.sizeof(pkv.AttnShape) == 40 and pkv.AttnShape.num_pool_blocks.offset == 32


def test_status_strings():
    L = pkv.lib()
    seen = {L.pkv_status_string(c) for c in range(0, -7, -1)}
    assert len(seen) == 7 and b"unknown status" not in seen
    assert L.pkv_status_string(-99) == b"unknown status"


def test_partition_and_workspace():
    sh = pkv.make_shape(128, 40, 8, 2048, 70000, partition_size=512)
    assert pkv.pkv_attn_partition_size(sh) == 512
    a16 = lambda x: (x + 15) // 16 * 16
    rec = (5 * 128 + 32) * 4             # one record: 5 rows of 128 floats + 16 (max, sum) pairs
    slots = 8 * 128 + 2048               # (request, KV head) segments + stream wavefronts
    assert pkv.pkv_attn_workspace_bytes(sh) == slots * rec + a16(129 * 4)
    sh.max_context_len = 512             # neither the bound nor the partition changes the size:
    sh.partition_size = 16               # runs are folded per (wavefront, segment) before they leave LDS
    assert pkv.pkv_attn_workspace_bytes(sh) == slots * rec + a16(129 * 4)
    # head dimensions 64 and 256: the record rows follow D
    for D, G in ((64, 5), (256, 5), (256, 8), (64, 16)):
        shd = pkv.make_shape(128, 8 * G, 8, 2048, 70000, head_dim=D)
        assert pkv.pkv_attn_workspace_bytes(shd) == slots * (G * D + 32) * 4 + a16(129 * 4)
    sh = pkv.make_shape(4, 8, 2, 19, 128)
    P = pkv.pkv_attn_partition_size(sh)
    assert P % 16 == 0 and 16 <= P <= 65536
    assert pkv.pkv_attn_workspace_bytes(pkv.make_shape(0, 8, 2, 19, 128)) == 0


@pytest.mark.parametrize("kw", [
    dict(head_dim=96), dict(head_dim=32), dict(head_dim=512), dict(head_dim=256, num_q_heads=32), dict(block_size=48), dict(block_size=128), dict(block_size=8),
    dict(block_size=32, partition_size=16), dict(block_size=64, num_pool_blocks=2 ** 29), dict(num_q_heads=9), dict(num_kv_heads=0), dict(num_q_heads=16384 + 4096, num_kv_heads=4096 + 1024),
    dict(partition_size=24), dict(partition_size=65536 + 16), dict(num_seqs=2049), dict(partition_size=-16),
    dict(max_blocks_per_seq=0), dict(num_seqs=-1), dict(max_context_len=20 * 16),
    dict(max_context_len=-1), dict(num_pool_blocks=0), dict(num_pool_blocks=2 ** 31),
])
def test_bad_shapes(kw):
    base = dict(num_seqs=4, num_q_heads=8, num_kv_heads=2, max_blocks_per_seq=19,
                num_pool_blocks=128)
    base.update(kw)
    sh = pkv.make_shape(**base)
    with pytest.raises(pkv.PkvError) as e:
        pkv.pkv_attn_workspace_bytes(sh)
    assert e.value.status == pkv.PKV_ERR_SHAPE
    L = pkv.lib()
    rc = L.paged_decode_attn(16, 16, 16, 16, 16, 1.0, 16, ctypes.byref(sh), None, 0, None)
    assert rc == pkv.PKV_ERR_SHAPE


def test_attn_argument_errors_before_launch():
    L = pkv.lib()
    sh = pkv.make_shape(4, 8, 2, 19, 128, partition_size=16)
    need = pkv.pkv_attn_workspace_bytes(sh)
    assert need > 0
    call = lambda *a: L.paged_decode_attn(*a)
    assert call(None, 16, 16, 16, 16, 1.0, 16, ctypes.byref(sh), 16, need, None) == pkv.PKV_ERR_NULL
    assert call(16, 16, 16, 16, 16, 1.0, None, ctypes.byref(sh), 16, need, None) == pkv.PKV_ERR_NULL
    assert call(16, 16, 16, 16, 16, 1.0, 16, None, 16, need, None) == pkv.PKV_ERR_NULL
    assert call(24, 16, 16, 16, 16, 1.0, 16, ctypes.byref(sh), 16, need, None) == pkv.PKV_ERR_ALIGN
    assert call(16, 16, 16, 18, 16, 1.0, 16, ctypes.byref(sh), 16, need, None) == pkv.PKV_ERR_ALIGN
    assert call(16, 16, 16, 16, 16, 1.0, 16, ctypes.byref(sh), None, need, None) == pkv.PKV_ERR_WORKSPACE
    assert call(16, 16, 16, 16, 16, 1.0, 16, ctypes.byref(sh), 16, need - 1, None) == pkv.PKV_ERR_WORKSPACE
    assert call(16, 16, 16, 16, 16, 1.0, 16, ctypes.byref(sh), 24, need, None) == pkv.PKV_ERR_ALIGN
    sh0 = pkv.make_shape(0, 8, 2, 19, 128)
    assert call(None, None, None, None, None, 1.0, None, ctypes.byref(sh0), None, 0, None) == pkv.PKV_OK


def test_copy_argument_errors_before_launch():
    L = pkv.lib()
    for fn, args in ((L.kv_blocks_gather, lambda a, b, c: (a, b, c)),
                     (L.kv_blocks_scatter, lambda a, b, c: (c, a, b))):
        # (pool, ids, staging) reordered per entry point
        assert fn(*args(16, 16, 16), 0, 32768, 64, None) == pkv.PKV_OK
        assert fn(*args(None, None, None), 0, 32768, 64, None) == pkv.PKV_OK
        assert fn(*args(16, 16, 16), -1, 32768, 64, None) == pkv.PKV_ERR_SHAPE
        assert fn(*args(16, 16, 16), 4, 0, 64, None) == pkv.PKV_ERR_SHAPE
        assert fn(*args(16, 16, 16), 4, 32768, -1, None) == pkv.PKV_ERR_SHAPE
        assert fn(*args(16, 16, 16), 4, 40, 64, None) == pkv.PKV_ERR_ALIGN
        assert fn(*args(None, 16, 16), 4, 32768, 64, None) == pkv.PKV_ERR_NULL
        assert fn(*args(16, None, 16), 4, 32768, 64, None) == pkv.PKV_ERR_NULL
        assert fn(*args(16, 16, None), 4, 32768, 64, None) == pkv.PKV_ERR_NULL
        assert fn(*args(24, 16, 16), 4, 32768, 64, None) == pkv.PKV_ERR_ALIGN
        assert fn(*args(16, 18, 16), 4, 32768, 64, None) == pkv.PKV_ERR_ALIGN


def test_append_argument_errors_before_launch():
    L = pkv.lib()
    sh = pkv.make_shape(4, 8, 2, 19, 128)
    call = lambda *a: L.kv_append(*a)
    assert call(None, 16, 16, 16, 16, 16, ctypes.byref(sh), None) == pkv.PKV_ERR_NULL
    assert call(16, 16, 16, None, 16, 16, ctypes.byref(sh), None) == pkv.PKV_ERR_NULL
    assert call(16, 16, 16, 16, 16, 16, None, None) == pkv.PKV_ERR_NULL
    assert call(16, 24, 16, 16, 16, 16, ctypes.byref(sh), None) == pkv.PKV_ERR_ALIGN
    assert call(16, 16, 16, 16, 18, 16, ctypes.byref(sh), None) == pkv.PKV_ERR_ALIGN
    bad = pkv.make_shape(4, 8, 3, 19, 128)
    assert call(16, 16, 16, 16, 16, 16, ctypes.byref(bad), None) == pkv.PKV_ERR_SHAPE
    sh0 = pkv.make_shape(0, 8, 2, 19, 128)
    assert call(None, None, None, None, None, None, ctypes.byref(sh0), None) == pkv.PKV_OK


def test_layers_argument_errors_before_launch():
    L = pkv.lib()
    sh = pkv.make_shape(4, 8, 2, 19, 128, partition_size=16)
    need = pkv.pkv_attn_workspace_bytes(sh)
    arr = lambda *v: (ctypes.c_void_p * len(v))(*v)
    good = arr(16, 32, 48)
    call = lambda q, k, v, o, n, ws=16, nbytes=need, shape=sh, tables=16: L.paged_decode_attn_layers(
        q, k, v, tables, 16, 1.0, o, n, ctypes.byref(shape), ws, nbytes, None)
    assert call(good, good, good, good, -1) == pkv.PKV_ERR_SHAPE
    assert call(None, None, None, None, 0) == pkv.PKV_OK
    assert call(None, good, good, good, 3) == pkv.PKV_ERR_NULL
    assert call(good, good, arr(16, None, 48), good, 3) == pkv.PKV_ERR_NULL
    # a bad pointer in the last layer is found before anything is launched
    assert call(good, good, good, arr(16, 32, 40), 3) == pkv.PKV_ERR_ALIGN
    assert call(good, good, good, good, 3, nbytes=need - 1) == pkv.PKV_ERR_WORKSPACE
    assert call(good, good, good, good, 3, tables=18) == pkv.PKV_ERR_ALIGN
    bad = pkv.make_shape(4, 9, 2, 19, 128)
    assert call(good, good, good, good, 3, shape=bad) == pkv.PKV_ERR_SHAPE
    sh0 = pkv.make_shape(0, 8, 2, 19, 128)
    assert call(None, None, None, None, 3, ws=None, nbytes=0, shape=sh0) == pkv.PKV_OK


def test_offload_reload_argument_errors_before_launch():
    L = pkv.lib()
    # offload(pool, ids, staging, host, ...), reload(host, staging, pool, ids, ...)
    off = lambda pool, ids, stg, host, *a: L.kv_blocks_offload(pool, ids, stg, host, *a, None)
    rel = lambda pool, ids, stg, host, *a: L.kv_blocks_reload(host, stg, pool, ids, *a, None)
    for fn in (off, rel):
        assert fn(None, None, None, None, 0, 32768, 64) == pkv.PKV_OK
        assert fn(16, 16, 16, 16, -1, 32768, 64) == pkv.PKV_ERR_SHAPE
        assert fn(16, 16, 16, 16, 4, 40, 64) == pkv.PKV_ERR_ALIGN
        assert fn(None, 16, 16, 16, 4, 32768, 64) == pkv.PKV_ERR_NULL
        assert fn(16, 16, None, 16, 4, 32768, 64) == pkv.PKV_ERR_NULL
        assert fn(16, 16, 16, None, 4, 32768, 64) == pkv.PKV_ERR_NULL
        assert fn(16, 18, 16, 16, 4, 32768, 64) == pkv.PKV_ERR_ALIGN
        # an address that is not page-locked host memory is refused, nothing is enqueued
        assert fn(16, 16, 16, 4096, 4, 32768, 64) == pkv.PKV_ERR_HOST
        buf = ctypes.create_string_buffer(4 * 32768)
        assert fn(16, 16, 16, ctypes.addressof(buf), 4, 32768, 64) == pkv.PKV_ERR_HOST


def test_headers_are_plain_c(tmp_path):
    """Both public headers compile as strict C99 and a C program links against the libraries."""
    import subprocess
    src = tmp_path / "use_abi.c"
    src.write_text(r'''
#include <stdio.h>
#include "pkv.h"
#include "pascal_sched.h"
int main(void) {
  pkv_attn_shape sh = {4, 8, 2, 128, 16, 19, 0, 0, 128};
  size_t bytes = 0;
  pascal_config cfg = {2, 64, 16, 500, 5000, 1, 0, 0, 0.1};
  pascal_sched* s = 0;
  int32_t rid = -1, inst = -1;
  if (pkv_attn_workspace_bytes(&sh, &bytes) != PKV_OK || bytes == 0) return 1;
  if (kv_blocks_gather(0, 0, 0, 0, 32768, 4, 0) != PKV_OK) return 2;
  if (pascal_create(&cfg, &s) != PASCAL_OK) return 3;
  if (pascal_submit(s, 40, 0.0, &rid, &inst) != PASCAL_OK || rid != 0) return 4;
  pascal_destroy(s);
  printf("%d %s\n", pkv_version(), pascal_status_string(0));
  return 0;
}
''')
    exe = tmp_path / "use_abi"
    pkg = os.path.join(ROOT, "paper_2602_11530_amd")
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror",
                           "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe),
                           "-L", pkg, "-lpkv", "-lpascal_sched", f"-Wl,-rpath,{pkg}",
                           "-Wl,-rpath,/opt/rocm/lib", "-L/opt/rocm/lib"])
    out = subprocess.check_output([str(exe)]).decode().split()
    assert int(out[0]) >= 1000 and out[1] == "ok"


def test_move_argument_errors_before_launch():
    L = pkv.lib()
    f = lambda sp, si, dp, di, n, bb=32768, a=64, b=64: L.kv_blocks_move(sp, si, dp, di, n, bb, a, b, None)
    assert f(None, None, None, None, 0) == pkv.PKV_OK
    assert f(16, 16, 32, 16, -1) == pkv.PKV_ERR_SHAPE
    assert f(16, 16, 32, 16, 4, bb=0) == pkv.PKV_ERR_SHAPE
    assert f(16, 16, 32, 16, 4, a=-1) == pkv.PKV_ERR_SHAPE
    assert f(16, 16, 32, 16, 4, bb=40) == pkv.PKV_ERR_ALIGN
    assert f(None, 16, 32, 16, 4) == pkv.PKV_ERR_NULL
    assert f(16, 16, 32, None, 4) == pkv.PKV_ERR_NULL
    assert f(16, 16, 24, 16, 4) == pkv.PKV_ERR_ALIGN
    assert f(16, 18, 32, 16, 4) == pkv.PKV_ERR_ALIGN


def test_fp8kv_argument_errors_before_launch():
    L = pkv.lib()
    sh = pkv.make_shape(4, 8, 2, 19, 128, partition_size=16)
    need = pkv.pkv_attn_workspace_bytes(sh)
    f = lambda q=16, k=16, v=16, t=16, l=16, ks=0.01, vs=0.02, o=16, shape=sh, ws=16, nb=need: \
        L.paged_decode_attn_fp8kv(q, k, v, t, l, 1.0, ks, vs, o, ctypes.byref(shape), ws, nb, None)
    for ks, vs in ((0.0, 1.0), (1.0, -2.0), (float("nan"), 1.0), (1.0, float("inf"))):
        assert f(ks=ks, vs=vs) == pkv.PKV_ERR_SHAPE
    assert f(shape=pkv.make_shape(4, 8, 2, 19, 128, head_dim=96)) == pkv.PKV_ERR_SHAPE
    assert f(shape=pkv.make_shape(4, 32, 2, 19, 128, head_dim=256)) == pkv.PKV_ERR_SHAPE   # G = 16 at D = 256
    assert f(k=None) == pkv.PKV_ERR_NULL and f(t=None) == pkv.PKV_ERR_NULL
    assert f(v=24) == pkv.PKV_ERR_ALIGN and f(l=18) == pkv.PKV_ERR_ALIGN
    assert f(nb=need - 1) == pkv.PKV_ERR_WORKSPACE and f(ws=None) == pkv.PKV_ERR_WORKSPACE
    sh0 = pkv.make_shape(0, 8, 2, 19, 128)
    assert f(q=None, k=None, v=None, t=None, l=None, o=None, shape=sh0, ws=None, nb=0) == pkv.PKV_OK
    g = lambda kn=16, vn=16, k=16, v=16, t=16, l=16, ks=0.01, vs=0.02, shape=sh: \
        L.kv_append_fp8(kn, vn, k, v, t, l, ks, vs, ctypes.byref(shape), None)
    assert g(ks=0.0) == pkv.PKV_ERR_SHAPE and g(vs=float("nan")) == pkv.PKV_ERR_SHAPE
    assert g(shape=pkv.make_shape(4, 8, 2, 19, 128, head_dim=96)) == pkv.PKV_ERR_SHAPE
    assert g(kn=None) == pkv.PKV_ERR_NULL and g(v=None) == pkv.PKV_ERR_NULL
    assert g(vn=24) == pkv.PKV_ERR_ALIGN and g(t=18) == pkv.PKV_ERR_ALIGN
    assert g(kn=None, vn=None, k=None, v=None, t=None, l=None, shape=sh0) == pkv.PKV_OK


def test_stream_probe_argument_errors():
    L = pkv.lib()
    f = lambda k=16, v=16, slabs=1024, blocks=100, sink=None: L.pkv_probe_stream_read(k, v, slabs, blocks, sink, None)
    assert f(slabs=0) == pkv.PKV_ERR_SHAPE and f(blocks=-1) == pkv.PKV_ERR_SHAPE
    assert f(blocks=2 ** 31) == pkv.PKV_ERR_SHAPE
    assert f(k=None) == pkv.PKV_ERR_NULL and f(v=None) == pkv.PKV_ERR_NULL
    assert f(k=24) == pkv.PKV_ERR_ALIGN and f(v=8) == pkv.PKV_ERR_ALIGN and f(sink=6) == pkv.PKV_ERR_ALIGN
    assert f(k=None, v=None, blocks=0) == pkv.PKV_OK


def test_static_call_and_fault_counter_argument_errors():
    L = pkv.lib()
    sh = pkv.make_shape(4, 8, 2, 19, 128)
    f = lambda q=16, k=16, v=16, t=16, l=16, o=16, shape=sh: \
        L.paged_decode_attn_static(q, k, v, t, l, 1.0, o, ctypes.byref(shape), None)
    assert f(shape=pkv.make_shape(4, 9, 2, 19, 128)) == pkv.PKV_ERR_SHAPE
    # 2048 requests x 8 KV heads of 16-head records exceed the library's fixed workspace
    big = pkv.make_shape(2048, 128, 8, 4, 64)
    assert pkv.pkv_attn_workspace_bytes(big) > pkv.STATIC_WORKSPACE_BYTES
    assert f(shape=big) == pkv.PKV_ERR_WORKSPACE
    assert f(q=None) == pkv.PKV_ERR_NULL and f(o=24) == pkv.PKV_ERR_ALIGN
    sh0 = pkv.make_shape(0, 8, 2, 19, 128)
    assert f(q=None, k=None, v=None, t=None, l=None, o=None, shape=sh0) == pkv.PKV_OK
    assert L.pkv_set_id_fault_counter(2) == pkv.PKV_ERR_ALIGN
    assert L.pkv_set_id_fault_counter(None) == pkv.PKV_OK
