/* Walks the argument-validation layer of libpkv (include/pkv.h) with every class of bad argument,
 * against a build of the library whose host code is instrumented with AddressSanitizer and
 * UndefinedBehaviorSanitizer.  Nothing here reaches a launch, so no GPU is needed; a read through
 * a bad pointer, an overflowing size computation or a misaligned access in the validation code
 * ends the run with a report.  Built and run by tests/test_abi_sanitizers.py. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "pkv.h"

static int failures = 0;
#define EXPECT(call, want)                                                              \
  do {                                                                                  \
    int got_ = (call);                                                                  \
    if (got_ != (want)) { printf("line %d: got %d, want %d\n", __LINE__, got_, (want)); failures++; } \
  } while (0)

int main(void) {
  void* p16 = (void*)(uintptr_t)4096;      /* aligned, never dereferenced by the host */
  void* p8 = (void*)(uintptr_t)4104;       /* 8-byte aligned only */
  int32_t* i4 = (int32_t*)(uintptr_t)8192;
  int32_t* i2 = (int32_t*)(uintptr_t)8194;
  pkv_attn_shape ok = {4, 8, 2, 128, 16, 19, 16, 0, 128};
  size_t need = 0, bytes = 0;
  EXPECT(pkv_attn_workspace_bytes(&ok, &need), PKV_OK);
  EXPECT(pkv_attn_workspace_bytes(&ok, NULL), PKV_ERR_NULL);
  EXPECT(pkv_attn_workspace_bytes(NULL, &bytes), PKV_ERR_NULL);
  EXPECT(pkv_attn_partition_size(&ok), 16);
  EXPECT(pkv_attn_partition_size(NULL), PKV_ERR_NULL);

  /* extreme sizes: every product in the checks must be formed without overflow */
  {
    pkv_attn_shape s = ok;
    s.num_seqs = 2048; s.num_q_heads = 128; s.num_kv_heads = 8; s.max_blocks_per_seq = INT32_MAX / 64;
    s.block_size = 64; s.num_pool_blocks = INT64_MAX;
    EXPECT(pkv_attn_workspace_bytes(&s, &bytes), PKV_ERR_SHAPE);
    s.num_pool_blocks = ((int64_t)1 << 31) / (8 * 4) - 1;
    s.max_context_len = 0; s.partition_size = 65536;
    EXPECT(pkv_attn_workspace_bytes(&s, &bytes) == PKV_OK || pkv_attn_workspace_bytes(&s, &bytes) == PKV_ERR_SHAPE, 1);
    s.max_blocks_per_seq = INT32_MAX;
    EXPECT(pkv_attn_workspace_bytes(&s, &bytes), PKV_ERR_SHAPE);
    s = ok; s.num_pool_blocks = INT64_MAX;                 /* the slab count must not be formed by a product */
    EXPECT(pkv_attn_workspace_bytes(&s, &bytes), PKV_ERR_SHAPE);
    s = ok; s.num_pool_blocks = INT64_MAX / 2; s.num_kv_heads = 8; s.num_q_heads = 8; s.block_size = 64; s.partition_size = 64;
    EXPECT(pkv_attn_workspace_bytes(&s, &bytes), PKV_ERR_SHAPE);
    s = ok; s.num_q_heads = INT32_MAX; s.num_kv_heads = INT32_MAX; s.num_seqs = 2048; s.max_blocks_per_seq = INT32_MAX / 16;
    EXPECT(pkv_attn_workspace_bytes(&s, &bytes), PKV_ERR_SHAPE);
    s = ok; s.head_dim = 256; s.num_q_heads = 32;
    EXPECT(pkv_attn_workspace_bytes(&s, &bytes), PKV_ERR_SHAPE);
    s = ok; s.partition_size = -16;
    EXPECT(pkv_attn_workspace_bytes(&s, &bytes), PKV_ERR_SHAPE);
    s = ok; s.max_context_len = INT32_MAX;
    EXPECT(pkv_attn_workspace_bytes(&s, &bytes), PKV_ERR_SHAPE);
  }

  /* attention, all four entry points */
  EXPECT(paged_decode_attn(p16, p16, p16, i4, i4, 1.f, p16, NULL, p16, need, NULL), PKV_ERR_NULL);
  EXPECT(paged_decode_attn(NULL, p16, p16, i4, i4, 1.f, p16, &ok, p16, need, NULL), PKV_ERR_NULL);
  EXPECT(paged_decode_attn(p16, p16, p8, i4, i4, 1.f, p16, &ok, p16, need, NULL), PKV_ERR_ALIGN);
  EXPECT(paged_decode_attn(p16, p16, p16, i2, i4, 1.f, p16, &ok, p16, need, NULL), PKV_ERR_ALIGN);
  EXPECT(paged_decode_attn(p16, p16, p16, i4, i4, 1.f, p16, &ok, p16, need - 1, NULL), PKV_ERR_WORKSPACE);
  EXPECT(paged_decode_attn(p16, p16, p16, i4, i4, 1.f, p16, &ok, p8, need, NULL), PKV_ERR_ALIGN);
  EXPECT(paged_decode_attn_fp8kv(p16, p16, p16, i4, i4, 1.f, 0.f, 1.f, p16, &ok, p16, need, NULL), PKV_ERR_SHAPE);
  EXPECT(paged_decode_attn_fp8kv(p16, p16, p16, i4, i4, 1.f, 1.f, (float)NAN, p16, &ok, p16, need, NULL), PKV_ERR_SHAPE);
  EXPECT(paged_decode_attn_fp8kv(p16, NULL, p16, i4, i4, 1.f, 1.f, 1.f, p16, &ok, p16, need, NULL), PKV_ERR_NULL);
  EXPECT(paged_decode_attn_fp8kv(p16, p16, p16, i4, i4, 1.f, 1.f, 1.f, p16, NULL, p16, need, NULL), PKV_ERR_NULL);
  EXPECT(paged_decode_attn_static(p16, p16, p16, i4, i4, 1.f, p8, &ok, NULL), PKV_ERR_ALIGN);
  EXPECT(paged_decode_attn_static(p16, p16, p16, i4, i4, 1.f, p16, NULL, NULL), PKV_ERR_NULL);
  {
    const void* good[3] = {p16, p16, p16};
    const void* bad[3] = {p16, p16, p8};
    const void* holes[3] = {p16, NULL, p16};
    void* outs[3] = {p16, p16, p16};
    EXPECT(paged_decode_attn_layers(good, good, bad, i4, i4, 1.f, outs, 3, &ok, p16, need, NULL), PKV_ERR_ALIGN);
    EXPECT(paged_decode_attn_layers(good, holes, good, i4, i4, 1.f, outs, 3, &ok, p16, need, NULL), PKV_ERR_NULL);
    EXPECT(paged_decode_attn_layers(NULL, good, good, i4, i4, 1.f, outs, 3, &ok, p16, need, NULL), PKV_ERR_NULL);
    EXPECT(paged_decode_attn_layers(good, good, good, i4, i4, 1.f, outs, -1, &ok, p16, need, NULL), PKV_ERR_SHAPE);
    EXPECT(paged_decode_attn_layers(good, good, good, i4, i4, 1.f, outs, 0, &ok, p16, need, NULL), PKV_OK);
  }

  /* copies */
  EXPECT(kv_blocks_gather(p16, i4, p16, -1, 32768, 64, NULL), PKV_ERR_SHAPE);
  EXPECT(kv_blocks_gather(p16, i4, p16, 4, 40, 64, NULL), PKV_ERR_ALIGN);
  EXPECT(kv_blocks_gather(p16, i4, p16, (int64_t)1 << 40, 32768, 64, NULL), PKV_ERR_SHAPE);
  EXPECT(kv_blocks_gather(p16, i4, p16, 4, (int64_t)1 << 40, 64, NULL), PKV_ERR_SHAPE);
  EXPECT(kv_blocks_gather(p16, i4, p16, 4, INT64_MAX - 15, 64, NULL), PKV_ERR_SHAPE);
  EXPECT(kv_blocks_scatter(p16, p16, i2, 4, 32768, 64, NULL), PKV_ERR_ALIGN);
  EXPECT(kv_blocks_scatter(NULL, p16, i4, 4, 32768, 64, NULL), PKV_ERR_NULL);
  EXPECT(kv_blocks_move(p16, i4, p16, i4, 4, 32768, -1, 64, NULL), PKV_ERR_SHAPE);
  EXPECT(kv_blocks_move(p16, i4, p8, i4, 4, 32768, 64, 64, NULL), PKV_ERR_ALIGN);
  EXPECT(kv_blocks_move(p16, NULL, p16, i4, 4, 32768, 64, 64, NULL), PKV_ERR_NULL);
  EXPECT(kv_blocks_move(NULL, NULL, NULL, NULL, 0, 32768, 64, 64, NULL), PKV_OK);
  {
    /* a pageable buffer: refused whether or not a device exists */
    char* buf = (char*)malloc(4 * 32768);
    EXPECT(kv_blocks_offload(p16, i4, p16, buf, 4, 32768, 64, NULL), PKV_ERR_HOST);
    EXPECT(kv_blocks_reload(buf, p16, p16, i4, 4, 32768, 64, NULL), PKV_ERR_HOST);
    EXPECT(kv_blocks_offload(p16, i4, p16, NULL, 4, 32768, 64, NULL), PKV_ERR_NULL);
    free(buf);
  }

  /* append, both element sizes */
  EXPECT(kv_append(p16, p16, p16, p16, i4, i4, NULL, NULL), PKV_ERR_NULL);
  EXPECT(kv_append(p16, p8, p16, p16, i4, i4, &ok, NULL), PKV_ERR_ALIGN);
  EXPECT(kv_append_fp8(p16, p16, p16, p16, i4, i4, -1.f, 1.f, &ok, NULL), PKV_ERR_SHAPE);
  EXPECT(kv_append_fp8(p16, p16, p16, NULL, i4, i4, 1.f, 1.f, &ok, NULL), PKV_ERR_NULL);

  /* the measurement aid */
  EXPECT(pkv_probe_stream_read(p16, p16, 0, 10, NULL, NULL), PKV_ERR_SHAPE);
  EXPECT(pkv_probe_stream_read(p16, p16, INT64_MAX, (int64_t)INT32_MAX + 1, NULL, NULL), PKV_ERR_SHAPE);
  EXPECT(pkv_probe_stream_read(p16, NULL, 64, 10, NULL, NULL), PKV_ERR_NULL);
  EXPECT(pkv_probe_stream_read(p8, p16, 64, 10, NULL, NULL), PKV_ERR_ALIGN);
  EXPECT(pkv_probe_stream_read(p16, p16, 64, 10, i2, NULL), PKV_ERR_ALIGN);
  EXPECT(pkv_probe_stream_read(NULL, NULL, INT64_MAX, 0, NULL, NULL), PKV_OK);

  EXPECT(pkv_set_id_fault_counter(i2), PKV_ERR_ALIGN);
  EXPECT(pkv_set_id_fault_counter(NULL), PKV_OK);
  for (int s = 1; s >= -8; --s)
    if (!pkv_status_string(s)[0]) failures++;
  if (!pkv_last_launch_error()) failures++;
  if (pkv_version() < 1000) failures++;
  printf("abi walk: %d failures\n", failures);
  return failures != 0;
}
