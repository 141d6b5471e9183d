/* Runs every function of the fp64 checker (oracle/pkv_oracle.c) on inputs read from a file,
 * with every array in a heap allocation of exactly its size, so that AddressSanitizer and
 * UndefinedBehaviorSanitizer see any read or write outside an array, any misaligned access and
 * any integer overflow.  Built and run by tests/test_oracle_sanitizers.py (host only, no GPU).
 *
 * Input file: 16 int64 header words
 *   S Hq Hkv D B MAXB NB n_ids scale_bits n_move NB2 0...
 * then q [S*Hq*D] u16, k_pool, v_pool [NB*Hkv*B*D] u16, tables [S*MAXB] i32, lens [S] i32,
 * ids [n_ids] i32 (gather source), ids2 [n_ids] i32 (scatter destination),
 * k_new, v_new [S*Hkv*D] u16, move_src [n_move] i32, move_dst [n_move] i32, pool2 [NB2*Hkv*B*D] u16.
 * Output file: ref [S*Hq*D] f64, staging, scattered pool, moved pool2, appended k and v pools. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int pkv_oracle_paged_decode_attn(const uint16_t*, const uint16_t*, const uint16_t*, const int32_t*,
                                 const int32_t*, float, double*, int64_t, int64_t, int64_t, int64_t,
                                 int64_t, int64_t, int64_t, int);
int pkv_oracle_kv_blocks_gather(const uint8_t*, const int32_t*, uint8_t*, int64_t, int64_t, int64_t);
int pkv_oracle_kv_blocks_scatter(const uint8_t*, uint8_t*, const int32_t*, int64_t, int64_t, int64_t);
int pkv_oracle_kv_blocks_move(const uint8_t*, const int32_t*, uint8_t*, const int32_t*, int64_t,
                              int64_t, int64_t, int64_t);
int pkv_oracle_kv_append(const uint16_t*, const uint16_t*, uint16_t*, uint16_t*, const int32_t*,
                         const int32_t*, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t);

static void* rd(FILE* f, size_t bytes) {
  void* p = malloc(bytes ? bytes : 1);   /* exactly the array, nothing after it */
  if (!p || (bytes && fread(p, 1, bytes, f) != bytes)) { fprintf(stderr, "short input\n"); exit(3); }
  return p;
}
static void wr(FILE* f, const void* p, size_t bytes) {
  if (bytes && fwrite(p, 1, bytes, f) != bytes) { fprintf(stderr, "short output\n"); exit(3); }
}

int main(int argc, char** argv) {
  if (argc != 3) return 2;
  FILE* in = fopen(argv[1], "rb");
  FILE* out = fopen(argv[2], "wb");
  if (!in || !out) return 2;
  int64_t h[16];
  if (fread(h, sizeof h[0], 16, in) != 16) return 3;
  const int64_t S = h[0], Hq = h[1], Hkv = h[2], D = h[3], B = h[4], MAXB = h[5], NB = h[6],
                n_ids = h[7], n_move = h[9], NB2 = h[10];
  float scale;
  const uint32_t sb = (uint32_t)h[8];
  memcpy(&scale, &sb, 4);
  const size_t pool_elems = (size_t)(NB * Hkv * B * D), pool2_elems = (size_t)(NB2 * Hkv * B * D);
  const size_t block_bytes = (size_t)(Hkv * B * D) * 2;
  uint16_t* q = rd(in, (size_t)(S * Hq * D) * 2);
  uint16_t* k = rd(in, pool_elems * 2);
  uint16_t* v = rd(in, pool_elems * 2);
  int32_t* tables = rd(in, (size_t)(S * MAXB) * 4);
  int32_t* lens = rd(in, (size_t)S * 4);
  int32_t* ids = rd(in, (size_t)n_ids * 4);
  int32_t* ids2 = rd(in, (size_t)n_ids * 4);
  uint16_t* k_new = rd(in, (size_t)(S * Hkv * D) * 2);
  uint16_t* v_new = rd(in, (size_t)(S * Hkv * D) * 2);
  int32_t* msrc = rd(in, (size_t)n_move * 4);
  int32_t* mdst = rd(in, (size_t)n_move * 4);
  uint16_t* pool2 = rd(in, pool2_elems * 2);
  fclose(in);

  double* ref = malloc((size_t)(S * Hq * D) * sizeof(double) + 1);
  int rc = pkv_oracle_paged_decode_attn(q, k, v, tables, lens, scale, ref, S, Hq, Hkv, D, B, MAXB, NB, 0);
  if (rc) { fprintf(stderr, "attn rc=%d\n", rc); return 4; }
  wr(out, ref, (size_t)(S * Hq * D) * sizeof(double));

  uint8_t* staging = malloc((size_t)n_ids * block_bytes + 1);
  rc = pkv_oracle_kv_blocks_gather((const uint8_t*)k, ids, staging, n_ids, (int64_t)block_bytes, NB);
  if (rc) { fprintf(stderr, "gather rc=%d\n", rc); return 4; }
  wr(out, staging, (size_t)n_ids * block_bytes);

  uint8_t* pool_copy = malloc(pool_elems * 2 + 1);
  memcpy(pool_copy, k, pool_elems * 2);
  rc = pkv_oracle_kv_blocks_scatter(staging, pool_copy, ids2, n_ids, (int64_t)block_bytes, NB);
  if (rc) { fprintf(stderr, "scatter rc=%d\n", rc); return 4; }
  wr(out, pool_copy, pool_elems * 2);

  rc = pkv_oracle_kv_blocks_move((const uint8_t*)k, msrc, (uint8_t*)pool2, mdst, n_move,
                                 (int64_t)block_bytes, NB, NB2);
  if (rc) { fprintf(stderr, "move rc=%d\n", rc); return 4; }
  wr(out, pool2, pool2_elems * 2);

  rc = pkv_oracle_kv_append(k_new, v_new, k, v, tables, lens, S, Hkv, D, B, MAXB, NB);
  if (rc) { fprintf(stderr, "append rc=%d\n", rc); return 4; }
  wr(out, k, pool_elems * 2);
  wr(out, v, pool_elems * 2);
  fclose(out);

  /* error paths must refuse without touching memory: ids outside the pool, negative sizes */
  int32_t bad[2] = {0, (int32_t)NB};
  if (n_ids >= 2 && pkv_oracle_kv_blocks_gather((const uint8_t*)k, bad, staging, 2, (int64_t)block_bytes, NB) == 0) return 5;
  bad[1] = -1;
  if (n_ids >= 2 && pkv_oracle_kv_blocks_scatter(staging, pool_copy, bad, 2, (int64_t)block_bytes, NB) == 0) return 5;
  if (pkv_oracle_paged_decode_attn(q, k, v, tables, lens, scale, ref, S, Hq, 0, D, B, MAXB, NB, 0) == 0) return 5;

  free(q); free(k); free(v); free(tables); free(lens); free(ids); free(ids2); free(k_new);
  free(v_new); free(msrc); free(mdst); free(pool2); free(ref); free(staging); free(pool_copy);
  puts("sanitized run ok");
  return 0;
}
