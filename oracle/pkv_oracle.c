/*
 * CPU checker for the paged-decode hot path.  TEST INFRASTRUCTURE ONLY: it is
 * called by the tests, by the smoke check and by the benchmark's cpu_baseline
 * leg, never by the product path, and it shares no code with the HIP library.
 *
 * What it computes is the plain definition, in fp64, with no blocking, no
 * running maximum and no partitioning:
 *
 *   The decode stage reuses each request's whole KV cache for every generated
 *   token (paper Section II-A), and the serving engine keeps that cache per
 *   request in fixed-size pages (Section II-B; the paged serving engine named
 *   in Section VI).  For request s, query head h, with kvh = h div G
 *   (G = Hq / Hkv consecutive query heads share one KV head):
 *
 *     x_t  = scale * sum_d q[s,h,d] * K[tbl[s][t div B], kvh, t mod B, d]
 *     m    = max_t x_t ;  w_t = exp(x_t - m) ;  Z = sum_t w_t
 *     ref[s,h,e] = sum_t (w_t / Z) * V[tbl[s][t div B], kvh, t mod B, e]
 *
 *   over t = 0 .. L_s - 1 (L_s counts the token being decoded: its K,V row is
 *   already in the pool).  L_s = 0 gives a zero row.  Table entries at or
 *   beyond ceil(L_s/B) and slots at or beyond L_s in the last block are never
 *   read.  Inputs are bf16 bit patterns widened exactly; scale is the fp32
 *   value the library is given, widened.
 *
 *   Eviction to and reload from the backing store (Section II-B) and
 *   migration of a request's whole KV cache at the phase boundary
 *   (Section IV-B, "KV cache transfer overhead") move whole pages:
 *     gather : staging[i] = pool[ids[i]]     scatter : pool[ids[i]] = staging[i]
 *     move   : dst[dst_ids[i]] = src[src_ids[i]]   (two pools on one device)
 *   bytewise, everything else untouched.
 *
 *   Before attention the decode step stores the new token's K and V rows at
 *   position L_s - 1 of each request's cache (Section II-A: the cache is updated
 *   with each newly generated token); pinned by numpy indexing.
 *
 * Pool layout: [NB, Hkv, B, D] row-major for K and for V.
 *
 *   8-bit pools (a reading: the paper fixes no quantised cache format).  K and V
 *   bytes are OCP FP8 E4M3: sign, 4 exponent bits (bias 7), 3 mantissa bits;
 *   exponent field 0 is subnormal (m * 2^-9), there are no infinities, 0x7F and
 *   0xFF are NaN.  One fp32 scale per pool: K = k_scale * e4m3(byte),
 *   V = v_scale * e4m3(byte); the attention above is then taken over those
 *   values.  Pinned against a library decode of all 256 bytes, a dense brute
 *   force over de-quantised rows, and the bf16 function on a pool holding the
 *   same values.
 *
 * Parity pins (tests, CPU only): dense brute force written in numpy on tiny
 * inputs, a library fp64 attention on de-paged tensors, closed forms (L = 1,
 * scale = 0, V == 1, a two-token ln 2 case), shift, paging and GQA
 * invariances; the copies are pinned by numpy fancy indexing.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double widen_bf16(uint16_t bits) {
  uint32_t u = ((uint32_t)bits) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

/* One OCP FP8 E4M3 byte, exactly. */
double pkv_oracle_e4m3(uint8_t b) {
  const int e = (b >> 3) & 15, m = b & 7;
  double v;
  if (e == 15 && m == 7) return NAN;
  if (e == 0) v = ldexp((double)m, -9);
  else v = ldexp(1.0 + m / 8.0, e - 7);
  return (b & 0x80) ? -v : v;
}

/* fp32 -> E4M3 byte: round to nearest, ties to even, magnitudes above 448 saturate to 448
 * (there is no infinity to overflow to); NaN gives the NaN byte with the input's sign.
 * Written from the format: below 2^-6 the grid is m * 2^-9, m = 0..7; from there on
 * (1 + m/8) * 2^(e-7), e = 1..15, with (e, m) = (15, 7) left out. */
uint8_t pkv_oracle_to_e4m3(float y) {
  const uint8_t sign = signbit(y) ? 0x80 : 0x00;
  if (isnan(y)) return (uint8_t)(sign | 0x7F);
  double a = fabs((double)y);
  if (a > 448.0) a = 448.0;
  if (a < ldexp(1.0, -6)) {
    const int m = (int)nearbyint(ldexp(a, 9));        /* 0..8, ties to even */
    return (uint8_t)(sign | m);                       /* m == 8 is the byte of 2^-6 */
  }
  int ex;
  const double f = frexp(a, &ex);                     /* a = f * 2^ex, f in [0.5, 1) */
  int e = ex - 1;                                     /* a = (2f) * 2^e, 2f in [1, 2) */
  int m = (int)nearbyint((2.0 * f - 1.0) * 8.0);      /* 0..8, ties to even */
  if (m == 8) { m = 0; e += 1; }
  return (uint8_t)(sign | ((e + 7) << 3) | m);
}

/* Element idx of a K or V pool: a bf16 bit pattern, or an E4M3 byte times the pool's scale. */
static double kv_value(const void* pool, int64_t idx, int fp8, double pool_scale) {
  if (fp8) return pool_scale * pkv_oracle_e4m3(((const uint8_t*)pool)[idx]);
  return widen_bf16(((const uint16_t*)pool)[idx]);
}

int pkv_oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* Returns 0, or -1 on a bad argument, -2 if a dereferenced table entry is
 * outside [0, NB), -3 on allocation failure.  threads <= 0 means "all". */
static int attn_definition(const uint16_t* q, const void* k_pool, const void* v_pool, int fp8,
                           double k_scale, double v_scale, const int32_t* block_tables,
                           const int32_t* context_lens, float scale, double* ref,
                           int64_t S, int64_t Hq, int64_t Hkv, int64_t D, int64_t B,
                           int64_t MAXB, int64_t NB, int threads) {
  if (S < 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || B <= 0 || MAXB <= 0 || Hq % Hkv) return -1;
  const int64_t G = Hq / Hkv;
  for (int64_t s = 0; s < S; ++s) {
    int64_t L = context_lens[s];
    if (L < 0 || (L + B - 1) / B > MAXB) return -1;
    for (int64_t j = 0; j < (L + B - 1) / B; ++j) {
      int64_t pb = block_tables[s * MAXB + j];
      if (pb < 0 || pb >= NB) return -2;
    }
  }
  int fail = 0;
#ifdef _OPENMP
  if (threads <= 0) threads = omp_get_max_threads();
#pragma omp parallel for collapse(2) schedule(dynamic, 1) num_threads(threads)
#endif
  for (int64_t s = 0; s < S; ++s) {
    for (int64_t h = 0; h < Hq; ++h) {
      const int64_t L = context_lens[s];
      double* o = ref + (s * Hq + h) * D;
      for (int64_t e = 0; e < D; ++e) o[e] = 0.0;
      if (L == 0) continue;
      const int64_t kvh = h / G;
      const uint16_t* qrow = q + (s * Hq + h) * D;
      double* x = (double*)malloc(sizeof(double) * (size_t)L);
      if (!x) { fail = 1; continue; }
      /* scores */
      for (int64_t t = 0; t < L; ++t) {
        const int64_t pb = block_tables[s * MAXB + t / B];
        const int64_t krow = ((pb * Hkv + kvh) * B + t % B) * D;
        double dot = 0.0;
        for (int64_t d = 0; d < D; ++d) dot += widen_bf16(qrow[d]) * kv_value(k_pool, krow + d, fp8, k_scale);
        x[t] = (double)scale * dot;
      }
      /* softmax weights */
      double m = x[0];
      for (int64_t t = 1; t < L; ++t) if (x[t] > m) m = x[t];
      double Z = 0.0;
      for (int64_t t = 0; t < L; ++t) { x[t] = exp(x[t] - m); Z += x[t]; }
      /* weighted sum of V rows */
      for (int64_t t = 0; t < L; ++t) {
        const int64_t pb = block_tables[s * MAXB + t / B];
        const int64_t vrow = ((pb * Hkv + kvh) * B + t % B) * D;
        const double w = x[t] / Z;
        for (int64_t e = 0; e < D; ++e) o[e] += w * kv_value(v_pool, vrow + e, fp8, v_scale);
      }
      free(x);
    }
  }
  return fail ? -3 : 0;
}

int pkv_oracle_paged_decode_attn(const uint16_t* q, const uint16_t* k_pool,
                                 const uint16_t* v_pool, const int32_t* block_tables,
                                 const int32_t* context_lens, float scale, double* ref,
                                 int64_t S, int64_t Hq, int64_t Hkv, int64_t D, int64_t B,
                                 int64_t MAXB, int64_t NB, int threads) {
  return attn_definition(q, k_pool, v_pool, 0, 1.0, 1.0, block_tables, context_lens, scale, ref,
                         S, Hq, Hkv, D, B, MAXB, NB, threads);
}

/* The same definition over E4M3 pools; k_scale and v_scale are the fp32 values the library is
 * given, widened. */
int pkv_oracle_paged_decode_attn_fp8kv(const uint16_t* q, const uint8_t* k_pool,
                                       const uint8_t* v_pool, const int32_t* block_tables,
                                       const int32_t* context_lens, float scale, float k_scale,
                                       float v_scale, double* ref, int64_t S, int64_t Hq,
                                       int64_t Hkv, int64_t D, int64_t B, int64_t MAXB, int64_t NB,
                                       int threads) {
  return attn_definition(q, k_pool, v_pool, 1, (double)k_scale, (double)v_scale, block_tables,
                         context_lens, scale, ref, S, Hq, Hkv, D, B, MAXB, NB, threads);
}

/* The append step for E4M3 pools: the new rows are divided by their pool's scale in fp32 (the
 * precision the device takes that decision in) and rounded to E4M3 as above. */
int pkv_oracle_kv_append_fp8(const uint16_t* k_new, const uint16_t* v_new, uint8_t* k_pool,
                             uint8_t* v_pool, const int32_t* block_tables,
                             const int32_t* context_lens, float k_scale, float v_scale, int64_t S,
                             int64_t Hkv, int64_t D, int64_t B, int64_t MAXB, int64_t NB) {
  for (int64_t s = 0; s < S; ++s) {
    const int64_t L = context_lens[s];
    if (L <= 0) continue;
    const int64_t t = L - 1;
    if (t / B >= MAXB) return -1;
    const int64_t pb = block_tables[s * MAXB + t / B];
    if (pb < 0 || pb >= NB) return -2;
    for (int64_t h = 0; h < Hkv; ++h) {
      const int64_t dst = ((pb * Hkv + h) * B + t % B) * D;
      for (int64_t d = 0; d < D; ++d) {
        const float kx = (float)widen_bf16(k_new[(s * Hkv + h) * D + d]);
        const float vx = (float)widen_bf16(v_new[(s * Hkv + h) * D + d]);
        k_pool[dst + d] = pkv_oracle_to_e4m3(kx / k_scale);
        v_pool[dst + d] = pkv_oracle_to_e4m3(vx / v_scale);
      }
    }
  }
  return 0;
}

/* staging[i] = pool[ids[i]], whole pages of block_bytes bytes. */
int pkv_oracle_kv_blocks_gather(const uint8_t* pool, const int32_t* ids, uint8_t* staging,
                                int64_t n, int64_t block_bytes, int64_t NB) {
  if (n < 0 || block_bytes <= 0) return -1;
  for (int64_t i = 0; i < n; ++i) {
    if (ids[i] < 0 || ids[i] >= NB) return -2;
    memcpy(staging + i * block_bytes, pool + (int64_t)ids[i] * block_bytes, (size_t)block_bytes);
  }
  return 0;
}

/* pool[ids[i]] = staging[i]; a page listed twice is an error (-4). */
int pkv_oracle_kv_blocks_scatter(const uint8_t* staging, uint8_t* pool, const int32_t* ids,
                                 int64_t n, int64_t block_bytes, int64_t NB) {
  if (n < 0 || block_bytes <= 0) return -1;
  uint8_t* seen = (uint8_t*)calloc((size_t)(NB > 0 ? NB : 1), 1);
  if (!seen) return -3;
  for (int64_t i = 0; i < n; ++i) {
    if (ids[i] < 0 || ids[i] >= NB) { free(seen); return -2; }
    if (seen[ids[i]]) { free(seen); return -4; }
    seen[ids[i]] = 1;
  }
  free(seen);
  for (int64_t i = 0; i < n; ++i)
    memcpy(pool + (int64_t)ids[i] * block_bytes, staging + i * block_bytes, (size_t)block_bytes);
  return 0;
}

/* dst[dst_ids[i]] = src[src_ids[i]], whole pages; the two pools are distinct buffers here.
 * A destination listed twice is an error (-4). */
int pkv_oracle_kv_blocks_move(const uint8_t* src, const int32_t* src_ids, uint8_t* dst,
                              const int32_t* dst_ids, int64_t n, int64_t block_bytes,
                              int64_t src_NB, int64_t dst_NB) {
  if (n < 0 || block_bytes <= 0) return -1;
  uint8_t* seen = (uint8_t*)calloc((size_t)(dst_NB > 0 ? dst_NB : 1), 1);
  if (!seen) return -3;
  for (int64_t i = 0; i < n; ++i) {
    if (src_ids[i] < 0 || src_ids[i] >= src_NB || dst_ids[i] < 0 || dst_ids[i] >= dst_NB) { free(seen); return -2; }
    if (seen[dst_ids[i]]) { free(seen); return -4; }
    seen[dst_ids[i]] = 1;
  }
  free(seen);
  for (int64_t i = 0; i < n; ++i)
    memcpy(dst + (int64_t)dst_ids[i] * block_bytes, src + (int64_t)src_ids[i] * block_bytes, (size_t)block_bytes);
  return 0;
}

/* The new token's K and V rows of every request go to position L_s - 1 of its
 * paged cache (the cache is updated with each generated token, Section II-A;
 * L_s already counts that token).  Requests with L_s <= 0 are skipped. */
int pkv_oracle_kv_append(const uint16_t* k_new, const uint16_t* v_new, uint16_t* k_pool,
                         uint16_t* v_pool, const int32_t* block_tables,
                         const int32_t* context_lens, int64_t S, int64_t Hkv, int64_t D, int64_t B,
                         int64_t MAXB, int64_t NB) {
  for (int64_t s = 0; s < S; ++s) {
    const int64_t L = context_lens[s];
    if (L <= 0) continue;
    const int64_t t = L - 1;
    if (t / B >= MAXB) return -1;
    const int64_t pb = block_tables[s * MAXB + t / B];
    if (pb < 0 || pb >= NB) return -2;
    for (int64_t h = 0; h < Hkv; ++h) {
      const int64_t dst = ((pb * Hkv + h) * B + t % B) * D;
      for (int64_t d = 0; d < D; ++d) {
        k_pool[dst + d] = k_new[(s * Hkv + h) * D + d];
        v_pool[dst + d] = v_new[(s * Hkv + h) * D + d];
      }
    }
  }
  return 0;
}
