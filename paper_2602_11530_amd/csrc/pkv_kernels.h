// Internal launch interface between the C-ABI layer and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace pkv {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // one 16-byte lane load

constexpr int kBlockTokens = 16;     // tokens per streaming unit (one MFMA tile of keys); a physical
                                     // block of B = 16, 32 or 64 tokens holds B/16 units per KV head
constexpr int kMaxBlockSize = 64;
constexpr int kMaxPartition = 65536; // tokens covered by one partial result, upper bound
constexpr int kMaxGroup = 16;        // query heads per KV head
constexpr int kMaxSeqs = 2048;       // per-request prefix arrays live in LDS

// The attention pass is a persistent launch sized for the 256 compute units of
// an MI355X: two 4-wave workgroups per unit, each wavefront streaming an equal
// share of the batch's KV blocks.
#ifndef PKV_STREAM_GROUPS
#define PKV_STREAM_GROUPS 512
#endif
constexpr int kStreamWavesPerGroup = 4;
constexpr int kStreamGroups = PKV_STREAM_GROUPS;
constexpr int kStreamWaves = kStreamGroups * kStreamWavesPerGroup;

// How the batch's KV blocks are laid out as one stream and cut into shares.
//   Segment (s, kvh) holds the nblk_s = ceil(L_s/16) 16-token units ("blocks" below;
//   a physical block of B tokens is B/16 of them in a row) of request s for KV
//   head kvh; segments follow each other in (s, kvh) order; position pos of the
//   stream is block b of segment (s, kvh) with
//       pos = Hkv * cumB[s] + kvh * nblk_s + b,     cumB[s] = sum_{s'<s} nblk_s'.
//   Wavefront w owns positions [w*T/W, (w+1)*T/W), T = Hkv * cumB[S].
//   A run is a maximal stretch of one wavefront's share inside one segment and
//   one partition (P tokens of the request); every run yields one partial result
//   (max, sum, un-normalised row) per query head of the group.  The runs of one
//   segment inside one share are folded into one record before it leaves the
//   wavefront, stored at
//       slot = s * Hkv + kvh + w,
//   which is unique and increases along the stream (from one record to the next
//   the segment, the wavefront or both advance), so the records of a segment are
//   the consecutive slots from (its index + the owner of its first block) to
//   (its index + the owner of its last block); slots skipped where a share and a
//   segment end together belong to nobody and are never read.
__host__ __device__ inline int64_t share_start(int64_t w, int64_t T, int64_t W) { return w * T / W; }
// The wavefront whose share holds position pos.
__host__ __device__ inline int share_owner(int64_t pos, int64_t T, int64_t W) {
  return (int)(((pos + 1) * W - 1) / T);
}

// One partial record: G un-normalised rows of D floats, then (reference max in
// log2 units, partial sum) for up to kMaxGroup heads.  Rows are 16-byte multiples.
__host__ __device__ inline int record_floats(int G, int D) { return G * D + 2 * kMaxGroup; }

struct AttnLaunch {
  const uint16_t* q;
  const void* k_pool;   // bf16, or e4m3 bytes when kv_fp8
  const void* v_pool;
  const int32_t* block_tables;
  const int32_t* context_lens;
  uint16_t* out;
  float* ws_rec;   // [slots][record_floats(G)] partial records, see record_floats()
  int32_t* ws_cum; // [S + 1] cumB, written by the stream pass for the merge
  float scale_log2e;   // softmax scale x log2(e) (x the K pool's scale for an e4m3 pool)
  float out_scale;     // applied to the normalised row: 1, or the V pool's scale
  int kv_fp8;          // the pools hold one-byte e4m3 values
  int32_t* id_faults;  // optional device counter of refused block ids (nullptr: not reported)
  int S, Hq, Hkv, G, MAXB;
  int D;           // head dimension: 64, 128 or 256
  int waves;       // persistent wavefronts of the stream pass: kStreamWaves, or half of it for D = 256
  int upb;         // 16-token units per physical block (B / 16)
  int P;           // partition size, tokens
  int max_ctx;     // context lengths are clamped to [0, max_ctx] (<= MAXB * 16)
  int NB;          // physical blocks per pool; ids outside [0, NB) are never followed
  int rec_buffered; // finished records a wavefront keeps in LDS before writing them out (>= 1)
};

// Stream pass: kStreamWaves persistent wavefronts, each writing its runs' partial records.
hipError_t launch_attn_stream(const AttnLaunch& a, hipStream_t stream);
// Merge: one wavefront per (request, query head).
hipError_t launch_attn_reduce(const AttnLaunch& a, hipStream_t stream);

// Whole-block copies; `gather` selects the direction.
// `id_faults` (optional, device): incremented once per listed block that is skipped because an
// id lies outside its pool.
hipError_t launch_kv_block_copy(const void* src, void* dst, const int32_t* block_ids,
                                int64_t n_blocks, int64_t block_bytes, int64_t num_pool_blocks,
                                bool gather, int32_t* id_faults, hipStream_t stream);

// Pool to pool: dst[dst_ids[i]] = src[src_ids[i]], no staging image in between.
hipError_t launch_kv_block_move(const void* src, const int32_t* src_ids, int64_t src_pool_blocks,
                                void* dst, const int32_t* dst_ids, int64_t dst_pool_blocks,
                                int64_t n_blocks, int64_t block_bytes, int32_t* id_faults,
                                hipStream_t stream);

// New token's K and V rows into slot context_lens[s] - 1 of every request.
hipError_t launch_kv_append(const uint16_t* k_new, const uint16_t* v_new, uint16_t* k_pool,
                            uint16_t* v_pool, const int32_t* block_tables,
                            const int32_t* context_lens, int S, int Hkv, int D, int MAXB, int B,
                            int max_ctx, int NB, int32_t* id_faults, hipStream_t stream);

// The same for one-byte E4M3 pools: rows are divided by the pool's scale and rounded to E4M3.
hipError_t launch_kv_append_fp8(const uint16_t* k_new, const uint16_t* v_new, void* k_pool,
                                void* v_pool, const int32_t* block_tables,
                                const int32_t* context_lens, float k_scale, float v_scale, int S,
                                int Hkv, int D, int MAXB, int B, int max_ctx, int NB,
                                int32_t* id_faults, hipStream_t stream);

// Measurement aid: the stream pass's load pattern with no arithmetic (see stream_probe.hip).
hipError_t launch_stream_read_probe(const void* k_buf, const void* v_buf, uint32_t num_slabs,
                                    int64_t total_blocks, void* sink, hipStream_t stream);

}  // namespace pkv
