// Internal launch interface between the C-ABI layer and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace pkv {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // one 16-byte lane load

constexpr int kHeadDim = 128;       // D
constexpr int kBlockTokens = 16;    // B
constexpr int kMaxPartition = 1024; // tokens: 64 blocks, one block id per lane of a wavefront
constexpr int kMaxGroup = 16;       // query heads per KV head

struct AttnLaunch {
  const uint16_t* q;
  const uint16_t* k_pool;
  const uint16_t* v_pool;
  const int32_t* block_tables;
  const int32_t* context_lens;
  uint16_t* out;
  float* ws_acc;   // [S][NP][Hq][D] un-normalised partial outputs
  float2* ws_ml;   // [S][NP][Hq]    (running max in log2 units, partial sum)
  float scale_log2e;
  int S, Hq, Hkv, G, MAXB;
  int P;           // partition size, tokens
  int NP;          // partitions launched per request = ceil(max_context_len / P)
  int max_ctx;     // context lengths are clamped to [0, max_ctx] (<= MAXB * 16)
  int NB;          // physical blocks per pool; ids outside [0, NB) are never followed
};

// Partition kernel: one wavefront per (request, KV head, partition).
hipError_t launch_attn_partition(const AttnLaunch& a, hipStream_t stream);
// Split-K merge: one wavefront per (request, query head); only when NP > 1.
hipError_t launch_attn_reduce(const AttnLaunch& a, hipStream_t stream);

// Whole-block copies; `gather` selects the direction.
hipError_t launch_kv_block_copy(const void* src, void* dst, const int32_t* block_ids,
                                int64_t n_blocks, int64_t block_bytes, int64_t num_pool_blocks,
                                bool gather, hipStream_t stream);

}  // namespace pkv
