// KV append for gfx950: the decode step's new K and V rows go into their slot
// of the paged pools before attention runs (paper Section II-A: the KV cache is
// updated with each newly generated token).  One 16-byte chunk per lane; a row of
// one KV head is 16 lanes; a few hundred KiB per call, so latency is all there is.
#include "pkv_kernels.h"

namespace pkv {
namespace {

constexpr int kAppendThreads = 256;

__global__ __launch_bounds__(kAppendThreads) void kv_append_kernel(
    const u32x4* __restrict__ k_new, const u32x4* __restrict__ v_new, u32x4* __restrict__ k_pool,
    u32x4* __restrict__ v_pool, const int32_t* __restrict__ block_tables,
    const int32_t* __restrict__ context_lens, int S, int Hkv, int D, int MAXB, int B, int max_ctx,
    int NB, int32_t* __restrict__ id_faults) {
  const int kRowChunks = D * 2 / 16;   // 16-byte chunks per row
  const int64_t idx = (int64_t)blockIdx.x * kAppendThreads + threadIdx.x;   // (s, kvh, chunk)
  const int64_t total = (int64_t)S * Hkv * kRowChunks;
  if (idx >= total) return;
  const int chunk = (int)(idx % kRowChunks);
  const int kvh = (int)((idx / kRowChunks) % Hkv);
  const int s = (int)(idx / ((int64_t)kRowChunks * Hkv));
  const int L = min(max(context_lens[s], 0), max_ctx);
  if (L <= 0) return;
  const int t = L - 1;
  const int id = block_tables[(int64_t)s * MAXB + t / B];
  if ((unsigned)id >= (unsigned)NB) {   // never follow a corrupt id; report it once per request
    if (id_faults && kvh == 0 && chunk == 0) atomicAdd(id_faults, 1);
    return;
  }
  const int64_t dst = (((int64_t)id * Hkv + kvh) * B + t % B) * kRowChunks + chunk;
  k_pool[dst] = k_new[idx];
  v_pool[dst] = v_new[idx];
}

}  // namespace

hipError_t launch_kv_append(const uint16_t* k_new, const uint16_t* v_new, uint16_t* k_pool,
                            uint16_t* v_pool, const int32_t* block_tables,
                            const int32_t* context_lens, int S, int Hkv, int D, int MAXB, int B,
                            int max_ctx, int NB, int32_t* id_faults, hipStream_t stream) {
  const int64_t total = (int64_t)S * Hkv * (D * 2 / 16);
  dim3 grid((unsigned)((total + kAppendThreads - 1) / kAppendThreads));
  hipLaunchKernelGGL(kv_append_kernel, grid, dim3(kAppendThreads), 0, stream, (const u32x4*)k_new,
                     (const u32x4*)v_new, (u32x4*)k_pool, (u32x4*)v_pool, block_tables,
                     context_lens, S, Hkv, D, MAXB, B, max_ctx, NB, id_faults);
  return hipGetLastError();
}

}  // namespace pkv
