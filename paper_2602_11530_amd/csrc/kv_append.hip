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

// The same step for one-byte E4M3 pools: every element is divided by its pool's scale in fp32,
// clamped to the format's range (+-448: there is no infinity to overflow to) and rounded to
// nearest even by the hardware conversion.  One lane takes eight dims: 16 bytes in, 8 bytes out.
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float to_range(float y) {
  return (y != y) ? y : fminf(fmaxf(y, -448.f), 448.f);   // NaN stays NaN
}
// two bf16 of one dword, scaled -> two e4m3 bytes in the chosen half of `old`
template <bool kHigh>
__device__ __forceinline__ int quantise2(uint32_t pair, float scale, int old) {
  const float a = __uint_as_float(pair << 16) / scale;
  const float b = __uint_as_float(pair & 0xffff0000u) / scale;
  return __builtin_amdgcn_cvt_pk_fp8_f32(to_range(a), to_range(b), old, kHigh);
}

__global__ __launch_bounds__(kAppendThreads) void kv_append_fp8_kernel(
    const u32x4* __restrict__ k_new, const u32x4* __restrict__ v_new, u32x2* __restrict__ k_pool,
    u32x2* __restrict__ v_pool, const int32_t* __restrict__ block_tables,
    const int32_t* __restrict__ context_lens, float k_scale, float v_scale, int S, int Hkv, int D,
    int MAXB, int B, int max_ctx, int NB, int32_t* __restrict__ id_faults) {
  const int kRowChunks = D / 8;   // eight dims per lane
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
  if ((unsigned)id >= (unsigned)NB) {
    if (id_faults && kvh == 0 && chunk == 0) atomicAdd(id_faults, 1);
    return;
  }
  const int64_t dst = (((int64_t)id * Hkv + kvh) * B + t % B) * kRowChunks + chunk;
  const u32x4 kx = k_new[idx], vx = v_new[idx];
  u32x2 k8, v8;
  k8.x = quantise2<true>(kx.y, k_scale, quantise2<false>(kx.x, k_scale, 0));
  k8.y = quantise2<true>(kx.w, k_scale, quantise2<false>(kx.z, k_scale, 0));
  v8.x = quantise2<true>(vx.y, v_scale, quantise2<false>(vx.x, v_scale, 0));
  v8.y = quantise2<true>(vx.w, v_scale, quantise2<false>(vx.z, v_scale, 0));
  k_pool[dst] = k8;
  v_pool[dst] = v8;
}

}  // namespace

hipError_t launch_kv_append_fp8(const uint16_t* k_new, const uint16_t* v_new, void* k_pool,
                                void* v_pool, const int32_t* block_tables,
                                const int32_t* context_lens, float k_scale, float v_scale, int S,
                                int Hkv, int D, int MAXB, int B, int max_ctx, int NB,
                                int32_t* id_faults, hipStream_t stream) {
  const int64_t total = (int64_t)S * Hkv * (D / 8);
  dim3 grid((unsigned)((total + kAppendThreads - 1) / kAppendThreads));
  hipLaunchKernelGGL(kv_append_fp8_kernel, grid, dim3(kAppendThreads), 0, stream,
                     (const u32x4*)k_new, (const u32x4*)v_new, (u32x2*)k_pool, (u32x2*)v_pool,
                     block_tables, context_lens, k_scale, v_scale, S, Hkv, D, MAXB, B, max_ctx, NB,
                     id_faults);
  return hipGetLastError();
}

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
