// KV-block gather / scatter for gfx950: whole physical blocks move between a
// paged pool and a contiguous staging image (eviction / reload of a preempted
// request, paper Section II-B; whole-cache migration at the phase boundary,
// Section IV-B).  Pure 16-byte loads and stores, no arithmetic: bit-exact.
#include "pkv_kernels.h"

namespace pkv {
namespace {

// Loads and stores are nontemporal.  Neither side is reused soon enough to be
// worth a cache line, and in a decode loop the choice matters more for the next
// kernel than for this one: with ordinary or write-through (sc1) stores the copy
// itself gets up to 20 % faster but the attention call that follows slows by
// 17-30 % while the lines drain; nontemporal stores are the best total.
#ifndef PKV_COPY_THREADS
#define PKV_COPY_THREADS 256
#endif
#ifndef PKV_COPY_CHUNKS
#define PKV_COPY_CHUNKS 8
#endif
#ifndef PKV_COPY_GRID
#define PKV_COPY_GRID 0        // 0: one workgroup per slice; N: N persistent workgroups
#endif
// cache policy per side: 0 nontemporal, 1 plain, 2 sc1, 3 sc0 sc1 nt (stores); 0 nontemporal, 1 plain, 2 sc1 (loads)
#ifndef PKV_COPY_POOL_LD
#define PKV_COPY_POOL_LD 0
#endif
#ifndef PKV_COPY_POOL_ST
#define PKV_COPY_POOL_ST 0
#endif
#ifndef PKV_COPY_STAGE_LD
#define PKV_COPY_STAGE_LD 0
#endif
#ifndef PKV_COPY_STAGE_ST
#define PKV_COPY_STAGE_ST 0
#endif
constexpr int kCopyThreads = PKV_COPY_THREADS;
constexpr int kChunksPerThread = PKV_COPY_CHUNKS;                 // 16-byte chunks
constexpr int kChunksPerGroup = kCopyThreads * kChunksPerThread;  // 32 KiB per workgroup
constexpr int kCopyGrid = PKV_COPY_GRID;

template <int kPolicy>
__device__ __forceinline__ u32x4 ld16(const u32x4* p) {
  if (kPolicy == 0) return __builtin_nontemporal_load(p);
  if (kPolicy == 1) return *p;
  u32x4 v;
  asm volatile("global_load_dwordx4 %0, %1, off sc1\n\ts_waitcnt vmcnt(0)" : "=v"(v) : "v"(p) : "memory");
  return v;
}
template <int kPolicy>
__device__ __forceinline__ void st16(u32x4* p, u32x4 v) {
  if (kPolicy == 0) __builtin_nontemporal_store(v, p);
  else if (kPolicy == 1) *p = v;
  else if (kPolicy == 2) asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(p), "v"(v) : "memory");
  else asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt" : : "v"(p), "v"(v) : "memory");
}

// One workgroup moves one slice (kChunksPerGroup chunks of one block): all
// loads first, then all stores.
template <int kLd, int kSt>
__device__ __forceinline__ void copy_slice(const u32x4* __restrict__ s, u32x4* __restrict__ d,
                                           int64_t slice, int64_t chunks_per_block) {
  const int64_t c0 = slice * kChunksPerGroup + threadIdx.x;
  if ((slice + 1) * kChunksPerGroup <= chunks_per_block) {
    // Whole slice inside the block (always, for 32 KiB blocks): all loads are
    // issued before the first store, with no per-lane guard in the way.
    u32x4 v[kChunksPerThread];
#pragma unroll
    for (int u = 0; u < kChunksPerThread; ++u) v[u] = ld16<kLd>(s + c0 + (int64_t)u * kCopyThreads);
#pragma unroll
    for (int u = 0; u < kChunksPerThread; ++u) st16<kSt>(d + c0 + (int64_t)u * kCopyThreads, v[u]);
  } else {
    // Ragged last slice of an odd block size.
    for (int u = 0; u < kChunksPerThread; ++u) {
      const int64_t c = c0 + (int64_t)u * kCopyThreads;
      if (c < chunks_per_block) st16<kSt>(d + c, ld16<kLd>(s + c));
    }
  }
}

// kMode 0: staging[i] = pool[ids_a[i]]; 1: pool[ids_a[i]] = staging[i];
// 2: dst[ids_b[i]] = src[ids_a[i]].  A unit is one slice of one listed block;
// the physical ids are wave-uniform, so the pool-side base address is scalar;
// byte offsets are 64-bit (a pool passes 2 GiB at the long-context sizes).
template <int kMode>
__global__ __launch_bounds__(kCopyThreads) void kv_block_copy_kernel(
    const u32x4* __restrict__ src, u32x4* __restrict__ dst, const int32_t* __restrict__ ids_a,
    const int32_t* __restrict__ ids_b, int64_t chunks_per_block, int64_t src_pool_blocks,
    int64_t dst_pool_blocks, int64_t n_blocks, int slices) {
  const int64_t n_units = n_blocks * slices;
  for (int64_t u = blockIdx.x; u < n_units; u += gridDim.x) {
    const int64_t i = u / slices, slice = u - i * slices;
    int64_t from = i, to = i;
    if (kMode == 0 || kMode == 2) {
      from = ids_a[i];
      if (from < 0 || from >= src_pool_blocks) continue;   // never follow a corrupt id
    }
    if (kMode == 1) {
      to = ids_a[i];
      if (to < 0 || to >= dst_pool_blocks) continue;
    }
    if (kMode == 2) {
      to = ids_b[i];
      if (to < 0 || to >= dst_pool_blocks) continue;
    }
    constexpr int kLd = kMode == 1 ? PKV_COPY_STAGE_LD : PKV_COPY_POOL_LD;
    constexpr int kSt = kMode == 0 ? PKV_COPY_STAGE_ST : PKV_COPY_POOL_ST;
    copy_slice<kLd, kSt>(src + from * chunks_per_block, dst + to * chunks_per_block, slice, chunks_per_block);
  }
}

template <int kMode>
hipError_t launch(const void* src, void* dst, const int32_t* ids_a, const int32_t* ids_b,
                  int64_t src_pool_blocks, int64_t dst_pool_blocks, int64_t n_blocks,
                  int64_t block_bytes, hipStream_t stream) {
  const int64_t chunks = block_bytes / 16;
  const int64_t slices = (chunks + kChunksPerGroup - 1) / kChunksPerGroup;
  const int64_t units = n_blocks * slices;
  int64_t groups = kCopyGrid > 0 ? (units < kCopyGrid ? units : kCopyGrid) : units;
  if (groups > 0x7fffffff) groups = 0x7fffffff;   // the kernel strides over the rest
  hipLaunchKernelGGL(kv_block_copy_kernel<kMode>, dim3((unsigned)groups), dim3(kCopyThreads), 0,
                     stream, (const u32x4*)src, (u32x4*)dst, ids_a, ids_b, chunks, src_pool_blocks,
                     dst_pool_blocks, n_blocks, (int)slices);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_kv_block_copy(const void* src, void* dst, const int32_t* block_ids,
                                int64_t n_blocks, int64_t block_bytes, int64_t num_pool_blocks,
                                bool gather, hipStream_t stream) {
  return gather ? launch<0>(src, dst, block_ids, nullptr, num_pool_blocks, n_blocks, n_blocks,
                            block_bytes, stream)
                : launch<1>(src, dst, block_ids, nullptr, n_blocks, num_pool_blocks, n_blocks,
                            block_bytes, stream);
}

hipError_t launch_kv_block_move(const void* src, const int32_t* src_ids, int64_t src_pool_blocks,
                                void* dst, const int32_t* dst_ids, int64_t dst_pool_blocks,
                                int64_t n_blocks, int64_t block_bytes, hipStream_t stream) {
  return launch<2>(src, dst, src_ids, dst_ids, src_pool_blocks, dst_pool_blocks, n_blocks,
                   block_bytes, stream);
}

}  // namespace pkv
