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
constexpr int kCopyThreads = 256;
constexpr int kChunksPerThread = 8;                               // 16-byte chunks
constexpr int kChunksPerGroup = kCopyThreads * kChunksPerThread;  // 32 KiB per workgroup

// One workgroup moves one 32 KiB slice: all loads first, then all stores.
__device__ __forceinline__ void copy_slice(const u32x4* __restrict__ s, u32x4* __restrict__ d,
                                           int64_t chunks_per_block) {
  const int64_t c0 = (int64_t)blockIdx.y * kChunksPerGroup + threadIdx.x;
  if (((int64_t)blockIdx.y + 1) * kChunksPerGroup <= chunks_per_block) {
    // Whole slice inside the block (always, for 32 KiB blocks): all loads are
    // issued before the first store, with no per-lane guard in the way.
    u32x4 v[kChunksPerThread];
#pragma unroll
    for (int u = 0; u < kChunksPerThread; ++u) v[u] = __builtin_nontemporal_load(s + c0 + (int64_t)u * kCopyThreads);
#pragma unroll
    for (int u = 0; u < kChunksPerThread; ++u) __builtin_nontemporal_store(v[u], d + c0 + (int64_t)u * kCopyThreads);
  } else {
    // Ragged last slice of an odd block size.
    for (int u = 0; u < kChunksPerThread; ++u) {
      const int64_t c = c0 + (int64_t)u * kCopyThreads;
      if (c < chunks_per_block) __builtin_nontemporal_store(__builtin_nontemporal_load(s + c), d + c);
    }
  }
}

// blockIdx.x = index into block_ids, blockIdx.y = 32 KiB slice of that block.
// The physical id is wave-uniform, so the pool-side base address is scalar;
// byte offsets are 64-bit (a pool passes 2 GiB at the long-context sizes).
template <bool kGather>
__global__ __launch_bounds__(kCopyThreads) void kv_block_copy_kernel(
    const u32x4* __restrict__ src, u32x4* __restrict__ dst, const int32_t* __restrict__ block_ids,
    int64_t chunks_per_block, int64_t num_pool_blocks) {
  const int64_t i = blockIdx.x;
  const int64_t phys = block_ids[i];
  if (phys < 0 || phys >= num_pool_blocks) return;   // never follow a corrupt id
  const int64_t pool_base = phys * chunks_per_block;
  const int64_t stage_base = i * chunks_per_block;
  copy_slice(src + (kGather ? pool_base : stage_base), dst + (kGather ? stage_base : pool_base),
             chunks_per_block);
}

// Pool to pool: block src_ids[i] of one pool becomes block dst_ids[i] of another.
__global__ __launch_bounds__(kCopyThreads) void kv_block_move_kernel(
    const u32x4* __restrict__ src, const int32_t* __restrict__ src_ids, int64_t src_pool_blocks,
    u32x4* __restrict__ dst, const int32_t* __restrict__ dst_ids, int64_t dst_pool_blocks,
    int64_t chunks_per_block) {
  const int64_t from = src_ids[blockIdx.x], to = dst_ids[blockIdx.x];
  if (from < 0 || from >= src_pool_blocks || to < 0 || to >= dst_pool_blocks) return;
  copy_slice(src + from * chunks_per_block, dst + to * chunks_per_block, chunks_per_block);
}

}  // namespace

hipError_t launch_kv_block_copy(const void* src, void* dst, const int32_t* block_ids,
                                int64_t n_blocks, int64_t block_bytes, int64_t num_pool_blocks,
                                bool gather, hipStream_t stream) {
  const int64_t chunks = block_bytes / 16;
  const int64_t slices = (chunks + kChunksPerGroup - 1) / kChunksPerGroup;
  // grid.x carries the block list (up to 2^31-1), grid.y the slices of a block.
  dim3 grid((unsigned)n_blocks, (unsigned)slices, 1);
  if (gather)
    hipLaunchKernelGGL(kv_block_copy_kernel<true>, grid, dim3(kCopyThreads), 0, stream,
                       (const u32x4*)src, (u32x4*)dst, block_ids, chunks, num_pool_blocks);
  else
    hipLaunchKernelGGL(kv_block_copy_kernel<false>, grid, dim3(kCopyThreads), 0, stream,
                       (const u32x4*)src, (u32x4*)dst, block_ids, chunks, num_pool_blocks);
  return hipGetLastError();
}

hipError_t launch_kv_block_move(const void* src, const int32_t* src_ids, int64_t src_pool_blocks,
                                void* dst, const int32_t* dst_ids, int64_t dst_pool_blocks,
                                int64_t n_blocks, int64_t block_bytes, hipStream_t stream) {
  const int64_t chunks = block_bytes / 16;
  const int64_t slices = (chunks + kChunksPerGroup - 1) / kChunksPerGroup;
  dim3 grid((unsigned)n_blocks, (unsigned)slices, 1);
  hipLaunchKernelGGL(kv_block_move_kernel, grid, dim3(kCopyThreads), 0, stream, (const u32x4*)src,
                     src_ids, src_pool_blocks, (u32x4*)dst, dst_ids, dst_pool_blocks, chunks);
  return hipGetLastError();
}

}  // namespace pkv
