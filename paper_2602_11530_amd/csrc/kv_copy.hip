// KV-block gather / scatter for gfx950: whole physical blocks move between a
// paged pool and a contiguous staging image (eviction / reload of a preempted
// request, paper Section II-B; whole-cache migration at the phase boundary,
// Section IV-B).  Pure 16-byte loads and stores, no arithmetic: bit-exact.
#include "pkv_kernels.h"

namespace pkv {
namespace {

// Cache policy.  The pool side is always nontemporal: neither the blocks read
// nor the blocks written are touched again soon, and ordinary stores would leave
// dirty lines whose write-back slows the kernel that runs next (an attention
// call measured 17-30 % slower after such a copy).  The staging side depends on
// the image's size.  An image that fits the 256 MB memory-side cache of an
// MI355X is written with write-through stores and read back with ordinary
// loads, so that the scatter (or the copy engine) that follows finds it on
// chip: gather + scatter of 153 MB per pool run 22 % faster that way (6.66
// instead of 5.44 TB/s read+write), with no effect on the next kernel.  The
// gain holds up to an image of about 280 MB, is gone at 310 MB, and beyond that
// a cached image only evicts itself (8 % slower than streaming at 370 MB), so
// larger images are streamed with nontemporal accesses on both sides.
constexpr int kCopyThreads = 256;
constexpr int kChunksPerThread = 8;                               // 16-byte chunks
constexpr int kChunksPerGroup = kCopyThreads * kChunksPerThread;  // 32 KiB per workgroup
constexpr int64_t kCachedStagingBytes = (int64_t)256 << 20;       // staging images up to this size stay on chip

enum Policy { kStream, kPlain, kWriteThrough };

template <int kPolicy>
__device__ __forceinline__ u32x4 ld16(const u32x4* p) {
  if (kPolicy == kStream) return __builtin_nontemporal_load(p);
  return *p;
}
template <int kPolicy>
__device__ __forceinline__ void st16(u32x4* p, u32x4 v) {
  if (kPolicy == kStream) __builtin_nontemporal_store(v, p);
  else if (kPolicy == kWriteThrough)
    // opaque to the compiler, so the wait states a wide store needs before its data
    // registers may be overwritten are spelled out
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
  else *p = v;
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
template <int kMode, bool kCachedStaging>
__global__ __launch_bounds__(kCopyThreads) void kv_block_copy_kernel(
    const u32x4* __restrict__ src, u32x4* __restrict__ dst, const int32_t* __restrict__ ids_a,
    const int32_t* __restrict__ ids_b, int64_t chunks_per_block, int64_t src_pool_blocks,
    int64_t dst_pool_blocks, int64_t n_blocks, int slices, int32_t* __restrict__ id_faults) {
  const int64_t n_units = n_blocks * slices;
  for (int64_t u = blockIdx.x; u < n_units; u += gridDim.x) {
    const int64_t i = u / slices, slice = u - i * slices;
    int64_t from = i, to = i;
    if (kMode == 0 || kMode == 2) from = ids_a[i];
    if (kMode == 1) to = ids_a[i];
    if (kMode == 2) to = ids_b[i];
    if (from < 0 || from >= src_pool_blocks || to < 0 || to >= dst_pool_blocks) {
      // never follow a corrupt id; the skipped block is reported once
      if (id_faults && slice == 0 && threadIdx.x == 0) atomicAdd(id_faults, 1);
      continue;
    }
    constexpr int kLd = (kMode == 1 && kCachedStaging) ? kPlain : kStream;
    constexpr int kSt = (kMode == 0 && kCachedStaging) ? kWriteThrough : kStream;
    copy_slice<kLd, kSt>(src + from * chunks_per_block, dst + to * chunks_per_block, slice,
                         chunks_per_block);
  }
}

template <int kMode>
hipError_t launch(const void* src, void* dst, const int32_t* ids_a, const int32_t* ids_b,
                  int64_t src_pool_blocks, int64_t dst_pool_blocks, int64_t n_blocks,
                  int64_t block_bytes, int32_t* id_faults, hipStream_t stream) {
  const int64_t chunks = block_bytes / 16;
  const int64_t slices = (chunks + kChunksPerGroup - 1) / kChunksPerGroup;
  const int64_t units = n_blocks * slices;
  // one workgroup per slice (the hardware dispatcher balances them better than a
  // persistent grid did: 5.4 against 5.2-5.3 TB/s); a list of more than kMaxGroups slices
  // (256 GiB of 32 KiB slices, or very many tiny blocks) is walked with a stride, which
  // keeps the launch below 2^32 work-items
  constexpr int64_t kMaxGroups = (int64_t)1 << 23;
  const dim3 grid((unsigned)(units > kMaxGroups ? kMaxGroups : units));
  const bool cached = kMode != 2 && n_blocks * block_bytes <= kCachedStagingBytes;
  auto kernel = cached ? kv_block_copy_kernel<kMode, true> : kv_block_copy_kernel<kMode, false>;
  hipLaunchKernelGGL(kernel, grid, dim3(kCopyThreads), 0, stream, (const u32x4*)src, (u32x4*)dst,
                     ids_a, ids_b, chunks, src_pool_blocks, dst_pool_blocks, n_blocks, (int)slices,
                     id_faults);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_kv_block_copy(const void* src, void* dst, const int32_t* block_ids,
                                int64_t n_blocks, int64_t block_bytes, int64_t num_pool_blocks,
                                bool gather, int32_t* id_faults, hipStream_t stream) {
  return gather ? launch<0>(src, dst, block_ids, nullptr, num_pool_blocks, n_blocks, n_blocks,
                            block_bytes, id_faults, stream)
                : launch<1>(src, dst, block_ids, nullptr, n_blocks, num_pool_blocks, n_blocks,
                            block_bytes, id_faults, stream);
}

hipError_t launch_kv_block_move(const void* src, const int32_t* src_ids, int64_t src_pool_blocks,
                                void* dst, const int32_t* dst_ids, int64_t dst_pool_blocks,
                                int64_t n_blocks, int64_t block_bytes, int32_t* id_faults,
                                hipStream_t stream) {
  return launch<2>(src, dst, src_ids, dst_ids, src_pool_blocks, dst_pool_blocks, n_blocks,
                   block_bytes, id_faults, stream);
}

}  // namespace pkv
