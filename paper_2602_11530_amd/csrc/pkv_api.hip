// C-ABI layer of libpkv: argument validation (all of it before any launch, so
// it can be exercised without a GPU), launch geometry, status codes.
#include "../../include/pkv.h"

#include "pkv_kernels.h"

#include <atomic>

// Workspace of paged_decode_attn_static: device memory that exists from the
// moment the library is loaded on a GPU until the process ends, so that entry
// point never allocates.  In host code this name is only a handle for
// hipGetSymbolAddress; the address kernels are given is looked up per device.
constexpr size_t kStaticScratchBytes = PKV_STATIC_WORKSPACE_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

thread_local hipError_t g_last_launch_error = hipSuccess;
thread_local int32_t* g_id_faults = nullptr;   // see pkv_set_id_fault_counter

inline bool misaligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Library's partition choice when the caller leaves it open.  With the stream
// decomposition a partition only bounds how many tokens one partial result may
// stand for before it is folded into its segment's record, so the largest value
// is the cheapest.
constexpr int kDefaultPartition = pkv::kMaxPartition;

// Query heads.  Keeps every size product far inside 64 bits and the merge launch (one
// wavefront per (request, head)) below 2^32 work-items at the largest batch.
constexpr int kMaxHeads = 16384;

struct Geometry {
  int G, P, max_ctx;
  int64_t slots;   // upper bound on partial-record slots
};

int check_shape(const pkv_attn_shape* sh, Geometry* g) {
  if (!sh) return PKV_ERR_NULL;
  if (sh->num_seqs < 0 || sh->num_seqs > pkv::kMaxSeqs) return PKV_ERR_SHAPE;
  if (sh->num_q_heads <= 0 || sh->num_kv_heads <= 0 || sh->num_q_heads > kMaxHeads)
    return PKV_ERR_SHAPE;
  const int D = sh->head_dim;
  if (D != 64 && D != 128 && D != 256) return PKV_ERR_SHAPE;
  const int B = sh->block_size;
  if (B != 16 && B != 32 && B != pkv::kMaxBlockSize) return PKV_ERR_SHAPE;
  if (sh->num_q_heads % sh->num_kv_heads != 0) return PKV_ERR_SHAPE;
  const int G = sh->num_q_heads / sh->num_kv_heads;
  if (G > pkv::kMaxGroup) return PKV_ERR_SHAPE;
  // a wavefront parks a whole record (G rows of D floats) in its 16 KiB share of LDS
  if (D == 256 && G > 8) return PKV_ERR_SHAPE;
  if (sh->max_blocks_per_seq <= 0) return PKV_ERR_SHAPE;
  if ((int64_t)sh->max_blocks_per_seq * B > INT32_MAX) return PKV_ERR_SHAPE;
  const int cap = sh->max_blocks_per_seq * B;
  if (sh->max_context_len < 0 || sh->max_context_len > cap) return PKV_ERR_SHAPE;
  const int max_ctx = sh->max_context_len ? sh->max_context_len : cap;
  int P = sh->partition_size;
  if (P < 0) return PKV_ERR_SHAPE;
  if (P == 0) P = kDefaultPartition;
  if (P % B != 0 || P < B || P > pkv::kMaxPartition) return PKV_ERR_SHAPE;
  // 4 KiB slabs (16 tokens of one KV head) are numbered in 32 bits on the device
  if (sh->num_pool_blocks < 1 ||
      sh->num_pool_blocks > INT32_MAX / ((int64_t)sh->num_kv_heads * (B / pkv::kBlockTokens)))
    return PKV_ERR_SHAPE;
  // stream positions, slots and rows are 32-bit on the device
  const int64_t max_blocks = (max_ctx + pkv::kBlockTokens - 1) / pkv::kBlockTokens;
  if ((int64_t)sh->num_kv_heads * sh->num_seqs * max_blocks > INT32_MAX) return PKV_ERR_SHAPE;
  if ((int64_t)sh->num_seqs * sh->num_q_heads > INT32_MAX) return PKV_ERR_SHAPE;
  g->G = G;
  g->P = P;
  g->max_ctx = max_ctx;
  // one record per (wavefront, request, KV head) that meet: slot = segment + wavefront
  g->slots = (int64_t)sh->num_kv_heads * sh->num_seqs + pkv::kStreamWaves;
  return PKV_OK;
}

// Workspace: the partial records, then the prefix array.
struct WorkspaceLayout {
  size_t rec_bytes, cum_bytes;
  size_t total() const { return rec_bytes + cum_bytes; }
};

WorkspaceLayout workspace_layout(const pkv_attn_shape* sh, const Geometry& g) {
  WorkspaceLayout w;
  w.rec_bytes = (size_t)g.slots * pkv::record_floats(g.G, sh->head_dim) * sizeof(float);
  w.cum_bytes = ((size_t)(sh->num_seqs + 1) * sizeof(int32_t) + 15) & ~(size_t)15;
  return w;
}

size_t workspace_bytes(const pkv_attn_shape* sh, const Geometry& g) {
  return sh->num_seqs == 0 ? 0 : workspace_layout(sh, g).total();
}

int launch_status(hipError_t e) {
  if (e == hipSuccess) return PKV_OK;
  g_last_launch_error = e;
  return PKV_ERR_LAUNCH;
}

// Every GPU holds its own copy of `scratch` at its own address; the address is
// looked up once per device, with that device current, and kept.
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

int static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return launch_status(e);
  if (dev < 0 || dev >= kMaxDevices) return launch_status(hipErrorInvalidDevice);
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return launch_status(e);
    if (!p) return launch_status(hipErrorInvalidSymbol);
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return PKV_OK;
}

}  // namespace

extern "C" {

int pkv_version(void) { return 1003; }

const char* pkv_status_string(int status) {
  switch (status) {
    case PKV_OK: return "ok";
    case PKV_ERR_NULL: return "a required pointer is NULL";
    case PKV_ERR_SHAPE: return "unsupported or inconsistent sizes";
    case PKV_ERR_ALIGN: return "a pointer or byte count is not 16-byte aligned";
    case PKV_ERR_WORKSPACE: return "workspace missing or too small";
    case PKV_ERR_LAUNCH: return "HIP refused the launch";
    case PKV_ERR_HOST: return "the host buffer is not pinned host memory";
    default: return "unknown status";
  }
}

const char* pkv_last_launch_error(void) { return hipGetErrorString(g_last_launch_error); }

int pkv_set_id_fault_counter(int32_t* device_counter) {
  if (reinterpret_cast<uintptr_t>(device_counter) & 3u) return PKV_ERR_ALIGN;
  g_id_faults = device_counter;
  return PKV_OK;
}

int pkv_probe_stream_read(const void* k_buf, const void* v_buf, int64_t num_slabs,
                          int64_t total_blocks, void* sink, void* stream) {
  if (num_slabs < 1 || total_blocks < 0 || total_blocks > INT32_MAX) return PKV_ERR_SHAPE;
  if (total_blocks == 0) return PKV_OK;
  if (!k_buf || !v_buf) return PKV_ERR_NULL;
  if (misaligned16(k_buf) || misaligned16(v_buf) || (reinterpret_cast<uintptr_t>(sink) & 3u))
    return PKV_ERR_ALIGN;
  // slab numbers are 32-bit on the device; a larger buffer is used up to 2^30 slabs (4 TiB)
  const uint32_t slabs = num_slabs > ((int64_t)1 << 30) ? (1u << 30) : (uint32_t)num_slabs;
  return launch_status(pkv::launch_stream_read_probe(k_buf, v_buf, slabs, total_blocks, sink,
                                                     static_cast<hipStream_t>(stream)));
}

int pkv_attn_partition_size(const pkv_attn_shape* shape) {
  Geometry g;
  const int rc = check_shape(shape, &g);
  return rc != PKV_OK ? rc : g.P;
}

int pkv_attn_workspace_bytes(const pkv_attn_shape* shape, size_t* out_bytes) {
  if (!out_bytes) return PKV_ERR_NULL;
  Geometry g;
  const int rc = check_shape(shape, &g);
  if (rc != PKV_OK) return rc;
  *out_bytes = workspace_bytes(shape, g);
  return PKV_OK;
}

// Validation shared by the single-layer and the multi-layer call; fills the
// launch descriptor except for the per-layer pointers.
static int prepare_attn(const int32_t* block_tables, const int32_t* context_lens, float scale,
                        const pkv_attn_shape* shape, void* workspace, size_t workspace_bytes_given,
                        pkv::AttnLaunch* a, bool* empty) {
  Geometry g;
  const int rc = check_shape(shape, &g);
  if (rc != PKV_OK) return rc;
  *empty = shape->num_seqs == 0;
  if (*empty) return PKV_OK;
  if (!block_tables || !context_lens) return PKV_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(block_tables) & 3u) || (reinterpret_cast<uintptr_t>(context_lens) & 3u))
    return PKV_ERR_ALIGN;
  const size_t need = workspace_bytes(shape, g);
  if (need) {
    if (!workspace || workspace_bytes_given < need) return PKV_ERR_WORKSPACE;
    if (misaligned16(workspace)) return PKV_ERR_ALIGN;
  }
  a->block_tables = block_tables;
  a->context_lens = context_lens;
  a->S = shape->num_seqs;
  a->Hq = shape->num_q_heads;
  a->Hkv = shape->num_kv_heads;
  a->G = g.G;
  a->D = shape->head_dim;
  // a D = 256 wavefront needs the registers of a whole SIMD lane: one wavefront per SIMD
  a->waves = shape->head_dim == 256 ? pkv::kStreamWaves / 2 : pkv::kStreamWaves;
  a->id_faults = g_id_faults;
  a->MAXB = shape->max_blocks_per_seq;
  a->upb = shape->block_size / pkv::kBlockTokens;
  a->P = g.P;
  a->max_ctx = g.max_ctx;
  a->NB = (int)shape->num_pool_blocks;
  a->scale_log2e = scale * 1.4426950408889634f;
  a->out_scale = 1.f;
  a->kv_fp8 = 0;
  const WorkspaceLayout lay = workspace_layout(shape, g);
  char* ws = static_cast<char*>(workspace);
  a->ws_rec = reinterpret_cast<float*>(ws);
  a->ws_cum = reinterpret_cast<int32_t*>(ws + lay.rec_bytes);
  return PKV_OK;
}

static int check_layer_pointers(const void* q, const void* k_pool, const void* v_pool, const void* out) {
  if (!q || !k_pool || !v_pool || !out) return PKV_ERR_NULL;
  if (misaligned16(q) || misaligned16(k_pool) || misaligned16(v_pool) || misaligned16(out))
    return PKV_ERR_ALIGN;
  return PKV_OK;
}

static int launch_layer(pkv::AttnLaunch& a, const void* q, const void* k_pool, const void* v_pool,
                        void* out, hipStream_t st) {
  a.q = static_cast<const uint16_t*>(q);
  a.k_pool = k_pool;
  a.v_pool = v_pool;
  a.out = static_cast<uint16_t*>(out);
  hipError_t e = pkv::launch_attn_stream(a, st);
  if (e != hipSuccess) return launch_status(e);
  e = pkv::launch_attn_reduce(a, st);
  if (e != hipSuccess) return launch_status(e);
  return PKV_OK;
}

int paged_decode_attn(const void* q, const void* k_pool, const void* v_pool,
                      const int32_t* block_tables, const int32_t* context_lens, float scale,
                      void* out, const pkv_attn_shape* shape, void* workspace,
                      size_t workspace_bytes_given, void* stream) {
  pkv::AttnLaunch a;
  bool empty = false;
  int rc = prepare_attn(block_tables, context_lens, scale, shape, workspace, workspace_bytes_given,
                        &a, &empty);
  if (rc != PKV_OK || empty) return rc;
  rc = check_layer_pointers(q, k_pool, v_pool, out);
  if (rc != PKV_OK) return rc;
  return launch_layer(a, q, k_pool, v_pool, out, static_cast<hipStream_t>(stream));
}

int paged_decode_attn_fp8kv(const void* q, const void* k_pool, const void* v_pool,
                            const int32_t* block_tables, const int32_t* context_lens, float scale,
                            float k_scale, float v_scale, void* out, const pkv_attn_shape* shape,
                            void* workspace, size_t workspace_bytes_given, void* stream) {
  Geometry g;
  int rc = check_shape(shape, &g);
  if (rc != PKV_OK) return rc;
  if (!(k_scale > 0.f) || !(v_scale > 0.f) || !(k_scale < __builtin_inff()) ||
      !(v_scale < __builtin_inff()))
    return PKV_ERR_SHAPE;
  pkv::AttnLaunch a;
  bool empty = false;
  rc = prepare_attn(block_tables, context_lens, scale, shape, workspace, workspace_bytes_given, &a,
                    &empty);
  if (rc != PKV_OK || empty) return rc;
  rc = check_layer_pointers(q, k_pool, v_pool, out);
  if (rc != PKV_OK) return rc;
  // K = k_scale * e4m3: the factor joins the softmax scale; V = v_scale * e4m3: applied once
  // to the normalised row
  a.scale_log2e = scale * k_scale * 1.4426950408889634f;
  a.out_scale = v_scale;
  a.kv_fp8 = 1;
  return launch_layer(a, q, k_pool, v_pool, out, static_cast<hipStream_t>(stream));
}

int paged_decode_attn_static(const void* q, const void* k_pool, const void* v_pool,
                             const int32_t* block_tables, const int32_t* context_lens, float scale,
                             void* out, const pkv_attn_shape* shape, void* stream) {
  Geometry g;
  int rc = check_shape(shape, &g);
  if (rc != PKV_OK) return rc;
  if (shape->num_seqs == 0) return PKV_OK;
  if (workspace_bytes(shape, g) > kStaticScratchBytes) return PKV_ERR_WORKSPACE;
  rc = check_layer_pointers(q, k_pool, v_pool, out);
  if (rc != PKV_OK) return rc;
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc != PKV_OK) return rc;
  pkv::AttnLaunch a;
  bool empty = false;
  rc = prepare_attn(block_tables, context_lens, scale, shape, ws, kStaticScratchBytes, &a, &empty);
  if (rc != PKV_OK || empty) return rc;
  return launch_layer(a, q, k_pool, v_pool, out, static_cast<hipStream_t>(stream));
}

int paged_decode_attn_layers(const void* const* q, const void* const* k_pools,
                             const void* const* v_pools, const int32_t* block_tables,
                             const int32_t* context_lens, float scale, void* const* out,
                             int32_t num_layers, const pkv_attn_shape* shape, void* workspace,
                             size_t workspace_bytes_given, void* stream) {
  if (num_layers < 0) return PKV_ERR_SHAPE;
  pkv::AttnLaunch a;
  bool empty = false;
  int rc = prepare_attn(block_tables, context_lens, scale, shape, workspace, workspace_bytes_given,
                        &a, &empty);
  if (rc != PKV_OK || empty || num_layers == 0) return rc;
  if (!q || !k_pools || !v_pools || !out) return PKV_ERR_NULL;
  // every layer is checked before the first launch: an error enqueues nothing
  for (int32_t l = 0; l < num_layers; ++l) {
    rc = check_layer_pointers(q[l], k_pools[l], v_pools[l], out[l]);
    if (rc != PKV_OK) return rc;
  }
  for (int32_t l = 0; l < num_layers; ++l) {
    rc = launch_layer(a, q[l], k_pools[l], v_pools[l], out[l], static_cast<hipStream_t>(stream));
    if (rc != PKV_OK) return rc;
  }
  return PKV_OK;
}

int kv_append(const void* k_new, const void* v_new, void* k_pool, void* v_pool,
              const int32_t* block_tables, const int32_t* context_lens,
              const pkv_attn_shape* shape, void* stream) {
  Geometry g;
  const int rc = check_shape(shape, &g);
  if (rc != PKV_OK) return rc;
  if (shape->num_seqs == 0) return PKV_OK;
  if (!k_new || !v_new || !k_pool || !v_pool || !block_tables || !context_lens) return PKV_ERR_NULL;
  if (misaligned16(k_new) || misaligned16(v_new) || misaligned16(k_pool) || misaligned16(v_pool) ||
      (reinterpret_cast<uintptr_t>(block_tables) & 3u) || (reinterpret_cast<uintptr_t>(context_lens) & 3u))
    return PKV_ERR_ALIGN;
  const hipError_t e = pkv::launch_kv_append(
      static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new),
      static_cast<uint16_t*>(k_pool), static_cast<uint16_t*>(v_pool), block_tables, context_lens,
      shape->num_seqs, shape->num_kv_heads, shape->head_dim, shape->max_blocks_per_seq,
      shape->block_size, g.max_ctx, (int)shape->num_pool_blocks, g_id_faults,
      static_cast<hipStream_t>(stream));
  return launch_status(e);
}

int kv_append_fp8(const void* k_new, const void* v_new, void* k_pool, void* v_pool,
                  const int32_t* block_tables, const int32_t* context_lens, float k_scale,
                  float v_scale, const pkv_attn_shape* shape, void* stream) {
  Geometry g;
  const int rc = check_shape(shape, &g);
  if (rc != PKV_OK) return rc;
  if (!(k_scale > 0.f) || !(v_scale > 0.f) || !(k_scale < __builtin_inff()) ||
      !(v_scale < __builtin_inff()))
    return PKV_ERR_SHAPE;
  if (shape->num_seqs == 0) return PKV_OK;
  if (!k_new || !v_new || !k_pool || !v_pool || !block_tables || !context_lens) return PKV_ERR_NULL;
  if (misaligned16(k_new) || misaligned16(v_new) || misaligned16(k_pool) || misaligned16(v_pool) ||
      (reinterpret_cast<uintptr_t>(block_tables) & 3u) || (reinterpret_cast<uintptr_t>(context_lens) & 3u))
    return PKV_ERR_ALIGN;
  const hipError_t e = pkv::launch_kv_append_fp8(
      static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new), k_pool, v_pool,
      block_tables, context_lens, k_scale, v_scale, shape->num_seqs, shape->num_kv_heads,
      shape->head_dim, shape->max_blocks_per_seq, shape->block_size, g.max_ctx,
      (int)shape->num_pool_blocks, g_id_faults, static_cast<hipStream_t>(stream));
  return launch_status(e);
}

// Host-visible checks of a block copy; *empty is set when there is nothing to do.
static int check_copy(const void* pool, const void* staging, const int32_t* block_ids,
                      int64_t n_blocks, int64_t block_bytes, int64_t num_pool_blocks, bool* empty) {
  *empty = false;
  if (n_blocks < 0 || block_bytes <= 0 || num_pool_blocks < 0) return PKV_ERR_SHAPE;
  if (block_bytes % 16 != 0) return PKV_ERR_ALIGN;
  if (n_blocks > INT32_MAX || block_bytes > ((int64_t)1 << 30)) return PKV_ERR_SHAPE;
  *empty = n_blocks == 0;
  if (*empty) return PKV_OK;
  if (!pool || !staging || !block_ids) return PKV_ERR_NULL;
  if (misaligned16(pool) || misaligned16(staging) || (reinterpret_cast<uintptr_t>(block_ids) & 3u))
    return PKV_ERR_ALIGN;
  return PKV_OK;
}

// The far end of an offload or reload must be page-locked host memory: only
// then is the copy asynchronous and done by the DMA engines at link speed.
static int check_pinned(const void* host, size_t bytes) {
  // the first and the last byte must both lie in page-locked host memory
  const char* ends[2] = {static_cast<const char*>(host), static_cast<const char*>(host) + (bytes - 1)};
  for (const char* p : ends) {
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
      (void)hipGetLastError();   // an unknown pointer is reported as an error; clear it
      return PKV_ERR_HOST;
    }
    if (attr.type != hipMemoryTypeHost) return PKV_ERR_HOST;
  }
  return PKV_OK;
}

static int copy_call(const void* pool, const void* staging, const int32_t* block_ids,
                     int64_t n_blocks, int64_t block_bytes, int64_t num_pool_blocks, bool gather,
                     void* stream) {
  bool empty = false;
  const int rc = check_copy(pool, staging, block_ids, n_blocks, block_bytes, num_pool_blocks, &empty);
  if (rc != PKV_OK || empty) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const hipError_t e =
      gather ? pkv::launch_kv_block_copy(pool, const_cast<void*>(staging), block_ids, n_blocks,
                                         block_bytes, num_pool_blocks, true, g_id_faults, st)
             : pkv::launch_kv_block_copy(staging, const_cast<void*>(pool), block_ids, n_blocks,
                                         block_bytes, num_pool_blocks, false, g_id_faults, st);
  return launch_status(e);
}

int kv_blocks_gather(const void* pool, const int32_t* block_ids, void* staging, int64_t n_blocks,
                     int64_t block_bytes, int64_t num_pool_blocks, void* stream) {
  return copy_call(pool, staging, block_ids, n_blocks, block_bytes, num_pool_blocks, true, stream);
}

int kv_blocks_scatter(const void* staging, void* pool, const int32_t* block_ids, int64_t n_blocks,
                      int64_t block_bytes, int64_t num_pool_blocks, void* stream) {
  return copy_call(pool, staging, block_ids, n_blocks, block_bytes, num_pool_blocks, false, stream);
}

int kv_blocks_move(const void* src_pool, const int32_t* src_ids, void* dst_pool,
                   const int32_t* dst_ids, int64_t n_blocks, int64_t block_bytes,
                   int64_t src_pool_blocks, int64_t dst_pool_blocks, void* stream) {
  if (n_blocks < 0 || block_bytes <= 0 || src_pool_blocks < 0 || dst_pool_blocks < 0) return PKV_ERR_SHAPE;
  if (block_bytes % 16 != 0) return PKV_ERR_ALIGN;
  if (n_blocks > INT32_MAX || block_bytes > ((int64_t)1 << 30)) return PKV_ERR_SHAPE;
  if (n_blocks == 0) return PKV_OK;
  if (!src_pool || !dst_pool || !src_ids || !dst_ids) return PKV_ERR_NULL;
  if (misaligned16(src_pool) || misaligned16(dst_pool) || (reinterpret_cast<uintptr_t>(src_ids) & 3u) ||
      (reinterpret_cast<uintptr_t>(dst_ids) & 3u))
    return PKV_ERR_ALIGN;
  return launch_status(pkv::launch_kv_block_move(src_pool, src_ids, src_pool_blocks, dst_pool, dst_ids,
                                                 dst_pool_blocks, n_blocks, block_bytes, g_id_faults,
                                                 static_cast<hipStream_t>(stream)));
}

int kv_blocks_offload(const void* pool, const int32_t* block_ids, void* staging, void* host_dst,
                      int64_t n_blocks, int64_t block_bytes, int64_t num_pool_blocks, void* stream) {
  bool empty = false;
  int rc = check_copy(pool, staging, block_ids, n_blocks, block_bytes, num_pool_blocks, &empty);
  if (rc != PKV_OK || empty) return rc;
  if (!host_dst) return PKV_ERR_NULL;
  rc = check_pinned(host_dst, (size_t)n_blocks * (size_t)block_bytes);
  if (rc != PKV_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e = pkv::launch_kv_block_copy(pool, staging, block_ids, n_blocks, block_bytes,
                                           num_pool_blocks, true, g_id_faults, st);
  if (e != hipSuccess) return launch_status(e);
  e = hipMemcpyAsync(host_dst, staging, (size_t)n_blocks * (size_t)block_bytes,
                     hipMemcpyDeviceToHost, st);
  return launch_status(e);
}

int kv_blocks_reload(const void* host_src, void* staging, void* pool, const int32_t* block_ids,
                     int64_t n_blocks, int64_t block_bytes, int64_t num_pool_blocks, void* stream) {
  bool empty = false;
  int rc = check_copy(pool, staging, block_ids, n_blocks, block_bytes, num_pool_blocks, &empty);
  if (rc != PKV_OK || empty) return rc;
  if (!host_src) return PKV_ERR_NULL;
  rc = check_pinned(host_src, (size_t)n_blocks * (size_t)block_bytes);
  if (rc != PKV_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e = hipMemcpyAsync(staging, host_src, (size_t)n_blocks * (size_t)block_bytes,
                                hipMemcpyHostToDevice, st);
  if (e != hipSuccess) return launch_status(e);
  e = pkv::launch_kv_block_copy(staging, pool, block_ids, n_blocks, block_bytes, num_pool_blocks,
                                false, g_id_faults, st);
  return launch_status(e);
}

}  // extern "C"
