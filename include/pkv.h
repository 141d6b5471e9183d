/*
 * pkv — paged KV-cache decode attention and KV-block migration for MI355X (gfx950).
 *
 * C ABI.  Every pointer marked "device" is HIP device memory owned by the
 * caller; every pointer marked "host" is ordinary host memory read only during
 * the call.  The library allocates nothing, frees nothing and keeps no state
 * between calls (apart from the calling thread's fault-counter setting, see
 * pkv_set_id_fault_counter, and the address of the static workspace, see
 * paged_decode_attn_static), so calls on different streams may overlap as long
 * as their outputs (and workspaces) do not.  Every call validates its host-visible
 * arguments first, then enqueues its kernels on `stream` and returns without
 * synchronising.
 *
 * Pool layout.  A layer's K pool and V pool are each
 *     bf16 [num_pool_blocks][num_kv_heads][block_size][head_dim], row-major,
 * so one physical block is one contiguous image of
 *     num_kv_heads * block_size * head_dim * 2 bytes  (32 KiB at 8 x 16 x 128).
 * block_size is 16, 32 or 64 tokens; head_dim is 64, 128 or 256.
 *
 * Status codes: 0 = PKV_OK; negative = error.  Every argument error (NULL,
 * SHAPE, ALIGN, WORKSPACE, HOST) is found before the first launch and enqueues
 * nothing.  PKV_ERR_LAUNCH means HIP refused a launch or a copy part-way: what
 * the call had enqueued before (an earlier layer of paged_decode_attn_layers,
 * the stream pass of an attention call, the first half of an offload or reload)
 * stays enqueued, and the outputs of that call are undefined.
 */
#ifndef PKV_H_
#define PKV_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PKV_OK 0
#define PKV_ERR_NULL (-1)      /* a required pointer is NULL                          */
#define PKV_ERR_SHAPE (-2)     /* unsupported or inconsistent sizes                   */
#define PKV_ERR_ALIGN (-3)     /* a pointer or byte count is not 16-byte aligned      */
#define PKV_ERR_WORKSPACE (-4) /* workspace missing or smaller than required          */
#define PKV_ERR_LAUNCH (-5)    /* HIP refused the launch; see pkv_last_launch_error() */
#define PKV_ERR_HOST (-6)      /* a host buffer of an offload/reload is not pinned memory */

/* Sizes of one attention call.  The batch changes at every decode step
 * (continuous batching, paper Section II-B), so nothing here is fixed at
 * library start-up. */
typedef struct {
  int32_t num_seqs;           /* S: requests in this step's batch, 0..2048              */
  int32_t num_q_heads;        /* Hq, 1..16384                                            */
  int32_t num_kv_heads;       /* Hkv; Hq % Hkv == 0; query heads h*G..h*G+G-1 share
                                 KV head h (G = Hq/Hkv, 1 <= G <= 16)                    */
  int32_t head_dim;           /* D: 64, 128 or 256 (256 only with G <= 8)                */
  int32_t block_size;         /* B: tokens per physical block: 16, 32 or 64              */
  int32_t max_blocks_per_seq; /* MAXB: row stride of block_tables, >= ceil(L_s/B)        */
  int32_t partition_size;     /* P: split-K partition, the most tokens of a request that
                                 one partial result (max, sum, row) may cover: a multiple
                                 of B in [B, 65536], or 0 to let the library choose.
                                 Partial results of one request and KV head that the same
                                 wavefront produced are merged on chip; the merge pass
                                 combines the rest.  P does not change the workspace.    */
  int32_t max_context_len;    /* host upper bound on every context_lens[s]; 0 means
                                 MAXB*B.  A smaller bound only shrinks the launch;
                                 a request longer than the bound is attended up to it.   */
  int64_t num_pool_blocks;    /* NB: physical blocks in k_pool and in v_pool;
                                 1 <= NB and NB * Hkv * B/16 < 2^31                      */
} pkv_attn_shape;

/* The split-K partition size (tokens) a call with this shape will use:
 * shape->partition_size if non-zero, else the library's choice.
 * Returns a negative status on a bad shape. */
int pkv_attn_partition_size(const pkv_attn_shape* shape /* host */);

/* Bytes of device workspace paged_decode_attn needs for this shape (0 only for
 * an empty batch).  `out_bytes` is host memory. */
int pkv_attn_workspace_bytes(const pkv_attn_shape* shape /* host */, size_t* out_bytes);

/*
 * Decode-step attention of every request in the batch over its whole paged KV
 * cache — the memory-bandwidth-bound decoding stage of paper Section II-A,
 * whose time grows with the KV footprint (Section IV-B, discussion of the
 * reasoning-placement algorithm):
 *
 *   out[s,h,:] = sum_t softmax_t( scale * q[s,h,:] . K[s,t,kvh,:] ) * V[s,t,kvh,:]
 *   for t in [0, context_lens[s]),   kvh = h / G,
 *   K[s,t] = k_pool[ block_tables[s][t / B] ][kvh][t % B][:]   (V alike).
 *
 * context_lens[s] includes the token being decoded (its K,V row is already in
 * the pool).  A request with context_lens[s] == 0 gets an all-zero output row.
 * Table entries at index >= ceil(context_lens[s]/B) and slots past the last
 * valid token are never read, whatever they hold.  Dereferenced block ids must
 * lie in [0, num_pool_blocks); the device never follows an id outside that
 * range (the tokens of such a block are left out of the softmax, so a
 * corrupt table gives a wrong row, not a memory fault), and a negative
 * context_lens[s] counts as 0.  Several requests may map the same block.
 * NaN or Inf inside the rows a request does attend over propagates as in IEEE
 * arithmetic and stays where it belongs: a NaN in a K row turns the rows of
 * that KV head's query group into NaN, a NaN V element turns that output
 * element into NaN, an infinite V element leaves it non-finite (NaN or Inf);
 * every other output element is unaffected.
 *
 * Arithmetic: bf16 inputs, fp32 scores, softmax statistics and accumulation,
 * one round-to-nearest-even to bf16 at the end.  The result does not depend on
 * which physical blocks hold the rows.  The work is spread evenly over the GPU
 * by cutting the batch's KV blocks into equal shares, so where a request's
 * partial sums are split (and with it the last bits of its row) depends on the
 * lengths of the requests ahead of it in the batch.
 *
 *   q            device  bf16  [S][Hq][D]
 *   k_pool       device  bf16  [NB][Hkv][B][D]
 *   v_pool       device  bf16  [NB][Hkv][B][D]
 *   block_tables device  int32 [S][MAXB]
 *   context_lens device  int32 [S]
 *   scale        fp32 softmax scale (1/sqrt(D) for the configs here)
 *   out          device  bf16  [S][Hq][D], written in full
 *   shape        host
 *   workspace    device, >= pkv_attn_workspace_bytes(), 16-byte aligned; may be
 *                NULL when that size is 0.  Contents need no initialisation and
 *                are undefined afterwards.  Calls that overlap in time need
 *                separate workspaces.
 *   stream       hipStream_t (NULL = the default stream)
 */
int paged_decode_attn(const void* q, const void* k_pool, const void* v_pool,
                      const int32_t* block_tables, const int32_t* context_lens, float scale,
                      void* out, const pkv_attn_shape* shape, void* workspace,
                      size_t workspace_bytes, void* stream);

/*
 * The same attention for num_layers layers in one call.  A request has the same
 * context length and the same block ids in every layer of the model, so one
 * block table and one length array serve all layers while each layer has its
 * own q, K pool, V pool and output (the decode iteration of paper Section II-A
 * runs the attention of every layer over that layer's KV cache).  Equivalent to
 * calling paged_decode_attn for l = 0 .. num_layers-1 in order on `stream`
 * with the one workspace; the layers run one after the other.  All arguments of
 * all layers are validated before the first launch.
 *
 *   q, k_pools, v_pools, out   host arrays [num_layers] of device pointers, each
 *                              as the argument of the same name above
 *   num_layers                 >= 0; 0 is a no-op returning PKV_OK
 * Everything else as for paged_decode_attn.
 */
int paged_decode_attn_layers(const void* const* q, const void* const* k_pools,
                             const void* const* v_pools, const int32_t* block_tables,
                             const int32_t* context_lens, float scale, void* const* out,
                             int32_t num_layers, const pkv_attn_shape* shape, void* workspace,
                             size_t workspace_bytes, void* stream);

/*
 * The same attention over KV pools stored in 8 bits: K and V are OCP FP8 E4M3
 * bytes (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; no infinities,
 * 0x7F and 0xFF are NaN, largest finite value 448), one fp32 scale per pool:
 *
 *     K[.] = k_scale * e4m3(k_pool byte),     V[.] = v_scale * e4m3(v_pool byte),
 *
 * everything else as in paged_decode_attn (q and out bf16, fp32 arithmetic).
 * The paper's decode step is bound by the bytes of the KV cache it reads
 * (Section II-A); a one-byte cache halves them.  The paper fixes no quantised
 * format: this one (per-pool scales, E4M3) is the library's choice.  The bytes
 * are widened exactly (every E4M3 value is a bf16 value), k_scale joins the
 * softmax scale and v_scale multiplies the normalised row, so the result is the
 * attention of the de-quantised pools to the same tolerance as the bf16 call.
 *
 *   k_pool, v_pool  device  e4m3 [NB][Hkv][B][D], one byte per element: a block
 *                   is Hkv * B * D bytes (16 KiB at 8 x 16 x 128); the copies
 *                   (gather, scatter, move, offload, reload) take such a pool as
 *                   it is, with that block_bytes
 *   k_scale,v_scale positive finite fp32 (PKV_ERR_SHAPE otherwise)
 *   shape           as for paged_decode_attn: every head_dim and block_size
 * NaN bytes inside a request's valid rows propagate as NaN; unused slots and
 * unused blocks may hold any bytes.
 */
int paged_decode_attn_fp8kv(const void* q, const void* k_pool, const void* v_pool,
                            const int32_t* block_tables, const int32_t* context_lens, float scale,
                            float k_scale, float v_scale, void* out, const pkv_attn_shape* shape,
                            void* workspace, size_t workspace_bytes, void* stream);

/*
 * paged_decode_attn for callers that cannot allocate device memory or carry a
 * workspace around: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, same kernels and bit-identical results,
 * but the workspace is a fixed array of PKV_STATIC_WORKSPACE_BYTES that every
 * GPU the library runs on holds from load time until the process ends.  The
 * call allocates and frees nothing (no hipMalloc, no hipFree, no allocating
 * library routine); the first call on a device looks the array's address up
 * and should therefore be made once outside a graph capture.
 *
 * Returns PKV_ERR_WORKSPACE, enqueuing nothing, when pkv_attn_workspace_bytes()
 * for `shape` exceeds PKV_STATIC_WORKSPACE_BYTES (set max_context_len to the
 * batch's longest context to keep the bound tight).  All calls on one GPU share
 * the one array: two calls of this entry point that overlap in time on the same
 * GPU (different streams, or graphs replayed concurrently) race and give
 * undefined rows.  The array's contents need no initialisation between calls
 * and are undefined afterwards.
 */
#define PKV_STATIC_WORKSPACE_BYTES (32u << 20)
int paged_decode_attn_static(const void* q, const void* k_pool, const void* v_pool,
                             const int32_t* block_tables, const int32_t* context_lens,
                             float scale, void* out, const pkv_attn_shape* shape, void* stream);

/*
 * staging[i] = pool[block_ids[i]] for i in [0, n_blocks): the send side of
 * evicting a preempted request's KV cache (paper Section II-B) or of shipping
 * a request's entire KV cache at the reasoning-to-answering transition
 * (Section IV-B, "KV cache transfer overhead").  Whole blocks move, unused
 * slots included; the copy is bit-exact.
 *
 *   pool       device, num_pool_blocks blocks of block_bytes bytes
 *   block_ids  device int32 [n_blocks]; an id outside [0, num_pool_blocks) is
 *              skipped on the device (its staging image is left as it was)
 *   staging    device, n_blocks * block_bytes bytes, contiguous, must not
 *              overlap the listed blocks
 *   block_bytes  multiple of 16, at most 1 GiB
 *   n_blocks == 0 is a no-op returning PKV_OK.
 */
int kv_blocks_gather(const void* pool, const int32_t* block_ids, void* staging,
                     int64_t n_blocks, int64_t block_bytes, int64_t num_pool_blocks,
                     void* stream);

/*
 * pool[block_ids[i]] = staging[i]: the receive side — reloading a resumed
 * request (Section II-B) or installing a migrated one (Section IV-B) into
 * freshly allocated blocks.  Ids must be distinct (unchecked); an id outside
 * [0, num_pool_blocks) is skipped; every pool byte outside the listed blocks is
 * left untouched.
 */
int kv_blocks_scatter(const void* staging, void* pool, const int32_t* block_ids,
                      int64_t n_blocks, int64_t block_bytes, int64_t num_pool_blocks,
                      void* stream);

/*
 * dst_pool[dst_ids[i]] = src_pool[src_ids[i]]: migration of a request's KV cache
 * between two instances whose pools live on the same GPU (Section IV-B moves the
 * entire KV cache at the phase transition; an MI355X holds the pools of several
 * instances of a 32B model), in one pass without a staging image: each byte is
 * read once and written once, half the traffic of gather followed by scatter.
 * The two pools may be one and the same only if no block is both read and
 * written (unchecked); dst ids must be distinct.  An entry whose source or
 * destination id is out of range is skipped.
 *
 *   src_pool, dst_pool  device, src_pool_blocks / dst_pool_blocks blocks of
 *                       block_bytes bytes
 *   src_ids, dst_ids    device int32 [n_blocks]
 */
int kv_blocks_move(const void* src_pool, const int32_t* src_ids, void* dst_pool,
                   const int32_t* dst_ids, int64_t n_blocks, int64_t block_bytes,
                   int64_t src_pool_blocks, int64_t dst_pool_blocks, void* stream);

/*
 * Eviction of a preempted request to the backing store: the listed blocks are
 * gathered into `staging` and that image is copied to page-locked host memory,
 * both on `stream` (paper Section II-B: a preempted request's KV cache is
 * offloaded to CPU memory, which serves only as backing storage, Section VII).
 * After the stream reaches this point host_dst[i] is the byte image of
 * pool[block_ids[i]] and the blocks may be handed to other requests.
 *
 *   pool, block_ids, staging, sizes   as for kv_blocks_gather (all device)
 *   host_dst   host, pinned (hipHostMalloc or an equivalent allocator),
 *              n_blocks * block_bytes bytes; PKV_ERR_HOST if it is anything else
 * The device part runs at HBM speed; the host copy is bound by the PCIe link
 * and is carried out by the copy engines, so decode attention on another stream
 * keeps the compute units meanwhile.
 */
int kv_blocks_offload(const void* pool, const int32_t* block_ids, void* staging, void* host_dst,
                      int64_t n_blocks, int64_t block_bytes, int64_t num_pool_blocks,
                      void* stream);

/*
 * Resumption of a preempted request: the image saved by kv_blocks_offload is
 * copied back into `staging` and scattered into freshly allocated blocks
 * (Section II-B: the request resumes once memory is available, reloading its KV
 * cache to the GPU).  Arguments as for kv_blocks_scatter plus the pinned host
 * source; ids must be distinct.
 */
int kv_blocks_reload(const void* host_src, void* staging, void* pool, const int32_t* block_ids,
                     int64_t n_blocks, int64_t block_bytes, int64_t num_pool_blocks,
                     void* stream);

/*
 * Writes the newly generated token's K and V rows into their slots: the step
 * that precedes attention in every decode iteration ("incrementally updating
 * [the KV caches] with each newly generated token", paper Section II-A).
 * context_lens[s] already counts the new token, so its row goes to position
 * t = context_lens[s] - 1:
 *
 *   k_pool[ block_tables[s][t / B] ][kvh][t % B][:] = k_new[s][kvh][:]   (V alike)
 *
 * for every request with context_lens[s] >= 1 (after clamping to
 * max_context_len) and every KV head.  A request with context_lens[s] <= 0, or
 * whose table entry lies outside [0, num_pool_blocks), is skipped.  Nothing else
 * in the pools is written; the copy is bit-exact.
 *
 *   k_new, v_new  device  bf16 [S][Hkv][D]
 *   k_pool,v_pool device  bf16 [NB][Hkv][B][D]
 *   block_tables  device  int32 [S][MAXB]
 *   context_lens  device  int32 [S]
 *   shape         host    (num_q_heads and partition_size are not used)
 */
int kv_append(const void* k_new, const void* v_new, void* k_pool, void* v_pool,
              const int32_t* block_tables, const int32_t* context_lens,
              const pkv_attn_shape* shape, void* stream);

/*
 * kv_append for E4M3 pools (see paged_decode_attn_fp8kv): the new rows arrive in
 * bf16 and are stored as
 *     byte = e4m3( x / pool_scale )
 * with the division in fp32, round to nearest even, and magnitudes beyond the
 * format's largest value saturating to +-448 (E4M3 has no infinity).  Everything
 * else as for kv_append.
 *
 *   k_new, v_new  device  bf16 [S][Hkv][D]
 *   k_pool,v_pool device  e4m3 [NB][Hkv][B][D]
 *   k_scale, v_scale  positive finite fp32 (PKV_ERR_SHAPE otherwise)
 */
int kv_append_fp8(const void* k_new, const void* v_new, void* k_pool, void* v_pool,
                  const int32_t* block_tables, const int32_t* context_lens, float k_scale,
                  float v_scale, const pkv_attn_shape* shape, void* stream);

/*
 * Optional report of block ids the kernels refused to follow.  No kernel of this
 * library ever dereferences a block id outside its pool: attention leaves the
 * tokens of such a block out, the copies and kv_append skip the entry.  That
 * keeps a corrupt table from becoming a memory fault, but it also means a request
 * can silently lose part of its KV cache (the whole-cache transfer of Section
 * IV-B is then no longer exact).  After this call, every call made by the calling
 * thread adds to *device_counter, on the device and in stream order, the number of
 * refused entries it met: one per skipped list entry of a copy or move, one per
 * skipped request of kv_append, one per refused 16-token unit and KV head in
 * attention (so any non-zero value means "a block id was out of range").
 *
 *   device_counter  device int32, 4-byte aligned, owned, zeroed and read by the
 *                   caller; it must stay valid while calls of this thread may
 *                   still run.  NULL (the initial state) switches the report off.
 * Returns PKV_OK, or PKV_ERR_ALIGN.  Allocates nothing, launches nothing.
 */
int pkv_set_id_fault_counter(int32_t* device_counter);

/*
 * Measurement aid (no part of the paper's method): streams total_blocks pairs of
 * 4 KiB slabs -- the K and the V rows of 16 tokens of one KV head at D = 128 in
 * bf16 -- out of two buffers with exactly the launch shape and load instructions
 * of paged_decode_attn's stream pass, at slab numbers drawn by a hash that visits
 * every slab once before it repeats one (so total_blocks <= num_slabs reads
 * nothing twice and no cache can help), and does nothing with the data.  Timed by the caller (events on `stream`), it gives the
 * rate the machine allows for that access pattern: 8192 * total_blocks bytes per
 * call.  bench.py reports it next to the attention rate.
 *
 *   k_buf, v_buf  device, 16-byte aligned, at least num_slabs * 4096 bytes each
 *                 (a layer's K and V pool will do: NB * Hkv * B/16 slabs)
 *   num_slabs     >= 1 (at most 2^30 are used)
 *   total_blocks  0 .. 2^31-1; 0 is a no-op
 *   sink          device, 4 bytes, or NULL; never written in practice (it keeps the
 *                 compiler from dropping the loads)
 */
int pkv_probe_stream_read(const void* k_buf, const void* v_buf, int64_t num_slabs,
                          int64_t total_blocks, void* sink, void* stream);

/* Static text for a status code. */
const char* pkv_status_string(int status);

/* Text of the HIP error behind the calling thread's most recent PKV_ERR_LAUNCH. */
const char* pkv_last_launch_error(void);

/* ABI version: major * 1000 + minor. */
int pkv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PKV_H_ */
