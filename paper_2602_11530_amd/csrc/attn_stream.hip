// Paged decode attention, stream pass, for gfx950 (wave64, MFMA).
//
// Decode attends over every running request's whole KV cache and is bound by
// memory bandwidth (paper Section II-A), and the batch mixes short answering
// contexts with long reasoning ones (Section III), so equal work per wavefront
// cannot come from a per-request grid.  Instead the batch's KV blocks form one
// stream (layout in pkv_kernels.h) that is cut into kStreamWaves equal shares:
// every wavefront reads the same number of blocks (+-1), starts streaming at
// once, never idles between requests, and there is no tail of late workgroups.
// A wavefront computes one partial result per run (a stretch of its share inside
// one request, one KV head and one P-token partition), folds the runs of one
// (request, KV head) into a single record while that record is still parked in
// LDS, and writes one record per (wavefront, request, KV head); the merge pass
// combines the records of each (request, query head).
//
// Per 16-token block, lane = 16*c + n, head_dim D = 128 (64 and 256 below):
//   S^T = K . Q^T   D/32 v_mfma_f32_16x16x32_bf16 (k = 32 dims each).
//         A = K rows: lane (n, c) loads the 16 bytes at dims 32*jj + 8*c of
//         token tau(n) = 4*(n%4) + n/4, straight from the pool (a 64-byte run
//         per token per load).  B = q: lane (n, c) holds the same dims of head n
//         (the GQA group padded to 16 rows).  The result leaves lane (n, c)
//         with head n's scores for tokens 4*i + c.
//   P     = exp2(score - m) in fp32, split into bf16 hi + lo parts so that the
//         weights keep ~16 mantissa bits through the second product.
//   O    += P . V   D/16 v_mfma_f32_16x16x16_bf16 per part.  V is loaded in its
//         natural order (lane (n, c) gets dims 8n..8n+7 of tokens 4*e + c, four
//         fully contiguous 1 KiB loads); the operand for output dims 8*n + i
//         pairs up the i-th halves of those four loads with v_perm_b32.  The
//         token order 4*e + c is exactly the one the scores came out in, so P
//         needs no shuffle between the two products.
//   D = 64:  lane (n, c) owns dims 4n..4n+3; its V loads are 8 bytes wide (four
//         fully contiguous 512-byte loads), two K steps, four output tiles.
//   D = 256: lane (n, c) owns dims 8n..8n+7 of each 128-dim half; eight K steps,
//         eight 16-byte V loads (a 256-byte run per token per load), sixteen
//         output tiles; a block is 16 KiB here and a wavefront needs more than half
//         of a SIMD's registers, so one wavefront per SIMD streams (half as many).
// The running maximum m is only raised when a score exceeds it by more than
// 2^kLazyLog2; any reference value gives the same softmax, and the bound keeps
// every weight within fp32/bf16 range.
//
// Where a block lives (physical id, KV head), how many of its tokens are valid
// and whether it closes a run is worked out 64 blocks at a time, one block per
// lane ("descriptors"), one window ahead of use; the streaming loop itself only
// reads a lane of those registers per block, so no memory access sits on the
// address path of the KV loads.
//
// Memory traffic.  The KV loads of a block (eight of 16 bytes at D = 128) are
// nontemporal and unconditional; a ring of kRing register buffers keeps
// kRing - 1 blocks (one) in flight per wavefront.  Finished records are parked in LDS and written in
// bursts of full-width write-through stores that the compiler's wait-count
// bookkeeping does not see (see store_record16).
#include "pkv_kernels.h"

namespace pkv {
namespace {

constexpr int kWindow = 64;       // descriptors per window: one per lane

// Register buffers per wavefront: the block being consumed and the block in
// flight behind it.  With 2048 wavefronts (1024 at D = 256) that is 16 MB on its
// way at any time, which keeps the memory system saturated; deeper rings (4 and
// 8 were measured, at every head dimension and pool format) only lengthen the
// queues: 0.5 % slower on the Qwen-32B-shaped batches, 2 to 5 % on the variants
// whose blocks are half the bytes, 5 to 20 % on batches of a few requests.
constexpr int kRing = 2;

// What depends on the head dimension and the pool format.
template <int kD, bool kFp8> struct Dim;
template <> struct Dim<64, false> {
  static constexpr int kKSteps = 2, kKLoads = 2, kVLoads = 4, kTiles = 4, kElemBytes = 2;
  typedef uint32_t VReg __attribute__((ext_vector_type(2)));
};
template <> struct Dim<128, false> {
  static constexpr int kKSteps = 4, kKLoads = 4, kVLoads = 4, kTiles = 8, kElemBytes = 2;
  typedef uint32_t VReg __attribute__((ext_vector_type(4)));
};
template <> struct Dim<256, false> {
  static constexpr int kKSteps = 8, kKLoads = 8, kVLoads = 8, kTiles = 16, kElemBytes = 2;
  typedef uint32_t VReg __attribute__((ext_vector_type(4)));
};
// K and V stored as one-byte e4m3 values: the values are widened to bf16 (exactly) in
// registers and then take the same path as a bf16 pool.  A K load is 16 bytes = 16 dims of one token and feeds two MFMA steps; a V load is
// the lane's dims of one token (4 bytes at D = 64, 8 bytes otherwise).
template <> struct Dim<64, true> {
  static constexpr int kKSteps = 2, kKLoads = 1, kVLoads = 4, kTiles = 4, kElemBytes = 1;
  typedef uint32_t VReg;
};
template <> struct Dim<128, true> {
  static constexpr int kKSteps = 4, kKLoads = 2, kVLoads = 4, kTiles = 8, kElemBytes = 1;
  typedef uint32_t VReg __attribute__((ext_vector_type(2)));
};
template <> struct Dim<256, true> {
  static constexpr int kKSteps = 8, kKLoads = 4, kVLoads = 8, kTiles = 16, kElemBytes = 1;
  typedef uint32_t VReg __attribute__((ext_vector_type(2)));
};
// First dim of output tiles 4t..4t+3 (they are consecutive dims) in the lane of column n.
template <int kD> __device__ __forceinline__ int tile_group_dim(int t, int n) {
  if (kD == 64) return 4 * n;
  if (kD == 128) return 8 * n + 4 * t;
  return 128 * (t >> 1) + 8 * n + 4 * (t & 1);
}
constexpr float kNegInf = -__builtin_huge_valf();
constexpr float kLazyLog2 = 8.f;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Two fp32 -> packed bf16, round to nearest even (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  const f32x2 f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}
// The same rounding, then the fp32 value of what was kept.
__device__ __forceinline__ float bf16_round(float x, uint32_t& bits) {
  bits = pack_bf16(x, 0.f) & 0xffffu;
  return __uint_as_float(bits << 16);
}

// Four e4m3 bytes of one dword -> four bf16 (exact: every e4m3 value is a bf16 value).
__device__ __forceinline__ u32x2 widen_e4m3x4(uint32_t w) {
  const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false);
  const f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
  return u32x2{pack_bf16(lo.x, lo.y), pack_bf16(hi.x, hi.y)};
}

// Stores of a finished run's record.  They are written as opaque instructions on
// purpose: gfx9-family hardware counts loads and stores in one counter, and once
// the compiler knows a store is pending it can no longer wait for "all but the N
// youngest loads" and drains the whole ring of KV loads at the next use.  Hidden
// from that bookkeeping, a wait sized for the loads alone is still sufficient
// (loads retire in order among themselves, so extra pending stores only make the
// same wait stricter), and the record itself is only read by the next kernel.
// sc1 makes the store write through instead of leaving a dirty line behind for a
// later eviction (measured while records were still written once per partition:
// 512-token partitions then cost 8 % instead of 13 % on the long-context batch).
__device__ __forceinline__ void store_record16(float* p, f32x4 v) {
  // the trailing s_nop covers the wait states a wide store needs before a vector
  // op may overwrite its data registers (the compiler cannot see that this is a store)
  asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
}

// One window of block descriptors: lane i describes stream index jbase + i.
struct Window {
  int slab;   // which slab (16 tokens of one KV head; 4 KiB at D = 128 in bf16), counted from the pool's start; 0 when not read
  int meta;   // bits 0-7 valid tokens (0..16), bit 8 closes a run, bit 9 first block of a segment here
  int qrow;   // s * Hq + kvh * G: first query/output row of the segment
  int slot;   // partial-record slot of the run this block belongs to
};
constexpr int kMetaLast = 1 << 8;
constexpr int kMetaSegFirst = 1 << 9;

template <int kD, bool kFp8>
__global__ __launch_bounds__(kStreamWavesPerGroup * 64) void attn_stream_kernel(AttnLaunch a) {
  typedef Dim<kD, kFp8> DD;
  typedef typename DD::VReg VReg;                 // one V load as it arrives
  typedef typename Dim<kD, false>::VReg VOp;      // the same rows as bf16
  constexpr int kKSteps = DD::kKSteps, kKLoads = DD::kKLoads, kVLoads = DD::kVLoads,
                kTiles = DD::kTiles, kElemBytes = DD::kElemBytes;
  static_assert(kWindow % kRing == 0, "the window must be a whole number of ring turns");
  extern __shared__ int smem[];
  int* cumB = smem;                  // [S+1] blocks before request s
  int* lens = smem + (a.S + 1);      // [S]   clamped context lengths
  // then room for rec_buffered finished records per wavefront, 16-byte aligned
  const int rec_floats = record_floats(a.G, kD);
  float* rec_stage = (float*)(smem + ((2 * (a.S + 1) + 3) & ~3)) +
                     (threadIdx.x >> 6) * a.rec_buffered * rec_floats;

  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int n = lane & 15, c = lane >> 4;
  const int G = a.G, S = a.S, Hkv = a.Hkv;
  const int bpp = a.P / kBlockTokens;   // blocks per partition

  // Prefix sums over the requests (wavefront 0 of every workgroup; S is small).
  if (wave == 0) {
    int runB = 0;
    for (int base = 0; base < S; base += 64) {
      const int i = base + lane;
      const int L = (i < S) ? min(max(a.context_lens[i], 0), a.max_ctx) : 0;
      const int nb = (L + kBlockTokens - 1) / kBlockTokens;
      int xb = nb;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int yb = __shfl_up(xb, o);
        if (lane >= o) xb += yb;
      }
      if (i < S) { lens[i] = L; cumB[i] = runB + xb - nb; }
      runB += __shfl(xb, 63);
    }
    if (lane == 0) cumB[S] = runB;
  }
  __syncthreads();
  if (blockIdx.x == 0) {   // the merge pass reads the same prefix array
    for (int i = threadIdx.x; i < S + 1; i += blockDim.x) a.ws_cum[i] = smem[i];
  }

  // Every participating wavefront gets at least one block, so that consecutive
  // runs of a segment always belong to the same or to adjacent wavefronts.
  const int64_t T = (int64_t)Hkv * cumB[S];
  const int W = (int)min((int64_t)a.waves, T);
  const int w = blockIdx.x * kStreamWavesPerGroup + wave;
  if (w >= W) return;
  const int pos0 = (int)share_start(w, T, W);
  const int nshare = (int)share_start(w + 1, T, W) - pos0;

  // Descriptors of stream indices jb .. jb+63 of this share.
  int search_steps = 0;
  while ((1 << search_steps) < S) ++search_steps;
  int refused = 0;   // table entries outside the pool met while describing this share
  auto describe = [&](int jb) -> Window {
    const int j = jb + lane;
    const bool live = j < nshare;
    const int pos = pos0 + min(j, nshare - 1);
    int lo = 0, hi = S;   // largest s with Hkv * cumB[s] <= pos
    for (int it = 0; it < search_steps; ++it) {
      const int mid = (lo + hi) >> 1;
      if (mid > lo && Hkv * cumB[mid] <= pos) lo = mid; else if (mid > lo) hi = mid;
    }
    const int s = lo;
    const int nb = cumB[s + 1] - cumB[s];
    const int o = pos - Hkv * cumB[s];
    const int kvh = o / nb;
    const int b = o - kvh * nb;
    int ntok = min(kBlockTokens, lens[s] - kBlockTokens * b);
    // unit b of the request lies in physical block b / upb, at unit b % upb of the KV head's rows
    const int tb = b / a.upb;
    const int id = live ? a.block_tables[(int64_t)s * a.MAXB + tb] : -1;
    const bool mapped = (unsigned)id < (unsigned)a.NB;   // ids outside the pool are never followed
    if (!mapped) ntok = 0;
    refused += __popcll(__ballot(live && !mapped));
    Window d;
    d.slab = mapped ? (id * Hkv + kvh) * a.upb + (b - tb * a.upb) : 0;
    const bool last = (b + 1 == nb) || ((b + 1) % bpp == 0) || (j + 1 == nshare);
    const bool seg_first = (b == 0) || (j == 0);
    d.meta = ntok | (last ? kMetaLast : 0) | (seg_first ? kMetaSegFirst : 0);
    d.qrow = s * a.Hq + kvh * G;
    d.slot = s * Hkv + kvh + w;
    return d;
  };

  Window dA = describe(0);
  Window dB = dA;   // described after the first KV loads are on their way (below)
  int jbase = 0;

  const int64_t slab_bytes = (int64_t)kBlockTokens * kD * kElemBytes;  // one (block, KV head) slab
  const int tau = 4 * (n & 3) + (n >> 2);
  const int koff = tau * (kD * kElemBytes / 16) + c;   // in 16-byte units within the slab
  // V, in units of one VReg: token 4*e + c, this lane's dims (of half h when D = 256)
  const int voff = kD == 256 ? 32 * c + n : lane;

  u32x4 qop[kKSteps];  // q as the B operand: dims 32*jj + 8*c .. +7 of head n; zero rows beyond the group
  float m = kNegInf;   // running reference maximum of head n (log2 units), same in all four c groups
  float l = 0.f;       // this lane's share of the softmax denominator
  f32x4 o[kTiles];     // o[i][r]: head 4*c + r, dim tile_group_dim(i / 4, n) + i % 4
#pragma unroll
  for (int i = 0; i < kTiles; ++i) o[i] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Issue the loads of stream index j (K in operand order, V
  // natural), nontemporal: the stream is read once and must not allocate in the
  // caches it passes through.  The loads are unconditional so that every wait in the loop knows
  // exactly how many are outstanding: a block that is unmapped, or an index past
  // the share's end, reads slab 0 (which always exists) and is masked or skipped.
  auto issue = [&](u32x4 (&k)[kKLoads], VReg (&v)[kVLoads], int j) {
    const int idx = j - jbase;   // 0 .. 2*kWindow-1
    const int sa = __builtin_amdgcn_readlane(dA.slab, idx & (kWindow - 1));
    const int sb = __builtin_amdgcn_readlane(dB.slab, idx & (kWindow - 1));
    int slab = (idx < kWindow) ? sa : sb;
    if (j >= nshare) slab = 0;
    const int64_t base = (int64_t)slab * slab_bytes;
    const u32x4* kp = (const u32x4*)((const char*)a.k_pool + base) + koff;
    const VReg* vp = (const VReg*)((const char*)a.v_pool + base) + voff;
#pragma unroll
    for (int jj = 0; jj < kKLoads; ++jj) k[jj] = __builtin_nontemporal_load(kp + 4 * jj);
    if (kD == 256) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[2 * e] = __builtin_nontemporal_load(vp + 128 * e);
        v[2 * e + 1] = __builtin_nontemporal_load(vp + 128 * e + 16);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = __builtin_nontemporal_load(vp + 64 * e);
    }
  };

  // Finished records wait in LDS and go out several at a time, with full-width
  // stores, and the rest when the share is done.  A store in the middle of the
  // stream is expensive out of proportion to its size: loads and stores retire
  // through one counter, so the KV loads issued after it cannot be consumed
  // before it has been acknowledged, and that costs one stall of several
  // microseconds per burst of stores however few bytes it carries.
  int nrec = 0;        // records parked in LDS
  int rec_slots = 0;   // lane r: slot of parked record r
  bool seg_open = false;   // the newest parked record belongs to the segment being streamed
  auto drain_records = [&]() {
    for (int r = 0; r < nrec; ++r) {
      const int slot = __builtin_amdgcn_readlane(rec_slots, r);
      float* dst = a.ws_rec + (int64_t)slot * rec_floats;
      const float* src = rec_stage + r * rec_floats;
      for (int f = 4 * lane; f < rec_floats; f += 256) store_record16(dst + f, *(const f32x4*)(src + f));
    }
    nrec = 0;
  };

  auto consume = [&](u32x4 (&kraw)[kKLoads], VReg (&vraw)[kVLoads], int j) {
    const int idx = j - jbase;   // always inside window A
    // The MFMA operands.  bf16 pools: the loaded registers themselves.  e4m3 pools: load L of
    // K holds dims 16*(4L + c) .. +15 of token tau(n), which feed steps 2L and 2L + 1 (the
    // contraction order is free as long as q follows it, see below); a V load holds the same
    // token and dims as in a bf16 pool, one byte each.
    u32x4 k[kKSteps];
    VOp v[kVLoads];
    if constexpr (kFp8) {
#pragma unroll
      for (int jj = 0; jj < kKSteps; ++jj) {
        const u32x2 a2 = widen_e4m3x4(kraw[jj >> 1][2 * (jj & 1)]);
        const u32x2 b2 = widen_e4m3x4(kraw[jj >> 1][2 * (jj & 1) + 1]);
        k[jj] = u32x4{a2.x, a2.y, b2.x, b2.y};
      }
#pragma unroll
      for (int e = 0; e < kVLoads; ++e) {
        if constexpr (kD == 64) {
          v[e] = widen_e4m3x4(vraw[e]);
        } else {
          const u32x2 a2 = widen_e4m3x4(vraw[e].x), b2 = widen_e4m3x4(vraw[e].y);
          v[e] = VOp{a2.x, a2.y, b2.x, b2.y};
        }
      }
    } else {
#pragma unroll
      for (int jj = 0; jj < kKSteps; ++jj) k[jj] = kraw[jj];
#pragma unroll
      for (int e = 0; e < kVLoads; ++e) v[e] = vraw[e];
    }
    const int meta = __builtin_amdgcn_readlane(dA.meta, idx);
    const int ntok = meta & 0xff;

    if (meta & kMetaSegFirst) {
      // A new (request, KV head): fetch its query group.
      seg_open = false;
      const int qrow = __builtin_amdgcn_readlane(dA.qrow, idx);
      const u32x4* qrow_p = (const u32x4*)(a.q + (int64_t)(qrow + min(n, G - 1)) * kD);
#pragma unroll
      for (int jj = 0; jj < kKSteps; ++jj) {
        // dims of step jj in this lane: 32*jj + 8*c .. +7, or, following the byte order of an
        // e4m3 K load, 64*(jj/2) + 16*c + 8*(jj%2) .. +7
        const u32x4 wq = kFp8 ? qrow_p[8 * (jj >> 1) + 2 * c + (jj & 1)] : qrow_p[4 * jj + c];
        qop[jj] = (n < G) ? wq : u32x4{0, 0, 0, 0};
      }
    }

    f32x4 sc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int jj = 0; jj < kKSteps; ++jj)
      sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k[jj]),
                                                   __builtin_bit_cast(bf16x8, qop[jj]), sc, 0, 0, 0);
    float x[4] = {sc.x * a.scale_log2e, sc.y * a.scale_log2e, sc.z * a.scale_log2e,
                  sc.w * a.scale_log2e};
    const bool edge = ntok < kBlockTokens;
    bool valid[4] = {true, true, true, true};
    if (edge) {
      // Last block of a request, or an unmapped one: masked slots may hold anything
      // (NaN included), so scores, weights and V rows are replaced by select,
      // never scaled by zero.  Element e of this lane is token 4*e + c.
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        valid[e] = 4 * e + c < ntok;
        x[e] = valid[e] ? x[e] : kNegInf;
        if (!valid[e]) {
          if (kD == 256) { v[2 * e] = VOp{}; v[2 * e + 1] = VOp{}; }
          else v[e] = VOp{};
        }
      }
    }
    const float mx = fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
    if (__any(mx > m + kLazyLog2)) {
      float mg = fmaxf(mx, __shfl_xor(mx, 16));
      mg = fmaxf(mg, __shfl_xor(mg, 32));
      const float mnew = fmaxf(m, mg);   // finite: some lane of the head saw a valid token
      const float alpha = __builtin_amdgcn_exp2f(m - mnew);
      l *= alpha;
      float ar[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) ar[r] = __shfl(alpha, 4 * c + r);
#pragma unroll
      for (int i = 0; i < kTiles; ++i) {
        o[i].x *= ar[0]; o[i].y *= ar[1]; o[i].z *= ar[2]; o[i].w *= ar[3];
      }
      m = mnew;
    }
    float pw[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) pw[e] = __builtin_amdgcn_exp2f(x[e] - m);
    if (edge) {
#pragma unroll
      for (int e = 0; e < 4; ++e) pw[e] = valid[e] ? pw[e] : 0.f;   // m may still be -inf here
    }
    l += (pw[0] + pw[1]) + (pw[2] + pw[3]);

    // P = hi + lo in bf16.
    uint32_t hb[4];
    float lo[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) lo[e] = pw[e] - bf16_round(pw[e], hb[e]);
    const u32x2 phi = {hb[0] | (hb[1] << 16), hb[2] | (hb[3] << 16)};
    const u32x2 plo = {pack_bf16(lo[0], lo[1]), pack_bf16(lo[2], lo[3])};
    const s16x4 pa = __builtin_bit_cast(s16x4, phi);
    const s16x4 pb = __builtin_bit_cast(s16x4, plo);
#pragma unroll
    for (int i = 0; i < kTiles; ++i) {
      // tile i needs, for tokens 4*e + c (e = 0..3), the bf16 of its dim: half (i & 1) of
      // word ((i % 8) >> 1) of the load that holds token e (and, for D = 256, half i / 8)
      const int wsel = (i & 7) >> 1, h = kD == 256 ? i >> 3 : 0, st = kD == 256 ? 2 : 1;
      const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
      const u32x2 vb = {__builtin_amdgcn_perm(v[st + h][wsel], v[h][wsel], sel),
                        __builtin_amdgcn_perm(v[3 * st + h][wsel], v[2 * st + h][wsel], sel)};
      const s16x4 vop = __builtin_bit_cast(s16x4, vb);
      o[i] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pa, vop, o[i], 0, 0, 0);
      o[i] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pb, vop, o[i], 0, 0, 0);
    }

    if (meta & kMetaLast) {
      // The run ends here.  The first run of a (request, KV head) in this share
      // parks its partial result in LDS as a new record, assembled in its memory
      // order; every later run of the same segment (the next P-token partitions)
      // is folded into that parked record with the split-K merge formula, so
      // memory sees one record per (wavefront, segment) however small P is.
      float lt = l + __shfl_xor(l, 16);
      lt += __shfl_xor(lt, 32);
      if (!seg_open) {
        if (nrec == a.rec_buffered) drain_records();
        const int slot = __builtin_amdgcn_readlane(dA.slot, idx);
        rec_slots = (lane == nrec) ? slot : rec_slots;
        ++nrec;
      }
      float* rec = rec_stage + (nrec - 1) * rec_floats;
      float keep[4] = {0.f, 0.f, 0.f, 0.f}, add[4] = {1.f, 1.f, 1.f, 1.f};
      if (seg_open) {
        // parked (m1, l1, rows1) and this run's (m, lt, o): weights 2^(m1-M) and 2^(m-M),
        // a side whose maximum is -inf (nothing valid seen) gets weight 0 by select
        const f32x2 ml = *(const f32x2*)(rec + G * kD + 2 * n);
        const float M = fmaxf(ml.x, m);
        const float w1 = (ml.x == kNegInf) ? 0.f : __builtin_amdgcn_exp2f(ml.x - M);
        const float w2 = (m == kNegInf) ? 0.f : __builtin_amdgcn_exp2f(m - M);
        lt = w1 * ml.y + w2 * lt;
        m = M;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          keep[r] = __shfl(w1, 4 * c + r);
          add[r] = __shfl(w2, 4 * c + r);
        }
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int h = 4 * c + r;
        if (h < G) {
#pragma unroll
          for (int t = 0; t < kTiles / 4; ++t) {
            f32x4* dst = (f32x4*)(rec + h * kD + tile_group_dim<kD>(t, n));
            f32x4 x4 = {o[4 * t][r], o[4 * t + 1][r], o[4 * t + 2][r], o[4 * t + 3][r]};
            if (seg_open) {
              const f32x4 p4 = *dst;
#pragma unroll
              for (int e = 0; e < 4; ++e) x4[e] = keep[r] * p4[e] + add[r] * x4[e];
            }
            *dst = x4;
          }
        }
      }
      if (c == 0) *(f32x2*)(rec + G * kD + 2 * n) = (n < G) ? f32x2{m, lt} : f32x2{kNegInf, 0.f};
      seg_open = true;
      m = kNegInf;
      l = 0.f;
#pragma unroll
      for (int i = 0; i < kTiles; ++i) o[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
  };

  // A ring of kRing register buffers: kRing - 1 blocks are always in flight
  // while one is consumed, and no buffer is ever copied.
  u32x4 kbuf[kRing][kKLoads];
  VReg vbuf[kRing][kVLoads];
#pragma unroll
  for (int i = 0; i < kRing - 1; ++i) issue(kbuf[i], vbuf[i], i);
  dB = describe(kWindow);
  for (int j = 0; j < nshare; j += kRing) {
#pragma unroll
    for (int i = 0; i < kRing; ++i) {
      constexpr int kAhead = kRing - 1;
      issue(kbuf[(i + kAhead) % kRing], vbuf[(i + kAhead) % kRing], j + i + kAhead);
      if (j + i < nshare) consume(kbuf[i], vbuf[i], j + i);
    }
    if (j + kRing == jbase + kWindow) {
      // The consumer leaves window A: B becomes A, and the window after it is
      // described now, 64 blocks before its first use.
      dA = dB;
      jbase += kWindow;
      dB = describe(jbase + kWindow);
    }
  }
  drain_records();
  // Refused ids are reported once per wavefront, after the stream: nothing in the loop waits on it.
  if (a.id_faults && refused && lane == 0) atomicAdd(a.id_faults, refused);
}

}  // namespace

hipError_t launch_attn_stream(const AttnLaunch& a_in, hipStream_t stream) {
  AttnLaunch a = a_in;
  // LDS per workgroup: the prefix arrays, then as many parked records per
  // wavefront as fit in 64 KiB (at most 8).
  const size_t cum_bytes = (size_t)((2 * (a.S + 1) + 3) & ~3) * sizeof(int);
  const size_t rec_bytes = (size_t)record_floats(a.G, a.D) * sizeof(float);
  const size_t room = (size_t)64 * 1024 - cum_bytes;
  a.rec_buffered = (int)(room / (kStreamWavesPerGroup * rec_bytes));
  if (a.rec_buffered > 8) a.rec_buffered = 8;
  if (a.rec_buffered < 1) return hipErrorInvalidValue;
  const size_t lds = cum_bytes + (size_t)kStreamWavesPerGroup * a.rec_buffered * rec_bytes;
  const dim3 grid(a.waves / kStreamWavesPerGroup), block(kStreamWavesPerGroup * 64);
  if (a.kv_fp8) {
    if (a.D == 64) hipLaunchKernelGGL((attn_stream_kernel<64, true>), grid, block, lds, stream, a);
    else if (a.D == 128) hipLaunchKernelGGL((attn_stream_kernel<128, true>), grid, block, lds, stream, a);
    else if (a.D == 256) hipLaunchKernelGGL((attn_stream_kernel<256, true>), grid, block, lds, stream, a);
    else return hipErrorInvalidValue;
  } else if (a.D == 64) hipLaunchKernelGGL((attn_stream_kernel<64, false>), grid, block, lds, stream, a);
  else if (a.D == 128) hipLaunchKernelGGL((attn_stream_kernel<128, false>), grid, block, lds, stream, a);
  else if (a.D == 256) hipLaunchKernelGGL((attn_stream_kernel<256, false>), grid, block, lds, stream, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace pkv
