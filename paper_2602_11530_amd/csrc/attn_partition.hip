// Paged decode attention, partition pass, for gfx950 (wave64, MFMA).
//
// One wavefront owns one (request, KV head, context partition) and streams that
// partition's K and V rows exactly once; the G query heads of the GQA group
// share every byte read (decode attends over the request's whole KV cache and
// is bound by memory bandwidth, paper Section II-A).  Both products run on the
// matrix cores with the group padded to 16 rows, which leaves the vector ALU
// with the softmax of 4 scores per lane per block and keeps the wave's time in
// its loads.
//
// Per 16-token block, lane = 16*c + n:
//   S^T = K . Q^T   four v_mfma_f32_16x16x32_bf16 (k = 32 dims each).
//         A = K rows: lane (n, c) loads the 16 bytes at dims 32*jj + 8*c of
//         token tau(n) = 4*(n%4) + n/4, straight from the pool (a 64-byte run
//         per token per load).  B = q: lane (n, c) holds the same dims of head n.
//         The result leaves lane (n, c) with head n's scores for tokens 4*i + c.
//   P     = exp2(score - m) in fp32, split into bf16 hi + lo parts so that the
//         weights keep ~16 mantissa bits through the second product.
//   O    += P . V   eight v_mfma_f32_16x16x16_bf16 per part.  V is loaded in its
//         natural order (lane (n, c) gets dims 8n..8n+7 of tokens 4*e + c, four
//         fully contiguous 1 KiB loads); the operand for output dims 8*n + i
//         pairs up the i-th halves of those four loads with v_perm_b32.  The
//         token order 4*e + c is exactly the one the scores came out in, so P
//         needs no shuffle between the two products.
// The running maximum m is only raised when a score exceeds it by more than
// 2^kLazyLog2; any reference value gives the same softmax, and the bound keeps
// every weight within fp32/bf16 range.
#include "pkv_kernels.h"

namespace pkv {
namespace {

#ifndef PKV_WAVES_PER_GROUP
#define PKV_WAVES_PER_GROUP 4
#endif
#ifndef PKV_MIN_WAVES_PER_EU
#define PKV_MIN_WAVES_PER_EU 1
#endif
constexpr int kWavesPerGroup = PKV_WAVES_PER_GROUP;
constexpr float kNegInf = -__builtin_huge_valf();
constexpr float kLazyLog2 = 8.f;
#ifndef PKV_RING
#define PKV_RING 4
#endif
constexpr int kRing = PKV_RING;   // 16-token blocks in flight per wavefront (register ring)

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

__global__ __launch_bounds__(kWavesPerGroup * 64)
__attribute__((amdgpu_waves_per_eu(PKV_MIN_WAVES_PER_EU))) void attn_partition_kernel(AttnLaunch a) {
  const int s = blockIdx.x / a.NP;
  const int p = blockIdx.x - s * a.NP;
  const int L = min(max(a.context_lens[s], 0), a.max_ctx);
  const int t0 = p * a.P;
  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int kvh = blockIdx.y * kWavesPerGroup + wave;
  const int n = lane & 15, c = lane >> 4;
  const int G = a.G;

  if (t0 >= L) {
    // Nothing to attend.  An empty request still owes a zero row when this
    // pass writes the output itself.
    if (L <= 0 && p == 0 && a.NP == 1 && kvh < a.Hkv && c == 0) {
      for (int h = 0; h < G; ++h)
        *(u32x4*)(a.out + ((int64_t)s * a.Hq + kvh * G + h) * kHeadDim + 8 * n) = u32x4{0, 0, 0, 0};
    }
    return;
  }
  const int t1 = min(L, t0 + a.P);
  const int nblk = (t1 - t0 + kBlockTokens - 1) / kBlockTokens;

  // This partition's physical block ids: lane i keeps entry i (a partition is at
  // most 64 blocks), read with one coalesced load; v_readlane hands block b's id
  // to the scalar unit with no memory access on the loads' address path.
  // Ids outside the pool become -1 and are never followed.
  int tbl = -1;
  if (lane < nblk) {
    const int id = a.block_tables[(int64_t)s * a.MAXB + t0 / kBlockTokens + lane];
    tbl = ((unsigned)id < (unsigned)a.NB) ? id : -1;
  }
  if (kvh >= a.Hkv) return;

  // q as the B operand of the score product: lane (n, c) holds dims
  // 32*jj + 8*c .. +7 of head n; heads beyond the group are zero rows.
  u32x4 qop[4];
  {
    const int hq = kvh * G + min(n, G - 1);
    const u32x4* qp = (const u32x4*)(a.q + ((int64_t)s * a.Hq + hq) * kHeadDim) + c;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const u32x4 w = qp[4 * jj];
      qop[jj] = (n < G) ? w : u32x4{0, 0, 0, 0};
    }
  }

  const int64_t head_elems = (int64_t)kBlockTokens * kHeadDim;  // one (block, KV head) slab
  const int64_t block_elems = (int64_t)a.Hkv * head_elems;
  const int tau = 4 * (n & 3) + (n >> 2);
  const int koff = tau * 16 + c;   // in 16-byte units within the slab

  float m = kNegInf;   // running reference maximum of head n (log2 units), same in all four c groups
  float l = 0.f;       // this lane's share of the softmax denominator
  f32x4 o[8];          // o[i][r]: head 4*c + r, dim 8*n + i
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Issue the eight 16-byte loads of block b (K in operand order, V natural) and
  // return its staged physical id.  The loads are issued unconditionally so that
  // every wait in the loop knows exactly how many are outstanding: an unmapped
  // block (-1) or one past the partition's end reads block 0 of KV head 0, which
  // always exists, and is masked out or skipped when its turn comes.
  auto issue = [&](u32x4 (&k)[4], u32x4 (&v)[4], int b) -> int {
    const bool live = b < nblk;
    const int phys = live ? __builtin_amdgcn_readlane(tbl, min(b, 63)) : -1;
    const int64_t base = (phys >= 0) ? (int64_t)phys * block_elems + (int64_t)kvh * head_elems : 0;
    const u32x4* kp = (const u32x4*)(a.k_pool + base) + koff;
    const u32x4* vp = (const u32x4*)(a.v_pool + base) + lane;
#pragma unroll
    for (int j = 0; j < 4; ++j) k[j] = kp[4 * j];
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = vp[64 * j];
    return phys;
  };

  auto consume = [&](u32x4 (&k)[4], u32x4 (&v)[4], int b, int phys) {
    f32x4 sc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int jj = 0; jj < 4; ++jj)
      sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k[jj]),
                                                   __builtin_bit_cast(bf16x8, qop[jj]), sc, 0, 0, 0);
    float x[4] = {sc.x * a.scale_log2e, sc.y * a.scale_log2e, sc.z * a.scale_log2e,
                  sc.w * a.scale_log2e};
    const bool edge = (b + 1 == nblk) || (phys < 0);
    bool valid[4] = {true, true, true, true};
    if (edge) {
      // Last or unmapped block: masked slots may hold anything (NaN included), so
      // scores, weights and V rows are replaced by select, never scaled by zero.
      const int tb = t0 + b * kBlockTokens + c;   // token of element 0; element e is tb + 4e
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        valid[e] = (tb + 4 * e < t1) && (phys >= 0);
        x[e] = valid[e] ? x[e] : kNegInf;
        if (!valid[e]) v[e] = u32x4{0, 0, 0, 0};
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
      for (int i = 0; i < 8; ++i) {
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
    for (int i = 0; i < 8; ++i) {
      const int wsel = i >> 1;
      const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
      const u32x2 vb = {__builtin_amdgcn_perm(v[1][wsel], v[0][wsel], sel),
                        __builtin_amdgcn_perm(v[3][wsel], v[2][wsel], sel)};
      const s16x4 vop = __builtin_bit_cast(s16x4, vb);
      o[i] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pa, vop, o[i], 0, 0, 0);
      o[i] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pb, vop, o[i], 0, 0, 0);
    }
  };

  // A ring of kRing register buffers: kRing - 1 blocks are always in flight
  // while one is consumed, and no buffer is ever copied.
  u32x4 kbuf[kRing][4], vbuf[kRing][4];
  int phys[kRing];
#pragma unroll
  for (int i = 0; i < kRing - 1; ++i) phys[i] = issue(kbuf[i], vbuf[i], i);
  for (int b = 0; b < nblk; b += kRing) {
#pragma unroll
    for (int i = 0; i < kRing; ++i) {
      constexpr int kAhead = kRing - 1;
      const int slot = (i + kAhead) % kRing;
      phys[slot] = issue(kbuf[slot], vbuf[slot], b + i + kAhead);
      if (b + i < nblk) consume(kbuf[i], vbuf[i], b + i, phys[i]);
    }
  }

  // Denominator of head n: sum the four c groups.
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);

  if (a.NP == 1) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int h = 4 * c + r;
      const float lh = __shfl(l, h);
      if (h < G) {
        const float inv = lh > 0.f ? 1.f / lh : 0.f;   // no mapped token at all: zero row
        u32x4 w;
        w.x = pack_bf16(o[0][r] * inv, o[1][r] * inv);
        w.y = pack_bf16(o[2][r] * inv, o[3][r] * inv);
        w.z = pack_bf16(o[4][r] * inv, o[5][r] * inv);
        w.w = pack_bf16(o[6][r] * inv, o[7][r] * inv);
        *(u32x4*)(a.out + ((int64_t)s * a.Hq + kvh * G + h) * kHeadDim + 8 * n) = w;
      }
    }
  } else {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int h = 4 * c + r;
      if (h < G) {
        const int64_t row = ((int64_t)s * a.NP + p) * a.Hq + kvh * G + h;
        float4* dst = (float4*)(a.ws_acc + row * kHeadDim + 8 * n);
        dst[0] = make_float4(o[0][r], o[1][r], o[2][r], o[3][r]);
        dst[1] = make_float4(o[4][r], o[5][r], o[6][r], o[7][r]);
      }
    }
    if (c == 0 && n < G) {
      const int64_t row = ((int64_t)s * a.NP + p) * a.Hq + kvh * G + n;
      a.ws_ml[row] = make_float2(m, l);
    }
  }
}

}  // namespace

hipError_t launch_attn_partition(const AttnLaunch& a, hipStream_t stream) {
  dim3 grid((unsigned)(a.S * a.NP), (unsigned)((a.Hkv + kWavesPerGroup - 1) / kWavesPerGroup), 1);
  hipLaunchKernelGGL(attn_partition_kernel, grid, dim3(kWavesPerGroup * 64), 0, stream, a);
  return hipGetLastError();
}

}  // namespace pkv
