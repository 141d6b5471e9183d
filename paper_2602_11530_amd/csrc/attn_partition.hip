// Paged decode attention, partition pass, for gfx950 (wave64).
//
// One wavefront owns one (request, KV head, context partition) and streams that
// partition's K and V rows exactly once; the G query heads of the GQA group
// share every byte read (decode attends over the request's whole KV cache and
// is bound by memory bandwidth, paper Section II-A).
//
// Lane map (natural pool layout, a K or V row is 128 bf16 = 16 lanes x 16 B):
//   lane = 16*r + c;  c = 16-byte column chunk (dims 8c..8c+7),  r = token row.
//   One 16-byte load per lane covers 4 consecutive tokens (1 KiB, contiguous);
//   a 16-token block of one KV head is 4 such loads for K and 4 for V.
// Scores: per-lane partial dot over 8 dims, then a 16-lane DPP all-reduce.
// Each token row r keeps its own online-softmax state; the four states are
// merged once at the end of the partition.
#include "pkv_kernels.h"

namespace pkv {
namespace {

constexpr int kWavesPerGroup = 4;
constexpr float kNegInf = -__builtin_huge_valf();

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// Sum over the 16 lanes of a DPP row; every lane of the row gets the total.
__device__ __forceinline__ float row16_allreduce_add(float x) {
  x += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
  x += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
  x += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), 0x141, 0xF, 0xF, true));  // row_half_mirror
  x += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), 0x140, 0xF, 0xF, true));  // row_mirror
  return x;
}

__device__ __forceinline__ void unpack8(const u32x4& w, float (&f)[8]) {
  f[0] = bf16_lo(w.x); f[1] = bf16_hi(w.x);
  f[2] = bf16_lo(w.y); f[3] = bf16_hi(w.y);
  f[4] = bf16_lo(w.z); f[5] = bf16_hi(w.z);
  f[6] = bf16_lo(w.w); f[7] = bf16_hi(w.w);
}

template <int G>
__global__ __launch_bounds__(kWavesPerGroup * 64) void attn_partition_kernel(AttnLaunch a) {
  __shared__ int s_blk[kMaxPartition / kBlockTokens];

  const int s = blockIdx.x / a.NP;
  const int p = blockIdx.x - s * a.NP;
  const int L = min(max(a.context_lens[s], 0), a.max_ctx);
  const int t0 = p * a.P;
  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int kvh = blockIdx.y * kWavesPerGroup + wave;
  const int r = lane >> 4, c = lane & 15;

  if (t0 >= L) {
    // Nothing to attend.  An empty request still owes a zero row when this
    // pass writes the output itself.
    if (L <= 0 && p == 0 && a.NP == 1 && kvh < a.Hkv && r == 0) {
#pragma unroll
      for (int h = 0; h < G; ++h)
        *(u32x4*)(a.out + ((int64_t)s * a.Hq + kvh * G + h) * kHeadDim + 8 * c) = u32x4{0, 0, 0, 0};
    }
    return;
  }
  const int t1 = min(L, t0 + a.P);
  const int nblk = (t1 - t0 + kBlockTokens - 1) / kBlockTokens;

  // Stage this partition's physical block ids in LDS (one coalesced read).
  for (int i = threadIdx.x; i < nblk; i += blockDim.x) {
    const int id = a.block_tables[(int64_t)s * a.MAXB + t0 / kBlockTokens + i];
    s_blk[i] = ((unsigned)id < (unsigned)a.NB) ? id : -1;
  }
  __syncthreads();
  if (kvh >= a.Hkv) return;

  // q for the group, fp32, pre-multiplied by scale*log2(e): softmax runs on exp2.
  float qf[G][8];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    const u32x4 w = *(const u32x4*)(a.q + ((int64_t)s * a.Hq + kvh * G + h) * kHeadDim + 8 * c);
    unpack8(w, qf[h]);
#pragma unroll
    for (int i = 0; i < 8; ++i) qf[h][i] *= a.scale_log2e;
  }

  float m[G], l[G], acc[G][8];
#pragma unroll
  for (int h = 0; h < G; ++h) {
    m[h] = kNegInf;
    l[h] = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[h][i] = 0.f;
  }

  const int64_t head_elems = (int64_t)kBlockTokens * kHeadDim;  // one (block, KV head) slab
  const int64_t block_elems = (int64_t)a.Hkv * head_elems;
  // Ids outside the pool were replaced by -1 when staged; such a block is read
  // from block 0 (always mapped) and masked out below.
  auto slab = [&](const uint16_t* pool, int b) -> const u32x4* {
    const int phys = max(__builtin_amdgcn_readfirstlane(s_blk[b]), 0);
    return (const u32x4*)(pool + (int64_t)phys * block_elems + (int64_t)kvh * head_elems) + lane;
  };

  u32x4 kq[4], vq[4];
  {
    const u32x4* kp = slab(a.k_pool, 0);
    const u32x4* vp = slab(a.v_pool, 0);
#pragma unroll
    for (int j = 0; j < 4; ++j) { kq[j] = kp[64 * j]; vq[j] = vp[64 * j]; }
  }

  for (int b = 0; b < nblk; ++b) {
    // Prefetch the next block's slabs while this one is consumed.
    u32x4 kn[4], vn[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) { kn[j] = kq[j]; vn[j] = vq[j]; }
    if (b + 1 < nblk) {
      const u32x4* kp = slab(a.k_pool, b + 1);
      const u32x4* vp = slab(a.v_pool, b + 1);
#pragma unroll
      for (int j = 0; j < 4; ++j) { kn[j] = kp[64 * j]; vn[j] = vp[64 * j]; }
    }

    const int tb = t0 + b * kBlockTokens + r;   // this lane's token for j = 0
    const bool mapped = s_blk[b] >= 0;
    float sc[4][G];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float kf[8];
      unpack8(kq[j], kf);
      const bool valid = (tb + 4 * j < t1) && mapped;
#pragma unroll
      for (int h = 0; h < G; ++h) {
        float d = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) d = __builtin_fmaf(qf[h][i], kf[i], d);
        d = row16_allreduce_add(d);
        sc[j][h] = valid ? d : kNegInf;   // select, never multiply: the slot may hold NaN
      }
      if (!valid) vq[j] = u32x4{0, 0, 0, 0};
    }

    float pw[4][G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const float mb = fmaxf(fmaxf(sc[0][h], sc[1][h]), fmaxf(sc[2][h], sc[3][h]));
      const float mn = fmaxf(m[h], mb);
      const float ms = (mn == kNegInf) ? 0.f : mn;   // row without a valid token yet
      const float alpha = __builtin_amdgcn_exp2f(m[h] - ms);
      float ps = 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        pw[j][h] = __builtin_amdgcn_exp2f(sc[j][h] - ms);
        ps += pw[j][h];
      }
      l[h] = l[h] * alpha + ps;
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[h][i] *= alpha;
      m[h] = mn;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float vf[8];
      unpack8(vq[j], vf);
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[h][i] = __builtin_fmaf(pw[j][h], vf[i], acc[h][i]);
    }

#pragma unroll
    for (int j = 0; j < 4; ++j) { kq[j] = kn[j]; vq[j] = vn[j]; }
  }

  // Merge the four token-row states (lanes c, c+16, c+32, c+48).
#pragma unroll
  for (int h = 0; h < G; ++h) {
    float ma = fmaxf(m[h], __shfl_xor(m[h], 16));
    ma = fmaxf(ma, __shfl_xor(ma, 32));
    const float f = (m[h] == kNegInf) ? 0.f : __builtin_amdgcn_exp2f(m[h] - ma);
    float lr = l[h] * f;
    lr += __shfl_xor(lr, 16);
    lr += __shfl_xor(lr, 32);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float x = acc[h][i] * f;
      x += __shfl_xor(x, 16);
      x += __shfl_xor(x, 32);
      acc[h][i] = x;
    }
    m[h] = ma;
    l[h] = lr;
  }

  if (r != 0) return;
  if (a.NP == 1) {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const float inv = l[h] > 0.f ? 1.f / l[h] : 0.f;   // no mapped token at all: zero row
      u32x4 w;
      w.x = f32_to_bf16_rne(acc[h][0] * inv) | (f32_to_bf16_rne(acc[h][1] * inv) << 16);
      w.y = f32_to_bf16_rne(acc[h][2] * inv) | (f32_to_bf16_rne(acc[h][3] * inv) << 16);
      w.z = f32_to_bf16_rne(acc[h][4] * inv) | (f32_to_bf16_rne(acc[h][5] * inv) << 16);
      w.w = f32_to_bf16_rne(acc[h][6] * inv) | (f32_to_bf16_rne(acc[h][7] * inv) << 16);
      *(u32x4*)(a.out + ((int64_t)s * a.Hq + kvh * G + h) * kHeadDim + 8 * c) = w;
    }
  } else {
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const int64_t row = ((int64_t)s * a.NP + p) * a.Hq + kvh * G + h;
      float4* dst = (float4*)(a.ws_acc + row * kHeadDim + 8 * c);
      dst[0] = make_float4(acc[h][0], acc[h][1], acc[h][2], acc[h][3]);
      dst[1] = make_float4(acc[h][4], acc[h][5], acc[h][6], acc[h][7]);
      if (c == 0) a.ws_ml[row] = make_float2(m[h], l[h]);
    }
  }
}

template <int G>
hipError_t launch_g(const AttnLaunch& a, hipStream_t stream) {
  dim3 grid((unsigned)(a.S * a.NP), (unsigned)((a.Hkv + kWavesPerGroup - 1) / kWavesPerGroup), 1);
  hipLaunchKernelGGL(attn_partition_kernel<G>, grid, dim3(kWavesPerGroup * 64), 0, stream, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_partition(const AttnLaunch& a, hipStream_t stream) {
  switch (a.G) {
    case 1: return launch_g<1>(a, stream);
    case 2: return launch_g<2>(a, stream);
    case 3: return launch_g<3>(a, stream);
    case 4: return launch_g<4>(a, stream);
    case 5: return launch_g<5>(a, stream);
    case 6: return launch_g<6>(a, stream);
    case 7: return launch_g<7>(a, stream);
    case 8: return launch_g<8>(a, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace pkv
