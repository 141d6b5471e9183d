// Split-K merge for paged decode attention on gfx950: combines the partial
// records (reference max, partial sum, un-normalised row) that the stream pass
// left for one (request, query head) into the final bf16 row.  The maxima are in
// log2 units.  One wavefront per row; the lanes fetch the records' statistics
// side by side, then stream the partial rows eight at a time so that the pass
// is not a chain of dependent loads.  Which slots hold a segment's records
// follows from the stream layout described in pkv_kernels.h.
#include "pkv_kernels.h"

namespace pkv {
namespace {

constexpr int kRowsPerGroup = 4;   // wavefronts per workgroup
constexpr int kBatch = 8;          // partial rows in flight per wavefront
constexpr float kNegInf = -__builtin_huge_valf();

// kPer = D / 64 consecutive floats of a row per lane
template <int kPer> struct Chunk { typedef float T __attribute__((ext_vector_type(kPer))); };
template <> struct Chunk<1> { typedef float T; };
template <int kPer> __device__ __forceinline__ float chunk_get(const typename Chunk<kPer>::T& v, int i) { return v[i]; }
template <> __device__ __forceinline__ float chunk_get<1>(const float& v, int) { return v; }

// fp32 -> bf16, round to nearest even (inputs here are finite)
__device__ __forceinline__ uint16_t bf16_bits(float x) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  const f32x2 f = {x, 0.f};
  return (uint16_t)(__builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2)) & 0xffffu);
}

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

template <int kD>
__global__ __launch_bounds__(kRowsPerGroup * 64) void attn_reduce_kernel(AttnLaunch a) {
  constexpr int kPer = kD / 64;
  typedef typename Chunk<kPer>::T Vec;
  const int row = blockIdx.x * kRowsPerGroup + (threadIdx.x >> 6);   // s*Hq + h
  if (row >= a.S * a.Hq) return;
  const int lane = threadIdx.x & 63;
  const int s = row / a.Hq, h = row - s * a.Hq;
  const int kvh = h / a.G, g = h - kvh * a.G;
  const int* cumB = a.ws_cum;
  const int nb = cumB[s + 1] - cumB[s];
  uint16_t* dst = a.out + (int64_t)row * kD + kPer * lane;
  if (nb <= 0) {   // an empty request owes a zero row
#pragma unroll
    for (int i = 0; i < kPer; ++i) dst[i] = 0;
    return;
  }

  const int64_t T = (int64_t)a.Hkv * cumB[a.S];
  const int64_t W = min((int64_t)a.waves, T);
  const int64_t pos_a = (int64_t)a.Hkv * cumB[s] + (int64_t)kvh * nb;   // the segment's first block
  const int seg = s * a.Hkv + kvh;
  const int first = seg + share_owner(pos_a, T, W);
  const int last = seg + share_owner(pos_a + nb - 1, T, W);
  const int np = last - first + 1;   // one record per wavefront that streamed part of this segment

  const int rec_floats = record_floats(a.G, kD);
  auto stats = [&](int p) -> float2 {   // (max, sum) of record p for this head
    return *(const float2*)(a.ws_rec + (int64_t)(first + p) * rec_floats + a.G * kD + 2 * g);
  };
  auto part_row = [&](int p) -> const float* {   // its un-normalised row
    return a.ws_rec + (int64_t)(first + p) * rec_floats + g * kD;
  };
  float M = kNegInf;
  for (int p0 = 0; p0 < np; p0 += 64) {
    const int p = p0 + lane;
    if (p < np) M = fmaxf(M, stats(p).x);
  }
  M = wave_max(M);

  float lsum = 0.f, acc[kPer];
#pragma unroll
  for (int i = 0; i < kPer; ++i) acc[i] = 0.f;
  for (int p0 = 0; p0 < np; p0 += 64) {
    const int p = p0 + lane;
    float w = 0.f;
    if (p < np) {
      const float2 ml = stats(p);
      // A record whose blocks were all unmapped carries max = -inf, sum = 0.
      w = (ml.x == kNegInf) ? 0.f : __builtin_amdgcn_exp2f(ml.x - M);
      lsum = __builtin_fmaf(w, ml.y, lsum);
    }
    const int cnt = min(64, np - p0);
    for (int j0 = 0; j0 < cnt; j0 += kBatch) {
      Vec v[kBatch];
      float wj[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int j = min(j0 + u, cnt - 1);   // clamped rows get weight 0
        wj[u] = (j0 + u < cnt) ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w), j)) : 0.f;
        v[u] = *((const Vec*)part_row(p0 + j) + lane);
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        // a weight of exactly zero must also silence whatever the row holds
#pragma unroll
        for (int i = 0; i < kPer; ++i)
          acc[i] = (wj[u] != 0.f) ? __builtin_fmaf(wj[u], chunk_get<kPer>(v[u], i), acc[i]) : acc[i];
      }
    }
  }
  lsum = wave_sum(lsum);
  const float inv = lsum > 0.f ? a.out_scale / lsum : 0.f;
  uint16_t r[kPer];
#pragma unroll
  for (int i = 0; i < kPer; ++i) r[i] = bf16_bits(acc[i] * inv);
  if (kPer == 1) dst[0] = r[0];
  else if (kPer == 2) *(uint32_t*)dst = r[0] | ((uint32_t)r[1] << 16);
  else *(uint2*)dst = make_uint2(r[0] | ((uint32_t)r[1] << 16), r[2] | ((uint32_t)r[3] << 16));
}

}  // namespace

hipError_t launch_attn_reduce(const AttnLaunch& a, hipStream_t stream) {
  const int rows = a.S * a.Hq;
  dim3 grid((unsigned)((rows + kRowsPerGroup - 1) / kRowsPerGroup), 1, 1);
  const dim3 block(kRowsPerGroup * 64);
  if (a.D == 64) hipLaunchKernelGGL(attn_reduce_kernel<64>, grid, block, 0, stream, a);
  else if (a.D == 128) hipLaunchKernelGGL(attn_reduce_kernel<128>, grid, block, 0, stream, a);
  else if (a.D == 256) hipLaunchKernelGGL(attn_reduce_kernel<256>, grid, block, 0, stream, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace pkv
