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

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

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

__global__ __launch_bounds__(kRowsPerGroup * 64) void attn_reduce_kernel(AttnLaunch a) {
  const int row = blockIdx.x * kRowsPerGroup + (threadIdx.x >> 6);   // s*Hq + h
  if (row >= a.S * a.Hq) return;
  const int lane = threadIdx.x & 63;
  const int s = row / a.Hq, h = row - s * a.Hq;
  const int kvh = h / a.G, g = h - kvh * a.G;
  const int* cumB = a.ws_cum;
  const int nb = cumB[s + 1] - cumB[s];
  uint32_t* dst = (uint32_t*)(a.out + (int64_t)row * kHeadDim) + lane;
  if (nb <= 0) { *dst = 0u; return; }   // an empty request owes a zero row

  const int64_t T = (int64_t)a.Hkv * cumB[a.S];
  const int64_t W = min((int64_t)kStreamWaves, T);
  const int64_t pos_a = (int64_t)a.Hkv * cumB[s] + (int64_t)kvh * nb;   // the segment's first block
  const int seg = s * a.Hkv + kvh;
  const int first = seg + share_owner(pos_a, T, W);
  const int last = seg + share_owner(pos_a + nb - 1, T, W);
  const int np = last - first + 1;   // one record per wavefront that streamed part of this segment

  const int rec_floats = record_floats(a.G);
  auto stats = [&](int p) -> float2 {   // (max, sum) of record p for this head
    return *(const float2*)(a.ws_rec + (int64_t)(first + p) * rec_floats + a.G * kHeadDim + 2 * g);
  };
  auto part_row = [&](int p) -> const float* {   // its un-normalised row
    return a.ws_rec + (int64_t)(first + p) * rec_floats + g * kHeadDim;
  };
  float M = kNegInf;
  for (int p0 = 0; p0 < np; p0 += 64) {
    const int p = p0 + lane;
    if (p < np) M = fmaxf(M, stats(p).x);
  }
  M = wave_max(M);

  float lsum = 0.f, o0 = 0.f, o1 = 0.f;
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
      float2 v[kBatch];
      float wj[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int j = min(j0 + u, cnt - 1);   // clamped rows get weight 0
        wj[u] = (j0 + u < cnt) ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w), j)) : 0.f;
        v[u] = *((const float2*)part_row(p0 + j) + lane);
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        // a weight of exactly zero must also silence whatever the row holds
        o0 = (wj[u] != 0.f) ? __builtin_fmaf(wj[u], v[u].x, o0) : o0;
        o1 = (wj[u] != 0.f) ? __builtin_fmaf(wj[u], v[u].y, o1) : o1;
      }
    }
  }
  lsum = wave_sum(lsum);
  const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
  const f32x2 r = {o0 * inv, o1 * inv};
  *dst = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, bf16x2));
}

}  // namespace

hipError_t launch_attn_reduce(const AttnLaunch& a, hipStream_t stream) {
  const int rows = a.S * a.Hq;
  dim3 grid((unsigned)((rows + kRowsPerGroup - 1) / kRowsPerGroup), 1, 1);
  hipLaunchKernelGGL(attn_reduce_kernel, grid, dim3(kRowsPerGroup * 64), 0, stream, a);
  return hipGetLastError();
}

}  // namespace pkv
