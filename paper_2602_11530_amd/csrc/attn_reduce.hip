// Split-K merge for paged decode attention on gfx950: combines the per-partition
// (running max, partial sum, un-normalised output) triples of one (request,
// query head) into the final bf16 row.  The maxima are in log2 units, as the
// partition pass leaves them.
#include "pkv_kernels.h"

namespace pkv {
namespace {

constexpr int kRowsPerGroup = 4;   // one wavefront per (request, query head)

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

__global__ __launch_bounds__(kRowsPerGroup * 64) void attn_reduce_kernel(AttnLaunch a) {
  const int row = blockIdx.x * kRowsPerGroup + (threadIdx.x >> 6);   // s*Hq + h
  if (row >= a.S * a.Hq) return;
  const int lane = threadIdx.x & 63;
  const int s = row / a.Hq, h = row - s * a.Hq;
  const int L = min(max(a.context_lens[s], 0), a.max_ctx);
  const int np = (L + a.P - 1) / a.P;   // partitions that were written
  uint32_t* dst = (uint32_t*)(a.out + (int64_t)row * kHeadDim) + lane;
  if (np <= 0) { *dst = 0u; return; }

  const int64_t base = ((int64_t)s * a.NP) * a.Hq + h;   // + p*Hq per partition
  float M = -__builtin_huge_valf();
  for (int p = 0; p < np; ++p) M = fmaxf(M, a.ws_ml[base + (int64_t)p * a.Hq].x);
  float lsum = 0.f, o0 = 0.f, o1 = 0.f;
  for (int p = 0; p < np; ++p) {
    const float2 ml = a.ws_ml[base + (int64_t)p * a.Hq];
    // A partition whose blocks were all unmapped carries max = -inf, sum = 0.
    const float w = (ml.x == -__builtin_huge_valf()) ? 0.f : __builtin_amdgcn_exp2f(ml.x - M);
    const float2 v = *((const float2*)(a.ws_acc + (base + (int64_t)p * a.Hq) * kHeadDim) + lane);
    lsum = __builtin_fmaf(w, ml.y, lsum);
    o0 = __builtin_fmaf(w, v.x, o0);
    o1 = __builtin_fmaf(w, v.y, o1);
  }
  const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
  *dst = f32_to_bf16_rne(o0 * inv) | (f32_to_bf16_rne(o1 * inv) << 16);
}

}  // namespace

hipError_t launch_attn_reduce(const AttnLaunch& a, hipStream_t stream) {
  const int rows = a.S * a.Hq;
  dim3 grid((unsigned)((rows + kRowsPerGroup - 1) / kRowsPerGroup), 1, 1);
  hipLaunchKernelGGL(attn_reduce_kernel, grid, dim3(kRowsPerGroup * 64), 0, stream, a);
  return hipGetLastError();
}

}  // namespace pkv
