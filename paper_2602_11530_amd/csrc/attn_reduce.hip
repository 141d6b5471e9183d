// Split-K merge for paged decode attention on gfx950: combines the partial
// records (reference max, partial sum, un-normalised row) that the stream pass
// left for one (request, query head) into the final bf16 row.  The maxima are in
// log2 units.  A wavefront fetches the records' statistics side by side, then
// streams the partial rows eight at a time so that the pass is not a chain of
// dependent loads.  A full batch gives a row a handful of records and one
// wavefront per row; a batch of a few requests spreads each (request, KV head)
// over hundreds of stream wavefronts, and then a workgroup shares the row.
// Which slots hold a segment's records follows from the stream layout described
// in pkv_kernels.h.
#include "pkv_kernels.h"

namespace pkv {
namespace {

constexpr int kRowsPerGroup = 4;   // wavefronts per workgroup
constexpr int kBatch = 8;          // partial rows in flight per wavefront
constexpr int kMaxWideWaves = 16;  // wavefronts of a workgroup that share one row (small batches)
constexpr float kNegInf = -__builtin_huge_valf();

// kPer = D / 64 consecutive floats of a row per lane
template <int kPer> struct Chunk { typedef float T __attribute__((ext_vector_type(kPer))); };
template <> struct Chunk<1> { typedef float T; };
template <int kPer> __device__ __forceinline__ float chunk_get(const typename Chunk<kPer>::T& v, int i) { return v[i]; }
template <> __device__ __forceinline__ float chunk_get<1>(const float& v, int) { return v; }

// fp32 -> bf16, round to nearest even (a NaN stays a NaN)
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

// Where the records of row (s, h) lie: the slots of its segment's first and last
// block's owners (see pkv_kernels.h).  Returns false for an empty request.
struct RowRecords {
  int first;   // slot of the first record
  int np;      // one record per wavefront that streamed part of this segment
  int g;       // head within its KV head's group
};
__device__ __forceinline__ bool locate_records(const AttnLaunch& a, int row, RowRecords& r) {
  const int s = row / a.Hq, h = row - s * a.Hq;
  const int kvh = h / a.G;
  r.g = h - kvh * a.G;
  const int* cumB = a.ws_cum;
  const int nb = cumB[s + 1] - cumB[s];
  if (nb <= 0) return false;
  const int64_t T = (int64_t)a.Hkv * cumB[a.S];
  const int64_t W = min((int64_t)a.waves, T);
  const int64_t pos_a = (int64_t)a.Hkv * cumB[s] + (int64_t)kvh * nb;   // the segment's first block
  const int seg = s * a.Hkv + kvh;
  r.first = seg + share_owner(pos_a, T, W);
  r.np = seg + share_owner(pos_a + nb - 1, T, W) - r.first + 1;
  return true;
}

// One wavefront folds `count` records of a row (records begin, begin + stride, ...
// counted from the row's first): on return M is their largest reference maximum,
// acc this lane's kPer floats of the sum of their rows weighted by 2^(m - M), and
// lsum the wave-wide sum of their partial sums with the same weights.  count = 0
// leaves (M, lsum, acc) = (-inf, 0, 0).
template <int kD>
__device__ __forceinline__ void fold_records(const AttnLaunch& a, const RowRecords& r, int begin,
                                             int stride, int count, int lane, float& M, float& lsum,
                                             float (&acc)[kD / 64]) {
  constexpr int kPer = kD / 64;
  typedef typename Chunk<kPer>::T Vec;
  const int rec_floats = record_floats(a.G, kD);
  auto record = [&](int i) -> const float* {
    return a.ws_rec + (int64_t)(r.first + begin + i * stride) * rec_floats;
  };
  auto stats = [&](int i) -> float2 {   // (max, sum) of record i for this head
    return *(const float2*)(record(i) + a.G * kD + 2 * r.g);
  };
  // the statistics of the first 64 records stay in registers for the second pass
  const float2 ml0 = (lane < count) ? stats(lane) : float2{kNegInf, 0.f};
  M = ml0.x;
  for (int i0 = 64; i0 < count; i0 += 64) {
    const int i = i0 + lane;
    if (i < count) M = fmaxf(M, stats(i).x);
  }
  M = wave_max(M);

  lsum = 0.f;
#pragma unroll
  for (int i = 0; i < kPer; ++i) acc[i] = 0.f;
  for (int i0 = 0; i0 < count; i0 += 64) {
    const int i = i0 + lane;
    float w = 0.f;
    if (i < count) {
      const float2 ml = i0 == 0 ? ml0 : stats(i);
      // A record whose blocks were all unmapped carries max = -inf, sum = 0.
      w = (ml.x == kNegInf) ? 0.f : __builtin_amdgcn_exp2f(ml.x - M);
      lsum = __builtin_fmaf(w, ml.y, lsum);
    }
    const int cnt = min(64, count - i0);
    for (int j0 = 0; j0 < cnt; j0 += kBatch) {
      Vec v[kBatch];
      float wj[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int j = min(j0 + u, cnt - 1);   // clamped rows get weight 0
        wj[u] = (j0 + u < cnt) ? __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w), j)) : 0.f;
        v[u] = *((const Vec*)(record(i0 + j) + r.g * kD) + lane);
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
}

// Normalise, scale, round once to bf16 and store this lane's kPer elements of the row.
template <int kPer>
__device__ __forceinline__ void store_row(uint16_t* dst, const float (&acc)[kPer], float lsum, float out_scale) {
  const float inv = lsum > 0.f ? out_scale / lsum : 0.f;
  uint16_t r[kPer];
#pragma unroll
  for (int i = 0; i < kPer; ++i) r[i] = bf16_bits(acc[i] * inv);
  if (kPer == 1) dst[0] = r[0];
  else if (kPer == 2) *(uint32_t*)dst = r[0] | ((uint32_t)r[1] << 16);
  else *(uint2*)dst = make_uint2(r[0] | ((uint32_t)r[1] << 16), r[2] | ((uint32_t)r[3] << 16));
}

// One wavefront per row: the shape of a full batch, where a row has a handful of records.
template <int kD>
__global__ __launch_bounds__(kRowsPerGroup * 64) void attn_reduce_kernel(AttnLaunch a) {
  constexpr int kPer = kD / 64;
  const int row = blockIdx.x * kRowsPerGroup + (threadIdx.x >> 6);   // s*Hq + h
  if (row >= a.S * a.Hq) return;
  const int lane = threadIdx.x & 63;
  uint16_t* dst = a.out + (int64_t)row * kD + kPer * lane;
  RowRecords r;
  if (!locate_records(a, row, r)) {   // an empty request owes a zero row
#pragma unroll
    for (int i = 0; i < kPer; ++i) dst[i] = 0;
    return;
  }
  float M, lsum, acc[kPer];
  fold_records<kD>(a, r, 0, 1, r.np, lane, M, lsum, acc);
  store_row<kPer>(dst, acc, lsum, a.out_scale);
}

// One workgroup per row, for a small batch: few segments share the stream's
// wavefronts, so a row has up to hundreds of records and a single wavefront
// would read them in a long chain of rounds.  Wavefront i of the group folds
// records i, i + n, i + 2n, ... (n = wavefronts in the group), the partial
// results meet in LDS and wavefront 0 folds those.
template <int kD>
__global__ __launch_bounds__(kMaxWideWaves * 64) void attn_reduce_wide_kernel(AttnLaunch a) {
  constexpr int kPer = kD / 64;
  __shared__ float part_stats[kMaxWideWaves][2];
  __shared__ float part_acc[kMaxWideWaves][kD];
  const int row = blockIdx.x;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int width = blockDim.x >> 6;
  uint16_t* dst = a.out + (int64_t)row * kD + kPer * lane;
  RowRecords r;
  if (!locate_records(a, row, r)) {   // the same for every wavefront of the group
    if (wave == 0) {
#pragma unroll
      for (int i = 0; i < kPer; ++i) dst[i] = 0;
    }
    return;
  }
  float M, lsum, acc[kPer];
  const int count = r.np > wave ? (r.np - wave + width - 1) / width : 0;
  fold_records<kD>(a, r, wave, width, count, lane, M, lsum, acc);
  if (lane == 0) { part_stats[wave][0] = M; part_stats[wave][1] = lsum; }
#pragma unroll
  for (int i = 0; i < kPer; ++i) part_acc[wave][kPer * lane + i] = acc[i];
  __syncthreads();
  if (wave != 0) return;
  float Mall = kNegInf;
  for (int w = 0; w < width; ++w) Mall = fmaxf(Mall, part_stats[w][0]);
  float lall = 0.f, total[kPer];
#pragma unroll
  for (int i = 0; i < kPer; ++i) total[i] = 0.f;
  for (int w = 0; w < width; ++w) {
    const float m = part_stats[w][0];
    if (m == kNegInf) continue;   // nothing valid behind this partial result: weight 0
    const float f = __builtin_amdgcn_exp2f(m - Mall);
    lall = __builtin_fmaf(f, part_stats[w][1], lall);
#pragma unroll
    for (int i = 0; i < kPer; ++i) total[i] = __builtin_fmaf(f, part_acc[w][kPer * lane + i], total[i]);
  }
  store_row<kPer>(dst, total, lall, a.out_scale);
}

}  // namespace

hipError_t launch_attn_reduce(const AttnLaunch& a, hipStream_t stream) {
  const int rows = a.S * a.Hq;
  // A segment's records come from the wavefronts that streamed it: about
  // waves / (S * Hkv) of them when the batch is large enough to occupy them all.
  // From 32 records per row on, the row gets a workgroup of its own with one
  // wavefront per four records (8 or 16 wavefronts); below that the wider group
  // costs more than the rounds it saves (measured at 8 and 16 records per row).
  const int64_t segments = (int64_t)a.S * a.Hkv;
  const int64_t per_row = a.waves / segments;
  if (per_row >= 32) {
    const int width = per_row >= 64 ? 16 : 8;
    const dim3 grid((unsigned)rows), block(width * 64);
    if (a.D == 64) hipLaunchKernelGGL(attn_reduce_wide_kernel<64>, grid, block, 0, stream, a);
    else if (a.D == 128) hipLaunchKernelGGL(attn_reduce_wide_kernel<128>, grid, block, 0, stream, a);
    else if (a.D == 256) hipLaunchKernelGGL(attn_reduce_wide_kernel<256>, grid, block, 0, stream, a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
  }
  dim3 grid((unsigned)((rows + kRowsPerGroup - 1) / kRowsPerGroup), 1, 1);
  const dim3 block(kRowsPerGroup * 64);
  if (a.D == 64) hipLaunchKernelGGL(attn_reduce_kernel<64>, grid, block, 0, stream, a);
  else if (a.D == 128) hipLaunchKernelGGL(attn_reduce_kernel<128>, grid, block, 0, stream, a);
  else if (a.D == 256) hipLaunchKernelGGL(attn_reduce_kernel<256>, grid, block, 0, stream, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace pkv
