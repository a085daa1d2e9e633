// dodo_score: the Scorer as a linear head d -> 1 (Eq. 6 / Eq. 15 of the Dodo paper).
//
// HBM-bound GEMV: every hidden row is read once, 16 bytes per lane per load,
// one wavefront per row with several loads in flight; the weight vector is
// staged once per workgroup in LDS as fp32.  The 64-lane reduction has a fixed
// order, so the scores are run-to-run deterministic.
#include "dodo_common.h"

namespace dodo {
namespace {

constexpr int kScoreThreads = 256;
constexpr int kUnroll = 8;  // 16-byte loads in flight per lane

template <int DTYPE>
struct Elems;
template <>
struct Elems<DODO_DTYPE_BF16> {
  static constexpr int kPerLoad = 8;
  __device__ static __forceinline__ float dot(const uint4& v, const float* w) {
    float a = bf16_lo(v.x) * w[0];
    a = fmaf(bf16_hi(v.x), w[1], a);
    a = fmaf(bf16_lo(v.y), w[2], a);
    a = fmaf(bf16_hi(v.y), w[3], a);
    a = fmaf(bf16_lo(v.z), w[4], a);
    a = fmaf(bf16_hi(v.z), w[5], a);
    a = fmaf(bf16_lo(v.w), w[6], a);
    a = fmaf(bf16_hi(v.w), w[7], a);
    return a;
  }
  __device__ static __forceinline__ float load_one(const void* p, int64_t i) {
    return __uint_as_float(static_cast<uint32_t>(static_cast<const uint16_t*>(p)[i]) << 16);
  }
};
template <>
struct Elems<DODO_DTYPE_F32> {
  static constexpr int kPerLoad = 4;
  __device__ static __forceinline__ float dot(const uint4& v, const float* w) {
    float a = __uint_as_float(v.x) * w[0];
    a = fmaf(__uint_as_float(v.y), w[1], a);
    a = fmaf(__uint_as_float(v.z), w[2], a);
    a = fmaf(__uint_as_float(v.w), w[3], a);
    return a;
  }
  __device__ static __forceinline__ float load_one(const void* p, int64_t i) {
    return static_cast<const float*>(p)[i];
  }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

template <int DTYPE>
__global__ __launch_bounds__(kScoreThreads) void score_kernel(const void* __restrict__ hidden,
                                                              const void* __restrict__ w, float bias, int64_t N,
                                                              int d, int64_t row_stride,
                                                              float* __restrict__ scores) {
  using E = Elems<DTYPE>;
  constexpr int kEPL = E::kPerLoad;     // elements per 16-byte load
  constexpr int kChunk = kWave * kEPL;  // elements one wave-wide load covers
  extern __shared__ float w_lds[];
  for (int c = threadIdx.x; c < d; c += kScoreThreads) w_lds[c] = E::load_one(w, c);
  __syncthreads();

  const int lane = lane_id();
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * (kScoreThreads / kWave) + threadIdx.x / kWave;
  const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (kScoreThreads / kWave);
  const int full_groups = d / (kChunk * kUnroll);
  const size_t esz = DTYPE == DODO_DTYPE_F32 ? 4 : 2;

  for (int64_t row = wave; row < N; row += nwaves) {
    const char* rp = static_cast<const char*>(hidden) + static_cast<size_t>(row) * row_stride * esz;
    float acc[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) acc[u] = 0.f;
    int c0 = lane * kEPL;
    for (int g = 0; g < full_groups; ++g) {
      uint4 v[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u)
        v[u] = load16_stream(rp + static_cast<size_t>(c0 + u * kChunk) * esz);
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) acc[u] += E::dot(v[u], &w_lds[c0 + u * kChunk]);
      c0 += kChunk * kUnroll;
    }
    for (; c0 < d; c0 += kChunk) {  // d is a multiple of 8: a 16-byte load never straddles the row end
      const uint4 v = *reinterpret_cast<const uint4*>(rp + static_cast<size_t>(c0) * esz);
      acc[0] += E::dot(v, &w_lds[c0]);
    }
    float s = 0.f;
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) s += acc[u];
    s = wave_sum(s) + bias;
    if (lane == 0) scores[row] = (s == 0.f) ? 0.f : s;  // -0 -> +0
  }
}

}  // namespace
}  // namespace dodo

extern "C" int dodo_score(const void* hidden, const void* w, float bias, int dtype, int64_t N, int32_t d,
                          int64_t row_stride, float* scores, void* stream) {
  using namespace dodo;
  if (N < 0 || d <= 0 || row_stride < d) return DODO_ERR_INVALID_ARG;
  if (N == 0) return DODO_OK;
  if (!hidden || !w || !scores) return DODO_ERR_INVALID_ARG;
  if (!dtype_ok(dtype)) return DODO_ERR_UNSUPPORTED;
  const int es = elem_bytes(dtype);
  if (d % 8 != 0 || d > 16384) return DODO_ERR_UNSUPPORTED;
  if (!aligned16(hidden) || (row_stride * es) % 16 != 0) return DODO_ERR_UNSUPPORTED;

  const int waves_per_block = kScoreThreads / kWave;
  int64_t blocks = (N + waves_per_block - 1) / waves_per_block;
  const int64_t cap = 256 * 4;  // 4 workgroups per CU keep >100 KB of loads in flight per CU
  if (blocks > cap) blocks = cap;
  const size_t lds = static_cast<size_t>(d) * sizeof(float);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dtype == DODO_DTYPE_BF16) {
    hipLaunchKernelGGL(score_kernel<DODO_DTYPE_BF16>, dim3(static_cast<unsigned>(blocks)), dim3(kScoreThreads), lds,
                       s, hidden, w, bias, N, d, row_stride, scores);
  } else {
    hipLaunchKernelGGL(score_kernel<DODO_DTYPE_F32>, dim3(static_cast<unsigned>(blocks)), dim3(kScoreThreads), lds, s,
                       hidden, w, bias, N, d, row_stride, scores);
  }
  return launch_status();
}
