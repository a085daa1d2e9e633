// dodo_score: the Scorer as a linear head d -> 1 (Eq. 6 / Eq. 15 of the Dodo paper).
//
// HBM-bound GEMV: every hidden row is read once, 16 bytes per lane per load,
// one wavefront per row with several loads in flight (and, for widths that
// split evenly, the next batch of loads in flight while the current one is
// reduced); the weight vector is staged once per workgroup in LDS as fp32.
// Summation order is fixed, so the scores are run-to-run deterministic.
#include "dodo_common.h"

namespace dodo {
namespace {

constexpr int kScoreThreads = 256;
constexpr int kUnroll = 8;  // 16-byte loads in flight per lane

// Layer dimension of a launch (grid y): layer l reads hidden + l * hidden_ls and w + l * w_ls (elements), writes
// scores + l * scores_ls and adds biases[l] (or the one bias when biases is null).  A single layer: all zero.
struct LayerDim {
  int64_t hidden_ls, w_ls, scores_ls;
  const float* biases;
};

template <int DTYPE>
struct Elems;
template <>
struct Elems<DODO_DTYPE_BF16> {
  static constexpr int kPerLoad = 8;
  // w points at 8 consecutive fp32 weights, 16-byte aligned
  __device__ static __forceinline__ float dot(const uint4& v, const float* w) {
    const float4 w0 = *reinterpret_cast<const float4*>(w), w1 = *reinterpret_cast<const float4*>(w + 4);
    float a = bf16_lo(v.x) * w0.x;
    a = fmaf(bf16_hi(v.x), w0.y, a);
    a = fmaf(bf16_lo(v.y), w0.z, a);
    a = fmaf(bf16_hi(v.y), w0.w, a);
    a = fmaf(bf16_lo(v.z), w1.x, a);
    a = fmaf(bf16_hi(v.z), w1.y, a);
    a = fmaf(bf16_lo(v.w), w1.z, a);
    a = fmaf(bf16_hi(v.w), w1.w, a);
    return a;
  }
  __device__ static __forceinline__ float load_one(const void* p, int64_t i) {
    return __uint_as_float(static_cast<uint32_t>(static_cast<const uint16_t*>(p)[i]) << 16);
  }
};
template <>
struct Elems<DODO_DTYPE_F32> {
  static constexpr int kPerLoad = 4;
  // w points at 4 consecutive fp32 weights, 16-byte aligned
  __device__ static __forceinline__ float dot(const uint4& v, const float* w) {
    const float4 w0 = *reinterpret_cast<const float4*>(w);
    float a = __uint_as_float(v.x) * w0.x;
    a = fmaf(__uint_as_float(v.y), w0.y, a);
    a = fmaf(__uint_as_float(v.z), w0.z, a);
    a = fmaf(__uint_as_float(v.w), w0.w, a);
    return a;
  }
  __device__ static __forceinline__ float load_one(const void* p, int64_t i) {
    return static_cast<const float*>(p)[i];
  }
};

__device__ __forceinline__ float wave_sum(float v) { return wave_sum64(v); }

// The weight vector as fp32 in LDS, staged by the whole workgroup.  16-byte loads, all of a thread's loads issued
// before the first is used (the kernel's first loads: one round trip instead of one per element); a weight
// vector that is not 16-byte aligned is fetched element by element.
template <int DTYPE>
__device__ __forceinline__ void stage_weights(const void* __restrict__ w, int d, float* __restrict__ w_lds) {
  using E = Elems<DTYPE>;
  constexpr int kEPL = E::kPerLoad;
  constexpr int kVecPerThread = 4;
  if ((reinterpret_cast<uintptr_t>(w) & 15u) == 0) {
    const int nvec = d / kEPL;  // d is a multiple of 8
    for (int v0 = threadIdx.x; v0 < nvec; v0 += kScoreThreads * kVecPerThread) {
      uint4 wv[kVecPerThread];
#pragma unroll
      for (int u = 0; u < kVecPerThread; ++u)
        wv[u] = static_cast<const uint4*>(w)[min(v0 + u * kScoreThreads, nvec - 1)];
#pragma unroll
      for (int u = 0; u < kVecPerThread; ++u) {
        const int v = v0 + u * kScoreThreads;
        if (v < nvec) {
          float* dst = w_lds + static_cast<size_t>(v) * kEPL;
          if (DTYPE == DODO_DTYPE_F32) {
            *reinterpret_cast<uint4*>(dst) = wv[u];
          } else {
            *reinterpret_cast<float4*>(dst) = make_float4(bf16_lo(wv[u].x), bf16_hi(wv[u].x), bf16_lo(wv[u].y), bf16_hi(wv[u].y));
            *reinterpret_cast<float4*>(dst + 4) = make_float4(bf16_lo(wv[u].z), bf16_hi(wv[u].z), bf16_lo(wv[u].w), bf16_hi(wv[u].w));
          }
        }
      }
    }
  } else {
    for (int c = threadIdx.x; c < d; c += kScoreThreads) w_lds[c] = E::load_one(w, c);
  }
}

template <int DTYPE>
__global__ __launch_bounds__(kScoreThreads) void score_kernel(const void* __restrict__ hidden_all,
                                                              const void* __restrict__ w_all, float bias, int64_t N,
                                                              int d, int64_t row_stride,
                                                              float* __restrict__ scores_all, LayerDim ld) {
  using E = Elems<DTYPE>;
  // all arguments in one round of scalar loads (the compiler would fetch them a few at a time, before each first use)
  asm volatile("" ::"s"(hidden_all), "s"(w_all), "s"(bias), "s"(N), "s"(d), "s"(row_stride), "s"(scores_all),
               "s"(ld.hidden_ls), "s"(ld.w_ls), "s"(ld.scores_ls), "s"(ld.biases));
  const int64_t layer = blockIdx.y;
  const size_t esz_l = DTYPE == DODO_DTYPE_F32 ? 4 : 2;
  const void* hidden = static_cast<const char*>(hidden_all) + layer * ld.hidden_ls * esz_l;
  const void* w = static_cast<const char*>(w_all) + layer * ld.w_ls * esz_l;
  float* scores = scores_all + layer * ld.scores_ls;
  if (ld.biases != nullptr) bias = ld.biases[layer];
  constexpr int kEPL = E::kPerLoad;     // elements per 16-byte load
  constexpr int kChunk = kWave * kEPL;  // elements one wave-wide load covers
  extern __shared__ __attribute__((aligned(16))) float w_lds[];
  stage_weights<DTYPE>(w, d, w_lds);
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

// Software-pipelined variant for widths that split evenly: d == nb * PB * (64 lanes * elements per
// load).  A row is read in nb batches of PB wave-wide 16-byte loads; the loads of the next batch
// (same row, or the wavefront's next row) are in flight while the current one is multiplied and
// reduced.  Same summation order per row as the generic kernel.
// SINGLE: the whole row is one batch (nb == 1); the weight fragments are then loop-invariant and
// stay in registers.
template <int DTYPE, int PB, bool SINGLE>
__global__ __launch_bounds__(kScoreThreads) void score_pipelined_kernel(const void* __restrict__ hidden_all,
                                                                        const void* __restrict__ w_all, float bias,
                                                                        int64_t N, int d, int nb_arg,
                                                                        int64_t row_stride,
                                                                        float* __restrict__ scores_all, LayerDim ld) {
  const int nb = SINGLE ? 1 : nb_arg;
  using E = Elems<DTYPE>;
  // all arguments in one round of scalar loads (the compiler would fetch them a few at a time, before each first use)
  asm volatile("" ::"s"(hidden_all), "s"(w_all), "s"(bias), "s"(N), "s"(d), "s"(row_stride), "s"(scores_all),
               "s"(ld.hidden_ls), "s"(ld.w_ls), "s"(ld.scores_ls), "s"(ld.biases));
  const int64_t layer = blockIdx.y;
  const size_t esz_l = DTYPE == DODO_DTYPE_F32 ? 4 : 2;
  const void* hidden = static_cast<const char*>(hidden_all) + layer * ld.hidden_ls * esz_l;
  const void* w = static_cast<const char*>(w_all) + layer * ld.w_ls * esz_l;
  float* scores = scores_all + layer * ld.scores_ls;
  if (ld.biases != nullptr) bias = ld.biases[layer];
  constexpr int kEPL = E::kPerLoad;
  constexpr int kChunk = kWave * kEPL;
  extern __shared__ __attribute__((aligned(16))) float w_lds[];
  stage_weights<DTYPE>(w, d, w_lds);
  __syncthreads();

  const int lane = lane_id();
  const int64_t wave = static_cast<int64_t>(blockIdx.x) * (kScoreThreads / kWave) + threadIdx.x / kWave;
  const int64_t nwaves = static_cast<int64_t>(gridDim.x) * (kScoreThreads / kWave);
  const size_t esz = DTYPE == DODO_DTYPE_F32 ? 4 : 2;
  const int lane_c = lane * kEPL;

  auto load_batch = [&](uint4 (&v)[PB], int64_t row, int bi) {
    const char* rp = static_cast<const char*>(hidden) + (static_cast<size_t>(row) * row_stride + bi * PB * kChunk + lane_c) * esz;
#pragma unroll
    for (int u = 0; u < PB; ++u) v[u] = load16_stream(rp + static_cast<size_t>(u * kChunk) * esz);
  };

  float acc = 0.f;
  auto consume = [&](const uint4 (&v)[PB], int64_t row, int bi) {
    float part[PB];
#pragma unroll
    for (int u = 0; u < PB; ++u) part[u] = E::dot(v[u], &w_lds[((SINGLE ? 0 : bi) * PB + u) * kChunk + lane_c]);
#pragma unroll
    for (int u = 0; u < PB; ++u) acc += part[u];
    if (bi == nb - 1) {  // the row is complete
      const float s = wave_sum(acc) + bias;
      if (lane == 0) scores[row] = (s == 0.f) ? 0.f : s;  // -0 -> +0
      acc = 0.f;
    }
  };
  auto advance = [&](int64_t& row, int& bi) {
    if (++bi == nb) {
      bi = 0;
      row += nwaves;
    }
  };

  // Two register buffers used alternately, so that no copy has to wait for the loads in flight.
  // Loads are issued unconditionally (past the end they re-read the last row and are discarded):
  // a branch around them would make the compiler wait for every outstanding load at the merge.
  auto load_clamped = [&](uint4 (&v)[PB], int64_t row, int bi) { load_batch(v, row < N ? row : N - 1, bi); };
  uint4 buf_a[PB], buf_b[PB];
  int64_t row_a = wave, row_b = wave;
  int bi_a = 0, bi_b = 0;
  advance(row_b, bi_b);  // b runs one batch ahead of a
  load_clamped(buf_a, row_a, bi_a);
  while (row_a < N) {
    load_clamped(buf_b, row_b, bi_b);
    __builtin_amdgcn_sched_barrier(0);  // keep the loads ahead of the arithmetic
    consume(buf_a, row_a, bi_a);
    advance(row_a, bi_a);
    advance(row_a, bi_a);  // a now names the batch after b
    load_clamped(buf_a, row_a, bi_a);
    __builtin_amdgcn_sched_barrier(0);
    if (row_b < N) consume(buf_b, row_b, bi_b);
    advance(row_b, bi_b);
    advance(row_b, bi_b);
  }
}

// Workgroups of `kernel` that fit on the device at once (all resident: the kernels stride over the
// rows, so a grid larger than this would run in uneven rounds).
template <typename K>
int resident_blocks(K kernel, size_t lds) {
  return compute_units() * resident_blocks_per_cu(reinterpret_cast<const void*>(kernel), kScoreThreads, lds, 2);
}

template <int DTYPE, int PB>
void launch_pipelined(const void* hidden, const void* w, float bias, int64_t N, int d, int nb, int64_t row_stride,
                      float* scores, unsigned blocks, size_t lds, hipStream_t s, int L, const LayerDim& ld) {
  if (nb == 1) {
    const int cap = resident_blocks(score_pipelined_kernel<DTYPE, PB, true>, lds);
    if (blocks > static_cast<unsigned>(cap)) blocks = cap;
    hipLaunchKernelGGL((score_pipelined_kernel<DTYPE, PB, true>), dim3(blocks, L), dim3(kScoreThreads), lds, s, hidden, w,
                       bias, N, d, nb, row_stride, scores, ld);
  } else {
    const int cap = resident_blocks(score_pipelined_kernel<DTYPE, PB, false>, lds);
    if (blocks > static_cast<unsigned>(cap)) blocks = cap;
    hipLaunchKernelGGL((score_pipelined_kernel<DTYPE, PB, false>), dim3(blocks, L), dim3(kScoreThreads), lds, s, hidden, w,
                       bias, N, d, nb, row_stride, scores, ld);
  }
}

template <int DTYPE>
bool try_pipelined(const void* hidden, const void* w, float bias, int64_t N, int d, int64_t row_stride, float* scores,
                   unsigned blocks, size_t lds, hipStream_t s, int L, const LayerDim& ld) {
  constexpr int kChunk = kWave * Elems<DTYPE>::kPerLoad;
  if (d % kChunk != 0) return false;
  const int chunks = d / kChunk;
  const int nb = (chunks + kUnroll - 1) / kUnroll;
  if (chunks % nb != 0) return false;
  const int pb = chunks / nb;
  switch (pb) {
    case 1: launch_pipelined<DTYPE, 1>(hidden, w, bias, N, d, nb, row_stride, scores, blocks, lds, s, L, ld); return true;
    case 2: launch_pipelined<DTYPE, 2>(hidden, w, bias, N, d, nb, row_stride, scores, blocks, lds, s, L, ld); return true;
    case 3: launch_pipelined<DTYPE, 3>(hidden, w, bias, N, d, nb, row_stride, scores, blocks, lds, s, L, ld); return true;
    case 4: launch_pipelined<DTYPE, 4>(hidden, w, bias, N, d, nb, row_stride, scores, blocks, lds, s, L, ld); return true;
    case 5: launch_pipelined<DTYPE, 5>(hidden, w, bias, N, d, nb, row_stride, scores, blocks, lds, s, L, ld); return true;
    case 6: launch_pipelined<DTYPE, 6>(hidden, w, bias, N, d, nb, row_stride, scores, blocks, lds, s, L, ld); return true;
    case 7: launch_pipelined<DTYPE, 7>(hidden, w, bias, N, d, nb, row_stride, scores, blocks, lds, s, L, ld); return true;
    case 8: launch_pipelined<DTYPE, 8>(hidden, w, bias, N, d, nb, row_stride, scores, blocks, lds, s, L, ld); return true;
    default: return false;
  }
}

}  // namespace
}  // namespace dodo

namespace dodo {
namespace {

int score_entry(const void* hidden, const void* w, float bias, int dtype, int64_t N, int32_t d, int64_t row_stride,
                float* scores, int32_t L, const LayerDim& ld, void* stream) {
  if (N < 0 || d <= 0 || row_stride < d || L < 0) return DODO_ERR_INVALID_ARG;
  if (N == 0 || L == 0) return DODO_OK;
  if (!hidden || !w || !scores) return DODO_ERR_INVALID_ARG;
  if (!dtype_ok(dtype)) return DODO_ERR_UNSUPPORTED;
  const int es = elem_bytes(dtype);
  if (d % 8 != 0 || d > 16384 || L > 65535) return DODO_ERR_UNSUPPORTED;
  if (!aligned16(hidden) || (row_stride * es) % 16 != 0 || (ld.hidden_ls * es) % 16 != 0) return DODO_ERR_UNSUPPORTED;

  const int waves_per_block = kScoreThreads / kWave;
  int64_t blocks = (N + waves_per_block - 1) / waves_per_block;
  const int64_t cap = 256 * 8;  // upper bound; each kernel trims it to what is resident at once
  if (blocks > cap) blocks = cap;
  const size_t lds = static_cast<size_t>(d) * sizeof(float);
  hipStream_t s = static_cast<hipStream_t>(stream);
  // widths that split evenly into batches of wave-wide loads (4096, 5120, 8192, ...) take the pipelined kernel
  const unsigned nblk = static_cast<unsigned>(blocks);
  if (dtype == DODO_DTYPE_BF16
          ? try_pipelined<DODO_DTYPE_BF16>(hidden, w, bias, N, d, row_stride, scores, nblk, lds, s, L, ld)
          : try_pipelined<DODO_DTYPE_F32>(hidden, w, bias, N, d, row_stride, scores, nblk, lds, s, L, ld))
    return launch_status();
  if (dtype == DODO_DTYPE_BF16) {
    const int64_t fit = resident_blocks(score_kernel<DODO_DTYPE_BF16>, lds);
    hipLaunchKernelGGL(score_kernel<DODO_DTYPE_BF16>, dim3(static_cast<unsigned>(blocks < fit ? blocks : fit), L),
                       dim3(kScoreThreads), lds, s, hidden, w, bias, N, d, row_stride, scores, ld);
  } else {
    const int64_t fit = resident_blocks(score_kernel<DODO_DTYPE_F32>, lds);
    hipLaunchKernelGGL(score_kernel<DODO_DTYPE_F32>, dim3(static_cast<unsigned>(blocks < fit ? blocks : fit), L),
                       dim3(kScoreThreads), lds, s, hidden, w, bias, N, d, row_stride, scores, ld);
  }
  return launch_status();
}

}  // namespace
}  // namespace dodo

extern "C" int dodo_score(const void* hidden, const void* w, float bias, int dtype, int64_t N, int32_t d,
                          int64_t row_stride, float* scores, void* stream) {
  return dodo::score_entry(hidden, w, bias, dtype, N, d, row_stride, scores, 1, dodo::LayerDim{0, 0, 0, nullptr}, stream);
}

extern "C" int dodo_score_layers(const void* hidden, const void* w, const float* biases, int dtype, int32_t L, int64_t N,
                                 int32_t d, int64_t row_stride, int64_t hidden_layer_stride, int64_t w_layer_stride,
                                 int64_t scores_layer_stride, float* scores, void* stream) {
  if (hidden_layer_stride < 0 || w_layer_stride < 0 || scores_layer_stride < 0) return DODO_ERR_INVALID_ARG;
  if (L > 1 && scores_layer_stride < N) return DODO_ERR_INVALID_ARG;
  return dodo::score_entry(hidden, w, 0.f, dtype, N, d, row_stride, scores, L,
                           dodo::LayerDim{hidden_layer_stride, w_layer_stride, scores_layer_stride, biases}, stream);
}
