// Selection of the autoregressive mode (Sec. 2.4 of the Dodo paper): a token is
// kept as a nugget if its score exceeds a threshold Lambda (Eq. 8), which does
// not look at later tokens.
//   dodo_threshold_from_sample  Lambda from a sample of scores: the (k+1)-th
//                               highest, k = nugget count of the sample size
//   dodo_select_threshold       kept tokens of whole sequences as packed index
//                               lists (same format as the TopK selection)
//   dodo_stream_append          one decode step: the token that leaves the
//                               window of uncompressed tokens is appended to
//                               its sequence's nugget cache if it is kept
// Integer and copy work only: results are unique and bit-exact.
#include "dodo_common.h"

namespace dodo {
namespace {

constexpr int kSampleThreads = 1024;
constexpr int kSampleBatch = 8;
constexpr int kThreshThreads = 1024;
constexpr int kThreshBatch = 4;  // 64-token groups per wavefront with their loads in flight together
constexpr int kAppendThreads = 256;

// Inverse of order_key on non-NaN keys.
__device__ __forceinline__ float key_to_score(uint32_t key) {
  if (key == 0u) return -__builtin_inff();  // NaN ranks lowest: everything that can be kept is kept
  return __uint_as_float((key & 0x80000000u) ? (key ^ 0x80000000u) : ~key);
}

// Key of the `rank`-th highest of n scores (1 <= rank <= n) by a 4-pass, 8-bit MSB radix select;
// one workgroup, the scores are re-read from global memory in every pass (they sit in L2).  For small samples,
// and for callers without a workspace; larger ones take the multi-workgroup form below.
__global__ __launch_bounds__(kSampleThreads) void kth_highest_kernel(const float* __restrict__ sample, int64_t n,
                                                                     int64_t rank, float* __restrict__ lambda_out) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t s_prefix;
  __shared__ unsigned long long s_remaining;
  const int tid = threadIdx.x, lane = lane_id(), wave = tid / kWave;
  uint32_t prefix = 0, mask = 0;
  unsigned long long remaining = static_cast<unsigned long long>(rank);
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    for (int i = tid; i < 256; i += kSampleThreads) hist[i] = 0;
    __syncthreads();
    // kSampleBatch 64-score groups per wavefront and iteration, their loads in flight together (the pass is bound
    // by the latency of these loads)
    for (int64_t i0 = static_cast<int64_t>(wave) * kWave * kSampleBatch; i0 < n; i0 += kSampleThreads * kSampleBatch) {
      float v[kSampleBatch];
#pragma unroll
      for (int u = 0; u < kSampleBatch; ++u) {
        const int64_t i = i0 + u * kWave + lane;
        v[u] = sample[i < n ? i : n - 1];
      }
#pragma unroll
      for (int u = 0; u < kSampleBatch; ++u) {
        const int64_t i = i0 + u * kWave + lane;
        const uint32_t key = order_key(v[u]);
        bool part = (i < n) && ((key & mask) == prefix);
        const uint32_t digit = (key >> shift) & 255u;
        // two rounds of wavefront aggregation absorb the hot bins, the rest goes lane by lane
#pragma unroll
        for (int round = 0; round < 2; ++round) {
          const uint64_t act = __ballot(part);
          if (act != 0) {
            const int leader = __ffsll(static_cast<long long>(act)) - 1;
            const uint32_t d0 = __builtin_amdgcn_readlane(digit, leader);
            const bool same = part && digit == d0;
            const uint64_t mm = __ballot(same);
            if (lane == leader) atomicAdd(&hist[d0], static_cast<uint32_t>(__popcll(mm)));
            part = part && !same;
          }
        }
        if (part) atomicAdd(&hist[digit], 1u);
      }
    }
    __syncthreads();
    if (tid == 0) {  // 256 bins, once per pass: a plain scan from the top
      unsigned long long above = 0;
      int d = 255;
      for (; d > 0; --d) {
        if (above + hist[d] >= remaining) break;
        above += hist[d];
      }
      s_prefix = prefix | (static_cast<uint32_t>(d) << shift);
      s_remaining = remaining - above;
    }
    __syncthreads();
    prefix = s_prefix;
    remaining = s_remaining;
    mask |= 255u << shift;
  }
  if (tid == 0) *lambda_out = key_to_score(prefix);
}

// The same selection with many workgroups, one launch per radix pass: every workgroup reads the histograms of the
// passes before (global, complete: they were made by earlier launches), derives the prefix and the remaining rank
// from them -- all workgroups the same -- and adds the histogram of its own part of the sample to the pass's
// global bins.  hist: 4 x 256 counters, cleared by the first launch's predecessor.
constexpr int kPassSampleThreads = 1024;
constexpr int kPassKeysPerBlock = 16384;

// Called by one whole wavefront: lane l owns bins 4l .. 4l+3 of every pass; the digit of a pass is where the
// count from the top reaches the remaining rank.  All lanes return the same values.
__device__ __forceinline__ void prefix_from_histograms(const uint32_t* hist_lds, int n_pass, unsigned long long rank,
                                                       uint32_t* prefix_out, uint32_t* mask_out,
                                                       unsigned long long* remaining_out) {
  const int lane = lane_id();
  uint32_t prefix = 0, mask = 0;
  unsigned long long remaining = rank;
  for (int p = 0; p < n_pass; ++p) {
    const int shift = 24 - 8 * p;
    const uint32_t b0 = hist_lds[256 * p + 4 * lane], b1 = hist_lds[256 * p + 4 * lane + 1],
                   b2 = hist_lds[256 * p + 4 * lane + 2], b3 = hist_lds[256 * p + 4 * lane + 3];
    unsigned long long suf = static_cast<unsigned long long>(b0) + b1 + b2 + b3;  // inclusive suffix sum over lanes
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const unsigned long long t = __shfl_down(suf, off, kWave);
      if (lane + off < kWave) suf += t;
    }
    const uint64_t ge = __ballot(suf >= remaining);
    // ge is empty only if the rank exceeds the sample size (excluded by the caller): then the lowest bin is taken
    const int L = ge != 0 ? 63 - __clzll(static_cast<long long>(ge)) : 0;
    unsigned long long above = suf - (static_cast<unsigned long long>(b0) + b1 + b2 + b3);  // counts in bins above this lane's
    int dsel = 0;
    if (above + b3 >= remaining) {
      dsel = 3;
    } else if (above + b3 + b2 >= remaining) {
      dsel = 2;
      above += b3;
    } else if (above + b3 + b2 + b1 >= remaining) {
      dsel = 1;
      above += static_cast<unsigned long long>(b3) + b2;
    } else {
      above += static_cast<unsigned long long>(b3) + b2 + b1;
    }
    const int digit = __shfl(4 * lane + dsel, L, kWave);
    const unsigned long long above_sel = __shfl(above, L, kWave);
    prefix |= static_cast<uint32_t>(digit) << shift;
    mask |= 255u << shift;
    remaining -= above_sel;
  }
  *prefix_out = prefix;
  *mask_out = mask;
  *remaining_out = remaining;
}

__global__ void clear_hist_kernel(uint32_t* hist) { hist[threadIdx.x] = 0; }

__global__ __launch_bounds__(kPassSampleThreads) void kth_pass_kernel(const float* __restrict__ sample, int64_t n,
                                                                      int64_t rank, int pass,
                                                                      uint32_t* __restrict__ hist_global) {
  __shared__ uint32_t prev[3 * 256];
  __shared__ uint32_t hist[256];
  __shared__ uint32_t s_prefix, s_mask;
  const int tid = threadIdx.x, lane = lane_id();
  for (int i = tid; i < 256 * pass; i += kPassSampleThreads) prev[i] = hist_global[i];
  for (int i = tid; i < 256; i += kPassSampleThreads) hist[i] = 0;
  __syncthreads();
  if (tid < kWave) {
    uint32_t prefix, mask;
    unsigned long long remaining;
    prefix_from_histograms(prev, pass, static_cast<unsigned long long>(rank), &prefix, &mask, &remaining);
    if (tid == 0) {
      s_prefix = prefix;
      s_mask = mask;
    }
  }
  __syncthreads();
  const uint32_t prefix = s_prefix, mask = s_mask;
  const int shift = 24 - 8 * pass;
  const int64_t lo = static_cast<int64_t>(blockIdx.x) * kPassKeysPerBlock;
  const int64_t hi = min(lo + kPassKeysPerBlock, n);
  constexpr int kBatch = 4;
  for (int64_t i0 = lo + tid; i0 < hi; i0 += kPassSampleThreads * kBatch) {
    float v[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int64_t i = i0 + u * kPassSampleThreads;
      v[u] = sample[i < hi ? i : hi - 1];
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int64_t i = i0 + u * kPassSampleThreads;
      const uint32_t key = order_key(v[u]);
      bool part = (i < hi) && ((key & mask) == prefix);
      const uint32_t digit = (key >> shift) & 255u;
#pragma unroll
      for (int round = 0; round < 2; ++round) {  // wavefront aggregation of the hot bins, as in the one-workgroup kernel
        const uint64_t act = __ballot(part);
        if (act != 0) {
          const int leader = __ffsll(static_cast<long long>(act)) - 1;
          const uint32_t d0 = __builtin_amdgcn_readlane(digit, leader);
          const bool same = part && digit == d0;
          const uint64_t mm = __ballot(same);
          if (lane == leader) atomicAdd(&hist[d0], static_cast<uint32_t>(__popcll(mm)));
          part = part && !same;
        }
      }
      if (part) atomicAdd(&hist[digit], 1u);
    }
  }
  __syncthreads();
  for (int i = tid; i < 256; i += kPassSampleThreads) {
    const uint32_t c = hist[i];
    if (c != 0) atomicAdd(&hist_global[256 * pass + i], c);
  }
}

__global__ __launch_bounds__(256) void kth_final_kernel(const uint32_t* __restrict__ hist_global, int64_t rank,
                                                        float* __restrict__ lambda_out) {
  __shared__ uint32_t prev[4 * 256];
  for (int i = threadIdx.x; i < 4 * 256; i += 256) prev[i] = hist_global[i];
  __syncthreads();
  if (threadIdx.x < kWave) {
    uint32_t prefix, mask;
    unsigned long long remaining;
    prefix_from_histograms(prev, 4, static_cast<unsigned long long>(rank), &prefix, &mask, &remaining);
    if (threadIdx.x == 0) *lambda_out = key_to_score(prefix);
  }
}

__global__ void fill_float_kernel(float* p, float v) { *p = v; }

// Stable compaction of { i : scores[i] > lambda } of one sequence per workgroup.
// COUNT_ONLY: counts[b] only.  Otherwise the workgroup finds its place in the packed list by
// summing the counts of the sequences before it, writes its indices there and cu_nuggets[b + 1].
template <bool COUNT_ONLY>
__global__ __launch_bounds__(kThreshThreads) void select_threshold_kernel(
    const float* __restrict__ scores, const int32_t* __restrict__ cu_seqlens, const float* __restrict__ lambda, int B,
    int32_t* __restrict__ counts, int32_t* __restrict__ cu_nuggets, int32_t* __restrict__ nugget_idx) {
  constexpr int kWaves = kThreshThreads / kWave;
  __shared__ int wave_cnt[kWaves];
  __shared__ int s_base;
  const int b = blockIdx.x;
  const int tid = threadIdx.x, lane = lane_id(), wave = tid / kWave;
  const int seq0 = cu_seqlens[b];
  const int n = cu_seqlens[b + 1] - seq0;
  const float lam = *lambda;
  const float* s = scores + seq0;
  // contiguous per-wavefront ranges keep the output in position order
  const int per_wave = ((n + kWaves * kWave - 1) / (kWaves * kWave)) * kWave;
  const int start = wave * per_wave;
  const int end = min(start + per_wave, n);
  int cnt = 0;
  for (int i0 = start; i0 < end; i0 += kWave * kThreshBatch) {
    float v[kThreshBatch];
#pragma unroll
    for (int u = 0; u < kThreshBatch; ++u) {
      const int i = i0 + u * kWave + lane;
      v[u] = s[i < end ? i : end - 1];  // unconditional loads: all in flight before the first use
    }
#pragma unroll
    for (int u = 0; u < kThreshBatch; ++u) {
      const int i = i0 + u * kWave + lane;
      cnt += __popcll(__ballot(i < end && v[u] > lam));  // false for NaN
    }
  }
  if (lane == 0) wave_cnt[wave] = cnt;
  if (!COUNT_ONLY && tid == 0) {
    int base = 0;
    for (int bb = 0; bb < b; ++bb) base += counts[bb];
    s_base = base;
  }
  __syncthreads();
  int total = 0, before = 0;
  for (int w = 0; w < kWaves; ++w) {
    if (w < wave) before += wave_cnt[w];
    total += wave_cnt[w];
  }
  if (COUNT_ONLY) {
    if (tid == 0) counts[b] = total;
    return;
  }
  int out_at = s_base + before;
  for (int i0 = start; i0 < end; i0 += kWave * kThreshBatch) {
    float v[kThreshBatch];
#pragma unroll
    for (int u = 0; u < kThreshBatch; ++u) {
      const int i = i0 + u * kWave + lane;
      v[u] = s[i < end ? i : end - 1];
    }
#pragma unroll
    for (int u = 0; u < kThreshBatch; ++u) {
      const int i = i0 + u * kWave + lane;
      const bool keep = i < end && v[u] > lam;
      const uint64_t km = __ballot(keep);
      if (keep) nugget_idx[out_at + popc_below_lane(km)] = i;
      out_at += __popcll(km);
    }
  }
  if (tid == 0) {
    cu_nuggets[b + 1] = s_base + total;
    if (b == 0) cu_nuggets[0] = 0;
  }
}

// One workgroup per sequence: append the leaving token's K and V rows if its score exceeds lambda.
__global__ __launch_bounds__(kAppendThreads) void stream_append_kernel(
    const float* __restrict__ scores, const float* __restrict__ lambda, const uint4* __restrict__ K_rows,
    const uint4* __restrict__ V_rows, int64_t row_stride_vec, int vec_per_row, int cap, int32_t* __restrict__ counts,
    int32_t* __restrict__ dropped, uint4* __restrict__ Kn, uint4* __restrict__ Vn) {
  const int b = blockIdx.x;
  if (!(scores[b] > *lambda)) return;  // uniform over the workgroup
  const int at = counts[b];
  if (at >= cap) {
    if (threadIdx.x == 0 && dropped != nullptr) atomicAdd(dropped, 1);
    return;
  }
  const uint4* ks = K_rows + b * row_stride_vec;
  const uint4* vs = V_rows + b * row_stride_vec;
  const int64_t dst = (static_cast<int64_t>(b) * cap + at) * vec_per_row;
  for (int c = threadIdx.x; c < vec_per_row; c += kAppendThreads) {
    Kn[dst + c] = ks[c];
    Vn[dst + c] = vs[c];
  }
  __syncthreads();  // every thread has read counts[b]
  if (threadIdx.x == 0) counts[b] = at + 1;
}

}  // namespace
}  // namespace dodo

extern "C" size_t dodo_threshold_from_sample_workspace_bytes(int64_t n) {
  return n > dodo::kPassKeysPerBlock ? 4 * 256 * sizeof(uint32_t) : 0;
}

extern "C" int dodo_threshold_from_sample(const float* sample, int64_t n, int64_t num, int64_t den, float* lambda_out,
                                          void* ws, size_t ws_bytes, void* stream) {
  using namespace dodo;
  if (n <= 0 || num <= 0 || den <= 0) return DODO_ERR_INVALID_ARG;
  if (!sample || !lambda_out) return DODO_ERR_INVALID_ARG;
  const int64_t k = dodo_nugget_count(n, num, den);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t need = dodo_threshold_from_sample_workspace_bytes(n);
  if (k >= n) {
    hipLaunchKernelGGL(fill_float_kernel, dim3(1), dim3(1), 0, s, lambda_out, -__builtin_inff());
  } else if (need > 0 && ws != nullptr && ws_bytes >= need && (reinterpret_cast<uintptr_t>(ws) & 3u) == 0 &&
             (n + kPassKeysPerBlock - 1) / kPassKeysPerBlock <= 0x7fffffffLL) {
    // large samples, given the workspace: one launch per radix pass over many workgroups
    uint32_t* hist = static_cast<uint32_t*>(ws);
    const unsigned blocks = static_cast<unsigned>((n + kPassKeysPerBlock - 1) / kPassKeysPerBlock);
    hipLaunchKernelGGL(clear_hist_kernel, dim3(1), dim3(4 * 256), 0, s, hist);
    for (int pass = 0; pass < 4; ++pass)
      hipLaunchKernelGGL(kth_pass_kernel, dim3(blocks), dim3(kPassSampleThreads), 0, s, sample, n, k + 1, pass, hist);
    hipLaunchKernelGGL(kth_final_kernel, dim3(1), dim3(256), 0, s, hist, k + 1, lambda_out);
  } else {
    hipLaunchKernelGGL(kth_highest_kernel, dim3(1), dim3(kSampleThreads), 0, s, sample, n, k + 1, lambda_out);
  }
  return launch_status();
}

extern "C" int dodo_select_threshold(const float* scores, const int32_t* cu_seqlens, int32_t B, const float* lambda,
                                     int32_t* counts, int32_t* cu_nuggets, int32_t* nugget_idx, void* stream) {
  using namespace dodo;
  if (B < 0) return DODO_ERR_INVALID_ARG;
  if (B == 0) return DODO_OK;
  if (!scores || !cu_seqlens || !lambda || !counts || !cu_nuggets || !nugget_idx) return DODO_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(select_threshold_kernel<true>, dim3(B), dim3(kThreshThreads), 0, s, scores, cu_seqlens, lambda, B,
                     counts, cu_nuggets, nugget_idx);
  int rc = launch_status();
  if (rc != DODO_OK) return rc;
  hipLaunchKernelGGL(select_threshold_kernel<false>, dim3(B), dim3(kThreshThreads), 0, s, scores, cu_seqlens, lambda, B,
                     counts, cu_nuggets, nugget_idx);
  return launch_status();
}

extern "C" int dodo_stream_append(const float* scores, const float* lambda, const void* K_rows, const void* V_rows,
                                  int dtype, int32_t B, int32_t H_kv, int32_t d_h, int64_t row_stride, int32_t cap,
                                  int32_t* counts, int32_t* dropped, void* Kn, void* Vn, void* stream) {
  using namespace dodo;
  if (B < 0 || H_kv <= 0 || d_h <= 0 || cap < 0) return DODO_ERR_INVALID_ARG;
  if (row_stride < static_cast<int64_t>(H_kv) * d_h) return DODO_ERR_INVALID_ARG;
  if (B == 0) return DODO_OK;
  if (!scores || !lambda || !K_rows || !V_rows || !counts || !Kn || !Vn) return DODO_ERR_INVALID_ARG;
  if (!dtype_ok(dtype)) return DODO_ERR_UNSUPPORTED;
  const int es = elem_bytes(dtype);
  if ((static_cast<int64_t>(H_kv) * d_h * es) % 16 != 0 || (row_stride * es) % 16 != 0) return DODO_ERR_UNSUPPORTED;
  if (!aligned16(K_rows) || !aligned16(V_rows) || !aligned16(Kn) || !aligned16(Vn)) return DODO_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(stream_append_kernel, dim3(B), dim3(kAppendThreads), 0, static_cast<hipStream_t>(stream), scores,
                     lambda, static_cast<const uint4*>(K_rows), static_cast<const uint4*>(V_rows), row_stride * es / 16,
                     H_kv * d_h * es / 16, cap, counts, dropped, static_cast<uint4*>(Kn), static_cast<uint4*>(Vn));
  return launch_status();
}
