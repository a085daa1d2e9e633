// dodo_select_topk: per-sequence TopK of the scorer output (Eq. 14 of the Dodo
// paper) plus the ordered, segmented compaction that writes the nugget index
// lists.  Integer work only, so the result is unique and bit-exact:
//   1. every fp32 score becomes an order-preserving uint32 key (NaN lowest,
//      -0 == +0), staged in LDS when the sequence fits (<= 36864 tokens);
//   2. a 4-pass, 8-bit MSB radix select finds the key T of the k-th best token
//      and how many tokens equal to T are still needed; after the first pass
//      the tokens that share the chosen top byte are collected in a list (if
//      they are few enough), so that the other three passes touch only those;
//   3. a stable compaction emits, in ascending position order, every token
//      with key > T and the first `need` tokens with key == T (lowest index
//      wins ties).
// One workgroup per sequence; histograms use LDS integer atomics with a
// wavefront-level pre-aggregation so that heavy ties do not serialise.
#include "dodo_common.h"

namespace dodo {
namespace {

constexpr int kStagedMaxKeys = 34 * 1024;  // 136 KiB of the 160 KiB LDS
constexpr int kCandCap = 8192;             // candidate list after the first pass: 16-bit positions, 16 KiB

__device__ __forceinline__ uint32_t order_key(float s) {
  uint32_t u = __float_as_uint(s);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;  // NaN ranks below everything
  if (u == 0x80000000u) u = 0u;                    // -0 == +0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

template <int THREADS, bool STAGED>
__global__ __launch_bounds__(THREADS) void select_topk_kernel(const float* __restrict__ scores,
                                                              const int32_t* __restrict__ cu_seqlens,
                                                              const int32_t* __restrict__ cu_nuggets, uint32_t flags,
                                                              int max_n, int32_t* __restrict__ nugget_idx) {
  constexpr int kWaves = THREADS / kWave;
  extern __shared__ uint32_t keys_lds[];  // max_n keys, then kCandCap 16-bit positions (STAGED only)
  __shared__ uint32_t hist[256];
  __shared__ uint32_t s_prefix, s_remaining, s_cand;
  __shared__ int wave_gt[kWaves], wave_eq[kWaves];

  const int b = blockIdx.x;
  const int tid = threadIdx.x, lane = lane_id(), wave = tid / kWave;
  const int seq0 = cu_seqlens[b];
  const int n = cu_seqlens[b + 1] - seq0;
  const int nug0 = cu_nuggets[b];
  int k = cu_nuggets[b + 1] - nug0;
  if (k <= 0 || n <= 0 || n > max_n) return;  // uniform over the workgroup
  if (k > n) k = n;
  const bool force = (flags & DODO_TOPK_FORCE_LAST) != 0;
  const int n_free = force ? n - 1 : n;  // tokens that compete on score
  const int k_free = force ? k - 1 : k;
  const float* s = scores + seq0;
  int32_t* out = nugget_idx + nug0;

  if (k_free > 0) {
    if (STAGED) {
      // batches of 8 loads in flight per thread: one global-memory latency per batch, not per key
      constexpr int kBatch = 8;
      for (int i0 = tid; i0 < n_free; i0 += THREADS * kBatch) {
        float v[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
          const int i = i0 + u * THREADS;
          v[u] = s[i < n_free ? i : n_free - 1];
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
          const int i = i0 + u * THREADS;
          if (i < n_free) keys_lds[i] = order_key(v[u]);
        }
      }
      __syncthreads();
    }
    auto key_at = [&](int i) -> uint32_t { return STAGED ? keys_lds[i] : order_key(s[i]); };

    // ---- radix select: key of the k_free-th best token ----
    // One pass: histogram of the pass's digit over the items that still match the prefix, then the
    // digit that holds the `remaining`-th largest.  An item is a token (first pass, or no list) or
    // an entry of the candidate list.
    uint32_t prefix = 0, mask = 0, remaining = static_cast<uint32_t>(k_free);
    auto radix_pass = [&](int shift, int n_items, auto item_key) {
      for (int i = tid; i < 256; i += THREADS) hist[i] = 0;
      __syncthreads();
      // four independent 64-item chunks per iteration, so that their dependency chains overlap
      constexpr int kChunks = 4;
      for (int i0 = wave * kWave * kChunks; i0 < n_items; i0 += THREADS * kChunks) {
        uint32_t digit[kChunks];
        bool part[kChunks];
#pragma unroll
        for (int u = 0; u < kChunks; ++u) {
          const int i = i0 + u * kWave + lane;
          const uint32_t key = (i < n_items) ? item_key(i) : 0u;
          part[u] = (i < n_items) && ((key & mask) == prefix);
          digit[u] = (key >> shift) & 255u;
        }
        // two rounds of wavefront aggregation absorb the hot bins (ties, shared exponents)
#pragma unroll
        for (int round = 0; round < 2; ++round) {
#pragma unroll
          for (int u = 0; u < kChunks; ++u) {
            const uint64_t act = __ballot(part[u]);
            if (act != 0) {
              const int leader = __ffsll(static_cast<long long>(act)) - 1;
              const uint32_t d0 = __builtin_amdgcn_readlane(digit[u], leader);
              const bool same = part[u] && digit[u] == d0;
              const uint64_t mm = __ballot(same);
              if (lane == leader) atomicAdd(&hist[d0], static_cast<uint32_t>(__popcll(mm)));
              part[u] = part[u] && !same;
            }
          }
        }
#pragma unroll
        for (int u = 0; u < kChunks; ++u)
          if (part[u]) atomicAdd(&hist[digit[u]], 1u);
      }
      __syncthreads();
      if (wave == 0) {
        // lane l owns bins 4l..4l+3; inclusive suffix sum over lanes
        const uint32_t b0 = hist[4 * lane], b1 = hist[4 * lane + 1], b2 = hist[4 * lane + 2], b3 = hist[4 * lane + 3];
        uint32_t suf = b0 + b1 + b2 + b3;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
          const uint32_t t = __shfl_down(suf, off, kWave);
          if (lane + off < kWave) suf += t;
        }
        const uint64_t ge = __ballot(suf >= remaining);  // non-empty: suf(lane 0) = #candidates >= remaining
        const int L = 63 - __clzll(static_cast<long long>(ge));
        if (lane == L) {
          uint32_t above = suf - (b0 + b1 + b2 + b3);  // candidates in bins above this lane's
          int dsel;
          uint32_t in_bin;
          if (above + b3 >= remaining) {
            dsel = 3;
            in_bin = b3;
          } else if (above + b3 + b2 >= remaining) {
            dsel = 2;
            above += b3;
            in_bin = b2;
          } else if (above + b3 + b2 + b1 >= remaining) {
            dsel = 1;
            above += b3 + b2;
            in_bin = b1;
          } else {
            dsel = 0;
            above += b3 + b2 + b1;
            in_bin = b0;
          }
          s_prefix = prefix | (static_cast<uint32_t>(4 * L + dsel) << shift);
          s_remaining = remaining - above;
          s_cand = in_bin;  // items that carry the chosen digit
        }
      }
      __syncthreads();
      prefix = s_prefix;
      remaining = s_remaining;
      mask |= 255u << shift;
    };
    radix_pass(24, n_free, key_at);
    const int n_cand = static_cast<int>(s_cand);
    if (STAGED && n_cand <= kCandCap) {
      // positions of the tokens that share the chosen top byte, in any order
      uint16_t* cand = reinterpret_cast<uint16_t*>(keys_lds + max_n);
      __syncthreads();  // everyone has read s_cand
      if (tid == 0) s_cand = 0;
      __syncthreads();
      for (int i0 = wave * kWave; i0 < n_free; i0 += THREADS) {
        const int i = i0 + lane;
        const bool is_c = i < n_free && (keys_lds[i] & mask) == prefix;
        const uint64_t cm = __ballot(is_c);
        if (cm != 0) {
          const int leader = __ffsll(static_cast<long long>(cm)) - 1;
          uint32_t base = 0;
          if (lane == leader) base = atomicAdd(&s_cand, static_cast<uint32_t>(__popcll(cm)));
          base = __builtin_amdgcn_readlane(base, leader);
          const uint32_t at = base + popc_below_lane(cm);
          if (is_c && at < static_cast<uint32_t>(kCandCap)) cand[at] = static_cast<uint16_t>(i);  // at < n_cand always
        }
      }
      __syncthreads();
      auto cand_key = [&](int c) -> uint32_t { return keys_lds[cand[c]]; };
      for (int pass = 1; pass < 4; ++pass) radix_pass(24 - 8 * pass, n_cand, cand_key);
    } else {
      for (int pass = 1; pass < 4; ++pass) radix_pass(24 - 8 * pass, n_free, key_at);
    }
    const uint32_t T = prefix;                        // key of the k_free-th best token
    const int need_eq = static_cast<int>(remaining);  // tokens equal to T still to take, lowest index first

    // ---- stable compaction over contiguous per-wavefront ranges ----
    const int per_wave = ((n_free + kWaves * kWave - 1) / (kWaves * kWave)) * kWave;
    const int start = wave * per_wave;
    const int end = min(start + per_wave, n_free);
    int cnt_gt = 0, cnt_eq = 0;
    for (int i0 = start; i0 < end; i0 += kWave) {
      const int i = i0 + lane;
      const uint32_t key = (i < end) ? key_at(i) : 0u;
      cnt_gt += __popcll(__ballot(i < end && key > T));
      cnt_eq += __popcll(__ballot(i < end && key == T));
    }
    if (lane == 0) {
      wave_gt[wave] = cnt_gt;
      wave_eq[wave] = cnt_eq;
    }
    __syncthreads();
    int eq_base = 0, out_base = 0;
    for (int w = 0; w < wave; ++w) {
      const int e = wave_eq[w];
      out_base += wave_gt[w] + max(0, min(e, need_eq - eq_base));
      eq_base += e;
    }
    for (int i0 = start; i0 < end; i0 += kWave) {
      const int i = i0 + lane;
      const uint32_t key = (i < end) ? key_at(i) : 0u;
      const bool is_eq = i < end && key == T;
      const uint64_t eq_mask = __ballot(is_eq);
      const bool sel = (i < end && key > T) || (is_eq && eq_base + popc_below_lane(eq_mask) < need_eq);
      const uint64_t sel_mask = __ballot(sel);
      const int pos = out_base + popc_below_lane(sel_mask);
      if (sel && pos < k_free) out[pos] = i;  // pos < k_free always holds; the test keeps a logic slip in bounds
      eq_base += __popcll(eq_mask);
      out_base += __popcll(sel_mask);
    }
  }
  if (force && tid == 0) out[k - 1] = n - 1;
}

template <int THREADS>
int launch_select(const float* scores, const int32_t* cu_seqlens, const int32_t* cu_nuggets, int32_t B, int32_t max_n,
                  uint32_t flags, int32_t* nugget_idx, hipStream_t stream) {
  if (max_n <= kStagedMaxKeys) {
    const size_t lds = static_cast<size_t>(max_n) * sizeof(uint32_t) + kCandCap * sizeof(uint16_t);
    auto kern = select_topk_kernel<THREADS, true>;
    if (lds > 48 * 1024) {
      DODO_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       static_cast<int>(lds)));
    }
    hipLaunchKernelGGL(kern, dim3(B), dim3(THREADS), lds, stream, scores, cu_seqlens, cu_nuggets, flags, max_n,
                       nugget_idx);
  } else {
    hipLaunchKernelGGL((select_topk_kernel<THREADS, false>), dim3(B), dim3(THREADS), 0, stream, scores, cu_seqlens,
                       cu_nuggets, flags, max_n, nugget_idx);
  }
  return launch_status();
}

}  // namespace
}  // namespace dodo

extern "C" size_t dodo_select_topk_workspace_bytes(int32_t B, int32_t max_n) {
  (void)B;
  (void)max_n;
  return 0;  // keys live in LDS (or are re-read from the score array); no global scratch
}

extern "C" int dodo_select_topk(const float* scores, const int32_t* cu_seqlens, const int32_t* cu_nuggets, int32_t B,
                                int32_t max_n, int32_t max_k, uint32_t flags, int32_t* nugget_idx, void* ws,
                                size_t ws_bytes, void* stream) {
  using namespace dodo;
  (void)ws;
  (void)ws_bytes;
  if (B < 0) return DODO_ERR_INVALID_ARG;
  if (B == 0) return DODO_OK;
  if (!scores || !cu_seqlens || !cu_nuggets || !nugget_idx) return DODO_ERR_INVALID_ARG;
  if (max_n <= 0 || max_k <= 0 || max_k > max_n) return DODO_ERR_INVALID_ARG;
  if (flags & ~DODO_TOPK_FORCE_LAST) return DODO_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // about four keys per thread: the kernel is latency-bound (few barriers matter more than lanes)
  if (max_n <= 1024) return launch_select<256>(scores, cu_seqlens, cu_nuggets, B, max_n, flags, nugget_idx, s);
  if (max_n <= 2048) return launch_select<512>(scores, cu_seqlens, cu_nuggets, B, max_n, flags, nugget_idx, s);
  return launch_select<1024>(scores, cu_seqlens, cu_nuggets, B, max_n, flags, nugget_idx, s);
}
