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
// Long sequences (given a workspace) are cut into chunks with a workgroup
// each: the chunks' histograms of a pass are added up in the workspace, every
// workgroup waits until all have contributed (bounded) and then picks the
// digit from the same totals; the compaction hands out output offsets and the
// tie budget in chunk (= position) order in the same way.  The result is the
// same bit for bit; one compute unit's instruction issue no longer bounds it.
#include "dodo_common.h"

namespace dodo {
namespace {

constexpr int kStagedMaxKeys = 34 * 1024;  // 136 KiB of the 160 KiB LDS
constexpr int kCandCap = 8192;             // candidate list after the first pass: 16-bit positions, 16 KiB
constexpr int kMultiMinKeys = 8192;        // sequences longer than this are worth several workgroups
constexpr int kMultiChunkKeys = 4096;      // aimed-at keys per workgroup
constexpr int kMaxChunks = 16;
// workspace of the chunked form: a header whose first word is the status word, then per sequence 4 histograms,
// 6 arrival counters (4 passes, counts, done) and the chunks' counts
constexpr int kWsHeader = 16;
constexpr int kWsHist = 0, kWsArrive = 4 * 256, kWsCounts = kWsArrive + 8, kWsPerSeq = kWsCounts + 2 * kMaxChunks;
constexpr uint32_t kStatusWaitFailed = 1u;
constexpr int kMaxPolls = 1 << 17;         // bound of a wait for the other chunks (~0.1 s, never reached in a healthy run)

// MULTI: G consecutive workgroups share a sequence (chunk c = blockIdx % G); lds_keys = keys that fit in LDS.
template <int THREADS, bool STAGED, bool MULTI>
__global__ __launch_bounds__(THREADS) void select_topk_kernel(const float* __restrict__ scores,
                                                              const int32_t* __restrict__ cu_seqlens,
                                                              const int32_t* __restrict__ cu_nuggets, uint32_t flags,
                                                              int max_n, int lds_keys, int G, uint32_t* __restrict__ ws,
                                                              int32_t* __restrict__ nugget_idx) {
  constexpr int kWaves = THREADS / kWave;
  extern __shared__ uint32_t keys_lds[];  // lds_keys keys, then kCandCap 16-bit positions (STAGED only)
  __shared__ uint32_t hist[256], hist_own[256];
  __shared__ uint32_t s_prefix, s_remaining, s_cand;
  __shared__ int wave_gt[kWaves], wave_eq[kWaves];
  __shared__ int s_ok, s_out_base, s_eq_base;

  // (a latency-bound kernel: all arguments in one round of scalar loads, the sequence's four boundaries in a second)
  asm volatile("" ::"s"(scores), "s"(cu_seqlens), "s"(cu_nuggets), "s"(flags), "s"(max_n), "s"(lds_keys), "s"(G), "s"(ws),
               "s"(nugget_idx));
  const int b = MULTI ? blockIdx.x / G : blockIdx.x;
  const int chunk = MULTI ? blockIdx.x % G : 0;
  const int tid = threadIdx.x, lane = lane_id(), wave = tid / kWave;
  const int seq0 = cu_seqlens[b], seq1 = cu_seqlens[b + 1];
  const int nug0 = cu_nuggets[b], nug1 = cu_nuggets[b + 1];
  asm volatile("" ::"s"(seq0), "s"(seq1), "s"(nug0), "s"(nug1));
  const int n = seq1 - seq0;
  int k = nug1 - nug0;
  if (k <= 0 || n <= 0 || n > max_n) return;  // uniform over the workgroup
  if (k > n) k = n;
  const bool force = (flags & DODO_TOPK_FORCE_LAST) != 0;
  const int n_free = force ? n - 1 : n;  // tokens that compete on score
  const int k_free = force ? k - 1 : k;
  int32_t* out = nugget_idx + nug0;
  // this workgroup's tokens: [lo, lo + n_own) of the sequence (all of them without chunks)
  const int chunk_len = MULTI ? ((n_free + G - 1) / G + kWave - 1) / kWave * kWave : n_free;
  const int lo = chunk * chunk_len;
  const int n_own = max(0, min(chunk_len, n_free - lo));
  const float* s = scores + seq0 + lo;
  uint32_t* gws = MULTI ? ws + kWsHeader + static_cast<int64_t>(b) * kWsPerSeq : nullptr;
  // Waits until all G chunks have passed sync point `which` (thread 0 polls; device-scope accesses, which go to
  // the level where all XCDs agree).  Whatever this workgroup published before is acknowledged first.
  bool all_ok = true;
  auto sync_chunks = [&](int which) {
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
    __syncthreads();
    if (tid == 0) {
      __hip_atomic_fetch_add(gws + kWsArrive + which, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      // (exactly G: a counter that was not zero when the call began never gets there, and the call reports it;
      // once a wait has run out this workgroup only announces itself at the later ones)
      int polls = 0, ok = all_ok ? 1 : 0;
      while (ok && __hip_atomic_load(gws + kWsArrive + which, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) !=
                       static_cast<uint32_t>(G)) {
        if (++polls > kMaxPolls) {
          ok = 0;
          break;
        }
        __builtin_amdgcn_s_sleep(8);
      }
      s_ok = ok;
    }
    __syncthreads();
    all_ok = all_ok && s_ok != 0;
  };

  if (k_free > 0) {
    if (STAGED) {
      // batches of 8 loads in flight per thread: one global-memory latency per batch, not per key
      constexpr int kBatch = 8;
      const int n_free = n_own;
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
    const int n_free = n_own;  // below, "the tokens" are this workgroup's; positions are relative to lo
    int pass_no = 0;

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
      if (MULTI) {
        // add this chunk's bins to the sequence's, wait for the other chunks, continue with the totals
        if (tid < 256) {
          const uint32_t v = hist[tid];
          hist_own[tid] = v;
          if (v != 0) __hip_atomic_fetch_add(gws + kWsHist + 256 * pass_no + tid, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        sync_chunks(pass_no);
        if (tid < 256)
          hist[tid] = __hip_atomic_load(gws + kWsHist + 256 * pass_no + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (!all_ok && tid == 0) hist[255] = remaining;  // (a failed wait: keep the scan below well-defined)
        __syncthreads();
      }
      ++pass_no;
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
          s_cand = MULTI ? hist_own[4 * L + dsel] : in_bin;  // this workgroup's items that carry the chosen digit
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
      uint16_t* cand = reinterpret_cast<uint16_t*>(keys_lds + lds_keys);
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
    if (MULTI) {
      // the chunks' counts, then offsets and the tie budget in chunk order
      if (tid == 0) {
        int gt = 0, eq = 0;
        for (int w = 0; w < kWaves; ++w) {
          gt += wave_gt[w];
          eq += wave_eq[w];
        }
        __hip_atomic_store(gws + kWsCounts + chunk, static_cast<uint32_t>(gt), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(gws + kWsCounts + kMaxChunks + chunk, static_cast<uint32_t>(eq), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
      }
      sync_chunks(4);
      if (tid == 0) {
        int ob = 0, eb = 0;
        for (int c2 = 0; c2 < chunk; ++c2) {
          const int gt = static_cast<int>(__hip_atomic_load(gws + kWsCounts + c2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
          const int eq = static_cast<int>(
              __hip_atomic_load(gws + kWsCounts + kMaxChunks + c2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
          ob += gt + max(0, min(eq, need_eq - eb));
          eb += eq;
        }
        s_out_base = ob;
        s_eq_base = eb;
      }
      __syncthreads();
      out_base = s_out_base;
      eq_base = s_eq_base;
    }
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
      if (sel && pos < k_free && all_ok) out[pos] = lo + i;  // pos < k_free always holds; the test keeps a logic slip in bounds
      eq_base += __popcll(eq_mask);
      out_base += __popcll(sel_mask);
    }
  }
  if (force && tid == 0 && chunk == 0) out[k - 1] = n - 1;
  if (MULTI && k_free > 0) {
    // A wait that ran out means a broken run (the chunks of a sequence were not running at the same time, or the
    // workspace was not zero-filled): the caller learns it from the status word, and the sequence's list is filled
    // with a valid index so that nothing downstream reads out of bounds.
    if (!all_ok) {
      for (int i = tid; i < k; i += THREADS) out[i] = n - 1;
      if (tid == 0) __hip_atomic_fetch_or(ws, kStatusWaitFailed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // Leave the sequence's part of the workspace zero-filled for the next call, also after a failure: whoever
    // is last to be done with it clears it.
    __syncthreads();
    if (tid == 0) {
      const uint32_t before = __hip_atomic_fetch_add(gws + kWsArrive + 5, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_ok = before + 1 == static_cast<uint32_t>(G);
    }
    __syncthreads();
    if (s_ok) {
      for (int i = tid; i < kWsPerSeq; i += THREADS)
        __hip_atomic_store(gws + i, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

// Chunks per sequence of the chunked form, or 0 when it does not apply (short sequences, or more workgroups than
// compute units: all chunks of a sequence must be resident at the same time, since they wait for each other).
int chunk_count(int32_t B, int32_t max_n) {
  if (max_n <= kMultiMinKeys) return 0;
  int G = (max_n + kMultiChunkKeys - 1) / kMultiChunkKeys;
  if (G > kMaxChunks) G = kMaxChunks;
  const int room = compute_units() / B;
  if (G > room) G = room;
  if (G < 2) return 0;
  const int chunk_len = ((max_n + G - 1) / G + kWave - 1) / kWave * kWave;
  return chunk_len <= kStagedMaxKeys ? G : 0;
}

template <int THREADS>
int launch_select(const float* scores, const int32_t* cu_seqlens, const int32_t* cu_nuggets, int32_t B, int32_t max_n,
                  uint32_t flags, int32_t* nugget_idx, hipStream_t stream) {
  if (max_n <= kStagedMaxKeys) {
    const size_t lds = static_cast<size_t>(max_n) * sizeof(uint32_t) + kCandCap * sizeof(uint16_t);
    auto kern = select_topk_kernel<THREADS, true, false>;
    if (lds > 48 * 1024) {
      {
      const int rc_lds = allow_dynamic_lds(reinterpret_cast<const void*>(kern), static_cast<int>(lds));
      if (rc_lds != DODO_OK) return rc_lds;
    }
    }
    hipLaunchKernelGGL(kern, dim3(B), dim3(THREADS), lds, stream, scores, cu_seqlens, cu_nuggets, flags, max_n, max_n, 1,
                       static_cast<uint32_t*>(nullptr), nugget_idx);
  } else {
    hipLaunchKernelGGL((select_topk_kernel<THREADS, false, false>), dim3(B), dim3(THREADS), 0, stream, scores, cu_seqlens,
                       cu_nuggets, flags, max_n, 0, 1, static_cast<uint32_t*>(nullptr), nugget_idx);
  }
  return launch_status();
}

int launch_select_chunked(const float* scores, const int32_t* cu_seqlens, const int32_t* cu_nuggets, int32_t B,
                          int32_t max_n, int G, uint32_t flags, int32_t* nugget_idx, uint32_t* ws, hipStream_t stream) {
  const int chunk_len = ((max_n + G - 1) / G + kWave - 1) / kWave * kWave;
  const size_t lds = static_cast<size_t>(chunk_len) * sizeof(uint32_t) + kCandCap * sizeof(uint16_t);
  auto kern = select_topk_kernel<1024, true, true>;
  if (lds > 48 * 1024) {
    {
      const int rc_lds = allow_dynamic_lds(reinterpret_cast<const void*>(kern), static_cast<int>(lds));
      if (rc_lds != DODO_OK) return rc_lds;
    }
  }
  hipLaunchKernelGGL(kern, dim3(B * G), dim3(1024), lds, stream, scores, cu_seqlens, cu_nuggets, flags, max_n, chunk_len, G,
                     ws, nugget_idx);
  return launch_status();
}

}  // namespace
}  // namespace dodo

extern "C" size_t dodo_select_topk_workspace_bytes(int32_t B, int32_t max_n) {
  using namespace dodo;
  if (B <= 0 || max_n <= 0) return 0;
  return chunk_count(B, max_n) > 0 ? (kWsHeader + static_cast<size_t>(B) * kWsPerSeq) * sizeof(uint32_t) : 0;
}

extern "C" int dodo_select_topk(const float* scores, const int32_t* cu_seqlens, const int32_t* cu_nuggets, int32_t B,
                                int32_t max_n, int32_t max_k, uint32_t flags, int32_t* nugget_idx, void* ws,
                                size_t ws_bytes, void* stream) {
  using namespace dodo;
  if (B < 0) return DODO_ERR_INVALID_ARG;
  if (B == 0) return DODO_OK;
  if (!scores || !cu_seqlens || !cu_nuggets || !nugget_idx) return DODO_ERR_INVALID_ARG;
  if (max_n <= 0 || max_k <= 0 || max_k > max_n) return DODO_ERR_INVALID_ARG;
  if (flags & ~DODO_TOPK_FORCE_LAST) return DODO_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // long sequences, given the workspace: several workgroups per sequence
  const int G = chunk_count(B, max_n);
  if (G > 0 && ws != nullptr && ws_bytes >= (kWsHeader + static_cast<size_t>(B) * kWsPerSeq) * sizeof(uint32_t) &&
      (reinterpret_cast<uintptr_t>(ws) & 3u) == 0)
    return launch_select_chunked(scores, cu_seqlens, cu_nuggets, B, max_n, G, flags, nugget_idx, static_cast<uint32_t*>(ws), s);
  // about four keys per thread: the kernel is latency-bound (few barriers matter more than lanes)
  if (max_n <= 1024) return launch_select<256>(scores, cu_seqlens, cu_nuggets, B, max_n, flags, nugget_idx, s);
  if (max_n <= 2048) return launch_select<512>(scores, cu_seqlens, cu_nuggets, B, max_n, flags, nugget_idx, s);
  return launch_select<1024>(scores, cu_seqlens, cu_nuggets, B, max_n, flags, nugget_idx, s);
}
