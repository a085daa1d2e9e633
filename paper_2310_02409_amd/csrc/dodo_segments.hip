// dodo_segment_plan: the segment form of the autoregressive objective (Sec. 2.4,
// "Learning", of the Dodo paper).  Every token i has its own splitting index
// i - tau in Eq. 9, so the sequence dimension cannot be batched; the paper chunks
// the text into segments whose tokens share one splitting index.  Segment c of a
// text (tokens c*S .. (c+1)*S - 1) gets t_c = max(0, c*S - tau): its tokens see
// the nuggets among the text's first t_c tokens and, causally, the uncompressed
// tokens from t_c on.  Each segment then is one entry of the batched attention
// call (dodo_nugget_attention_segments): a prefix of the text's nugget list, a
// window of the text's own K/V rows, and the segment's tokens as the query block.
// Integer work only: bit-exact.
#include "dodo_common.h"

namespace dodo {
namespace {

constexpr int kPlanThreads = 256;

__global__ __launch_bounds__(kPlanThreads) void segment_plan_kernel(
    const int32_t* __restrict__ nugget_idx, const int32_t* __restrict__ cu_seqlens,
    const int32_t* __restrict__ cu_nuggets, int B, int seg_len, int tau, int capacity, int32_t* __restrict__ seg_cu_q,
    int32_t* __restrict__ seg_nug_start, int32_t* __restrict__ seg_nug_len, int32_t* __restrict__ seg_loc_start,
    int32_t* __restrict__ seg_loc_len, int32_t* __restrict__ n_segments_out) {
  const int e = blockIdx.x * kPlanThreads + threadIdx.x;
  if (e > capacity) return;
  // text b and segment c of entry e: texts own consecutive runs of ceil(n_b / seg_len) entries
  int b = 0, first = 0;
  int64_t total = 0;
  bool found = false;
  for (int bb = 0; bb < B; ++bb) {
    const int n = cu_seqlens[bb + 1] - cu_seqlens[bb];
    const int segs = (n + seg_len - 1) / seg_len;
    if (!found && e < total + segs) {
      b = bb;
      first = static_cast<int>(total);
      found = true;
    }
    total += segs;
  }
  const int N = cu_seqlens[B];
  if (e == 0 && n_segments_out != nullptr) *n_segments_out = static_cast<int32_t>(min<int64_t>(total, 0x7fffffff));
  if (e == capacity) {
    seg_cu_q[capacity] = N;  // closes the cumulative array
    return;
  }
  if (!found) {  // beyond the last segment: an empty entry
    seg_cu_q[e] = N;
    seg_nug_start[e] = 0;
    seg_nug_len[e] = 0;
    seg_loc_start[e] = 0;
    seg_loc_len[e] = 0;
    return;
  }
  const int c = e - first;
  const int s0 = cu_seqlens[b], n = cu_seqlens[b + 1] - s0;
  const int q_begin = c * seg_len, q_end = min(q_begin + seg_len, n);
  const int t = max(0, q_begin - tau);
  // nuggets among the first t tokens: the index list ascends, so they are a prefix of it
  const int k0 = cu_nuggets[b], k = cu_nuggets[b + 1] - k0;
  int lo = 0, hi = k;  // first position whose index is >= t
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (nugget_idx[k0 + mid] < t) lo = mid + 1; else hi = mid;
  }
  seg_cu_q[e] = s0 + q_begin;
  seg_nug_start[e] = k0;
  seg_nug_len[e] = lo;
  seg_loc_start[e] = s0 + t;
  seg_loc_len[e] = q_end - t;
}

}  // namespace
}  // namespace dodo

extern "C" int dodo_segment_plan(const int32_t* nugget_idx, const int32_t* cu_seqlens, const int32_t* cu_nuggets,
                                 int32_t B, int32_t seg_len, int32_t tau, int32_t capacity, int32_t* seg_cu_q,
                                 int32_t* seg_nug_start, int32_t* seg_nug_len, int32_t* seg_loc_start,
                                 int32_t* seg_loc_len, int32_t* n_segments_out, void* stream) {
  using namespace dodo;
  if (B < 0 || seg_len <= 0 || tau < 0 || capacity < 0) return DODO_ERR_INVALID_ARG;
  if (!seg_cu_q) return DODO_ERR_INVALID_ARG;
  if (capacity > 0 && (!seg_nug_start || !seg_nug_len || !seg_loc_start || !seg_loc_len)) return DODO_ERR_INVALID_ARG;
  if (!cu_seqlens || (B > 0 && (!cu_nuggets || !nugget_idx))) return DODO_ERR_INVALID_ARG;
  const unsigned blocks = static_cast<unsigned>((static_cast<int64_t>(capacity) + 1 + kPlanThreads - 1) / kPlanThreads);
  hipLaunchKernelGGL(segment_plan_kernel, dim3(blocks), dim3(kPlanThreads), 0, static_cast<hipStream_t>(stream),
                     nugget_idx, cu_seqlens, cu_nuggets, B, seg_len, tau, capacity, seg_cu_q, seg_nug_start, seg_nug_len,
                     seg_loc_start, seg_loc_len, n_segments_out);
  return launch_status();
}
