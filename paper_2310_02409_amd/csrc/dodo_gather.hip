// dodo_gather_nuggets: sub-selection of the chosen tokens' K and V rows into
// the compact nugget cache (Eq. 5 of the Dodo paper: nuggets are existing token
// states, re-used rather than recomputed).
//
// Pure HBM copy: one workgroup per destination row and tensor moves the row's K or V
// (H_kv*d_h elements, 8 KiB for LLaMA-7B in bf16) with 16-byte loads that
// are all issued before the first store.  The destination row's sequence is
// found on the device from cu_nuggets (one boundary per lane and a ballot for up
// to 64 sequences, a binary search beyond), so nothing is read back to the host.
// dodo_gather_nuggets_layers does the same for the K/V of several layers with the
// one index list they share (Sec. 2.1), in one launch: the grid's second
// dimension is the layer.
#include "dodo_common.h"

namespace dodo {
namespace {

constexpr int kGatherThreads = 512;  // upper bound: the launch picks a size that gives every thread the same number of pieces
constexpr int kMaxVec = 4;  // 16-byte vectors per thread per tensor held in registers at once

// Copies row src_tok of K or of V (of the layer given by blockIdx.y) to row dst_tok of the nugget cache.
template <bool HEAD_MAJOR>
__device__ __forceinline__ void copy_row(const uint4* __restrict__ src, int64_t src_tok, int64_t dst_tok, int64_t Kt,
                                         int vec_per_head, int vec_per_row, int64_t token_stride_vec,
                                         int64_t src_layer_stride_vec, int64_t dst_layer_stride_vec,
                                         uint4* __restrict__ dst_base) {
  const int64_t layer = blockIdx.y;
  const uint4* from = src + layer * src_layer_stride_vec + src_tok * token_stride_vec;
  uint4* to = dst_base + layer * dst_layer_stride_vec;

  const int threads = blockDim.x;
  for (int c0 = threadIdx.x; c0 < vec_per_row; c0 += threads * kMaxVec) {
    uint4 v[kMaxVec];
#pragma unroll
    for (int u = 0; u < kMaxVec; ++u) {
      const int c = c0 + u * threads;
      if (c < vec_per_row) v[u] = load16_stream(from + c);
    }
#pragma unroll
    for (int u = 0; u < kMaxVec; ++u) {
      const int c = c0 + u * threads;
      if (c < vec_per_row) {
        int64_t dst;
        if (HEAD_MAJOR) {
          const int h = c / vec_per_head;
          dst = (static_cast<int64_t>(h) * Kt + dst_tok) * vec_per_head + (c - h * vec_per_head);
        } else {
          dst = dst_tok * vec_per_row + c;
        }
        store16_stream(to + dst, v[u]);
      }
    }
  }
}

template <bool HEAD_MAJOR>
__global__ __launch_bounds__(kGatherThreads) void gather_kernel(
    const uint4* __restrict__ K, const uint4* __restrict__ V, const int32_t* __restrict__ nugget_idx,
    const int32_t* __restrict__ cu_seqlens, const int32_t* __restrict__ cu_nuggets, int B, int64_t Kt,
    int vec_per_head, int vec_per_row, int64_t token_stride_vec, int64_t src_layer_stride_vec,
    int64_t dst_layer_stride_vec, uint4* __restrict__ Kn, uint4* __restrict__ Vn) {
  // two workgroups per destination row, one for its K and one for its V: rows are few (a handful per compute
  // unit in a launch that lasts microseconds), and halves spread more evenly over the compute units
  const int64_t dst_tok = blockIdx.x >> 1;
  const uint4* src = (blockIdx.x & 1) ? V : K;
  uint4* dst = (blockIdx.x & 1) ? Vn : Kn;
  // Sequence b with cu_nuggets[b] <= dst_tok < cu_nuggets[b+1].  The lookups before the row copy are dependent
  // loads, each a full memory latency, in a kernel that lasts a few of them.  For up to 64 sequences everything the
  // row address needs is fetched at once: every lane takes one boundary of cu_nuggets and one sequence start, all
  // lanes the index entry (nugget_idx has room for Kt entries, so the load is in bounds even when Kt is only an
  // upper bound of the nugget count); a ballot finds b and a lane read hands over its start.
  int b;
  if (B <= kWave) {
    const int lane = lane_id();
    const int bound = cu_nuggets[min(lane + 1, B)];  // upper boundary of sequence `lane`
    const int start = cu_seqlens[min(lane, B)];      // first token of sequence `lane`
    const int idx = nugget_idx[dst_tok];
    asm volatile("" ::"v"(bound), "v"(start), "s"(idx));  // all three requested before the first branch, one wait
    const uint64_t above = __ballot(lane < B && bound > dst_tok);  // sequences that end after dst_tok
    if (above == 0) return;  // dst_tok >= cu_nuggets[B]: Kt may be an upper bound of the nugget count
    b = __ffsll(static_cast<long long>(above)) - 1;
    const int64_t src_tok = static_cast<int64_t>(__shfl(start, b, kWave)) + idx;
    copy_row<HEAD_MAJOR>(src, src_tok, dst_tok, Kt, vec_per_head, vec_per_row, token_stride_vec, src_layer_stride_vec,
                         dst_layer_stride_vec, dst);
    return;
  }
  if (dst_tok >= cu_nuggets[B]) return;
  int lo = 0, hi = B;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu_nuggets[mid] <= dst_tok) lo = mid; else hi = mid;
  }
  b = lo;
  const int64_t src_tok = static_cast<int64_t>(cu_seqlens[b]) + nugget_idx[dst_tok];
  copy_row<HEAD_MAJOR>(src, src_tok, dst_tok, Kt, vec_per_head, vec_per_row, token_stride_vec, src_layer_stride_vec,
                       dst_layer_stride_vec, dst);
}

int gather_entry(const void* K, const void* V, int dtype, const int32_t* nugget_idx, const int32_t* cu_seqlens,
                 const int32_t* cu_nuggets, int32_t B, int64_t Kt, int32_t L, int32_t H_kv, int32_t d_h,
                 int64_t token_stride, int64_t src_layer_stride, int64_t dst_layer_stride, void* Kn, void* Vn, int layout,
                 void* stream) {
  if (B < 0 || Kt < 0 || L < 0 || H_kv <= 0 || d_h <= 0) return DODO_ERR_INVALID_ARG;
  if (token_stride < static_cast<int64_t>(H_kv) * d_h) return DODO_ERR_INVALID_ARG;
  if (layout != DODO_LAYOUT_TOKEN_MAJOR && layout != DODO_LAYOUT_HEAD_MAJOR) return DODO_ERR_INVALID_ARG;
  if (L > 1 && (src_layer_stride < 0 || dst_layer_stride < Kt * H_kv * d_h)) return DODO_ERR_INVALID_ARG;
  if (Kt == 0 || B == 0 || L == 0) return DODO_OK;
  if (!K || !V || !nugget_idx || !cu_seqlens || !cu_nuggets || !Kn || !Vn) return DODO_ERR_INVALID_ARG;
  if (!dtype_ok(dtype)) return DODO_ERR_UNSUPPORTED;
  if (Kt > 0x3fffffffLL || L > 65535) return DODO_ERR_UNSUPPORTED;
  const int es = elem_bytes(dtype);
  if ((static_cast<int64_t>(d_h) * es) % 16 != 0 || (token_stride * es) % 16 != 0) return DODO_ERR_UNSUPPORTED;
  if ((src_layer_stride * es) % 16 != 0 || (dst_layer_stride * es) % 16 != 0) return DODO_ERR_UNSUPPORTED;
  if (!aligned16(K) || !aligned16(V) || !aligned16(Kn) || !aligned16(Vn)) return DODO_ERR_UNSUPPORTED;

  const int vec_per_head = d_h * es / 16;
  const int vec_per_row = vec_per_head * H_kv;
  const int64_t stride_vec = token_stride * es / 16;
  const int64_t src_l = src_layer_stride * es / 16, dst_l = dst_layer_stride * es / 16;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // workgroup size: the row's 16-byte pieces divided evenly over the threads (a 10 KiB row is two pieces each for
  // 320 threads rather than three for some of 256 and two for the rest), between one and eight wavefronts
  const int passes = vec_per_row >= 512 ? vec_per_row / 256 : 1;
  int threads = ((vec_per_row + passes - 1) / passes + kWave - 1) / kWave * kWave;
  if (threads > kGatherThreads) threads = kGatherThreads;
  const dim3 grid(static_cast<unsigned>(2 * Kt), static_cast<unsigned>(L)), block(static_cast<unsigned>(threads));
  if (layout == DODO_LAYOUT_HEAD_MAJOR) {
    hipLaunchKernelGGL(gather_kernel<true>, grid, block, 0, s, static_cast<const uint4*>(K),
                       static_cast<const uint4*>(V), nugget_idx, cu_seqlens, cu_nuggets, B, Kt, vec_per_head,
                       vec_per_row, stride_vec, src_l, dst_l, static_cast<uint4*>(Kn), static_cast<uint4*>(Vn));
  } else {
    hipLaunchKernelGGL(gather_kernel<false>, grid, block, 0, s, static_cast<const uint4*>(K),
                       static_cast<const uint4*>(V), nugget_idx, cu_seqlens, cu_nuggets, B, Kt, vec_per_head,
                       vec_per_row, stride_vec, src_l, dst_l, static_cast<uint4*>(Kn), static_cast<uint4*>(Vn));
  }
  return launch_status();
}

}  // namespace
}  // namespace dodo

extern "C" int dodo_gather_nuggets(const void* K, const void* V, int dtype, const int32_t* nugget_idx,
                                   const int32_t* cu_seqlens, const int32_t* cu_nuggets, int32_t B, int64_t Kt,
                                   int32_t H_kv, int32_t d_h, int64_t token_stride, void* Kn, void* Vn, int layout,
                                   void* stream) {
  return dodo::gather_entry(K, V, dtype, nugget_idx, cu_seqlens, cu_nuggets, B, Kt, 1, H_kv, d_h, token_stride, 0, 0, Kn,
                            Vn, layout, stream);
}

extern "C" int dodo_gather_nuggets_layers(const void* K, const void* V, int dtype, const int32_t* nugget_idx,
                                          const int32_t* cu_seqlens, const int32_t* cu_nuggets, int32_t B, int64_t Kt,
                                          int32_t L, int32_t H_kv, int32_t d_h, int64_t token_stride,
                                          int64_t src_layer_stride, int64_t dst_layer_stride, void* Kn, void* Vn,
                                          int layout, void* stream) {
  return dodo::gather_entry(K, V, dtype, nugget_idx, cu_seqlens, cu_nuggets, B, Kt, L, H_kv, d_h, token_stride,
                            src_layer_stride, dst_layer_stride, Kn, Vn, layout, stream);
}
