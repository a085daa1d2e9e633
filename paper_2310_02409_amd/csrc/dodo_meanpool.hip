// dodo_meanpool_nuggets: the compaction of the pooling baseline the Dodo paper
// compares with (Sec. 5.1): every sequence is cut evenly into k_b chunks and the
// K and V rows of a chunk are averaged into one row, giving a cache of the same
// shape as the nugget cache (same downstream attention calls).
//
// HBM-bound: every K and V row is read once.  One workgroup per output row and
// tensor; a thread owns a 16-byte piece of the row and walks the chunk's tokens in
// order, twelve tokens' loads in flight.  Sums and the division are done in double and
// rounded once to the storage type, in the same order as the plain definition,
// so the result is bit-exact.
#include "dodo_common.h"

namespace dodo {
namespace {

constexpr int kPoolThreads = 512;  // upper bound: the launch gives every thread one 16-byte piece of the row if it can
constexpr int kTokensInFlight = 12;  // (chunks of 10 tokens at 10x: one batch; a load under a condition costs more than a surplus one)

// double -> bf16 bits with one rounding (to nearest, ties to even); finite inputs and NaN
__device__ __forceinline__ uint16_t f64_to_bf16_bits(double v) {
  if (v != v) return 0x7fc0;
  // the float conversion may round across a bf16 tie, so the decision is taken on the double itself:
  // bf16 neighbours of |v| below and above, the nearer wins, ties to the even one
  const double av = fabs(v);
  const float f = static_cast<float>(av);
  uint32_t mag = __float_as_uint(f) & 0x7fff0000u;
  if (static_cast<double>(__uint_as_float(mag)) > av) mag -= 0x10000u;
  const uint32_t up = mag + 0x10000u;  // (overflow to inf is a valid encoding)
  const double dl = av - static_cast<double>(__uint_as_float(mag));
  const double du = static_cast<double>(__uint_as_float(up)) - av;
  const uint32_t pick = (dl < du) ? mag : (du < dl) ? up : ((mag >> 16) & 1u) ? up : mag;
  return static_cast<uint16_t>((pick >> 16) | (v < 0.0 || (v == 0.0 && __double_as_longlong(v) < 0) ? 0x8000u : 0u));
}

template <int DTYPE>
struct Piece;  // a 16-byte piece of a row as doubles
template <>
struct Piece<DODO_DTYPE_BF16> {
  static constexpr int kElems = 8;
  __device__ static __forceinline__ void add(const uint4& v, double* acc) {
    acc[0] += static_cast<double>(bf16_lo(v.x)); acc[1] += static_cast<double>(bf16_hi(v.x));
    acc[2] += static_cast<double>(bf16_lo(v.y)); acc[3] += static_cast<double>(bf16_hi(v.y));
    acc[4] += static_cast<double>(bf16_lo(v.z)); acc[5] += static_cast<double>(bf16_hi(v.z));
    acc[6] += static_cast<double>(bf16_lo(v.w)); acc[7] += static_cast<double>(bf16_hi(v.w));
  }
  __device__ static __forceinline__ uint4 round(const double* acc, double inv) {
    uint4 o;
    o.x = f64_to_bf16_bits(acc[0] * inv) | (static_cast<uint32_t>(f64_to_bf16_bits(acc[1] * inv)) << 16);
    o.y = f64_to_bf16_bits(acc[2] * inv) | (static_cast<uint32_t>(f64_to_bf16_bits(acc[3] * inv)) << 16);
    o.z = f64_to_bf16_bits(acc[4] * inv) | (static_cast<uint32_t>(f64_to_bf16_bits(acc[5] * inv)) << 16);
    o.w = f64_to_bf16_bits(acc[6] * inv) | (static_cast<uint32_t>(f64_to_bf16_bits(acc[7] * inv)) << 16);
    return o;
  }
};
template <>
struct Piece<DODO_DTYPE_F32> {
  static constexpr int kElems = 4;
  __device__ static __forceinline__ void add(const uint4& v, double* acc) {
    acc[0] += static_cast<double>(__uint_as_float(v.x)); acc[1] += static_cast<double>(__uint_as_float(v.y));
    acc[2] += static_cast<double>(__uint_as_float(v.z)); acc[3] += static_cast<double>(__uint_as_float(v.w));
  }
  __device__ static __forceinline__ uint4 round(const double* acc, double inv) {
    return make_uint4(__float_as_uint(static_cast<float>(acc[0] * inv)), __float_as_uint(static_cast<float>(acc[1] * inv)),
                      __float_as_uint(static_cast<float>(acc[2] * inv)), __float_as_uint(static_cast<float>(acc[3] * inv)));
  }
};

template <int DTYPE, bool HEAD_MAJOR>
__global__ __launch_bounds__(kPoolThreads) void meanpool_kernel(
    const uint4* __restrict__ K, const uint4* __restrict__ V, const int32_t* __restrict__ cu_seqlens,
    const int32_t* __restrict__ cu_nuggets, int B, int64_t Kt, int vec_per_head, int vec_per_row,
    int64_t token_stride_vec, uint4* __restrict__ Kn, uint4* __restrict__ Vn) {
  using P = Piece<DTYPE>;
  // two workgroups per output row, one for its K and one for its V (as in the gather kernel)
  const int64_t dst_tok = blockIdx.x >> 1;
  const uint4* __restrict__ src = (blockIdx.x & 1) ? V : K;
  uint4* __restrict__ dst_base = (blockIdx.x & 1) ? Vn : Kn;
  // Sequence b with cu_nuggets[b] <= dst_tok < cu_nuggets[b+1], its first token and its lengths.  For up to 64
  // sequences every lane fetches the boundaries of one sequence, all in one round of loads before the first
  // branch; a ballot finds b and lane reads hand its values over.  More sequences: a binary search.
  int seq0, nug0;
  int64_t n, k;
  if (B <= kWave) {
    const int lane = lane_id();
    const int lo_i = min(lane, B), hi_i = min(lane + 1, B);
    const int nug_lo = cu_nuggets[lo_i], nug_hi = cu_nuggets[hi_i];
    const int seq_lo = cu_seqlens[lo_i], seq_hi = cu_seqlens[hi_i];
    asm volatile("" ::"v"(nug_lo), "v"(nug_hi), "v"(seq_lo), "v"(seq_hi));  // one wait for all four
    const uint64_t above = __ballot(lane < B && nug_hi > dst_tok);  // sequences that end after dst_tok
    if (above == 0) return;  // dst_tok >= cu_nuggets[B]: Kt may be an upper bound of the row count
    const int b = __ffsll(static_cast<long long>(above)) - 1;
    nug0 = __shfl(nug_lo, b, kWave);
    seq0 = __shfl(seq_lo, b, kWave);
    k = __shfl(nug_hi, b, kWave) - nug0;
    n = __shfl(seq_hi, b, kWave) - seq0;
  } else {
    if (dst_tok >= cu_nuggets[B]) return;
    int lo = 0, hi = B;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (cu_nuggets[mid] <= dst_tok) lo = mid; else hi = mid;
    }
    nug0 = cu_nuggets[lo];
    seq0 = cu_seqlens[lo];
    k = cu_nuggets[lo + 1] - nug0;
    n = cu_seqlens[lo + 1] - seq0;
  }
  const int64_t j = dst_tok - nug0;
  // chunk boundaries floor(j n / k) and floor((j + 1) n / k): in 32 bits when the products fit (a 64-bit division by
  // a run-time value is some hundred vector instructions)
  int64_t t0, t1;
  if ((j + 1) * n <= 0xffffffffLL) {
    t0 = static_cast<uint32_t>(j * n) / static_cast<uint32_t>(k);
    t1 = static_cast<uint32_t>((j + 1) * n) / static_cast<uint32_t>(k);
  } else {
    t0 = j * n / k;
    t1 = (j + 1) * n / k;
  }
  const double inv = t1 > t0 ? 1.0 / static_cast<double>(t1 - t0) : 0.0;
  const uint4* rows = src + (seq0 + t0) * token_stride_vec;
  const int len = static_cast<int>(t1 - t0);

  const int threads = blockDim.x;
  for (int c = threadIdx.x; c < vec_per_row; c += threads) {
    double acc[P::kElems];
#pragma unroll
    for (int e = 0; e < P::kElems; ++e) acc[e] = 0.0;
    for (int t = 0; t < len; t += kTokensInFlight) {
      uint4 vv[kTokensInFlight];
#pragma unroll
      for (int u = 0; u < kTokensInFlight; ++u) {
        const int64_t tt = min(t + u, len - 1);  // unconditional loads; the surplus is not added
        vv[u] = load16_stream(rows + tt * token_stride_vec + c);
      }
#pragma unroll
      for (int u = 0; u < kTokensInFlight; ++u)
        if (t + u < len) P::add(vv[u], acc);
    }
    int64_t dst;
    if (HEAD_MAJOR) {
      const int h = c / vec_per_head;
      dst = (static_cast<int64_t>(h) * Kt + dst_tok) * vec_per_head + (c - h * vec_per_head);
    } else {
      dst = dst_tok * vec_per_row + c;
    }
    store16_stream(dst_base + dst, P::round(acc, inv));
  }
}

}  // namespace
}  // namespace dodo

extern "C" int dodo_meanpool_nuggets(const void* K, const void* V, int dtype, const int32_t* cu_seqlens,
                                     const int32_t* cu_nuggets, int32_t B, int64_t Kt, int32_t H_kv, int32_t d_h,
                                     int64_t token_stride, void* Kn, void* Vn, int layout, void* stream) {
  using namespace dodo;
  if (B < 0 || Kt < 0 || H_kv <= 0 || d_h <= 0) return DODO_ERR_INVALID_ARG;
  if (token_stride < static_cast<int64_t>(H_kv) * d_h) return DODO_ERR_INVALID_ARG;
  if (layout != DODO_LAYOUT_TOKEN_MAJOR && layout != DODO_LAYOUT_HEAD_MAJOR) return DODO_ERR_INVALID_ARG;
  if (Kt == 0 || B == 0) return DODO_OK;
  if (!K || !V || !cu_seqlens || !cu_nuggets || !Kn || !Vn) return DODO_ERR_INVALID_ARG;
  if (!dtype_ok(dtype)) return DODO_ERR_UNSUPPORTED;
  if (Kt > 0x7fffffffLL) return DODO_ERR_UNSUPPORTED;
  const int es = elem_bytes(dtype);
  if ((static_cast<int64_t>(d_h) * es) % 16 != 0 || (token_stride * es) % 16 != 0) return DODO_ERR_UNSUPPORTED;
  if (!aligned16(K) || !aligned16(V) || !aligned16(Kn) || !aligned16(Vn)) return DODO_ERR_UNSUPPORTED;
  const int vec_per_head = d_h * es / 16;
  const int vec_per_row = vec_per_head * H_kv;
  const int64_t stride_vec = token_stride * es / 16;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (Kt > 0x3fffffffLL) return DODO_ERR_UNSUPPORTED;
  int threads = (vec_per_row + kWave - 1) / kWave * kWave;
  if (threads > kPoolThreads) threads = kPoolThreads;
  const dim3 grid(static_cast<unsigned>(2 * Kt)), block(static_cast<unsigned>(threads));
  auto go = [&](auto kern) {
    hipLaunchKernelGGL(kern, grid, block, 0, s, static_cast<const uint4*>(K), static_cast<const uint4*>(V), cu_seqlens,
                       cu_nuggets, B, Kt, vec_per_head, vec_per_row, stride_vec, static_cast<uint4*>(Kn),
                       static_cast<uint4*>(Vn));
  };
  const bool hm = layout == DODO_LAYOUT_HEAD_MAJOR;
  if (dtype == DODO_DTYPE_BF16) {
    if (hm) go(meanpool_kernel<DODO_DTYPE_BF16, true>); else go(meanpool_kernel<DODO_DTYPE_BF16, false>);
  } else {
    if (hm) go(meanpool_kernel<DODO_DTYPE_F32, true>); else go(meanpool_kernel<DODO_DTYPE_F32, false>);
  }
  return launch_status();
}
