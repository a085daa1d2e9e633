// dodo_meanpool_nuggets: the compaction of the pooling baseline the Dodo paper
// compares with (Sec. 5.1): every sequence is cut evenly into k_b chunks and the
// K and V rows of a chunk are averaged into one row, giving a cache of the same
// shape as the nugget cache (same downstream attention calls).
//
// HBM-bound: every K and V row is read once.  One workgroup per output row; a
// thread owns 16-byte pieces of the row and walks the chunk's tokens in order,
// four tokens' loads in flight.  Sums and the division are done in double and
// rounded once to the storage type, in the same order as the plain definition,
// so the result is bit-exact.
#include "dodo_common.h"

namespace dodo {
namespace {

constexpr int kPoolThreads = 256;
constexpr int kTokensInFlight = 4;

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
  const int64_t dst_tok = blockIdx.x;
  if (dst_tok >= cu_nuggets[B]) return;
  int lo = 0, hi = B;  // sequence b with cu_nuggets[b] <= dst_tok < cu_nuggets[b+1]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu_nuggets[mid] <= dst_tok) lo = mid; else hi = mid;
  }
  const int b = lo;
  const int64_t n = cu_seqlens[b + 1] - cu_seqlens[b];
  const int64_t k = cu_nuggets[b + 1] - cu_nuggets[b];
  const int64_t j = dst_tok - cu_nuggets[b];
  const int64_t t0 = j * n / k, t1 = (j + 1) * n / k;
  const double inv = t1 > t0 ? 1.0 / static_cast<double>(t1 - t0) : 0.0;
  const uint4* ksrc = K + (cu_seqlens[b] + t0) * token_stride_vec;
  const uint4* vsrc = V + (cu_seqlens[b] + t0) * token_stride_vec;
  const int len = static_cast<int>(t1 - t0);

  for (int c = threadIdx.x; c < vec_per_row; c += kPoolThreads) {
    double ak[P::kElems], av[P::kElems];
#pragma unroll
    for (int e = 0; e < P::kElems; ++e) ak[e] = av[e] = 0.0;
    for (int t = 0; t < len; t += kTokensInFlight) {
      uint4 kk[kTokensInFlight], vv[kTokensInFlight];
#pragma unroll
      for (int u = 0; u < kTokensInFlight; ++u) {
        const int64_t tt = min(t + u, len - 1);  // unconditional loads; the surplus is not added
        kk[u] = load16_stream(ksrc + tt * token_stride_vec + c);
        vv[u] = load16_stream(vsrc + tt * token_stride_vec + c);
      }
#pragma unroll
      for (int u = 0; u < kTokensInFlight; ++u)
        if (t + u < len) {
          P::add(kk[u], ak);
          P::add(vv[u], av);
        }
    }
    int64_t dst;
    if (HEAD_MAJOR) {
      const int h = c / vec_per_head;
      dst = (static_cast<int64_t>(h) * Kt + dst_tok) * vec_per_head + (c - h * vec_per_head);
    } else {
      dst = dst_tok * vec_per_row + c;
    }
    store16_stream(Kn + dst, P::round(ak, inv));
    store16_stream(Vn + dst, P::round(av, inv));
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
  const dim3 grid(static_cast<unsigned>(Kt)), block(kPoolThreads);
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
