// Bandwidth-bound nugget attention (Eq. 9 / Eq. 13 of the Dodo paper) for
// single-token decode and small query counts: every visible K and V row is
// read once with 16-byte loads, a group of lanes per row.
//
// One workgroup handles one (query row, head, split).  Its 256 threads form
// G = 256 / lanes-per-row groups; group g walks rows g, g+G, ... of the split,
// keeping an independent online-softmax state (running max, sum, d_h partial
// outputs spread over its lanes) in base 2.  Groups are merged through LDS in
// group order; splits are merged by a second kernel in split order.  No float
// atomics anywhere, so results are run-to-run deterministic.
#include "dodo_attn.h"

namespace dodo {
namespace {

constexpr int kRowsInFlight = 4;  // rows a group loads before it starts the arithmetic
constexpr float kNegInf = -__builtin_inff();

template <int DTYPE>
struct Vec16;
template <>
struct Vec16<DODO_DTYPE_BF16> {
  static constexpr int kElems = 8;
  __device__ static __forceinline__ void unpack(const uint4& v, float* f) {
    f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x); f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
    f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z); f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
  }
};
template <>
struct Vec16<DODO_DTYPE_F32> {
  static constexpr int kElems = 4;
  __device__ static __forceinline__ void unpack(const uint4& v, float* f) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
  }
};

__device__ __forceinline__ float exp2_guard(float x) { return __builtin_amdgcn_exp2f(x); }  // exp2(-inf) = 0

// partial record of one split in the workspace: [m, s, o[0..DH)] floats
template <int DH>
__host__ __device__ constexpr int partial_floats() { return DH + 2; }

template <int DTYPE, int DH, int kThreads>
__global__ __launch_bounds__(kThreads) void splitk_attention_kernel(
    const void* __restrict__ Q, const void* __restrict__ Kn, const void* __restrict__ Vn,
    const void* __restrict__ Kl, const void* __restrict__ Vl, const int32_t* __restrict__ cu_q,
    const int32_t* __restrict__ cu_nuggets, const int32_t* __restrict__ cu_local, int H, int H_kv, int max_q,
    int nsplit, int64_t nug_tok_stride, int64_t nug_head_stride, float scale_log2e, void* __restrict__ O,
    float* __restrict__ lse, float* __restrict__ ws) {
  using VT = Vec16<DTYPE>;
  constexpr int kEPL = VT::kElems;          // elements per lane
  constexpr int kLPR = DH / kEPL;           // lanes per K/V row
  constexpr int kGroups = kThreads / kLPR;  // rows processed side by side
  constexpr size_t kEs = DTYPE == DODO_DTYPE_F32 ? 4 : 2;

  __shared__ float part_m[kGroups], part_s[kGroups];
  __shared__ float part_o[kGroups][DH];

  int t = blockIdx.x;
  const int split = t % nsplit; t /= nsplit;
  const int h = t % H; t /= H;
  const int i = t % max_q;
  const int b = t / max_q;
  const int q0 = cu_q[b];
  const int q_b = cu_q[b + 1] - q0;
  if (i >= q_b) return;  // uniform over the workgroup
  const int k0 = cu_nuggets[b], k_b = cu_nuggets[b + 1] - k0;
  const int l0 = cu_local[b], m_b = cu_local[b + 1] - l0;
  const int n_local = max(0, min(m_b, m_b - q_b + i + 1));  // causal rule, bottom-right aligned
  const int n_vis = k_b + n_local;
  const int chunk = (n_vis + nsplit - 1) / nsplit;
  const int r0 = split * chunk;
  const int r1 = min(r0 + chunk, n_vis);
  const int kvh = h / (H / H_kv);

  const int g = threadIdx.x / kLPR;
  const int sub = threadIdx.x % kLPR;
  const int64_t row_id = static_cast<int64_t>(q0 + i) * H + h;

  float q[kEPL];
  {
    const uint4 qv = *reinterpret_cast<const uint4*>(static_cast<const char*>(Q) + (row_id * DH + sub * kEPL) * kEs);
    VT::unpack(qv, q);
#pragma unroll
    for (int e = 0; e < kEPL; ++e) q[e] *= scale_log2e;
  }
  const int64_t nug_base = static_cast<int64_t>(kvh) * nug_head_stride + sub * kEPL;
  const int64_t loc_base = static_cast<int64_t>(kvh) * DH + sub * kEPL;

  float m = kNegInf, ssum = 0.f;
  float o[kEPL];
#pragma unroll
  for (int e = 0; e < kEPL; ++e) o[e] = 0.f;

  for (int j0 = r0; j0 < r1; j0 += kGroups * kRowsInFlight) {
    uint4 kv[kRowsInFlight], vv[kRowsInFlight];
    bool valid[kRowsInFlight];
#pragma unroll
    for (int u = 0; u < kRowsInFlight; ++u) {
      // loads are unconditional (rows past the end re-read the last row of the range and are
      // discarded): a branch around them would serialise the loads behind a full wait
      const int jr = j0 + u * kGroups + g;
      valid[u] = jr < r1;
      const int j = valid[u] ? jr : r1 - 1;
      const bool nug = j < k_b;
      const int64_t off = nug ? (static_cast<int64_t>(k0 + j) * nug_tok_stride + nug_base) * kEs
                              : (static_cast<int64_t>(l0 + j - k_b) * H_kv * DH + loc_base) * kEs;
      kv[u] = load16_stream(static_cast<const char*>(nug ? Kn : Kl) + off);
      vv[u] = load16_stream(static_cast<const char*>(nug ? Vn : Vl) + off);
    }
    float logit[kRowsInFlight];
    float mx = m;
#pragma unroll
    for (int u = 0; u < kRowsInFlight; ++u) {
      float kf[kEPL];
      VT::unpack(kv[u], kf);
      float d = q[0] * kf[0];
#pragma unroll
      for (int e = 1; e < kEPL; ++e) d = fmaf(q[e], kf[e], d);
#pragma unroll
      for (int off = kLPR / 2; off >= 1; off >>= 1) d += __shfl_xor(d, off, kWave);
      logit[u] = valid[u] ? d : kNegInf;
      mx = fmaxf(mx, logit[u]);
    }
    if (mx != kNegInf) {  // uniform inside a group
      const float alpha = exp2_guard(m - mx);
      ssum *= alpha;
#pragma unroll
      for (int e = 0; e < kEPL; ++e) o[e] *= alpha;
#pragma unroll
      for (int u = 0; u < kRowsInFlight; ++u) {
        const float p = exp2_guard(logit[u] - mx);
        float vf[kEPL];
        VT::unpack(vv[u], vf);
        ssum += p;
#pragma unroll
        for (int e = 0; e < kEPL; ++e) o[e] = fmaf(p, vf[e], o[e]);
      }
      m = mx;
    }
  }

  // ---- merge the groups in group order ----
  if (sub == 0) {
    part_m[g] = m;
    part_s[g] = ssum;
  }
#pragma unroll
  for (int e = 0; e < kEPL; ++e) part_o[g][sub * kEPL + e] = o[e];
  __syncthreads();
  if (threadIdx.x < DH) {
    const int c = threadIdx.x;
    float M = kNegInf;
    for (int gg = 0; gg < kGroups; ++gg) M = fmaxf(M, part_m[gg]);
    float S = 0.f, oc = 0.f;
    if (M != kNegInf) {
      for (int gg = 0; gg < kGroups; ++gg) {
        const float wgt = exp2_guard(part_m[gg] - M);
        S = fmaf(part_s[gg], wgt, S);
        oc = fmaf(part_o[gg][c], wgt, oc);
      }
    }
    if (nsplit == 1) {
      const float val = (S > 0.f) ? oc / S : 0.f;
      if (DTYPE == DODO_DTYPE_F32) {
        static_cast<float*>(O)[row_id * DH + c] = val;
      } else {
        static_cast<uint16_t*>(O)[row_id * DH + c] = static_cast<uint16_t>(f32_to_bf16_bits(val));
      }
      if (lse != nullptr && c == 0) lse[row_id] = (S > 0.f) ? (M + __log2f(S)) * 0.6931471805599453f : kNegInf;
    } else {
      const int64_t slot = ((static_cast<int64_t>(b) * max_q + i) * H + h) * nsplit + split;
      float* rec = ws + slot * partial_floats<DH>();
      if (c == 0) {
        rec[0] = M;
        rec[1] = S;
      }
      rec[2 + c] = oc;
    }
  }
}

template <int DTYPE, int DH>
__global__ __launch_bounds__(DH) void splitk_combine_kernel(const float* __restrict__ ws,
                                                            const int32_t* __restrict__ cu_q, int H, int max_q,
                                                            int nsplit, void* __restrict__ O,
                                                            float* __restrict__ lse) {
  int t = blockIdx.x;
  const int h = t % H; t /= H;
  const int i = t % max_q;
  const int b = t / max_q;
  const int q0 = cu_q[b];
  if (i >= cu_q[b + 1] - q0) return;
  const int c = threadIdx.x;
  const float* rec = ws + (((static_cast<int64_t>(b) * max_q + i) * H + h) * nsplit) * partial_floats<DH>();
  float M = kNegInf;
  for (int s = 0; s < nsplit; ++s) M = fmaxf(M, rec[s * partial_floats<DH>()]);
  float S = 0.f, oc = 0.f;
  if (M != kNegInf) {
    for (int s = 0; s < nsplit; ++s) {
      const float* r = rec + s * partial_floats<DH>();
      const float wgt = exp2_guard(r[0] - M);
      S = fmaf(r[1], wgt, S);
      oc = fmaf(r[2 + c], wgt, oc);
    }
  }
  const int64_t row_id = static_cast<int64_t>(q0 + i) * H + h;
  const float val = (S > 0.f) ? oc / S : 0.f;
  if (DTYPE == DODO_DTYPE_F32) {
    static_cast<float*>(O)[row_id * DH + c] = val;
  } else {
    static_cast<uint16_t*>(O)[row_id * DH + c] = static_cast<uint16_t>(f32_to_bf16_bits(val));
  }
  if (lse != nullptr && c == 0) lse[row_id] = (S > 0.f) ? (M + __log2f(S)) * 0.6931471805599453f : kNegInf;
}

template <int DTYPE, int DH>
int launch_t(const AttnParams& p, int nsplit) {
  const int64_t rows = static_cast<int64_t>(p.B) * p.max_q * p.H;
  // few workgroups (about one per CU) with many rows each: 16 wavefronts per workgroup keep enough
  // loads in flight; otherwise 4 wavefronts and several workgroups per CU
  const bool wide = rows * nsplit <= 512 && static_cast<int64_t>(p.max_k) + p.max_local >= 512;
  if (wide) {
    hipLaunchKernelGGL((splitk_attention_kernel<DTYPE, DH, 1024>), dim3(static_cast<unsigned>(rows * nsplit)),
                       dim3(1024), 0, p.stream, p.Q, p.Kn, p.Vn, p.Kl, p.Vl, p.cu_q, p.cu_nuggets, p.cu_local, p.H,
                       p.H_kv, p.max_q, nsplit, p.nug_tok_stride, p.nug_head_stride, p.scale_log2e, p.O, p.lse,
                       static_cast<float*>(p.ws));
  } else {
    hipLaunchKernelGGL((splitk_attention_kernel<DTYPE, DH, 256>), dim3(static_cast<unsigned>(rows * nsplit)),
                       dim3(256), 0, p.stream, p.Q, p.Kn, p.Vn, p.Kl, p.Vl, p.cu_q, p.cu_nuggets, p.cu_local, p.H,
                       p.H_kv, p.max_q, nsplit, p.nug_tok_stride, p.nug_head_stride, p.scale_log2e, p.O, p.lse,
                       static_cast<float*>(p.ws));
  }
  int rc = launch_status();
  if (rc != DODO_OK || nsplit == 1) return rc;
  hipLaunchKernelGGL((splitk_combine_kernel<DTYPE, DH>), dim3(static_cast<unsigned>(rows)), dim3(DH), 0, p.stream,
                     static_cast<const float*>(p.ws), p.cu_q, p.H, p.max_q, nsplit, p.O, p.lse);
  return launch_status();
}

}  // namespace

int splitk_count(int32_t B, int32_t H, int32_t max_q, int32_t max_k, int32_t max_local) {
  const int64_t base = static_cast<int64_t>(B) * H * max_q;  // workgroups without splitting
  const int64_t rows = static_cast<int64_t>(max_k) + max_local;
  const int64_t want = (256 + base - 1) / base;            // aim at >= one (wide) workgroup per CU
  const int64_t room = rows / 256 > 0 ? rows / 256 : 1;    // keep >= 256 rows per split
  int64_t n = want < room ? want : room;
  if (n < 1) n = 1;
  if (n > 64) n = 64;
  return static_cast<int>(n);
}

size_t splitk_workspace_bytes(int32_t B, int32_t H, int32_t d_h, int32_t max_q, int nsplit) {
  if (nsplit <= 1) return 0;
  return static_cast<size_t>(B) * max_q * H * nsplit * (d_h + 2) * sizeof(float);
}

int launch_splitk_attention(const AttnParams& p) {
  const int nsplit = splitk_count(p.B, p.H, p.max_q, p.max_k, p.max_local);
  if (static_cast<int64_t>(p.B) * p.max_q * p.H * nsplit > 0x7fffffffLL) return DODO_ERR_UNSUPPORTED;
  if (p.dtype == DODO_DTYPE_BF16) {
    if (p.d_h == 128) return launch_t<DODO_DTYPE_BF16, 128>(p, nsplit);
    if (p.d_h == 64) return launch_t<DODO_DTYPE_BF16, 64>(p, nsplit);
  } else {
    if (p.d_h == 128) return launch_t<DODO_DTYPE_F32, 128>(p, nsplit);
    if (p.d_h == 64) return launch_t<DODO_DTYPE_F32, 64>(p, nsplit);
  }
  return DODO_ERR_UNSUPPORTED;
}

}  // namespace dodo
