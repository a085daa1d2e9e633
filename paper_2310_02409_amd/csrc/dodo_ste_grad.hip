// dodo_ste_score_grad: the gradient that the straight-through estimator hands
// to the scores (Sec. 2.5, Eq. 17-18 of the Dodo paper).  The score s_i is
// added to the attention logits of nugget i (minus a detached copy, so the
// forward pass is unchanged); its gradient is therefore the sum, over query rows
// j and heads h (and layers: one call per layer, accumulating), of the gradient
// of the loss in the softmax input xi[j, i]:
//     grad[i] = grad_scale * sum_h sum_j P[j,i] * (dP[j,i] - D[j]),
//     P[j,i] = exp(scale q_j.k_i - lse[j]),  dP[j,i] = dO[j].v_i,  D[j] = dO[j].O[j],
// with O and lse as the forward attention call returned them (lse covers the
// local keys as well, so only nugget columns are touched here).
//
// Two contractions (Q K^T and dO V^T) restricted to the nugget columns:
// 4 k q d_h flop per (sequence, head).  bf16 with d_h = 128 runs on the matrix
// cores: each of a workgroup's 4 wavefronts owns 64 nuggets of one (sequence,
// head), whose K and V fragments stay in its registers; the workgroup walks over
// the sequence's query rows in tiles of 32 (Q and dO rows stream into a 3-stage
// LDS ring by 16-byte direct loads, two tiles ahead, shared by the 4 wavefronts),
// and a wavefront computes S and dP with v_mfma_f32_32x32x16_bf16 so that a nugget
// is a lane and a query row an accumulator register, and adds P (dP - D) into a
// per-lane sum.  No atomics: per-head sums go to the workspace and a last kernel
// adds them in head order.  Other types and head sizes take a plain kernel.
#include "dodo_common.h"

namespace dodo {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef __attribute__((address_space(3))) void lds_void;

constexpr int kDH = 128;
constexpr int kRowBytes = kDH * 2;
constexpr int kGradWaves = 4;
constexpr int kGradThreads = kGradWaves * kWave;
constexpr int kWaveNug = 64;                       // nuggets per wavefront
constexpr int kNugTile = kGradWaves * kWaveNug;    // nuggets per workgroup
constexpr int kQTile = 32;                         // query rows per step
constexpr int kStagesSte = 3;
constexpr int kStageBytesSte = 2 * kQTile * kRowBytes;  // Q tile, dO tile
constexpr int kLoadsPerTileSte = 4;                // direct loads per wavefront per tile
constexpr int kMaxQLds = 12288;                    // query rows of a sequence whose lse and D fit in LDS next to the stages
constexpr float kLog2e = 1.4426950408889634f;

// D[h][row] = dO[row,h] . O[row,h] and lse2[h][row] = lse[row,h] * log2(e), head-major so that the rows of a head are
// contiguous.  16 lanes per (row, head), 8 channels per lane and step (d_h % 8 == 0).
template <int DTYPE>
__global__ __launch_bounds__(256) void ste_rowdot_kernel(const void* __restrict__ dO, const void* __restrict__ O,
                                                         const float* __restrict__ lse, int64_t Sq, int H, int d_h,
                                                         float* __restrict__ aux_lse2, float* __restrict__ aux_D,
                                                         float* __restrict__ partial, int64_t n_partial) {
  // per-head sums that no workgroup writes later must read as zero: cleared here, by the first threads
  const int64_t gid = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  for (int64_t i = gid; i < n_partial; i += static_cast<int64_t>(gridDim.x) * blockDim.x) partial[i] = 0.f;
  const int64_t t = gid / 16;
  const int sub = threadIdx.x % 16;
  const bool live = t < Sq * H;
  float acc = 0.f;
  if (live) {
    for (int c0 = sub * 8; c0 < d_h; c0 += 128) {
      float a[8], o[8];
      if (DTYPE == DODO_DTYPE_F32) {
        const float4* pa = reinterpret_cast<const float4*>(static_cast<const float*>(dO) + t * d_h + c0);
        const float4* po = reinterpret_cast<const float4*>(static_cast<const float*>(O) + t * d_h + c0);
        const float4 a0 = pa[0], a1 = pa[1], o0 = po[0], o1 = po[1];
        a[0] = a0.x; a[1] = a0.y; a[2] = a0.z; a[3] = a0.w; a[4] = a1.x; a[5] = a1.y; a[6] = a1.z; a[7] = a1.w;
        o[0] = o0.x; o[1] = o0.y; o[2] = o0.z; o[3] = o0.w; o[4] = o1.x; o[5] = o1.y; o[6] = o1.z; o[7] = o1.w;
      } else {
        const uint4 av = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(dO) + t * d_h + c0);
        const uint4 ov = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(O) + t * d_h + c0);
        const uint32_t aw[4] = {av.x, av.y, av.z, av.w}, ow[4] = {ov.x, ov.y, ov.z, ov.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          a[2 * e] = bf16_lo(aw[e]); a[2 * e + 1] = bf16_hi(aw[e]);
          o[2 * e] = bf16_lo(ow[e]); o[2 * e + 1] = bf16_hi(ow[e]);
        }
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) acc = fmaf(a[e], o[e], acc);
    }
  }
#pragma unroll
  for (int off = 8; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, kWave);
  if (live && sub == 0) {
    const int64_t row = t / H;
    const int h = static_cast<int>(t % H);
    aux_D[h * Sq + row] = acc;
    aux_lse2[h * Sq + row] = lse[t] * kLog2e;
  }
}

__global__ __launch_bounds__(kGradThreads, 2) void ste_grad_mfma_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ Kn, const uint16_t* __restrict__ Vn,
    const uint16_t* __restrict__ dO, const float* __restrict__ aux_lse2, const float* __restrict__ aux_D,
    const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_nuggets, int B, int H, int H_kv, int n_nug_tiles,
    int max_q_pad, int64_t Sq, int64_t Kt, int64_t nug_tok_stride, int64_t nug_head_stride, float scale_log2e,
    float* __restrict__ partial) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];  // kStages stages of (Q tile | dO tile), then lse2, D
  const uint32_t lds_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_void*)lds));
  // block i runs on XCD i % 8: the nugget tiles of one (sequence, head) sit on one XCD and share Q / dO in its L2
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int bh = (slot / n_nug_tiles) * 8 + xcd;
  const int tile = slot % n_nug_tiles;
  if (bh >= B * H) return;
  const int b = bh / H, h = bh % H;
  const int k0 = cu_nuggets[b], k_b = cu_nuggets[b + 1] - k0;
  if (tile * kNugTile >= k_b) return;  // uniform over the workgroup
  const int q0 = cu_q[b], q_b = cu_q[b + 1] - q0;
  const int kvh = h / (H / H_kv);

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int lane = tid % kWave;
  const int n = lane & 31, g = lane >> 5;
  const int nug0 = tile * kNugTile + wave * kWaveNug;  // this wavefront's 64 nuggets
  const bool active = nug0 < k_b;                      // (the others only help to load)

  // lse (base 2) and D of all query rows of this (sequence, head); rows past the end get +inf, which makes their
  // weights 0
  float* lse2_l = reinterpret_cast<float*>(lds + kStagesSte * kStageBytesSte);
  float* dd_l = lse2_l + max_q_pad;
  for (int r = tid; r < max_q_pad; r += kGradThreads) {
    const bool ok = r < q_b;
    lse2_l[r] = ok ? aux_lse2[static_cast<int64_t>(h) * Sq + q0 + r] : __builtin_inff();
    dd_l[r] = ok ? aux_D[static_cast<int64_t>(h) * Sq + q0 + r] : 0.f;
  }

  // K and V fragments of the two 32-nugget blocks (B operands: lane (n, g) holds channels 16 ks + 8 g .. + 8 of
  // nugget row n); rows past the sequence's last nugget re-read it, their sums are not stored
  bf16x8 kf[2][kDH / 16], vf[2][kDH / 16];
#pragma unroll
  for (int blk = 0; blk < 2; ++blk) {
    const int r = min(nug0 + 32 * blk + n, k_b - 1);
    const int64_t off = static_cast<int64_t>(k0 + r) * nug_tok_stride + static_cast<int64_t>(kvh) * nug_head_stride + 8 * g;
#pragma unroll
    for (int ks = 0; ks < kDH / 16; ++ks) {
      kf[blk][ks] = *reinterpret_cast<const bf16x8*>(Kn + off + 16 * ks);
      vf[blk][ks] = *reinterpret_cast<const bf16x8*>(Vn + off + 16 * ks);
    }
  }
  // (the loads above are complete before the first direct load below is counted: the fragments are read there)
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  // loader: a stage is 32 query rows of Q and of dO; wavefront w brings rows 8w .. 8w+7 of both, 4 rows (16 lanes
  // per 256-byte row) per instruction; the 16-byte piece at position pos of LDS row r is piece pos ^ (r & 15) of
  // the row, which keeps the fragment reads below conflict-free
  const int l_row = lane >> 4, l_pos = lane & 15;
  const int64_t row_stride = static_cast<int64_t>(H) * kDH;  // elements between query rows
  const uint16_t* q_base = Q + (static_cast<int64_t>(q0) * H + h) * kDH;
  const uint16_t* do_base = dO + (static_cast<int64_t>(q0) * H + h) * kDH;
  const int n_qtiles = (q_b + kQTile - 1) / kQTile;
  auto issue_tile = [&](int t) {
    const int tl = min(t, n_qtiles - 1);  // past the end: re-read the last tile into a stage nobody reads any more
    const uint32_t stage = lds_base + (t % kStagesSte) * kStageBytesSte;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int row = 8 * wave + 4 * u + l_row;
      const uint32_t voff = static_cast<uint32_t>(min(tl * kQTile + row, q_b - 1)) * static_cast<uint32_t>(row_stride * 2) +
                            ((l_pos ^ (row & 15)) << 4);
      const uint32_t dst = stage + (8 * wave + 4 * u) * kRowBytes;
      dma16_uniform(q_base, voff, __builtin_amdgcn_readfirstlane(dst));
      dma16_uniform(do_base, voff, __builtin_amdgcn_readfirstlane(dst + kQTile * kRowBytes));
    }
  };

  float ds[2] = {0.f, 0.f};
  if (n_qtiles > 0) {
    issue_tile(0);
    issue_tile(1);
  }
  for (int t = 0; t < n_qtiles; ++t) {
    __builtin_amdgcn_s_waitcnt(0x0f70 | kLoadsPerTileSte);  // this wavefront's part of tile t has landed, t+1 may be in flight
    __syncthreads();  // everyone's part has landed (first pass: lse2 / D too); tile t-1 has been read by everyone
    issue_tile(t + 2);
    if (!active) continue;
    const char* stg = lds + (t % kStagesSte) * kStageBytesSte;
    floatx16 acc_s[2], acc_p[2];
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        acc_s[blk][v] = 0.f;
        acc_p[blk][v] = 0.f;
      }
    const char* qrow = stg + n * kRowBytes;
    const char* drow = stg + kQTile * kRowBytes + n * kRowBytes;
#pragma unroll
    for (int ks = 0; ks < kDH / 16; ++ks) {
      const int piece = ((2 * ks + g) ^ (n & 15)) << 4;
      const bf16x8 qa = *reinterpret_cast<const bf16x8*>(qrow + piece);
      const bf16x8 da = *reinterpret_cast<const bf16x8*>(drow + piece);
#pragma unroll
      for (int blk = 0; blk < 2; ++blk) {
        acc_s[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kf[blk][ks], acc_s[blk], 0, 0, 0);
        acc_p[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(da, vf[blk][ks], acc_p[blk], 0, 0, 0);
      }
    }
    // accumulator v of a block is query row 8 (v / 4) + 4 g + v % 4 of the tile, for this lane's nugget
#pragma unroll
    for (int vq = 0; vq < 4; ++vq) {
      const float4 l2 = *reinterpret_cast<const float4*>(lse2_l + t * kQTile + 8 * vq + 4 * g);
      const float4 dd = *reinterpret_cast<const float4*>(dd_l + t * kQTile + 8 * vq + 4 * g);
      const float l2v[4] = {l2.x, l2.y, l2.z, l2.w};
      const float ddv[4] = {dd.x, dd.y, dd.z, dd.w};
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float p = __builtin_amdgcn_exp2f(acc_s[blk][4 * vq + e] * scale_log2e - l2v[e]);
          ds[blk] = fmaf(p, acc_p[blk][4 * vq + e] - ddv[e], ds[blk]);
        }
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0f70);  // drain the look-ahead loads before the wavefront ends

  // the two halves of a nugget's query rows sit in lanes n and n + 32
  if (active) {
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      const float both = ds[blk] + __shfl_xor(ds[blk], 32, kWave);
      const int i = nug0 + 32 * blk + n;
      if (g == 0 && i < k_b) partial[static_cast<int64_t>(h) * Kt + k0 + i] = both;
    }
  }
}

// One wavefront per (head, nugget): every lane takes query rows of its own and does the two dot products alone.
template <int DTYPE>
__global__ __launch_bounds__(kWave) void ste_grad_plain_kernel(
    const void* __restrict__ Q, const void* __restrict__ Kn, const void* __restrict__ Vn, const void* __restrict__ dO,
    const float* __restrict__ aux_lse2, const float* __restrict__ aux_D, const int32_t* __restrict__ cu_q,
    const int32_t* __restrict__ cu_nuggets, int B, int H, int H_kv, int d_h, int64_t Sq, int64_t Kt,
    int64_t nug_tok_stride, int64_t nug_head_stride, float scale_log2e, float* __restrict__ partial) {
  const int64_t kk = blockIdx.x;  // nugget (packed index)
  const int h = blockIdx.y;
  if (kk >= cu_nuggets[B]) return;
  int lo = 0, hi = B;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu_nuggets[mid] <= kk) lo = mid; else hi = mid;
  }
  const int b = lo;
  const int q0 = cu_q[b], q_b = cu_q[b + 1] - q0;
  const int kvh = h / (H / H_kv);
  const int64_t koff = kk * nug_tok_stride + static_cast<int64_t>(kvh) * nug_head_stride;
  float acc = 0.f;
  for (int j = threadIdx.x; j < q_b; j += kWave) {
    const int64_t qoff = (static_cast<int64_t>(q0 + j) * H + h) * d_h;
    float s = 0.f, dp = 0.f;
    for (int c = 0; c < d_h; ++c) {
      s = fmaf(load_elem<DTYPE>(Q, qoff + c), load_elem<DTYPE>(Kn, koff + c), s);
      dp = fmaf(load_elem<DTYPE>(dO, qoff + c), load_elem<DTYPE>(Vn, koff + c), dp);
    }
    const float p = __builtin_amdgcn_exp2f(s * scale_log2e - aux_lse2[static_cast<int64_t>(h) * Sq + q0 + j]);
    acc = fmaf(p, dp - aux_D[static_cast<int64_t>(h) * Sq + q0 + j], acc);
  }
#pragma unroll
  for (int off = kWave / 2; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, kWave);
  if (threadIdx.x == 0) partial[static_cast<int64_t>(h) * Kt + kk] = acc;
}

// grad[k] = (accumulate ? grad[k] : 0) + grad_scale * sum over heads, in head order.  A workgroup takes 8 nuggets:
// all of their per-head sums are fetched at once (thread (h mod 32, nugget)), then one thread per nugget adds them.
__global__ __launch_bounds__(256) void ste_reduce_heads_kernel(const float* __restrict__ partial, int H, int64_t Kt,
                                                               const int32_t* __restrict__ cu_nuggets, int B,
                                                               float grad_scale, int accumulate,
                                                               float* __restrict__ grad) {
  extern __shared__ float vals[];  // [H][8]
  const int kk = threadIdx.x & 7;
  const int64_t k = static_cast<int64_t>(blockIdx.x) * 8 + kk;
  const bool live = k < Kt && k < cu_nuggets[B];
  for (int h = threadIdx.x >> 3; h < H; h += 32) vals[h * 8 + kk] = live ? partial[static_cast<int64_t>(h) * Kt + k] : 0.f;
  __syncthreads();
  if (threadIdx.x < 8 && live) {
    float s = 0.f;
    for (int h = 0; h < H; ++h) s += vals[h * 8 + kk];
    s *= grad_scale;
    grad[k] = accumulate ? grad[k] + s : s;
  }
}

__global__ void fill_zero_kernel(float* __restrict__ p, int64_t n) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

}  // namespace
}  // namespace dodo

extern "C" size_t dodo_ste_score_grad_workspace_bytes(int64_t Sq, int32_t H, int64_t Kt) {
  if (Sq <= 0 || H <= 0 || Kt <= 0) return 0;
  return (static_cast<size_t>(2) * Sq * H + static_cast<size_t>(H) * Kt) * sizeof(float);
}

extern "C" int dodo_ste_score_grad(const void* Q, const void* Kn, const void* Vn, const void* dO, const void* O,
                                   const float* lse, const int32_t* cu_q, const int32_t* cu_nuggets, int32_t B,
                                   int32_t H, int32_t H_kv, int32_t d_h, int32_t max_q, int32_t max_k, int64_t Sq,
                                   int64_t Kt, float softmax_scale, float grad_scale, int accumulate, int dtype,
                                   int layout, float* grad_scores, void* ws, size_t ws_bytes, void* stream) {
  using namespace dodo;
  if (B < 0 || H <= 0 || H_kv <= 0 || d_h <= 0 || max_q < 0 || max_k < 0 || Sq < 0 || Kt < 0) return DODO_ERR_INVALID_ARG;
  if (H % H_kv != 0) return DODO_ERR_INVALID_ARG;
  if (layout != DODO_LAYOUT_TOKEN_MAJOR && layout != DODO_LAYOUT_HEAD_MAJOR) return DODO_ERR_INVALID_ARG;
  if (!(softmax_scale == softmax_scale) || !(grad_scale == grad_scale)) return DODO_ERR_INVALID_ARG;
  if (B == 0 || Kt == 0 || max_k == 0) return DODO_OK;
  if (!grad_scores || !cu_q || !cu_nuggets) return DODO_ERR_INVALID_ARG;
  if (!dtype_ok(dtype) || d_h % 8 != 0 || H > 4096) return DODO_ERR_UNSUPPORTED;  // (the last kernel keeps 8 values per head in LDS)
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (Sq == 0 || max_q == 0) {  // no query rows: the gradient of this layer is zero
    if (!accumulate) {
      hipLaunchKernelGGL(fill_zero_kernel, dim3(static_cast<unsigned>((Kt + 255) / 256)), dim3(256), 0, s, grad_scores, Kt);
      return launch_status();
    }
    return DODO_OK;
  }
  if (!Q || !Kn || !Vn || !dO || !O || !lse) return DODO_ERR_INVALID_ARG;
  if (!aligned16(Q) || !aligned16(Kn) || !aligned16(Vn) || !aligned16(dO) || !aligned16(O)) return DODO_ERR_UNSUPPORTED;
  if (Sq * H > 0x7fffffffLL || Kt > 0x7fffffffLL) return DODO_ERR_UNSUPPORTED;
  const size_t need = dodo_ste_score_grad_workspace_bytes(Sq, H, Kt);
  if (!ws || ws_bytes < need) return DODO_ERR_WORKSPACE_TOO_SMALL;
  float* aux_lse2 = static_cast<float*>(ws);
  float* aux_D = aux_lse2 + Sq * H;
  float* partial = aux_D + Sq * H;
  int64_t tok_stride, head_stride;
  if (layout == DODO_LAYOUT_TOKEN_MAJOR) {
    tok_stride = static_cast<int64_t>(H_kv) * d_h;
    head_stride = d_h;
  } else {
    tok_stride = d_h;
    head_stride = Kt * d_h;
  }
  const float scale_log2e = softmax_scale * kLog2e;
  const unsigned rd_blocks = static_cast<unsigned>((Sq * H * 16 + 255) / 256);
  if (dtype == DODO_DTYPE_BF16) {
    hipLaunchKernelGGL(ste_rowdot_kernel<DODO_DTYPE_BF16>, dim3(rd_blocks), dim3(256), 0, s, dO, O, lse, Sq, H, d_h,
                       aux_lse2, aux_D, partial, static_cast<int64_t>(H) * Kt);
  } else {
    hipLaunchKernelGGL(ste_rowdot_kernel<DODO_DTYPE_F32>, dim3(rd_blocks), dim3(256), 0, s, dO, O, lse, Sq, H, d_h,
                       aux_lse2, aux_D, partial, static_cast<int64_t>(H) * Kt);
  }
  int rc = launch_status();
  if (rc != DODO_OK) return rc;
  const bool mfma = dtype == DODO_DTYPE_BF16 && d_h == kDH && max_q <= kMaxQLds &&
                    static_cast<int64_t>(max_q) * H * kDH * 2 < 0x7fffffffLL;  // row offsets of a sequence in 32 bits
  if (mfma) {
    const int n_nug_tiles = (max_k + kNugTile - 1) / kNugTile;
    const int64_t bh8 = (static_cast<int64_t>(B) * H + 7) / 8 * 8;
    const int64_t grid = bh8 * n_nug_tiles;
    if (grid > 0x7fffffffLL) return DODO_ERR_UNSUPPORTED;
    const int max_q_pad = (max_q + kQTile - 1) / kQTile * kQTile;
    const int kLds = kStagesSte * kStageBytesSte + 2 * max_q_pad * static_cast<int>(sizeof(float));
    {
      const int rc_lds = allow_dynamic_lds(reinterpret_cast<const void*>(ste_grad_mfma_kernel), kLds);
      if (rc_lds != DODO_OK) return rc_lds;
    }
    hipLaunchKernelGGL(ste_grad_mfma_kernel, dim3(static_cast<unsigned>(grid)), dim3(kGradThreads), kLds, s,
                       static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(Kn),
                       static_cast<const uint16_t*>(Vn), static_cast<const uint16_t*>(dO), aux_lse2, aux_D, cu_q,
                       cu_nuggets, B, H, H_kv, n_nug_tiles, max_q_pad, Sq, Kt, tok_stride, head_stride, scale_log2e, partial);
  } else {
    if (H > 65535) return DODO_ERR_UNSUPPORTED;
    const dim3 grid(static_cast<unsigned>(Kt), static_cast<unsigned>(H));
    if (dtype == DODO_DTYPE_BF16) {
      hipLaunchKernelGGL(ste_grad_plain_kernel<DODO_DTYPE_BF16>, grid, dim3(kWave), 0, s, Q, Kn, Vn, dO, aux_lse2, aux_D,
                         cu_q, cu_nuggets, B, H, H_kv, d_h, Sq, Kt, tok_stride, head_stride, scale_log2e, partial);
    } else {
      hipLaunchKernelGGL(ste_grad_plain_kernel<DODO_DTYPE_F32>, grid, dim3(kWave), 0, s, Q, Kn, Vn, dO, aux_lse2, aux_D,
                         cu_q, cu_nuggets, B, H, H_kv, d_h, Sq, Kt, tok_stride, head_stride, scale_log2e, partial);
    }
  }
  rc = launch_status();
  if (rc != DODO_OK) return rc;
  hipLaunchKernelGGL(ste_reduce_heads_kernel, dim3(static_cast<unsigned>((Kt + 7) / 8)), dim3(256),
                     static_cast<size_t>(H) * 8 * sizeof(float), s, partial, H, Kt, cu_nuggets, B, grad_scale, accumulate,
                     grad_scores);
  return launch_status();
}
