// Query-block nugget attention on the matrix cores (Eq. 13 / Eq. 9 of the Dodo
// paper): each query row attends over all nuggets of its sequence, then over
// the causally visible part of the local (uncompressed) rows.  bf16 inputs,
// fp32 accumulation, d_h = 128.  Inputs must be finite.
//
// Work split: one workgroup (4 wavefronts) owns 128 consecutive query rows of
// one (sequence, head); each wavefront owns 32 of them; two workgroups share a
// CU so that one wavefront's softmax overlaps another's MFMAs.  Keys arrive in
// tiles of 64: first the dense nugget tiles, then the local tiles up to the
// causal diagonal.  K and V tiles go from global memory straight into LDS
// (16-byte direct loads, double-buffered, one barrier per tile), row-major with
// an XOR swizzle chosen so that both read patterns below are conflict-free.
// Per tile and wavefront:
//   S^T = K Q^T     v_mfma_f32_32x32x16_bf16, A = K rows (LDS), B = Q^T (registers)
//   online softmax in base 2 on the accumulators: lane <-> query row, so row
//   statistics and rescaling are lane-local; one exchange with lane^32
//   O^T += V^T P^T  A = V^T through the transposing LDS read (ds_read_b64_tr_b16),
//   B = P^T taken straight from the S^T accumulators.
// Re-using the accumulators as the B operand fixes which key sits in which
// k-slot; the V^T reads follow the same permutation, so no data crosses lanes.
#include "dodo_attn.h"

namespace dodo {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short shortx4;
typedef __attribute__((ext_vector_type(16))) float floatx16;

constexpr int kBM = 128;       // query rows per workgroup
constexpr int kBN = 64;        // keys per tile
constexpr int kDH = 128;       // head size
constexpr int kThreads = 256;  // 4 wavefronts x 32 query rows
constexpr int kRowBytes = kDH * 2;
constexpr int kTileBytes = kBN * kRowBytes;  // 16 KiB
constexpr float kNegInf = -__builtin_inff();

typedef __attribute__((ext_vector_type(8))) short shortx8;
typedef __attribute__((ext_vector_type(8))) float floatx8;

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void gbl_void;

__device__ __forceinline__ float exp2_hw(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  typedef __attribute__((ext_vector_type(2))) float floatx2;
  union {
    bf16x2 b;
    uint32_t u;
  } cvt;
  floatx2 f = {lo, hi};
  cvt.b = __builtin_convertvector(f, bf16x2);  // hardware round-to-nearest-even pack
  return cvt.u;
}

// Enqueues the direct global->LDS loads of one 64 x 128 tile (K or V).  Wavefront w
// fills LDS rows 16w .. 16w+15, 4 rows (1 KiB) per instruction; the lane at LDS
// position (row, pos) fetches the 16-byte piece that the swizzle stores there.
// Rows past the end of the region re-read its last row (finite data, masked later).
template <bool V_SWIZZLE>
__device__ __forceinline__ void issue_tile_load(const uint16_t* __restrict__ region, int64_t tok_stride, int cnt,
                                                char* lds_tile, int wave, int lane) {
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int chunk = wave * 4 + u;
    const int row = chunk * 4 + (lane >> 4);
    const int pos = lane & 15;
    const int piece = V_SWIZZLE ? ((((pos >> 2) ^ (row & 3)) << 2) | (pos & 3)) : (pos ^ (row & 15));
    const int grow = min(row, cnt - 1);
    const uint16_t* src = region + grow * tok_stride + piece * 8;
    __builtin_amdgcn_global_load_lds((gbl_void*)(src), (lds_void*)(lds_tile + chunk * 1024), 16, 0, 0);
  }
}

__global__ __launch_bounds__(kThreads, 2) void block_attention_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ Kn, const uint16_t* __restrict__ Vn,
    const uint16_t* __restrict__ Kl, const uint16_t* __restrict__ Vl, const int32_t* __restrict__ cu_q,
    const int32_t* __restrict__ cu_nuggets, const int32_t* __restrict__ cu_local, int B, int H, int H_kv,
    int n_qblocks, int64_t nug_tok_stride, int64_t nug_head_stride, float scale_log2e, uint16_t* __restrict__ O,
    float* __restrict__ lse) {
  __shared__ __attribute__((aligned(1024))) char lds[4 * kTileBytes];  // K[2], V[2]

  // heaviest query blocks (largest causal extent) are scheduled first
  const int bh = blockIdx.x % (B * H);
  const int qblk = n_qblocks - 1 - blockIdx.x / (B * H);
  const int b = bh / H, h = bh % H;
  const int q0 = cu_q[b], q_b = cu_q[b + 1] - q0;
  const int i0 = qblk * kBM;
  if (i0 >= q_b) return;  // uniform over the workgroup
  const int k0 = cu_nuggets[b], k_b = cu_nuggets[b + 1] - k0;
  const int l0 = cu_local[b], m_b = cu_local[b + 1] - l0;
  const int kvh = h / (H / H_kv);

  const int tid = threadIdx.x;
  const int wave = tid / kWave, lane = tid % kWave;
  const int j = lane & 31, g = lane >> 5;
  const int my_i = i0 + wave * 32 + j;  // this lane's query row inside the sequence
  const bool row_ok = my_i < q_b;
  const int shift = m_b - q_b + 1;  // query row i sees local rows [0, i + shift)
  const int my_vis = row_ok ? max(0, min(m_b, my_i + shift)) : 0;
  // local rows visible to the first / last query row of this wavefront and to the whole workgroup
  const int w_lo = max(0, min(m_b, i0 + wave * 32 + shift));
  const int w_hi = max(0, min(m_b, min(i0 + wave * 32 + 31, q_b - 1) + shift));
  const int wg_vis = max(0, min(m_b, min(i0 + kBM, q_b) - 1 + shift));

  const int n_nug_tiles = (k_b + kBN - 1) / kBN;
  const int n_loc_tiles = (wg_vis + kBN - 1) / kBN;
  const int n_tiles = n_nug_tiles + n_loc_tiles;

  const uint16_t* nugK = Kn + static_cast<int64_t>(k0) * nug_tok_stride + static_cast<int64_t>(kvh) * nug_head_stride;
  const uint16_t* nugV = Vn + static_cast<int64_t>(k0) * nug_tok_stride + static_cast<int64_t>(kvh) * nug_head_stride;
  const int64_t loc_stride = static_cast<int64_t>(H_kv) * kDH;
  const uint16_t* locK = Kl + (static_cast<int64_t>(l0) * H_kv + kvh) * kDH;
  const uint16_t* locV = Vl + (static_cast<int64_t>(l0) * H_kv + kvh) * kDH;

  auto issue_tile = [&](int tile) {
    const bool nug = tile < n_nug_tiles;
    const int base = nug ? tile * kBN : (tile - n_nug_tiles) * kBN;
    const int cnt = min(kBN, (nug ? k_b : wg_vis) - base);
    const int64_t stride = nug ? nug_tok_stride : loc_stride;
    const uint16_t* kp = (nug ? nugK : locK) + base * stride;
    const uint16_t* vp = (nug ? nugV : locV) + base * stride;
    issue_tile_load<false>(kp, stride, cnt, lds + (tile & 1) * kTileBytes, wave, lane);
    issue_tile_load<true>(vp, stride, cnt, lds + (2 + (tile & 1)) * kTileBytes, wave, lane);
  };

  if (n_tiles > 0) issue_tile(0);

  // Q^T fragments: lane (j, g) holds Q[my_i][16*ds + 8*g .. +8) for ds = 0..7
  bf16x8 qf[kDH / 16];
  {
    const uint16_t* qp = Q + (static_cast<int64_t>(q0 + (row_ok ? my_i : 0)) * H + h) * kDH + 8 * g;
#pragma unroll
    for (int ds = 0; ds < kDH / 16; ++ds) {
      const shortx8 raw = *reinterpret_cast<const shortx8*>(qp + 16 * ds);
      const shortx8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
      qf[ds] = __builtin_bit_cast(bf16x8, row_ok ? raw : zero);
    }
  }

  floatx16 acc_o[kDH / 32];
#pragma unroll
  for (int cb = 0; cb < kDH / 32; ++cb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc_o[cb][v] = 0.f;
  float m_run = kNegInf, l_run = 0.f;

  // per-lane constants of the LDS read patterns
  const int k_row_off = j * kRowBytes;  // K: row 32kb + j, piece (2ds + g) ^ (row & 15); (32kb + j) & 15 == j & 15
  const int k_sw = j & 15;
  // V^T via transposing read: lane supplies row 16t + 8e + 4g + (lane%16)/4, 8 bytes at channel 32cb + 16*half + 4*(lane%4)
  const int v_r = 4 * g + ((lane & 15) >> 2);
  const int v_in = 32 * ((lane >> 4) & 1) + 8 * (lane & 3);

  for (int tile = 0; tile < n_tiles; ++tile) {
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wavefront's part of the tile has landed
    __syncthreads();                      // everyone's part has landed; the other buffer is free
    if (tile + 1 < n_tiles) issue_tile(tile + 1);

    const bool is_nug = tile < n_nug_tiles;
    const int base = is_nug ? tile * kBN : (tile - n_nug_tiles) * kBN;
    const int cnt = min(kBN, (is_nug ? k_b : wg_vis) - base);
    if (!is_nug && base >= w_hi) continue;  // nothing of this tile is visible to this wavefront
    const bool need_mask = cnt < kBN || (!is_nug && base + kBN > w_lo);
    const char* kbuf = lds + (tile & 1) * kTileBytes;
    const char* vbuf = lds + (2 + (tile & 1)) * kTileBytes;

    // ---- S^T = K Q^T : two 32-key blocks; all 16 K fragments are requested before the first MFMA ----
    bf16x8 kf[2][kDH / 16];
#pragma unroll
    for (int ds = 0; ds < kDH / 16; ++ds)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
        kf[kb][ds] =
            *reinterpret_cast<const bf16x8*>(kbuf + kb * 32 * kRowBytes + k_row_off + (((2 * ds + g) ^ k_sw) << 4));
    floatx16 acc_s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc_s[kb][v] = 0.f;
#pragma unroll
    for (int ds = 0; ds < kDH / 16; ++ds)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
        acc_s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb][ds], qf[ds], acc_s[kb], 0, 0, 0);

    // ---- V^T fragments for the whole tile are requested now and land while the softmax runs ----
    // slot 8g+4e+r of k-step t <-> key 16t + 8e + 4g + r
    shortx4 vf[4][kDH / 32][2];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int cb = 0; cb < kDH / 32; ++cb)
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int r = 16 * t + 8 * e + v_r;
          const char* p = vbuf + r * kRowBytes + ((cb ^ (r & 3)) << 6) + v_in;
          vf[t][cb][e] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((shortx4 __attribute__((address_space(3)))*)(p));
        }

    // ---- online softmax (base 2); accumulator v of block kb <-> key 32kb + 8(v/4) + 4g + v%4 ----
    float tmax = kNegInf;
    if (need_mask) {
      const int limit = is_nug ? cnt : min(cnt, my_vis - base);  // keys [0, limit) of this tile are visible
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = 32 * kb + 8 * (v >> 2) + 4 * g + (v & 3);
          const float s = (key < limit) ? acc_s[kb][v] * scale_log2e : kNegInf;
          acc_s[kb][v] = s;
          tmax = fmaxf(tmax, s);
        }
    } else {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float s = acc_s[kb][v] * scale_log2e;
          acc_s[kb][v] = s;
          tmax = fmaxf(tmax, s);
        }
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
    const float m_new = fmaxf(m_run, tmax);
    const float m_use = (m_new == kNegInf) ? 0.f : m_new;
    float psum = 0.f;
    bf16x8 pf[4];  // P^T as B operand: pf[2kb + half] = accumulators 8*half .. 8*half+7 of block kb
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        floatx8 p;
#pragma unroll
        for (int v = 0; v < 8; ++v) {
          p[v] = exp2_hw(acc_s[kb][8 * half + v] - m_use);
          psum += p[v];
        }
        pf[2 * kb + half] = __builtin_convertvector(p, bf16x8);  // hardware RNE pack
      }
    }
    if (__any(m_new != m_run)) {  // rescale only when some row's maximum moved
      const float alpha = exp2_hw(m_run - m_use);  // m_run = -inf -> 0
      l_run *= alpha;
#pragma unroll
      for (int cb = 0; cb < kDH / 32; ++cb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc_o[cb][v] *= alpha;
      m_run = m_new;
    }
    l_run += psum;

    // ---- O^T += V^T P^T ----
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
      for (int cb = 0; cb < kDH / 32; ++cb) {
        const shortx8 a8 = __builtin_shufflevector(vf[t][cb][0], vf[t][cb][1], 0, 1, 2, 3, 4, 5, 6, 7);
        acc_o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a8), pf[t], acc_o[cb], 0, 0, 0);
      }
    }
  }

  // ---- epilogue: lane (j, g) holds channels 32cb + 8(v/4) + 4g + v%4 of query row my_i ----
  const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
  if (row_ok) {
    const float inv = (l_tot > 0.f) ? 1.f / l_tot : 0.f;
    uint16_t* op = O + (static_cast<int64_t>(q0 + my_i) * H + h) * kDH;
#pragma unroll
    for (int cb = 0; cb < kDH / 32; ++cb)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        const int c = 32 * cb + 8 * vq + 4 * g;
        uint2 out;
        out.x = pack2_bf16(acc_o[cb][4 * vq + 0] * inv, acc_o[cb][4 * vq + 1] * inv);
        out.y = pack2_bf16(acc_o[cb][4 * vq + 2] * inv, acc_o[cb][4 * vq + 3] * inv);
        *reinterpret_cast<uint2*>(op + c) = out;
      }
    if (lse != nullptr && g == 0) {
      lse[static_cast<int64_t>(q0 + my_i) * H + h] =
          (l_tot > 0.f) ? (m_run + __log2f(l_tot)) * 0.6931471805599453f : kNegInf;
    }
  }
}

}  // namespace

int launch_block_attention(const AttnParams& p) {
  if (p.dtype != DODO_DTYPE_BF16 || p.d_h != kDH) return DODO_ERR_UNSUPPORTED;
  const int n_qblocks = (p.max_q + kBM - 1) / kBM;
  const int64_t grid = static_cast<int64_t>(p.B) * p.H * n_qblocks;
  if (grid > 0x7fffffffLL) return DODO_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(block_attention_kernel, dim3(static_cast<unsigned>(grid)), dim3(kThreads), 0, p.stream,
                     static_cast<const uint16_t*>(p.Q), static_cast<const uint16_t*>(p.Kn),
                     static_cast<const uint16_t*>(p.Vn), static_cast<const uint16_t*>(p.Kl),
                     static_cast<const uint16_t*>(p.Vl), p.cu_q, p.cu_nuggets, p.cu_local, p.B, p.H, p.H_kv, n_qblocks,
                     p.nug_tok_stride, p.nug_head_stride, p.scale_log2e, static_cast<uint16_t*>(p.O), p.lse);
  return launch_status();
}

}  // namespace dodo
