// Query-block nugget attention on the matrix cores (Eq. 13 / Eq. 9 of the Dodo
// paper): each query row attends over all nuggets of its sequence, then over
// the causally visible part of the local (uncompressed) rows.  bf16 inputs,
// fp32 accumulation, d_h = 128.
//
// Work split: one workgroup (4 wavefronts) owns 128 consecutive query rows of
// one (sequence, head); each wavefront owns 32 of them.  Keys arrive in tiles
// of 64: first the dense nugget tiles, then the local tiles up to the causal
// diagonal.  Per tile and wavefront:
//   S^T = K Q^T     v_mfma_f32_32x32x16_bf16, A = K rows from LDS, B = Q^T held in registers
//   online softmax in base 2 on the accumulators (lane <-> query row, so all
//   row statistics and rescaling are lane-local; one exchange with lane^32)
//   O^T += V^T P^T  A = V^T from LDS (V is transposed while it is staged),
//   B = P^T straight from the S^T accumulators.
// The k-slot -> key permutation implied by re-using the accumulators as the B
// operand is mirrored in how V^T is read, so no data moves between lanes.
#include "dodo_attn.h"

namespace dodo {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float floatx16;

constexpr int kBM = 128;       // query rows per workgroup
constexpr int kBN = 64;        // keys per tile
constexpr int kDH = 128;       // head size
constexpr int kThreads = 256;  // 4 wavefronts x 32 query rows
constexpr int kKStride = kDH + 8;   // bf16 elements per K row in LDS (272 B: conflict-free 16-byte reads)
constexpr int kVtStride = kBN + 4;  // bf16 elements per V^T row in LDS (136 B)
constexpr float kNegInf = -__builtin_inff();

union Frag {
  uint4 u;
  bf16x8 v;
};

__device__ __forceinline__ float exp2_hw(float x) { return __builtin_amdgcn_exp2f(x); }

__global__ __launch_bounds__(kThreads) void block_attention_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ Kn, const uint16_t* __restrict__ Vn,
    const uint16_t* __restrict__ Kl, const uint16_t* __restrict__ Vl, const int32_t* __restrict__ cu_q,
    const int32_t* __restrict__ cu_nuggets, const int32_t* __restrict__ cu_local, int B, int H, int H_kv,
    int n_qblocks, int64_t nug_tok_stride, int64_t nug_head_stride, float scale_log2e, uint16_t* __restrict__ O,
    float* __restrict__ lse) {
  __shared__ __attribute__((aligned(16))) uint16_t Ks[kBN * kKStride];
  __shared__ __attribute__((aligned(16))) uint16_t Vt[kDH * kVtStride];

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
  const int my_i = i0 + wave * 32 + j;   // this lane's query row inside the sequence
  const bool row_ok = my_i < q_b;
  // local rows visible to this lane's query: [0, my_vis)
  const int my_vis = row_ok ? max(0, min(m_b, m_b - q_b + my_i + 1)) : 0;
  // local rows any query of this workgroup can see
  const int i_last = min(i0 + kBM, q_b) - 1;
  const int wg_vis = max(0, min(m_b, m_b - q_b + i_last + 1));

  // Q^T fragments: lane (j, g) holds Q[my_i][16*ds + 8*g .. +8) for ds = 0..7
  Frag qf[kDH / 16];
  {
    const uint16_t* qp = Q + (static_cast<int64_t>(q0 + (row_ok ? my_i : 0)) * H + h) * kDH + 8 * g;
#pragma unroll
    for (int ds = 0; ds < kDH / 16; ++ds) {
      qf[ds].u = row_ok ? *reinterpret_cast<const uint4*>(qp + 16 * ds) : make_uint4(0, 0, 0, 0);
    }
  }

  floatx16 acc_o[kDH / 32];
#pragma unroll
  for (int cb = 0; cb < kDH / 32; ++cb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc_o[cb][v] = 0.f;
  float m_run = kNegInf, l_run = 0.f;

  const int n_nug_tiles = (k_b + kBN - 1) / kBN;
  const int n_loc_tiles = (wg_vis + kBN - 1) / kBN;

  for (int tile = 0; tile < n_nug_tiles + n_loc_tiles; ++tile) {
    const bool is_nug = tile < n_nug_tiles;
    const int base = is_nug ? tile * kBN : (tile - n_nug_tiles) * kBN;  // first row of the tile in its region
    const int cnt = min(kBN, (is_nug ? k_b : wg_vis) - base);          // rows of the tile that exist
    const uint16_t* kbase;
    const uint16_t* vbase;
    int64_t tok_stride;
    if (is_nug) {
      const int64_t off = static_cast<int64_t>(k0 + base) * nug_tok_stride + static_cast<int64_t>(kvh) * nug_head_stride;
      kbase = Kn + off;
      vbase = Vn + off;
      tok_stride = nug_tok_stride;
    } else {
      const int64_t off = (static_cast<int64_t>(l0 + base) * H_kv + kvh) * kDH;
      kbase = Kl + off;
      vbase = Vl + off;
      tok_stride = static_cast<int64_t>(H_kv) * kDH;
    }

    __syncthreads();  // previous tile fully consumed
    // ---- stage K (row-major, padded) ----
#pragma unroll
    for (int u = 0; u < (kBN * kDH / 8) / kThreads; ++u) {
      const int id = tid + u * kThreads;
      const int key = id >> 4, cc = id & 15;
      uint4 val = make_uint4(0, 0, 0, 0);
      if (key < cnt) val = *reinterpret_cast<const uint4*>(kbase + key * tok_stride + cc * 8);
      *reinterpret_cast<uint4*>(&Ks[key * kKStride + cc * 8]) = val;
    }
    // ---- stage V transposed: two adjacent keys per thread give one dword per channel ----
#pragma unroll
    for (int u = 0; u < (kBN / 2 * kDH / 8) / kThreads; ++u) {
      const int id = tid + u * kThreads;
      const int kp = id >> 4, cc = id & 15;
      uint4 a = make_uint4(0, 0, 0, 0), c = make_uint4(0, 0, 0, 0);
      if (2 * kp < cnt) a = *reinterpret_cast<const uint4*>(vbase + (2 * kp) * tok_stride + cc * 8);
      if (2 * kp + 1 < cnt) c = *reinterpret_cast<const uint4*>(vbase + (2 * kp + 1) * tok_stride + cc * 8);
      const uint32_t av[4] = {a.x, a.y, a.z, a.w}, cv[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t even = (av[e] & 0xffffu) | (cv[e] << 16);          // channel 8cc+2e   of keys 2kp, 2kp+1
        const uint32_t odd = (av[e] >> 16) | (cv[e] & 0xffff0000u);       // channel 8cc+2e+1 of keys 2kp, 2kp+1
        *reinterpret_cast<uint32_t*>(&Vt[(cc * 8 + 2 * e) * kVtStride + 2 * kp]) = even;
        *reinterpret_cast<uint32_t*>(&Vt[(cc * 8 + 2 * e + 1) * kVtStride + 2 * kp]) = odd;
      }
    }
    __syncthreads();

    // ---- S^T = K Q^T : two 32-key blocks ----
    floatx16 acc_s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc_s[kb][v] = 0.f;
#pragma unroll
    for (int ds = 0; ds < kDH / 16; ++ds) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        Frag a;
        a.u = *reinterpret_cast<const uint4*>(&Ks[(kb * 32 + j) * kKStride + 16 * ds + 8 * g]);
        acc_s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, qf[ds].v, acc_s[kb], 0, 0, 0);
      }
    }

    // ---- online softmax (base 2); accumulator v of block kb <-> key 32kb + 8(v/4) + 4g + v%4 ----
    const int limit = is_nug ? cnt : min(cnt, my_vis - base);  // keys [0, limit) of this tile are visible
    float tmax = kNegInf;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = 32 * kb + 8 * (v >> 2) + 4 * g + (v & 3);
        const float s = (key < limit) ? acc_s[kb][v] * scale_log2e : kNegInf;
        acc_s[kb][v] = s;
        tmax = fmaxf(tmax, s);
      }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
    const float m_new = fmaxf(m_run, tmax);
    const float m_use = (m_new == kNegInf) ? 0.f : m_new;
    const float alpha = exp2_hw(m_run - m_use);  // m_run = -inf -> 0
    float psum = 0.f;
    Frag pf[4];  // P^T as B operand: pf[2kb + half] = accumulators 8*half .. 8*half+7 of block kb
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      float p[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        p[v] = exp2_hw(acc_s[kb][v] - m_use);
        psum += p[v];
      }
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        pf[2 * kb + half].u = make_uint4(pack_bf16(p[8 * half + 0], p[8 * half + 1]), pack_bf16(p[8 * half + 2], p[8 * half + 3]),
                                         pack_bf16(p[8 * half + 4], p[8 * half + 5]), pack_bf16(p[8 * half + 6], p[8 * half + 7]));
      }
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int cb = 0; cb < kDH / 32; ++cb)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc_o[cb][v] *= alpha;

    // ---- O^T += V^T P^T : slot 8g+4e+r of k-step t <-> key 16t + 8e + 4g + r ----
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
      for (int cb = 0; cb < kDH / 32; ++cb) {
        const uint16_t* vrow = &Vt[(cb * 32 + j) * kVtStride + 16 * t + 4 * g];
        const uint2 lo = *reinterpret_cast<const uint2*>(vrow);
        const uint2 hi = *reinterpret_cast<const uint2*>(vrow + 8);
        Frag a;
        a.u = make_uint4(lo.x, lo.y, hi.x, hi.y);
        acc_o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, pf[t].v, acc_o[cb], 0, 0, 0);
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
        out.x = pack_bf16(acc_o[cb][4 * vq + 0] * inv, acc_o[cb][4 * vq + 1] * inv);
        out.y = pack_bf16(acc_o[cb][4 * vq + 2] * inv, acc_o[cb][4 * vq + 3] * inv);
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
