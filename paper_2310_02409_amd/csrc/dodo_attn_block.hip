// Query-block nugget attention on the matrix cores (Eq. 13 / Eq. 9 of the Dodo
// paper): each query row attends over all nuggets of its sequence, then over
// the causally visible part of the local (uncompressed) rows.  bf16 inputs,
// fp32 accumulation, d_h = 128.  Inputs must be finite.
//
// Work split: one workgroup (4 wavefronts) owns 128*QB consecutive query rows
// of one (sequence, head); each wavefront owns QB blocks of 32 rows.  Keys
// arrive in tiles of 64: first the dense nugget tiles, then the local tiles up
// to the causal diagonal.  K and V tiles go from global memory straight into
// LDS (16-byte direct loads, several tiles in flight, one barrier per tile),
// row-major with an XOR swizzle chosen so that both read patterns below are
// conflict-free.  Per tile, wavefront and 32-row block:
//   S^T = K Q^T     v_mfma_f32_32x32x16_bf16, A = K rows (LDS), B = Q^T (registers)
//   online softmax in base 2 on the accumulators: lane <-> query row, so row
//   statistics and rescaling are lane-local; one exchange with lane^32
//   O^T += V^T P^T  A = V^T through the transposing LDS read (ds_read_b64_tr_b16),
//   B = P^T taken straight from the S^T accumulators.
// Re-using the accumulators as the B operand fixes which key sits in which
// k-slot; the V^T reads follow the same permutation, so no data crosses lanes.
// With QB = 2 every K / V fragment read from LDS feeds two MFMAs, which halves
// the LDS traffic per flop (at 32 rows per wavefront the 128 B/clk of LDS, not
// the matrix pipe, is the limit), and the softmax of one block runs under the
// MFMAs of the other.  That fast loop keeps a fixed exponent offset per row
// (the maximum of the first tile the row sees), so the output accumulators are
// touched by MFMAs only and can live in the accumulation registers; if some
// logit ever exceeds its row's offset by more than 2^64 the workgroup redoes
// its rows with the exact running-maximum loop.
#include <type_traits>

#include "dodo_attn.h"

namespace dodo {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short shortx4;
typedef __attribute__((ext_vector_type(8))) short shortx8;
typedef __attribute__((ext_vector_type(8))) float floatx8;
typedef __attribute__((ext_vector_type(16))) float floatx16;

constexpr int kBN = 64;        // keys per tile
constexpr int kDH = 128;       // head size
constexpr int kThreads = 256;  // 4 wavefronts
constexpr int kRowBytes = kDH * 2;
constexpr int kTileBytes = kBN * kRowBytes;  // 16 KiB per K or V tile
constexpr float kNegInf = -__builtin_inff();

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void gbl_void;

__device__ __forceinline__ float exp2_hw(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  typedef __attribute__((ext_vector_type(2))) float floatx2;
  const floatx2 f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));  // hardware round-to-nearest-even pack
}

// One 16-byte-per-lane direct global->LDS load: the lanes' data land at lds_base + 16*lane.
// Issued as inline assembly so that the compiler does not order every later LDS read behind all
// outstanding loads (it cannot tell the stages apart); the tile loop does that bookkeeping itself
// with explicit vmcnt waits and a barrier.  lds_base must be wavefront-uniform.
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_base) : "memory");
}

// Enqueues the direct global->LDS loads of one 64 x 128 tile (K or V).  Wavefront w
// fills LDS rows 16w .. 16w+15, 4 rows (1 KiB) per instruction; the lane at LDS
// position (row, pos) fetches the 16-byte piece that the swizzle stores there.
// Rows past the end of the region re-read its last row (finite data, masked later).
template <bool V_SWIZZLE>
__device__ __forceinline__ void issue_tile_load(const uint16_t* __restrict__ region, int64_t tok_stride, int cnt,
                                                uint32_t lds_tile, int wave, int lane) {
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int chunk = wave * 4 + u;
    const int row = chunk * 4 + (lane >> 4);
    const int pos = lane & 15;
    const int piece = V_SWIZZLE ? ((((pos >> 2) ^ (row & 3)) << 2) | (pos & 3)) : (pos ^ (row & 15));
    const int grow = min(row, cnt - 1);
    const uint16_t* src = region + grow * tok_stride + piece * 8;
    dma16(src, __builtin_amdgcn_readfirstlane(lds_tile + chunk * 1024));
  }
}

// Online-softmax update of one 32-row block for one 64-key tile.  acc holds the raw
// S^T accumulators (two 32-key blocks); accumulator v of block kb <-> key 32kb + 8(v/4) + 4g + v%4.
// Returns P^T as MFMA B operands: pf[2kb + half] = accumulators 8*half .. 8*half+7 of block kb.
template <bool MASK>
__device__ __forceinline__ void softmax_tile(floatx16 (&acc)[2], int limit, int g, float scale_log2e, float& m_run,
                                             float& l_run, floatx16 (&acc_o)[kDH / 32], bf16x8 (&pf)[4]) {
  float tmax = kNegInf;
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      float s = acc[kb][v] * scale_log2e;
      if (MASK) {
        const int key = 32 * kb + 8 * (v >> 2) + 4 * g + (v & 3);
        s = (key < limit) ? s : kNegInf;
      }
      acc[kb][v] = s;
      tmax = fmaxf(tmax, s);
    }
  tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
  const float m_new = fmaxf(m_run, tmax);
  const float m_use = (m_new == kNegInf) ? 0.f : m_new;
  float psum = 0.f;
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      floatx8 p;
#pragma unroll
      for (int v = 0; v < 8; ++v) {
        p[v] = exp2_hw(acc[kb][8 * half + v] - m_use);
        psum += p[v];
      }
      pf[2 * kb + half] = __builtin_convertvector(p, bf16x8);  // hardware RNE pack
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
}

template <int QB>
struct BlockCfg {
  static constexpr int kBM = 128 * QB;             // query rows per workgroup
  static constexpr int kStages = QB == 1 ? 2 : 4;  // K/V tiles resident in LDS
  static constexpr int kLdsBytes = kStages * 2 * kTileBytes;
  static constexpr int kMinBlocks = QB == 1 ? 2 : 1;
};

template <int QB>
__global__ __launch_bounds__(kThreads, BlockCfg<QB>::kMinBlocks) void block_attention_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ Kn, const uint16_t* __restrict__ Vn,
    const uint16_t* __restrict__ Kl, const uint16_t* __restrict__ Vl, const int32_t* __restrict__ cu_q,
    const int32_t* __restrict__ cu_nuggets, const int32_t* __restrict__ cu_local, int B, int H, int H_kv,
    int n_qblocks, int64_t nug_tok_stride, int64_t nug_head_stride, float scale_log2e, uint16_t* __restrict__ O,
    float* __restrict__ lse) {
  using Cfg = BlockCfg<QB>;
  constexpr int kBM = Cfg::kBM;
  constexpr int kStages = Cfg::kStages;
  extern __shared__ __attribute__((aligned(1024))) char lds[];  // stage s: K at 2s, V at 2s+1 (tiles of 16 KiB)
  const uint32_t lds_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_void*)lds));

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
  const int w_i0 = i0 + wave * (32 * QB);  // first query row of this wavefront
  const int shift = m_b - q_b + 1;         // query row i sees local rows [0, i + shift)
  int my_i[QB], my_vis[QB];
  bool row_ok[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    my_i[qb] = w_i0 + 32 * qb + j;  // this lane's query row inside the sequence
    row_ok[qb] = my_i[qb] < q_b;
    my_vis[qb] = row_ok[qb] ? max(0, min(m_b, my_i[qb] + shift)) : 0;
  }
  // local rows visible to the first / last query row of this wavefront and to the whole workgroup
  const int w_lo = max(0, min(m_b, w_i0 + shift));
  const int w_hi = max(0, min(m_b, min(w_i0 + 32 * QB - 1, q_b - 1) + shift));
  const int wg_vis = max(0, min(m_b, min(i0 + kBM, q_b) - 1 + shift));

  const int n_nug_tiles = (k_b + kBN - 1) / kBN;
  const int n_loc_tiles = (wg_vis + kBN - 1) / kBN;
  const int n_tiles = n_nug_tiles + n_loc_tiles;

  const uint16_t* nugK = Kn + static_cast<int64_t>(k0) * nug_tok_stride + static_cast<int64_t>(kvh) * nug_head_stride;
  const uint16_t* nugV = Vn + static_cast<int64_t>(k0) * nug_tok_stride + static_cast<int64_t>(kvh) * nug_head_stride;
  const int64_t loc_stride = static_cast<int64_t>(H_kv) * kDH;
  const uint16_t* locK = Kl + (static_cast<int64_t>(l0) * H_kv + kvh) * kDH;
  const uint16_t* locV = Vl + (static_cast<int64_t>(l0) * H_kv + kvh) * kDH;

  // Every call enqueues exactly 8 loads per lane (a tile past the end re-reads the
  // last one into a stage nobody reads), so the vmcnt arithmetic below is uniform.
  auto issue_tile = [&](int tile) {
    const int stage = tile % kStages;
    const int tl = min(tile, n_tiles - 1);
    const bool nug = tl < n_nug_tiles;
    const int base = nug ? tl * kBN : (tl - n_nug_tiles) * kBN;
    const int cnt = min(kBN, (nug ? k_b : wg_vis) - base);
    const int64_t stride = nug ? nug_tok_stride : loc_stride;
    const uint16_t* kp = (nug ? nugK : locK) + base * stride;
    const uint16_t* vp = (nug ? nugV : locV) + base * stride;
    issue_tile_load<false>(kp, stride, cnt, lds_base + (2 * stage) * kTileBytes, wave, lane);
    issue_tile_load<true>(vp, stride, cnt, lds_base + (2 * stage + 1) * kTileBytes, wave, lane);
  };

  // Q^T fragments: lane (j, g) holds Q[my_i][16*ds + 8*g .. +8) for ds = 0..7
  bf16x8 qf[QB][kDH / 16];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const uint16_t* qp = Q + (static_cast<int64_t>(q0 + (row_ok[qb] ? my_i[qb] : 0)) * H + h) * kDH + 8 * g;
#pragma unroll
    for (int ds = 0; ds < kDH / 16; ++ds) {
      const shortx8 raw = *reinterpret_cast<const shortx8*>(qp + 16 * ds);
      const shortx8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
      qf[qb][ds] = __builtin_bit_cast(bf16x8, row_ok[qb] ? raw : zero);
    }
  }

  floatx16 acc_o[QB][kDH / 32];
  float m_run[QB], l_run[QB];

  // per-lane constants of the LDS read patterns
  const int k_row_off = j * kRowBytes;  // K: row 32kb + j, piece (2ds + g) ^ (row & 15); (32kb + j) & 15 == j & 15
  const int k_sw = j & 15;
  // V^T via transposing read: lane supplies row 16t + 8e + 4g + (lane%16)/4, 8 bytes at channel 32cb + 16*half + 4*(lane%4)
  const int v_r = 4 * g + ((lane & 15) >> 2);
  const int v_in = 32 * ((lane >> 4) & 1) + 8 * (lane & 3);

  // One pass over all tiles.  FAST (QB = 2 only): software-pipelined slots with a fixed exponent
  // offset per row; returns true if some logit overflowed the offset (the pass must be redone
  // with FAST = false).  Otherwise: exact running-maximum softmax.
  auto run_pass = [&](auto fast_tag) -> bool {
    constexpr bool FAST = decltype(fast_tag)::value;
    bool bail = false;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      m_run[qb] = kNegInf;
      l_run[qb] = 0.f;
#pragma unroll
      for (int cb = 0; cb < kDH / 32; ++cb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc_o[qb][cb][v] = 0.f;
    }
    if (n_tiles > 0) {
#pragma unroll
      for (int t = 0; t < kStages - 1; ++t) issue_tile(t);
    }

    for (int tile = 0; tile < n_tiles; ++tile) {
      // this wavefront's part of tile `tile` has landed once at most (kStages-2) later tiles are in flight
      if (kStages == 2) {
        __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
      } else {
        __builtin_amdgcn_s_waitcnt(0x4f70);  // vmcnt(16): two younger tiles (8 loads each) may still be in flight
      }
      __syncthreads();  // everyone's part has landed; the stage read during the previous tile is free
      issue_tile(tile + kStages - 1);

      const bool is_nug = tile < n_nug_tiles;
      const int base = is_nug ? tile * kBN : (tile - n_nug_tiles) * kBN;
      const int cnt = min(kBN, (is_nug ? k_b : wg_vis) - base);
      if (!is_nug && base >= w_hi) continue;  // nothing of this tile is visible to this wavefront
      const bool need_mask = cnt < kBN || (!is_nug && base + kBN > w_lo);
      const char* kbuf = lds + (2 * (tile % kStages)) * kTileBytes;
      const char* vbuf = kbuf + kTileBytes;
      int limit[QB];  // keys [0, limit) of this tile are visible to this lane's row
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) limit[qb] = is_nug ? cnt : min(cnt, my_vis[qb] - base);

      // K fragment s = 2*ds + kb (order of use): row 32kb + j, 16 bytes at the swizzled position of piece 2ds + g
      auto read_k = [&](int s) -> bf16x8 {
        return *reinterpret_cast<const bf16x8*>(kbuf + (s & 1) * 32 * kRowBytes + k_row_off +
                                                ((((s >> 1) * 2 + g) ^ k_sw) << 4));
      };
      // V^T fragment s = 4*t + cb: slot 8g+4e+r of k-step t <-> key 16t + 8e + 4g + r
      auto read_vt = [&](int s) -> bf16x8 {
        const int t = s >> 2, cb = s & 3;
        shortx4 a[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int r = 16 * t + 8 * e + v_r;
          const char* p = vbuf + r * kRowBytes + ((cb ^ (r & 3)) << 6) + v_in;
          a[e] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((shortx4 __attribute__((address_space(3)))*)(p));
        }
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(a[0], a[1], 0, 1, 2, 3, 4, 5, 6, 7));
      };

      if constexpr (FAST) {
        // Each 32-key half of the tile runs four slots of 8 MFMAs:
        //   S(0) | S(1) + softmax(0) | PV(0) + softmax(1) | PV(1)
        // so that the VALU work of one 32-row block hides under the MFMAs of the other.
        auto fast_tile = [&](auto mask_tag) {
          constexpr bool MASK = decltype(mask_tag)::value;
          bf16x8 kf[8], kf_next[8];
#pragma unroll
          for (int ds = 0; ds < 8; ++ds) kf[ds] = read_k(2 * ds);
#pragma unroll
          for (int hf = 0; hf < 2; ++hf) {
            bf16x8 vf[8], pf[2][2];
            floatx16 acc_s[2];
            float tmax[2], psum[2];
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
              for (int v = 0; v < 16; ++v) acc_s[qb][v] = 0.f;

            // accumulator v of block qb <-> key 32hf + 8(v/4) + 4g + v%4: mask, track the raw
            // maximum, p = 2^(s*c - offset)
            auto soft_elem = [&](int qb, int v, float neg_m) -> float {
              float sv = acc_s[qb][v];
              if (MASK) {
                const int key = 32 * hf + 8 * (v >> 2) + 4 * g + (v & 3);
                sv = (key < limit[qb]) ? sv : kNegInf;
              }
              tmax[qb] = fmaxf(tmax[qb], sv);
              float pv = exp2_hw(fmaf(sv, scale_log2e, neg_m));
              asm volatile("" : "+v"(pv));  // keep the evaluation in its slot
              psum[qb] += pv;
              return pv;
            };
            // after a slot: rows that had no offset yet take this half's maximum and redo their P
            // (their accumulators are still zero, so nothing is rescaled); overflow raises `bail`
            auto settle = [&](int qb) {
              tmax[qb] = fmaxf(tmax[qb], __shfl_xor(tmax[qb], 32, kWave));
              const float t2 = tmax[qb] * scale_log2e;
              if (__any(m_run[qb] == kNegInf && t2 != kNegInf)) {
                if (m_run[qb] == kNegInf) m_run[qb] = t2;
                const float neg_m = (m_run[qb] == kNegInf) ? 0.f : -m_run[qb];
                psum[qb] = 0.f;
#pragma unroll
                for (int grp = 0; grp < 2; ++grp) {
                  floatx8 pg;
#pragma unroll
                  for (int u = 0; u < 8; ++u) pg[u] = soft_elem(qb, 8 * grp + u, neg_m);
                  pf[qb][grp] = __builtin_convertvector(pg, bf16x8);
                }
              }
              bail = bail || (!(t2 <= m_run[qb] + 64.f) && t2 != kNegInf);
              l_run[qb] += psum[qb];
            };

            // ---- slot 1: S(0) ----
#pragma unroll
            for (int ds = 0; ds < 8; ++ds)
              acc_s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ds], qf[0][ds], acc_s[0], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);

            // ---- slot 2: S(1) under softmax(0); this half's V^T fragments are requested on the way ----
            {
              const float neg_m = (m_run[0] == kNegInf) ? 0.f : -m_run[0];
              tmax[0] = kNegInf;
              psum[0] = 0.f;
              floatx8 pg;
#pragma unroll
              for (int ds = 0; ds < 8; ++ds) {
                acc_s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ds], qf[1][ds], acc_s[1], 0, 0, 0);
                vf[ds] = read_vt(8 * hf + ds);
                pg[(2 * ds) & 7] = soft_elem(0, 2 * ds, neg_m);
                pg[(2 * ds + 1) & 7] = soft_elem(0, 2 * ds + 1, neg_m);
                if ((ds & 3) == 3) pf[0][ds >> 2] = __builtin_convertvector(pg, bf16x8);
                __builtin_amdgcn_sched_barrier(0);
              }
              settle(0);
            }
            __builtin_amdgcn_sched_barrier(0);

            // ---- slot 3: PV(0) under softmax(1); the next half's K fragments are requested on the way ----
            {
              const float neg_m = (m_run[1] == kNegInf) ? 0.f : -m_run[1];
              tmax[1] = kNegInf;
              psum[1] = 0.f;
              floatx8 pg;
#pragma unroll
              for (int s = 0; s < 8; ++s) {
                acc_o[0][s & 3] =
                    __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[s], pf[0][s >> 2], acc_o[0][s & 3], 0, 0, 0);
                if (hf == 0) kf_next[s] = read_k(2 * s + 1);
                pg[(2 * s) & 7] = soft_elem(1, 2 * s, neg_m);
                pg[(2 * s + 1) & 7] = soft_elem(1, 2 * s + 1, neg_m);
                if ((s & 3) == 3) pf[1][s >> 2] = __builtin_convertvector(pg, bf16x8);
                __builtin_amdgcn_sched_barrier(0);
              }
              settle(1);
            }
            __builtin_amdgcn_sched_barrier(0);

            // ---- slot 4: PV(1) ----
#pragma unroll
            for (int s = 0; s < 8; ++s)
              acc_o[1][s & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[s], pf[1][s >> 2], acc_o[1][s & 3], 0, 0, 0);
            if (hf == 0) {
#pragma unroll
              for (int ds = 0; ds < 8; ++ds) kf[ds] = kf_next[ds];
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        };
        if (need_mask) {
          fast_tile(std::true_type{});
        } else {
          fast_tile(std::false_type{});
        }
      } else {
        // ---- S^T = K Q^T : two 32-key blocks ----
        floatx16 acc_s[QB][2];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc_s[qb][kb][v] = 0.f;
#pragma unroll
        for (int s = 0; s < 16; ++s) {
          const bf16x8 kf = read_k(s);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
            acc_s[qb][s & 1] =
                __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qb][s >> 1], acc_s[qb][s & 1], 0, 0, 0);
        }
        // ---- online softmax (base 2) of every 32-row block ----
        bf16x8 pf[QB][4];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          if (need_mask) {
            softmax_tile<true>(acc_s[qb], limit[qb], g, scale_log2e, m_run[qb], l_run[qb], acc_o[qb], pf[qb]);
          } else {
            softmax_tile<false>(acc_s[qb], kBN, g, scale_log2e, m_run[qb], l_run[qb], acc_o[qb], pf[qb]);
          }
        }
        // ---- O^T += V^T P^T ----
#pragma unroll
        for (int s = 0; s < 16; ++s) {
          const bf16x8 vt = read_vt(s);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
            acc_o[qb][s & 3] =
                __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt, pf[qb][s >> 2], acc_o[qb][s & 3], 0, 0, 0);
        }
      }
    }
    __builtin_amdgcn_s_waitcnt(0x0f70);  // drain the look-ahead loads before LDS is reused or the wavefront ends
    return bail;
  };

  if constexpr (QB == 2) {
    // the fast pass needs a positive scale (it tracks the maximum of the raw logits)
    bool redo = !(scale_log2e > 0.f);
    if (!redo) redo = run_pass(std::true_type{});
    if (__syncthreads_or(redo)) run_pass(std::false_type{});
  } else {
    run_pass(std::false_type{});
  }

  // ---- epilogue: lane (j, g) holds channels 32cb + 8(v/4) + 4g + v%4 of query row my_i ----
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32, kWave);
    if (row_ok[qb]) {
      const float inv = (l_tot > 0.f) ? 1.f / l_tot : 0.f;
      uint16_t* op = O + (static_cast<int64_t>(q0 + my_i[qb]) * H + h) * kDH;
#pragma unroll
      for (int cb = 0; cb < kDH / 32; ++cb)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          const int c = 32 * cb + 8 * vq + 4 * g;
          uint2 out;
          out.x = pack2_bf16(acc_o[qb][cb][4 * vq + 0] * inv, acc_o[qb][cb][4 * vq + 1] * inv);
          out.y = pack2_bf16(acc_o[qb][cb][4 * vq + 2] * inv, acc_o[qb][cb][4 * vq + 3] * inv);
          *reinterpret_cast<uint2*>(op + c) = out;
        }
      if (lse != nullptr && g == 0) {
        lse[static_cast<int64_t>(q0 + my_i[qb]) * H + h] =
            (l_tot > 0.f) ? (m_run[qb] + __log2f(l_tot)) * 0.6931471805599453f : kNegInf;
      }
    }
  }
}

template <int QB>
int launch_qb(const AttnParams& p) {
  using Cfg = BlockCfg<QB>;
  const int n_qblocks = (p.max_q + Cfg::kBM - 1) / Cfg::kBM;
  const int64_t grid = static_cast<int64_t>(p.B) * p.H * n_qblocks;
  if (grid > 0x7fffffffLL) return DODO_ERR_UNSUPPORTED;
  auto kern = block_attention_kernel<QB>;
  if (Cfg::kLdsBytes > 64 * 1024) {
    DODO_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                     Cfg::kLdsBytes));
  }
  hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(grid)), dim3(kThreads), Cfg::kLdsBytes, p.stream,
                     static_cast<const uint16_t*>(p.Q), static_cast<const uint16_t*>(p.Kn),
                     static_cast<const uint16_t*>(p.Vn), static_cast<const uint16_t*>(p.Kl),
                     static_cast<const uint16_t*>(p.Vl), p.cu_q, p.cu_nuggets, p.cu_local, p.B, p.H, p.H_kv, n_qblocks,
                     p.nug_tok_stride, p.nug_head_stride, p.scale_log2e, static_cast<uint16_t*>(p.O), p.lse);
  return launch_status();
}

}  // namespace

int launch_block_attention(const AttnParams& p) {
  if (p.dtype != DODO_DTYPE_BF16 || p.d_h != kDH) return DODO_ERR_UNSUPPORTED;
  // 256-row workgroups (64 rows per wavefront) once the query block is long enough to fill them
  if (p.max_q > 128) return launch_qb<2>(p);
  return launch_qb<1>(p);
}

}  // namespace dodo
