// Query-block nugget attention on the matrix cores (Eq. 13 / Eq. 9 of the Dodo
// paper): each query row attends over all nuggets of its sequence, then over
// the causally visible part of the local (uncompressed) rows.  bf16 inputs,
// fp32 accumulation, d_h = 128 or 64 (a template parameter: the tile loops, LDS
// layout and fragment counts follow from it).  Inputs must be finite.
//
// Work split: one workgroup owns NW*32 consecutive query rows of one (sequence,
// head); each wavefront owns 32 of them.  Keys arrive in tiles of 64: first the
// dense nugget tiles, then the local tiles up to the causal diagonal.  K and V
// tiles go from global memory straight into LDS (16-byte direct loads issued as
// inline assembly, so that the compiler does not order every later LDS read behind
// all outstanding loads: the tile loops keep that count themselves; several
// tiles in flight), row-major with an XOR swizzle chosen so that both read
// patterns below are conflict-free.  Per tile and wavefront:
//   S^T = K Q^T     v_mfma_f32_32x32x16_bf16, A = K rows (LDS), B = Q^T (registers)
//   online softmax in base 2 on the accumulators: lane <-> query row, so row
//   statistics and rescaling are lane-local; one exchange with lane^32
//   O^T += V^T P^T  A = V^T through the transposing LDS read (ds_read_b64_tr_b16),
//   B = P^T taken straight from the S^T accumulators.
// Re-using the accumulators as the B operand fixes which key sits in which
// k-slot; the V^T reads follow the same permutation, so no data crosses lanes.
//
// A single wavefront runs its MFMA and its softmax (VALU) work one after the
// other, and two wavefronts that share a SIMD drift into the same phase, so the
// matrix pipe idles while both do softmax.  The 8-wavefront kernel therefore
// runs two groups of four wavefronts (one of each per SIMD) half a tile apart,
// separated by workgroup barriers: while one group issues the 32 MFMAs of
// "PV(t-1), then S(t)", the other does the softmax of its tile.  Small query
// blocks (<= 128 rows) use a plain 4-wavefront kernel.
#include <type_traits>

#include "dodo_attn.h"

namespace dodo {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short shortx4;
typedef __attribute__((ext_vector_type(8))) short shortx8;
typedef __attribute__((ext_vector_type(8))) float floatx8;
typedef __attribute__((ext_vector_type(16))) float floatx16;

constexpr int kBN = 64;   // keys per tile
// What follows from the head size DH (128 or 64)
template <int DH>
struct HeadDims {
  static constexpr int kRowBytes = DH * 2;
  static constexpr int kTileBytes = kBN * kRowBytes;  // 16 KiB (DH = 128) or 8 KiB (DH = 64) per K or V tile
  static constexpr int kPieces = kRowBytes / 16;      // 16-byte pieces of a row
  static constexpr int kPiecesLog2 = DH == 128 ? 4 : 3;
  // Rows of 128 bytes cover half of the LDS banks, so two consecutive rows sit side by side and the swizzles take
  // the row's index from bit 1 on; rows of 256 bytes cover all banks and use the index as it is.
  static constexpr int kRowShift = DH == 128 ? 0 : 1;
  static constexpr int kChannelBlocks = DH / 32;      // 32-channel blocks of O^T = 64-byte granules of a V row
  static constexpr int kSteps = DH / 8;               // MFMAs per tile of S^T = K Q^T (2 key blocks x DH/16), and of
                                                      // O^T += V^T P^T (4 key steps x DH/32 channel blocks)
};
constexpr float kNegInf = -__builtin_inff();

typedef __attribute__((address_space(3))) void lds_void;

__device__ __forceinline__ float exp2_hw(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint32_t pack2_bf16(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  typedef __attribute__((ext_vector_type(2))) float floatx2;
  const floatx2 f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));  // hardware round-to-nearest-even pack
}

// Per-lane part of the tile loads.  A 64 x DH tile is 64 * P pieces of 16 bytes (P = 16 or 8 per row); wavefront
// w of NW fills LDS rows (64/NW)*w ..., 64/P rows (1 KiB) per instruction.  The lane at LDS position
// (row, pos) fetches the piece that the swizzle stores there:
//   K: piece = pos ^ (r & (P-1))                      (16-byte granules, for the 16-byte row reads)
//   V: piece = ((pos/4) ^ (r & (P/4-1)))*4 + pos%4    (64-byte granules, for the transposing reads)
// with r = row >> kRowShift.
template <int NW, int DH>
struct TileLoader {
  static constexpr int kP = HeadDims<DH>::kPieces;
  static constexpr int kRowsPerInstr = 64 / kP;
  static constexpr int kGranMask = HeadDims<DH>::kChannelBlocks - 1;
  static constexpr int kRowShift = HeadDims<DH>::kRowShift;
  static constexpr int kPerWave = (kBN / kRowsPerInstr) / NW;  // load instructions per wavefront per tile and tensor
  int row0;                // LDS row of this lane in the wavefront's first instruction
  uint32_t pos;            // 16-byte position inside the row
  uint32_t v_piece_bytes;  // the V swizzle term is the same for all of the wavefront's instructions
  uint32_t lds_chunk0;     // byte offset of the wavefront's first 1 KiB chunk inside a tile

  __device__ __forceinline__ void init(int wave, int lane) {
    row0 = wave * kPerWave * kRowsPerInstr + (lane >> HeadDims<DH>::kPiecesLog2);
    pos = lane & (kP - 1);
    v_piece_bytes = ((((pos >> 2) ^ ((row0 >> kRowShift) & kGranMask)) << 2) | (pos & 3)) * 16u;
    lds_chunk0 = wave * kPerWave * 1024;
  }
  // Rows past the end of the region re-read its last row (finite data, masked later).
  __device__ __forceinline__ void issue(const uint16_t* kbase, const uint16_t* vbase, uint32_t stride_bytes, int cnt,
                                        uint32_t lds_k, uint32_t lds_v) const {
#pragma unroll
    for (int u = 0; u < kPerWave; ++u) {
      const int row = row0 + kRowsPerInstr * u;
      const uint32_t roff = static_cast<uint32_t>(min(row, cnt - 1)) * stride_bytes;
      const uint32_t k_piece_bytes = (pos ^ ((row >> kRowShift) & (kP - 1))) * 16u;
      dma16_uniform(kbase, roff + k_piece_bytes, __builtin_amdgcn_readfirstlane(lds_k + lds_chunk0 + u * 1024));
      dma16_uniform(vbase, roff + v_piece_bytes, __builtin_amdgcn_readfirstlane(lds_v + lds_chunk0 + u * 1024));
    }
  }
  // 64 rows in the V arrangement only
  __device__ __forceinline__ void issue_rows_v(const uint16_t* base, uint32_t stride_bytes, int cnt, uint32_t lds_dst) const {
#pragma unroll
    for (int u = 0; u < kPerWave; ++u) {
      const uint32_t roff = static_cast<uint32_t>(min(row0 + kRowsPerInstr * u, cnt - 1)) * stride_bytes;
      dma16_uniform(base, roff + v_piece_bytes, __builtin_amdgcn_readfirstlane(lds_dst + lds_chunk0 + u * 1024));
    }
  }
  // 64 rows in the K arrangement only (also used for the query rows)
  __device__ __forceinline__ void issue_rows(const uint16_t* base, uint32_t stride_bytes, int cnt, uint32_t lds_dst) const {
#pragma unroll
    for (int u = 0; u < kPerWave; ++u) {
      const int row = row0 + kRowsPerInstr * u;
      const uint32_t roff = static_cast<uint32_t>(min(row, cnt - 1)) * stride_bytes;
      dma16_uniform(base, roff + (pos ^ ((row >> kRowShift) & (kP - 1))) * 16u, __builtin_amdgcn_readfirstlane(lds_dst + lds_chunk0 + u * 1024));
    }
  }
  // The same three with the rows taken through an index list: row r of the tile is token idx[r] of `base`
  // (idx points into LDS at the tile's first entry).
  __device__ __forceinline__ void issue_idx(const uint16_t* kbase, const uint16_t* vbase, uint32_t stride_bytes, int cnt,
                                            uint32_t lds_k, uint32_t lds_v, const int32_t* idx) const {
#pragma unroll
    for (int u = 0; u < kPerWave; ++u) {
      const int row = row0 + kRowsPerInstr * u;
      const uint32_t roff = static_cast<uint32_t>(idx[min(row, cnt - 1)]) * stride_bytes;
      const uint32_t k_piece_bytes = (pos ^ ((row >> kRowShift) & (kP - 1))) * 16u;
      dma16_uniform(kbase, roff + k_piece_bytes, __builtin_amdgcn_readfirstlane(lds_k + lds_chunk0 + u * 1024));
      dma16_uniform(vbase, roff + v_piece_bytes, __builtin_amdgcn_readfirstlane(lds_v + lds_chunk0 + u * 1024));
    }
  }
  __device__ __forceinline__ void issue_rows_v_idx(const uint16_t* base, uint32_t stride_bytes, int cnt, uint32_t lds_dst,
                                                   const int32_t* idx) const {
#pragma unroll
    for (int u = 0; u < kPerWave; ++u) {
      const uint32_t roff = static_cast<uint32_t>(idx[min(row0 + kRowsPerInstr * u, cnt - 1)]) * stride_bytes;
      dma16_uniform(base, roff + v_piece_bytes, __builtin_amdgcn_readfirstlane(lds_dst + lds_chunk0 + u * 1024));
    }
  }
  __device__ __forceinline__ void issue_rows_idx(const uint16_t* base, uint32_t stride_bytes, int cnt, uint32_t lds_dst,
                                                 const int32_t* idx) const {
#pragma unroll
    for (int u = 0; u < kPerWave; ++u) {
      const int row = row0 + kRowsPerInstr * u;
      const uint32_t roff = static_cast<uint32_t>(idx[min(row, cnt - 1)]) * stride_bytes;
      dma16_uniform(base, roff + (pos ^ ((row >> kRowShift) & (kP - 1))) * 16u, __builtin_amdgcn_readfirstlane(lds_dst + lds_chunk0 + u * 1024));
    }
  }
};

// Online-softmax update of one 32-row block for one 64-key tile.  acc holds the raw
// S^T accumulators (two 32-key blocks); accumulator v of block kb <-> key 32kb + 8(v/4) + 4g + v%4.
// Returns P^T as MFMA B operands: pf[2kb + half] = accumulators 8*half .. 8*half+7 of block kb.
template <bool MASK, int NCB>
__device__ __forceinline__ void softmax_tile(floatx16 (&acc)[2], int limit, int g, float scale_log2e, float& m_run,
                                             float& l_run, floatx16 (&acc_o)[NCB], bf16x8 (&pf)[4]) {
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
  // The running sums are rescaled unconditionally: a data-dependent skip would add a branch around
  // 64 live accumulators, which costs more in register copies than the multiplies it saves.
  const float alpha = exp2_hw(m_run - m_use);  // m_run = -inf -> 0
  l_run *= alpha;
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc_o[cb][v] *= alpha;
  m_run = m_new;
  l_run += psum;
}

// Softmax update with a fixed exponent offset per row (used by the two-group kernel): the offset
// m_off is the row maximum of the first tile the row sees and is never moved afterwards, so the
// output accumulators are not rescaled -- O = sum(p v) / sum(p) does not depend on the offset.
// An overflow of the fixed offset shows up as a non-finite row sum at the end, in which case the
// caller redoes the rows with softmax_tile.  Needs scale_log2e > 0.
template <bool MASK, bool SUMS>
__device__ __forceinline__ void softmax_fixed(floatx16 (&acc)[2], int limit, int g, float scale_log2e, float& m_off,
                                              float& l_run, bf16x8 (&pf)[4]) {
  if (MASK) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = 32 * kb + 8 * (v >> 2) + 4 * g + (v & 3);
        acc[kb][v] = (key < limit) ? acc[kb][v] : kNegInf;
      }
  }
  if (__any(m_off == kNegInf)) {  // some row of this wavefront has no offset yet (first visible tile)
    float tmax = kNegInf;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) tmax = fmaxf(tmax, acc[kb][v]);
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
    m_off = (m_off == kNegInf) ? tmax * scale_log2e : m_off;  // such rows have all-zero accumulators
  }
  const float neg = (m_off == kNegInf) ? 0.f : -m_off;
  float psum[2] = {0.f, 0.f};
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      floatx8 p;
#pragma unroll
      for (int v = 0; v < 8; ++v) p[v] = exp2_hw(fmaf(acc[kb][8 * half + v], scale_log2e, neg));
      if (SUMS) psum[kb] += ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
      pf[2 * kb + half] = __builtin_convertvector(p, bf16x8);  // hardware RNE pack
    }
  if (SUMS) l_run += psum[0] + psum[1];
}

// NW = 4: plain loop, two workgroups per CU.  NW = 8: two groups of four wavefronts in
// alternating MFMA / softmax phases, one workgroup per CU.
template <int NW, int DH>
struct BlockCfg {
  static constexpr int kThreads = NW * kWave;
  static constexpr int kBM = NW * 32;              // query rows per workgroup
  static constexpr int kStages = NW == 4 ? 2 : 4;  // K/V tiles resident in LDS
  static constexpr int kLdsBytes = kStages * 2 * HeadDims<DH>::kTileBytes;
  static constexpr int kMinBlocks = NW == 4 ? 2 : 1;
  // gather-free form: the sequence's index list sits in LDS after the stages (160 KiB per compute unit in all)
  static constexpr int kIdxCap = NW == 4 ? 4096 : 7680;  // (the 8-wavefront kernel has 1 KiB of static LDS besides)
  static constexpr int kIdxBytes = kIdxCap * 4;
};

// What a query block needs to know of its sequence: first rows and lengths of its queries, nuggets and local rows
// (and, gather-free form, the first token of its context).  Read with scalar loads by load_seq_geom, for both query
// blocks of a workgroup at the kernel's start, so that no block begins with a chain of dependent loads.
struct SeqGeom {
  int b, h, kvh;
  int q0, q_b, k0, k_b, l0, m_b;
  int64_t ctx0;
};
template <bool IDX>
__device__ __forceinline__ SeqGeom load_seq_geom(int bh, FastDiv div_H, int H, FastDiv div_G,
                                                 const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_nuggets,
                                                 const int32_t* __restrict__ nug_len, const int32_t* __restrict__ cu_local,
                                                 const int32_t* __restrict__ loc_len, const int32_t* __restrict__ cu_ctx) {
  SeqGeom g;
  g.b = static_cast<int>(fast_div(static_cast<uint32_t>(bh), div_H));
  g.h = bh - g.b * H;
  g.kvh = static_cast<int>(fast_div(static_cast<uint32_t>(g.h), div_G));
  const int32_t* k_end_p = nug_len != nullptr ? nug_len + g.b : cu_nuggets + g.b + 1;
  const int32_t* l_end_p = loc_len != nullptr ? loc_len + g.b : cu_local + g.b + 1;
  g.q0 = cu_q[g.b];
  const int q_end = cu_q[g.b + 1];
  g.k0 = cu_nuggets[g.b];
  const int k_end = *k_end_p;
  g.l0 = cu_local[g.b];
  const int l_end = *l_end_p;
  g.ctx0 = IDX ? cu_ctx[g.b] : 0;
  asm volatile("" ::"s"(g.q0), "s"(q_end), "s"(g.k0), "s"(k_end), "s"(g.l0), "s"(l_end), "s"(g.ctx0));  // one round of loads
  g.q_b = q_end - g.q0;
  g.k_b = nug_len != nullptr ? k_end : k_end - g.k0;
  g.m_b = loc_len != nullptr ? l_end : l_end - g.l0;
  return g;
}

// One query block (kBM rows) of one (sequence, head); called by the whole workgroup.
// IDX: Kn / Vn are the context's K / V and nugget j of sequence b is its token cu_ctx[b] + nug_idx[cu_nuggets[b] + j].
template <int NW, bool IDX, int DH>
__device__ __forceinline__ void attend_query_block(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ Kn, const uint16_t* __restrict__ Vn,
    const uint16_t* __restrict__ Kl, const uint16_t* __restrict__ Vl, const int32_t* __restrict__ nug_idx,
    int H, int H_kv, const SeqGeom& geom, int qblk,
    int64_t nug_tok_stride, int64_t nug_head_stride, float scale_log2e, uint16_t* __restrict__ O,
    float* __restrict__ lse) {
  using Cfg = BlockCfg<NW, DH>;
  using HD = HeadDims<DH>;
  constexpr int kDH = DH, kRowBytes = HD::kRowBytes, kTileBytes = HD::kTileBytes;
  constexpr int kP = HD::kPieces;           // 16-byte pieces of a row
  constexpr int kRowShift = HD::kRowShift;  // swizzles use row >> kRowShift
  constexpr int kNCB = HD::kChannelBlocks;  // 32-channel blocks of the output
  constexpr int kSteps = HD::kSteps;        // MFMAs of S^T per tile, and of O^T += V^T P^T
  constexpr int kBM = Cfg::kBM;
  constexpr int kStages = Cfg::kStages;
  extern __shared__ __attribute__((aligned(1024))) char lds[];  // stage s: K at 2s, V at 2s+1 (tiles of 16 KiB)
  const uint32_t lds_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_void*)lds));

  const int h = geom.h, kvh = geom.kvh;
  const int q0 = geom.q0, q_b = geom.q_b, k0 = geom.k0, k_b = geom.k_b, l0 = geom.l0, m_b = geom.m_b;
  const int i0 = qblk * kBM;
  if (i0 >= q_b) return;  // uniform over the workgroup

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int lane = tid % kWave;
  const int j = lane & 31, g = lane >> 5;
  const int w_i0 = i0 + wave * 32;  // first query row of this wavefront
  const int shift = m_b - q_b + 1;  // query row i sees local rows [0, i + shift)
  const int my_i = w_i0 + j;        // this lane's query row inside the sequence
  const bool row_ok = my_i < q_b;
  const int my_vis = row_ok ? max(0, min(m_b, my_i + shift)) : 0;
  // local rows visible to the first / last query row of this wavefront and to the whole workgroup
  const int w_lo = max(0, min(m_b, w_i0 + shift));
  const int w_hi = max(0, min(m_b, min(w_i0 + 31, q_b - 1) + shift));
  const int wg_vis = max(0, min(m_b, min(i0 + kBM, q_b) - 1 + shift));

  const int n_nug_tiles = (k_b + kBN - 1) / kBN;
  const int n_loc_tiles = (wg_vis + kBN - 1) / kBN;
  const int n_tiles = n_nug_tiles + n_loc_tiles;

  const int64_t nug_row0 = IDX ? geom.ctx0 : k0;  // IDX: the index list holds tokens of the sequence that starts here
  const uint16_t* nugK = Kn + nug_row0 * nug_tok_stride + static_cast<int64_t>(kvh) * nug_head_stride;
  const uint16_t* nugV = Vn + nug_row0 * nug_tok_stride + static_cast<int64_t>(kvh) * nug_head_stride;
  const int32_t* idx_l = reinterpret_cast<const int32_t*>(lds + Cfg::kLdsBytes);
  if (IDX) {
    // (a previous query block of this workgroup is past its last tile request: the caller's barrier)
    int32_t* dst = reinterpret_cast<int32_t*>(lds + Cfg::kLdsBytes);
    for (int t = threadIdx.x; t < min(k_b, Cfg::kIdxCap); t += Cfg::kThreads) dst[t] = nug_idx[k0 + t];
    __syncthreads();
  }
  const int64_t loc_stride = static_cast<int64_t>(H_kv) * kDH;
  const uint16_t* locK = Kl + (static_cast<int64_t>(l0) * H_kv + kvh) * kDH;
  const uint16_t* locV = Vl + (static_cast<int64_t>(l0) * H_kv + kvh) * kDH;

  TileLoader<NW, DH> loader;
  loader.init(wave, lane);
  // Every call enqueues the same number of loads per lane (a tile past the end re-reads the last
  // one into a stage nobody reads), so the vmcnt arithmetic of the loops is uniform.
  auto issue_tile = [&](int tile) {
    const int stage = tile % kStages;
    const int tl = min(tile, n_tiles - 1);
    const bool nug = tl < n_nug_tiles;
    const int base = nug ? tl * kBN : (tl - n_nug_tiles) * kBN;
    const int cnt = min(kBN, (nug ? k_b : wg_vis) - base);
    const int64_t stride = nug ? nug_tok_stride : loc_stride;
    if (IDX && nug) {
      loader.issue_idx(nugK, nugV, static_cast<uint32_t>(stride) * 2u, cnt, lds_base + (2 * stage) * kTileBytes,
                       lds_base + (2 * stage + 1) * kTileBytes, idx_l + base);
    } else {
      loader.issue((nug ? nugK : locK) + base * stride, (nug ? nugV : locV) + base * stride,
                   static_cast<uint32_t>(stride) * 2u, cnt, lds_base + (2 * stage) * kTileBytes,
                   lds_base + (2 * stage + 1) * kTileBytes);
    }
  };
  // per-tile bookkeeping shared by the phases
  struct TileInfo {
    bool visible, need_mask;
    int limit;
  };
  auto tile_info = [&](int tile) -> TileInfo {
    const bool is_nug = tile < n_nug_tiles;
    const int base = is_nug ? tile * kBN : (tile - n_nug_tiles) * kBN;
    const int cnt = min(kBN, (is_nug ? k_b : wg_vis) - base);
    TileInfo ti;
    ti.visible = is_nug || base < w_hi;  // some key of this tile is visible to this wavefront
    ti.need_mask = cnt < kBN || (!is_nug && base + kBN > w_lo);
    ti.limit = is_nug ? cnt : min(cnt, my_vis - base);  // keys [0, limit) are visible to this lane's row
    return ti;
  };

  // Prologue.  The first tile is requested before anything else; the workgroup's query rows follow,
  // through LDS like a K tile (whole rows per request; a lane fetching its own row from global
  // memory would touch 32 rows per instruction), into the stages that tiles 1.. (NW = 4) or 2..
  // (NW = 8) use later.  Q^T fragments: lane (j, g) holds Q[my_i][16*ds + 8*g .. +8) for ds = 0..7.
  // Rows past the end of the sequence re-read its last row; nothing of them is stored.
  constexpr int kLoadsPerTile = TileLoader<NW, DH>::kPerWave * 2;
  constexpr int kQSlot0 = NW == 8 ? 4 : 2;  // first 16 KiB slot of the query rows
  bf16x8 qf[kDH / 16];
  if (n_tiles > 0) {
    issue_tile(0);
#pragma unroll
    for (int c = 0; c < kBM / kBN; ++c) {
      const int r0 = i0 + kBN * c;
      const int64_t base_row = q0 + min(r0, q_b - 1);
      loader.issue_rows(Q + (base_row * H + h) * kDH, static_cast<uint32_t>(H) * kRowBytes, max(1, min(kBN, q_b - r0)),
                        lds_base + (kQSlot0 + c) * kTileBytes);
    }
    if (NW == 8) {
      issue_tile(1);
      __builtin_amdgcn_s_waitcnt(0x0f70 | kLoadsPerTile);  // tile 0 and Q landed, tile 1 in flight
    } else {
      __builtin_amdgcn_s_waitcnt(0x0f70);
    }
    __syncthreads();
    const char* qbuf = lds + kQSlot0 * kTileBytes + (wave * 32 + j) * kRowBytes;
#pragma unroll
    for (int ds = 0; ds < kDH / 16; ++ds)
      qf[ds] = *reinterpret_cast<const bf16x8*>(qbuf + (((2 * ds + g) ^ ((j >> kRowShift) & (kP - 1))) << 4));
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the fragments are in registers
    if (NW == 8) {
      __syncthreads();  // everyone has its fragments: the stages are free again
      issue_tile(2);
      issue_tile(3);
    }
  } else {
#pragma unroll
    for (int ds = 0; ds < kDH / 16; ++ds) qf[ds] = __builtin_bit_cast(bf16x8, make_uint4(0, 0, 0, 0));
  }

  floatx16 acc_o[kDH / 32];
#pragma unroll
  for (int cb = 0; cb < kDH / 32; ++cb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc_o[cb][v] = 0.f;
  float m_run = kNegInf, l_run = 0.f;

  // per-lane constants of the LDS read patterns
  const int k_row_off = j * kRowBytes;  // K: row 32kb + j, piece (2ds + g) ^ swizzle(row); swizzle(32kb + j) == swizzle(j)
  const int k_sw = (j >> kRowShift) & (kP - 1);
  // V^T via transposing read: lane supplies row 16t + 8e + 4g + (lane%16)/4, 8 bytes at channel 32cb + 16*half + 4*(lane%4)
  const int v_r = 4 * g + ((lane & 15) >> 2);
  const int v_in = 32 * ((lane >> 4) & 1) + 8 * (lane & 3);

  // Fragments are requested kAhead MFMAs before their use; the scheduling barriers keep the
  // compiler from hoisting every LDS read of a tile to the front (which would not fit in registers).
  constexpr int kAhead = 6;
  // S^T = K Q^T of one tile: K fragment s = 2*ds + kb is row 32kb + j, 16 bytes at the swizzled piece 2ds + g
  auto read_k = [&](int tile, int s) -> bf16x8 {
    const char* kbuf = lds + (2 * (tile % kStages)) * kTileBytes + k_row_off;
    return *reinterpret_cast<const bf16x8*>(kbuf + (s & 1) * 32 * kRowBytes + ((((s >> 1) * 2 + g) ^ k_sw) << 4));
  };
  auto compute_s = [&](int tile, floatx16 (&acc_s)[2]) {
    bf16x8 kf[kAhead];
#pragma unroll
    for (int s = 0; s < kAhead; ++s) kf[s] = read_k(tile, s);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc_s[kb][v] = 0.f;
#pragma unroll
    for (int s = 0; s < kSteps; ++s) {
      const bf16x8 cur = kf[s % kAhead];
      if (s + kAhead < kSteps) kf[s % kAhead] = read_k(tile, s + kAhead);
      acc_s[s & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, qf[s >> 1], acc_s[s & 1], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // O^T += V^T P^T of one tile: V^T fragment s = 4*t + cb; slot 8g+4e+r of k-step t <-> key 16t + 8e + 4g + r.
  // The two-group kernel takes the row sums of P from the matrix pipe as well, which has slack
  // there while the softmax phase has none: P^T is also multiplied with a 33rd block of V^T whose
  // only non-zero row is all ones, so accumulator row 0 of that block (lane j, g = 0, register 0)
  // collects sum_k P[k][query] -- of the bf16-rounded P, exactly what O^T is accumulated from.
  constexpr bool kOnesBlock = true;
  floatx16 acc_l;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc_l[v] = 0.f;
  const bf16x8 ones_frag = __builtin_bit_cast(
      bf16x8, j == 0 ? make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u) : make_uint4(0, 0, 0, 0));
  auto read_vt = [&](int tile, int s) -> bf16x8 {
    const char* vbuf = lds + (2 * (tile % kStages) + 1) * kTileBytes + v_in;
    const int t = s / kNCB, cb = s % kNCB;
    shortx4 a[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const int r = 16 * t + 8 * e + v_r;
      const char* p = vbuf + r * kRowBytes + ((cb ^ ((r >> kRowShift) & (kNCB - 1))) << 6);
      a[e] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((shortx4 __attribute__((address_space(3)))*)(p));
    }
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(a[0], a[1], 0, 1, 2, 3, 4, 5, 6, 7));
  };
  auto compute_pv = [&](int tile, const bf16x8 (&pf)[4]) {
    bf16x8 vf[kAhead];
#pragma unroll
    for (int s = 0; s < kAhead; ++s) vf[s] = read_vt(tile, s);
#pragma unroll
    for (int s = 0; s < kSteps; ++s) {
      const bf16x8 cur = vf[s % kAhead];
      if (s + kAhead < kSteps) vf[s % kAhead] = read_vt(tile, s + kAhead);
      acc_o[s % kNCB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, pf[s / kNCB], acc_o[s % kNCB], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  bool bail = false;
  auto softmax_fast = [&](const TileInfo& ti, floatx16 (&acc_s)[2], bf16x8 (&pf)[4]) {
    if (ti.need_mask) {
      softmax_fixed<true, !kOnesBlock>(acc_s, ti.limit, g, scale_log2e, m_run, l_run, pf);
    } else {
      softmax_fixed<false, !kOnesBlock>(acc_s, kBN, g, scale_log2e, m_run, l_run, pf);
    }
  };
  auto softmax = [&](const TileInfo& ti, floatx16 (&acc_s)[2], bf16x8 (&pf)[4]) {
    if (ti.need_mask) {
      softmax_tile<true, kNCB>(acc_s, ti.limit, g, scale_log2e, m_run, l_run, acc_o, pf);
    } else {
      softmax_tile<false, kNCB>(acc_s, kBN, g, scale_log2e, m_run, l_run, acc_o, pf);
    }
  };

  if constexpr (NW == 4) {
    // ---- plain loop: one barrier per tile, next tile in flight ----
    // (the first barrier also tells that every wavefront has taken its Q fragments out of stage 1)
    for (int tile = 0; tile < n_tiles; ++tile) {
      __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wavefront's part of the tile has landed
      __syncthreads();                      // everyone's part has landed; the other stage is free
      issue_tile(tile + 1);
      const TileInfo ti = tile_info(tile);
      if (!ti.visible) continue;
      floatx16 acc_s[2];
      bf16x8 pf[4];
      compute_s(tile, acc_s);
      softmax(ti, acc_s, pf);
      compute_pv(tile, pf);
    }
  } else {
    // ---- two groups of four wavefronts, half a tile apart ----
    // Phase p ends with a workgroup barrier.  Group 0 does in even phases 2t "PV(t-1) then S(t)"
    // (32 MFMAs) and in odd phases 2t+1 the softmax of tile t; group 1 does the softmax of tile
    // t-1 in phase 2t and the MFMAs in phase 2t+1, so in every phase one group feeds the matrix
    // pipe while the other runs VALU work.  Tile t is read during phases 2t .. 2t+3 and sits in
    // stage t % 4; tile t+4 is requested during phases 2t+4 (K) and 2t+5 (V) and has to be visible
    // at the barrier that ends phase 2t+7.
    const int grp = wave >> 2;
    floatx16 acc_s[2];
    bf16x8 pf[4];
    // One iteration = phases 2t and 2t+1.  The two groups run separate copies of the loop (same
    // number of barriers) so that each copy is straight-line code for the compiler.
    // The MFMA phase is one software pipeline over 32 fragments (16 of V^T, then 16 of K), each
    // requested kAhead MFMAs before its use into a ring of registers: slot i of the phase lives
    // in ring[i % kAhead].  The first kAhead fragments of V^T are requested at the end of the
    // softmax phase before, so no MFMA phase starts by waiting for LDS.  A tile that is invisible
    // to a wavefront (above the causal diagonal) is followed by invisible tiles only.
    bf16x8 ring[kAhead];
    auto pv_steps = [&](int t, auto k_prefetch_tag) {  // PV(t-1); requests the first K fragments of tile t
      constexpr bool K_PREFETCH = decltype(k_prefetch_tag)::value;
#pragma unroll
      for (int s = 0; s < kSteps; ++s) {
        const bf16x8 cur = ring[s % kAhead];
        if (s + kAhead < kSteps) {
          ring[s % kAhead] = read_vt(t - 1, s + kAhead);
        } else if (K_PREFETCH) {
          ring[s % kAhead] = read_k(t, s + kAhead - kSteps);
        }
        acc_o[s % kNCB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, pf[s / kNCB], acc_o[s % kNCB], 0, 0, 0);
        if (kOnesBlock && (s % kNCB) == kNCB - 1)
          acc_l = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones_frag, pf[s / kNCB], acc_l, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    auto s_steps = [&](int t) {  // S(t); its first kAhead fragments are in the ring already
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc_s[kb][v] = 0.f;
#pragma unroll
      for (int s = 0; s < kSteps; ++s) {
        const bf16x8 cur = ring[(kSteps + s) % kAhead];
        if (s + kAhead < kSteps) ring[(kSteps + s) % kAhead] = read_k(t, s + kAhead);
        acc_s[s & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, qf[s >> 1], acc_s[s & 1], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    auto valu_work = [&](int t) {  // softmax of tile t, then the first V^T fragments for PV(t)
      softmax_fast(tile_info(t), acc_s, pf);
#pragma unroll
      for (int s = 0; s < kAhead; ++s) ring[s] = read_vt(t, s);
    };
    // In the loop a wavefront requests tiles where it would otherwise idle at a barrier, after its
    // softmax: a request can take hundreds of cycles to issue when the memory pipeline is backed
    // up.  The wavefronts of group 1 bring K of tile t+2 (during phase 2t), those of group 0 its V
    // (during phase 2t+1), four requests per wavefront as in the prologue's split.
    TileLoader<4, DH> half_loader;
    half_loader.init(wave & 3, lane);
    auto issue_half = [&](int tile, auto v_tag) {
      constexpr bool IS_V = decltype(v_tag)::value;
      const int stage = tile % kStages;
      const int tl = min(tile, n_tiles - 1);
      const bool nug = tl < n_nug_tiles;
      const int base = nug ? tl * kBN : (tl - n_nug_tiles) * kBN;
      const int cnt = min(kBN, (nug ? k_b : wg_vis) - base);
      const int64_t stride = nug ? nug_tok_stride : loc_stride;
      if (IDX && nug) {
        if (IS_V) {
          half_loader.issue_rows_v_idx(nugV, static_cast<uint32_t>(stride) * 2u, cnt,
                                       lds_base + (2 * stage + 1) * kTileBytes, idx_l + base);
        } else {
          half_loader.issue_rows_idx(nugK, static_cast<uint32_t>(stride) * 2u, cnt, lds_base + (2 * stage) * kTileBytes,
                                     idx_l + base);
        }
      } else if (IS_V) {
        half_loader.issue_rows_v((nug ? nugV : locV) + base * stride, static_cast<uint32_t>(stride) * 2u, cnt,
                                 lds_base + (2 * stage + 1) * kTileBytes);
      } else {
        half_loader.issue_rows((nug ? nugK : locK) + base * stride, static_cast<uint32_t>(stride) * 2u, cnt,
                               lds_base + (2 * stage) * kTileBytes);
      }
    };
    auto end_odd_phase = [&](int t) {  // ends phase 2t+1: tile t+1 must have landed
      // younger requests of this wavefront in flight: two tiles' worth while the prologue's are pending, else one
      if (t == 0) {
        __builtin_amdgcn_s_waitcnt(0x0f70 | (2 * kLoadsPerTile));
      } else {
        __builtin_amdgcn_s_waitcnt(0x0f70 | (1 * kLoadsPerTile));
      }
      __syncthreads();
    };
    if (n_tiles > 0 && scale_log2e > 0.f) {
      // Tiles [0, n_vis) are visible to this wavefront.  Iteration t is one of four kinds, so that
      // each loop body is straight-line code: 0 = S(0) only, 1 = PV(t-1) and S(t) (the steady
      // state), 2 = PV(n_vis-1) only, 3 = nothing but the barriers the other wavefronts count on.
      const int n_vis = n_nug_tiles + min(n_loc_tiles, (w_hi + kBN - 1) / kBN);
      auto iteration = [&](int t, auto grp_tag, auto kind_tag) {
        constexpr int GRP = decltype(grp_tag)::value, KIND = decltype(kind_tag)::value;
        if (GRP == 1) {
          if (t >= 2) issue_half(t + 2, std::false_type{});
          if (KIND == 1 || KIND == 2) valu_work(t - 1);
          __syncthreads();
        }
        __builtin_amdgcn_s_setprio(1);
        if (KIND == 0) {
#pragma unroll
          for (int s = 0; s < kAhead; ++s) ring[(kSteps + s) % kAhead] = read_k(t, s);
          s_steps(t);
        } else if (KIND == 1) {
          pv_steps(t, std::true_type{});
          s_steps(t);
        } else if (KIND == 2) {
          pv_steps(t, std::false_type{});
        }
        __builtin_amdgcn_s_setprio(0);
        if (GRP == 0) {
          __syncthreads();
          if (t >= 2) issue_half(t + 2, std::true_type{});
          if (KIND == 0 || KIND == 1) valu_work(t);
        }
        end_odd_phase(t);
      };
      auto run = [&](auto grp_tag) {
        using K0 = std::integral_constant<int, 0>;
        using K1 = std::integral_constant<int, 1>;
        using K2 = std::integral_constant<int, 2>;
        using K3 = std::integral_constant<int, 3>;
        int t = 0;
        if (n_vis > 0) {
          iteration(0, grp_tag, K0{});
          for (t = 1; t < n_vis; ++t) iteration(t, grp_tag, K1{});
          iteration(t, grp_tag, K2{});
          ++t;
        }
        for (; t <= n_tiles; ++t) iteration(t, grp_tag, K3{});
      };
      if (grp == 0) {
        run(std::integral_constant<int, 0>{});
      } else {
        run(std::integral_constant<int, 1>{});
      }
      if (kOnesBlock) l_run = (g == 0) ? acc_l[0] : 0.f;
      const float l_row = l_run + __shfl_xor(l_run, 32, kWave);
      bail = !(l_row - l_row == 0.f);  // +inf or NaN: some logit overflowed the row's fixed offset
    } else {
      bail = n_tiles > 0;
    }
    // Rare: some logit overflowed its row's fixed offset (or the scale is not positive).  Redo the
    // workgroup's rows with the exact running-maximum softmax, one tile at a time.
    __builtin_amdgcn_s_waitcnt(0x0f70);
    if (__syncthreads_or(bail)) {
#pragma unroll
      for (int cb = 0; cb < kDH / 32; ++cb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc_o[cb][v] = 0.f;
      m_run = kNegInf;
      l_run = 0.f;
      for (int tile = 0; tile < n_tiles; ++tile) {
        issue_tile(tile);
        __builtin_amdgcn_s_waitcnt(0x0f70);
        __syncthreads();
        const TileInfo ti = tile_info(tile);
        if (ti.visible) {
          compute_s(tile, acc_s);
          softmax(ti, acc_s, pf);
          compute_pv(tile, pf);
        }
        __syncthreads();
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0f70);  // drain the look-ahead loads before the wavefront ends

  // ---- epilogue: lane (j, g) holds channels 32cb + 8(v/4) + 4g + v%4 of query row my_i ----
  // The 32 x 128 block of a wavefront goes through LDS (free by now) so that O is written with
  // full 256-byte rows, 16 bytes per lane; 16-byte pieces are XOR-swizzled with the row to keep
  // both the 8-byte writes and the 16-byte reads free of bank conflicts.
  if (NW == 4) __syncthreads();  // every wavefront is done with the K/V stages
  const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
  {
    const float inv = (l_tot > 0.f) ? 1.f / l_tot : 0.f;
    char* obuf = lds + wave * (32 * kRowBytes);
#pragma unroll
    for (int cb = 0; cb < kDH / 32; ++cb)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        const int piece = 4 * cb + vq;  // 16-byte piece of the row: channels 8*piece .. 8*piece+7; g picks the half
        uint2 out;
        out.x = pack2_bf16(acc_o[cb][4 * vq + 0] * inv, acc_o[cb][4 * vq + 1] * inv);
        out.y = pack2_bf16(acc_o[cb][4 * vq + 2] * inv, acc_o[cb][4 * vq + 3] * inv);
        *reinterpret_cast<uint2*>(obuf + j * kRowBytes + ((piece ^ ((j >> kRowShift) & (kP - 1))) << 4) + 8 * g) = out;
      }
    __builtin_amdgcn_wave_barrier();
    const int n_rows = min(32, q_b - w_i0);  // valid rows of this wavefront (may be <= 0)
    uint16_t* obase = O + (static_cast<int64_t>(q0 + w_i0) * H + h) * kDH;
#pragma unroll
    for (int it = 0; it < kP / 2; ++it) {  // 64 / kP rows per iteration, 16 bytes per lane
      const int row = (64 / kP) * it + (lane >> HD::kPiecesLog2), piece = lane & (kP - 1);
      const uint4 val = *reinterpret_cast<const uint4*>(obuf + row * kRowBytes + ((piece ^ ((row >> kRowShift) & (kP - 1))) << 4));
      if (row < n_rows) *reinterpret_cast<uint4*>(obase + static_cast<int64_t>(row) * H * kDH + piece * 8) = val;
    }
  }
  if (row_ok && lse != nullptr && g == 0) {
    lse[static_cast<int64_t>(q0 + my_i) * H + h] =
        (l_tot > 0.f) ? (m_run + __log2f(l_tot)) * 0.6931471805599453f : kNegInf;
  }
}

// Workgroups are handed to the 8 XCDs round-robin, each XCD has an L2 of its own: the query blocks
// of one (sequence, head) go to one XCD back to back (heaviest first), so that they start together
// and share the K/V tiles in that L2.  With pair != 0 a workgroup takes two query blocks, one
// after the other: a block i from the end and a block i from the start, so that under the causal
// mask all workgroups carry the same load (new workgroups are handed out in order, and a compute
// unit that finishes early is not refilled before the ones ahead of it in that order).
template <int NW, bool IDX, int DH>
__global__ __launch_bounds__((BlockCfg<NW, DH>::kThreads), (BlockCfg<NW, DH>::kMinBlocks)) void block_attention_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ Kn, const uint16_t* __restrict__ Vn,
    const uint16_t* __restrict__ Kl, const uint16_t* __restrict__ Vl, const int32_t* __restrict__ cu_q,
    const int32_t* __restrict__ cu_nuggets, const int32_t* __restrict__ nug_len,
    const int32_t* __restrict__ cu_local, const int32_t* __restrict__ loc_len, const int32_t* __restrict__ nug_idx,
    const int32_t* __restrict__ cu_ctx,
    int B, int H, int H_kv, int n_qblocks, int pair, int heavy_last, FastDiv div_groups, FastDiv div_H, FastDiv div_G,
    int64_t nug_tok_stride, int64_t nug_head_stride, float scale_log2e, uint16_t* __restrict__ O,
    float* __restrict__ lse) {
  // all arguments in one round of scalar loads (the compiler would fetch them a few at a time, before each first use)
  asm volatile("" ::"s"(Q), "s"(Kn), "s"(Vn), "s"(Kl), "s"(Vl), "s"(cu_q), "s"(cu_nuggets), "s"(nug_len), "s"(cu_local),
               "s"(loc_len), "s"(nug_idx), "s"(cu_ctx), "s"(B), "s"(H), "s"(H_kv), "s"(n_qblocks), "s"(pair),
               "s"(heavy_last), "s"(div_groups.mul), "s"(div_groups.shift), "s"(div_H.mul), "s"(div_H.shift),
               "s"(div_G.mul), "s"(div_G.shift), "s"(nug_tok_stride), "s"(nug_head_stride), "s"(scale_log2e), "s"(O),
               "s"(lse));
  const int n_groups = pair ? (n_qblocks + 1) >> 1 : n_qblocks;  // (div_groups divides by this)
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int j = static_cast<int>(fast_div(static_cast<uint32_t>(slot), div_groups));
  const int bh = j * 8 + xcd;
  const int heavy = n_qblocks - 1 - (slot - j * n_groups), light = n_qblocks - 1 - heavy;
  if (bh >= B * H) return;
  // Two neighbouring workgroups of an XCD (j even and odd) share two (sequence, head) pairs
  // crosswise: one takes the heavy block of the first pair and then the light block of the second,
  // the other the light block of the first and then the heavy block of the second.  Both carry the
  // same load, the two blocks that read the same K/V run at the same time and share it in L2, and
  // the bursts of first loads come from half of the compute units at a time.
  const int bh_other = (j ^ 1) * 8 + xcd;
  const bool cross = pair && light != heavy && bh_other < B * H;
  int bh1 = bh, q1 = heavy, bh2 = bh, q2 = (pair && light != heavy) ? light : -1;
  if (cross) {
    if (j & 1) {
      bh1 = bh_other;
      q1 = light;
      q2 = heavy;
    } else {
      bh2 = bh_other;
    }
  }
  // heavy_last: the batch's entries grow in cost with their index (segments of a text see more and more nuggets);
  // workgroups are handed out in index order, so the entries are walked from the back to keep the tail light
  if (heavy_last) {
    bh1 = B * H - 1 - bh1;
    bh2 = B * H - 1 - bh2;
  }
  // both blocks' sequence data are requested here, before the first block's work
  const SeqGeom g1 = load_seq_geom<IDX>(bh1, div_H, H, div_G, cu_q, cu_nuggets, nug_len, cu_local, loc_len, cu_ctx);
  const SeqGeom g2 = load_seq_geom<IDX>(q2 >= 0 ? bh2 : bh1, div_H, H, div_G, cu_q, cu_nuggets, nug_len, cu_local, loc_len, cu_ctx);
  attend_query_block<NW, IDX, DH>(Q, Kn, Vn, Kl, Vl, nug_idx, H, H_kv, g1, q1, nug_tok_stride, nug_head_stride, scale_log2e, O,
                                  lse);
  if (q2 >= 0) {
    __syncthreads();  // the first block's use of LDS is over
    attend_query_block<NW, IDX, DH>(Q, Kn, Vn, Kl, Vl, nug_idx, H, H_kv, g2, q2, nug_tok_stride, nug_head_stride, scale_log2e, O,
                                    lse);
  }
}

template <int NW, bool IDX, int DH>
int launch_nw(const AttnParams& p) {
  using Cfg = BlockCfg<NW, DH>;
  if (IDX && p.max_k > Cfg::kIdxCap) return DODO_ERR_UNSUPPORTED;
  constexpr int kLds = Cfg::kLdsBytes + (IDX ? Cfg::kIdxBytes : 0);
  const int n_qblocks = (p.max_q + Cfg::kBM - 1) / Cfg::kBM;
  // pairs of query blocks per workgroup, if that still leaves a workgroup for every compute unit
  const int64_t bh8 = (static_cast<int64_t>(p.B) * p.H + 7) / 8 * 8;
  const int pair = (n_qblocks >= 2 && bh8 * ((n_qblocks + 1) / 2) >= compute_units()) ? 1 : 0;
  const int64_t grid = bh8 * (pair ? (n_qblocks + 1) / 2 : n_qblocks);
  if (grid > 0x7fffffffLL) return DODO_ERR_UNSUPPORTED;
  auto kern = block_attention_kernel<NW, IDX, DH>;
  if (kLds > 64 * 1024) {
    const int rc = allow_dynamic_lds(reinterpret_cast<const void*>(kern), kLds);
    if (rc != DODO_OK) return rc;
  }
  hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(grid)), dim3(Cfg::kThreads), kLds, p.stream,
                     static_cast<const uint16_t*>(p.Q), static_cast<const uint16_t*>(p.Kn),
                     static_cast<const uint16_t*>(p.Vn), static_cast<const uint16_t*>(p.Kl),
                     static_cast<const uint16_t*>(p.Vl), p.cu_q, p.cu_nuggets, p.nug_len, p.cu_local, p.loc_len, p.nug_idx, p.cu_ctx, p.B, p.H, p.H_kv,
                     n_qblocks, pair, p.heavy_last, make_fast_div(static_cast<uint32_t>(pair ? (n_qblocks + 1) / 2 : n_qblocks)),
                     make_fast_div(static_cast<uint32_t>(p.H)), make_fast_div(static_cast<uint32_t>(p.H / p.H_kv)),
                     p.nug_tok_stride, p.nug_head_stride, p.scale_log2e, static_cast<uint16_t*>(p.O), p.lse);
  return launch_status();
}

template <int DH>
int launch_dh(const AttnParams& p) {
  // the K/V row offsets inside one tile are kept in 32 bits
  if (p.nug_tok_stride * 2 * kBN > 0x7fffffffLL || static_cast<int64_t>(p.H_kv) * DH * 2 * kBN > 0x7fffffffLL ||
      static_cast<int64_t>(p.H) * DH * 2 * kBN > 0x7fffffffLL)
    return DODO_ERR_UNSUPPORTED;
  if (p.nug_idx != nullptr) {
    // a token's byte offset from its sequence's first row is kept in 32 bits as well
    if (static_cast<int64_t>(p.max_n) * p.nug_tok_stride * 2 > 0x7fffffffLL) return DODO_ERR_UNSUPPORTED;
    return p.max_q > 128 ? launch_nw<8, true, DH>(p) : launch_nw<4, true, DH>(p);
  }
  if (p.max_q > 128) return launch_nw<8, false, DH>(p);
  return launch_nw<4, false, DH>(p);
}

}  // namespace

int launch_block_attention(const AttnParams& p) {
  if (p.dtype != DODO_DTYPE_BF16) return DODO_ERR_UNSUPPORTED;
  if (p.d_h == 128) return launch_dh<128>(p);
  if (p.d_h == 64) return launch_dh<64>(p);
  return DODO_ERR_UNSUPPORTED;
}

}  // namespace dodo
