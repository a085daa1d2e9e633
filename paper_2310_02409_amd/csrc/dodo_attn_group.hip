// Nugget attention for a few query vectors that read the same K/V rows, on the matrix cores (Eq. 13 / Eq. 9 of
// the Dodo paper with q_b small): the G query heads of one KV head (grouped-query attention) times the rows of a
// small query block -- at most 32 vectors, the width of one MFMA tile.  bf16, d_h = 128 or 64 (a template
// parameter: tile sizes, LDS layout and fragment counts follow from it).
//
// The work is bandwidth-bound (every K and V row is read once, and serves all the vectors), so the layout is built
// around keeping loads in flight: a workgroup owns one (sequence, KV head, split); each of its wavefronts streams
// its own share of the keys, 32 at a time, through a private two-stage LDS buffer filled by direct global->LDS
// loads -- no workgroup barrier in the loop, the wavefront's own vmcnt is all the synchronisation there is.  Per 32
// keys and wavefront:
//   S^T = K Q^T     8 x v_mfma_f32_32x32x16_bf16, A = K rows (LDS), B = Q^T (registers): lane <-> query vector
//   online softmax in base 2 on the accumulators (row statistics are lane-local, one exchange with lane^32)
//   O^T += V^T P^T  8 MFMAs, A = V^T through the transposing LDS read, B = P^T straight from the accumulators
// (the LDS swizzles and the k-slot <-> key permutation are those of the query-block kernel).  The wavefronts'
// partial (m, l, O) meet in LDS and are merged in wavefront order; with several splits the workgroup writes a
// partial record and the last split merges the records in split order, as in the split-K kernel (same workspace
// format), so results are deterministic.
#include "dodo_attn.h"

namespace dodo {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short shortx4;
typedef __attribute__((ext_vector_type(8))) float floatx8;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef __attribute__((address_space(3))) void lds_void;

constexpr int kKeys = 32;        // keys per tile
constexpr int kMaxVectors = 32;  // query vectors per workgroup: the N side of one MFMA tile
// What follows from the head size DH (128 or 64)
template <int DH>
struct GroupDims {
  static constexpr int kRowBytes = DH * 2;
  static constexpr int kP = kRowBytes / 16;           // 16-byte pieces of a row
  static constexpr int kPLog2 = DH == 128 ? 4 : 3;
  // rows of 128 bytes cover half of the LDS banks: two consecutive rows sit side by side and the swizzles take the
  // row's index from bit 1 on; rows of 256 bytes use the index as it is
  static constexpr int kRowShift = DH == 128 ? 0 : 1;
  static constexpr int kNCB = DH / 32;                // 32-channel blocks of O^T = 64-byte granules of a V row
  static constexpr int kKSteps = DH / 16;             // MFMAs of S^T per tile
  static constexpr int kRowsPerInstr = 64 / kP;       // a load instruction brings 1 KiB: 4 or 8 rows
  static constexpr int kInstrPerTensor = kKeys / kRowsPerInstr;
  static constexpr int kTensorBytes = kKeys * kRowBytes;  // K or V part of a stage: 8 or 4 KiB
  static constexpr int kStageBytes = 2 * kTensorBytes;
  static constexpr int kWaveLds = 2 * kStageBytes;        // two stages per wavefront: 32 or 16 KiB
  static constexpr int kLoadsPerTile = 2 * kInstrPerTensor;
  static constexpr int kPartStride = DH + 4;              // floats per vector of a partial in LDS (spreads the banks)
  static constexpr int kPartBytes = (kMaxVectors * kPartStride + 2 * kMaxVectors) * 4;  // a partial: O, then m and l
  // splits of the keys of a (sequence, KV head) pair over workgroups: the last split's staging (one float per
  // vector and other split in each of the first two wavefronts' regions, behind the partials) bounds their number
  static constexpr int kMaxSplits = DH == 128 ? 64 : 32;
  static_assert(kPartBytes + (kMaxVectors * (kMaxSplits - 1) + 3 * kMaxVectors) * 4 <= kWaveLds,
                "the merge's staging fits behind the partials");
};
constexpr float kNegInf = -__builtin_inff();

__device__ __forceinline__ float exp2_hw(float x) { return __builtin_amdgcn_exp2f(x); }  // exp2(-inf) = 0
constexpr int vmcnt_imm(int n) { return 0x0f70 | (n & 15) | ((n >> 4) << 14); }         // s_waitcnt vmcnt(n) only

// Online-softmax update for one 32-key tile.  acc holds the raw S^T accumulators: register v <-> key
// 8(v/4) + 4g + v%4 (g = lane / 32).  MASK: keys at or beyond `limit` are masked.  Returns P^T as the two MFMA B
// operands (k-step t covers keys 16t .. 16t+15).
// The exponent offset m_run of a vector is moved (and its sum and output accumulators rescaled) only when the tile's
// maximum exceeds it by more than kSlack: the result does not depend on the offset, the weights stay below
// 2^kSlack, and after the first tiles of a vector the output accumulators are hardly ever touched again (the rescale is
// a wavefront-uniform branch: taken if any vector of the wavefront moves).
constexpr float kSlack = 8.f;
template <bool MASK, int NCB>
__device__ __forceinline__ void softmax_tile32(floatx16& acc, int limit, int g, float scale_log2e, float& m_run,
                                               float& l_run, floatx16 (&acc_o)[NCB], bf16x8 (&pf)[2]) {
  float tmax = kNegInf;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    float s = acc[v] * scale_log2e;
    if (MASK) {
      const int key = 8 * (v >> 2) + 4 * g + (v & 3);
      s = (key < limit) ? s : kNegInf;
    }
    acc[v] = s;
    tmax = fmaxf(tmax, s);
  }
  tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));  // both lanes of a vector decide alike
  const bool move = tmax > m_run + kSlack;           // (m_run = -inf: any finite maximum moves it)
  if (__any(move)) {
    const float m_new = move ? tmax : m_run;
    const float alpha = exp2_hw(m_run - ((m_new == kNegInf) ? 0.f : m_new));  // 1 where nothing moves, 0 from -inf
    l_run *= alpha;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc_o[cb][v] *= alpha;
    m_run = m_new;
  }
  const float m_use = (m_run == kNegInf) ? 0.f : m_run;
  float psum = 0.f;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    floatx8 p;
#pragma unroll
    for (int v = 0; v < 8; ++v) {
      p[v] = exp2_hw(acc[8 * half + v] - m_use);
      psum += p[v];
    }
    pf[half] = __builtin_convertvector(p, bf16x8);  // hardware round-to-nearest-even pack
  }
  l_run += psum;
}

// NWV wavefronts per workgroup.  Grid: (KV head, sequence, split).
template <int DH, int NWV>
__global__ __launch_bounds__(NWV * kWave) void group_attention_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ Kn, const uint16_t* __restrict__ Vn,
    const uint16_t* __restrict__ Kl, const uint16_t* __restrict__ Vl, const int32_t* __restrict__ cu_q,
    const int32_t* __restrict__ cu_nuggets, const int32_t* __restrict__ nug_len, const int32_t* __restrict__ cu_local,
    const int32_t* __restrict__ loc_len, int H, int H_kv, int G, FastDiv div_G, int max_q, int row0, int rows_per,
    int nsplit,
    int64_t nug_tok_stride, int64_t nug_head_stride, float scale_log2e, uint16_t* __restrict__ O,
    float* __restrict__ lse, float* __restrict__ ws, uint32_t* __restrict__ flags) {
  using GD = GroupDims<DH>;
  constexpr int kDH = DH, kRowBytes = GD::kRowBytes, kP = GD::kP, kRowShift = GD::kRowShift, kNCB = GD::kNCB;
  constexpr int kTensorBytes = GD::kTensorBytes, kStageBytes = GD::kStageBytes, kWaveLds = GD::kWaveLds;
  constexpr int kPartStride = GD::kPartStride, kPartBytes = GD::kPartBytes, kMaxSplits = GD::kMaxSplits;
  constexpr int kThreads = NWV * kWave;
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int kvh = blockIdx.x, b = blockIdx.y, split = blockIdx.z;

  const int32_t* k_end_p = nug_len != nullptr ? nug_len + b : cu_nuggets + b + 1;
  const int32_t* l_end_p = loc_len != nullptr ? loc_len + b : cu_local + b + 1;
  const int q0 = cu_q[b], q_end = cu_q[b + 1];
  const int k0 = cu_nuggets[b], k_end = *k_end_p;
  const int l0 = cu_local[b], l_end = *l_end_p;
  asm volatile("" ::"s"(q0), "s"(q_end), "s"(k0), "s"(k_end), "s"(l0), "s"(l_end));  // one round of loads
  const int q_b = min(q_end - q0, max_q);  // query rows of the sequence; this launch takes rows row0 .. row0 + rows_per
  const int k_b = nug_len != nullptr ? k_end : k_end - k0;
  const int m_b = loc_len != nullptr ? l_end : l_end - l0;
  if (q_b <= row0) return;  // uniform over the workgroup and over the splits: nothing to write, nothing to wait for
  const int q_cnt = min(rows_per, q_b - row0);

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int lane = tid % kWave;
  const int j = lane & 31, g = lane >> 5;
  const int nv = q_cnt * G;  // query vectors of this workgroup: vector v = (row row0 + v / G, head kvh * G + v % G)
  const bool valid = j < nv;
  const int jv = valid ? j : 0;  // spare lanes repeat vector 0; nothing of them is stored
  const int my_il = static_cast<int>(fast_div(static_cast<uint32_t>(jv), div_G));
  const int my_i = row0 + my_il;
  const int my_h = kvh * G + (jv - my_il * G);
  // causal rule, bottom-right aligned: query row i sees local rows j <= m_b - q_b + i (the sequence's last row sees
  // all); the launch's last row bounds the local tiles
  const int wg_vis = max(0, min(m_b, m_b - q_b + row0 + q_cnt));
  const int my_vis = valid ? max(0, min(m_b, m_b - q_b + my_i + 1)) : 0;

  const int n_nug_tiles = (k_b + kKeys - 1) / kKeys;
  const int n_loc_tiles = (wg_vis + kKeys - 1) / kKeys;
  const int n_tiles = n_nug_tiles + n_loc_tiles;
  const int per_split = (n_tiles + nsplit - 1) / nsplit;
  const int t0 = min(n_tiles, split * per_split), t1 = min(n_tiles, t0 + per_split);
  // this wavefront's tiles: t0 + wave, t0 + wave + NWV, ...
  const int first = t0 + wave;
  const int n_mine = first < t1 ? (t1 - first + NWV - 1) / NWV : 0;
  const int last = first + (n_mine - 1) * NWV;

  // Q^T fragments: lane (j, g) holds channels 16 ds + 8 g .. + 8 of its vector for ds = 0..7
  bf16x8 qf[kDH / 16];
  {
    const uint16_t* qrow = Q + (static_cast<int64_t>(q0 + my_i) * H + my_h) * kDH + 8 * g;
#pragma unroll
    for (int ds = 0; ds < kDH / 16; ++ds) qf[ds] = *reinterpret_cast<const bf16x8*>(qrow + 16 * ds);
  }

  const uint16_t* nugK = Kn + static_cast<int64_t>(k0) * nug_tok_stride + static_cast<int64_t>(kvh) * nug_head_stride;
  const uint16_t* nugV = Vn + static_cast<int64_t>(k0) * nug_tok_stride + static_cast<int64_t>(kvh) * nug_head_stride;
  const int64_t loc_stride = static_cast<int64_t>(H_kv) * kDH;
  const uint16_t* locK = Kl + (static_cast<int64_t>(l0) * H_kv + kvh) * kDH;
  const uint16_t* locV = Vl + (static_cast<int64_t>(l0) * H_kv + kvh) * kDH;

  // Tile loads: an instruction brings 1 KiB (4 or 8 rows) of K or of V; the lane at LDS position (row, pos) fetches
  // the 16-byte piece that the swizzle stores there (K: pos ^ r; V: 64-byte granule (pos / 4) ^ r; r = row >>
  // kRowShift, taken modulo the number of pieces or granules).  Rows past the end of the region re-read its last row
  // (finite data, masked later).
  char* const lds_w = lds + wave * kWaveLds;
  const uint32_t lds_w_addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_void*)lds_w));
  const int ld_row0 = lane >> GD::kPLog2;
  const uint32_t ld_pos = lane & (kP - 1);
  auto k_piece_of = [&](int row) -> uint32_t { return (ld_pos ^ ((row >> kRowShift) & (kP - 1))) * 16u; };
  auto v_piece_of = [&](int row) -> uint32_t {
    return ((((ld_pos >> 2) ^ ((row >> kRowShift) & (kNCB - 1))) << 2) | (ld_pos & 3)) * 16u;
  };
  // Whole tiles (the usual case): the row term of instruction u goes into the scalar base, so the lanes' offsets
  // are loop constants (the V piece is the same for all of a lane's rows).
  const uint32_t nug_sb = static_cast<uint32_t>(nug_tok_stride) * 2u, loc_sb = static_cast<uint32_t>(loc_stride) * 2u;
  const uint32_t v_piece0 = v_piece_of(ld_row0);
  uint32_t k_piece0[GD::kInstrPerTensor];
#pragma unroll
  for (int u = 0; u < GD::kInstrPerTensor; ++u) k_piece0[u] = k_piece_of(ld_row0 + GD::kRowsPerInstr * u);
  auto issue_tile = [&](int tile, int stage) {
    const bool nug = tile < n_nug_tiles;
    const int base = nug ? tile * kKeys : (tile - n_nug_tiles) * kKeys;
    const int cnt = min(kKeys, (nug ? k_b : m_b) - base);
    const int64_t stride = nug ? nug_tok_stride : loc_stride;
    const uint16_t* kbase = (nug ? nugK : locK) + base * stride;
    const uint16_t* vbase = (nug ? nugV : locV) + base * stride;
    const uint32_t stride_bytes = nug ? nug_sb : loc_sb;
    const uint32_t dst = lds_w_addr + stage * kStageBytes;
    if (cnt == kKeys) {
      const uint32_t row_term = static_cast<uint32_t>(ld_row0) * stride_bytes;
#pragma unroll
      for (int u = 0; u < GD::kInstrPerTensor; ++u) {
        dma16_uniform(kbase + GD::kRowsPerInstr * u * stride, row_term + k_piece0[u],
                      __builtin_amdgcn_readfirstlane(dst + u * 1024));
        dma16_uniform(vbase + GD::kRowsPerInstr * u * stride, row_term + v_piece0,
                      __builtin_amdgcn_readfirstlane(dst + kTensorBytes + u * 1024));
      }
      return;
    }
#pragma unroll
    for (int u = 0; u < GD::kInstrPerTensor; ++u) {
      const int row = ld_row0 + GD::kRowsPerInstr * u;
      const uint32_t roff = static_cast<uint32_t>(min(row, cnt - 1)) * stride_bytes;
      dma16_uniform(kbase, roff + k_piece_of(row), __builtin_amdgcn_readfirstlane(dst + u * 1024));
      dma16_uniform(vbase, roff + v_piece_of(row), __builtin_amdgcn_readfirstlane(dst + kTensorBytes + u * 1024));
    }
  };

  floatx16 acc_o[kNCB];
#pragma unroll
  for (int cb = 0; cb < kNCB; ++cb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc_o[cb][v] = 0.f;
  float m_run = kNegInf, l_run = 0.f;

  // V^T through the transposing read: the lane supplies row 16t + 8e + 4g + (lane % 16) / 4, 8 bytes at channel
  // 32cb + 16 * ((lane / 16) % 2) + 4 * (lane % 4)
  const int v_r = 4 * g + ((lane & 15) >> 2);
  const int v_in = 32 * ((lane >> 4) & 1) + 8 * (lane & 3);

  if (n_mine > 0) {
    // Two tiles in flight per wavefront; every iteration requests one more (past the end: the last one again,
    // into the stage nobody reads any more), so the count of outstanding loads is the same at every wait.
    issue_tile(first, 0);
    issue_tile(min(first + NWV, last), 1);
    // the query fragments are waited for here, once: a wait for them inside the loop would also wait for the tile
    // in flight (loads complete in order)
#pragma unroll
    for (int ds = 0; ds < kDH / 16; ++ds) asm volatile("" ::"v"(qf[ds]));
    for (int n = 0; n < n_mine; ++n) {
      const int tile = first + n * NWV, stage = n & 1;
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(GD::kLoadsPerTile));  // this tile has landed, the next one is in flight
      const char* kbuf = lds_w + stage * kStageBytes;
      const char* vbuf = kbuf + kTensorBytes;
      // all fragment reads of the tile are requested up front
      bf16x8 kf[kDH / 16], vt[2][kNCB];
#pragma unroll
      for (int ds = 0; ds < kDH / 16; ++ds)
        kf[ds] = *reinterpret_cast<const bf16x8*>(kbuf + j * kRowBytes + (((2 * ds + g) ^ ((j >> kRowShift) & (kP - 1))) << 4));
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int cb = 0; cb < kNCB; ++cb) {
          shortx4 a[2];
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            const int r = 16 * t + 8 * e + v_r;
            const char* p = vbuf + r * kRowBytes + ((cb ^ ((r >> kRowShift) & (kNCB - 1))) << 6) + v_in;
            a[e] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((shortx4 __attribute__((address_space(3)))*)(p));
          }
          vt[t][cb] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(a[0], a[1], 0, 1, 2, 3, 4, 5, 6, 7));
        }
      // with every fragment of the tile in registers its stage is free: the tile after next is requested before the
      // arithmetic, so two tiles are in flight while the wavefront computes
      __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
      __builtin_amdgcn_sched_barrier(0);
      issue_tile(min(tile + 2 * NWV, last), stage);
      __builtin_amdgcn_sched_barrier(0);
      floatx16 acc_s;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc_s[v] = 0.f;
#pragma unroll
      for (int ds = 0; ds < kDH / 16; ++ds) acc_s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ds], qf[ds], acc_s, 0, 0, 0);
      const bool nug = tile < n_nug_tiles;
      const int base = nug ? tile * kKeys : (tile - n_nug_tiles) * kKeys;
      const int limit = nug ? k_b - base : my_vis - base;  // keys [0, limit) of the tile are visible to this lane's vector
      bf16x8 pf[2];
      if (__all(limit >= kKeys)) {
        softmax_tile32<false, kNCB>(acc_s, limit, g, scale_log2e, m_run, l_run, acc_o, pf);
      } else {
        softmax_tile32<true, kNCB>(acc_s, limit, g, scale_log2e, m_run, l_run, acc_o, pf);
      }
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int cb = 0; cb < kNCB; ++cb)
          acc_o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt[t][cb], pf[t], acc_o[cb], 0, 0, 0);
    }
  }
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // drain the look-ahead loads: the stages are reused below

  // ---- the wavefronts' partials meet in LDS: [vector][channel] floats, then m and l per vector ----
  // lane (j, g) holds channels 32cb + 8(v/4) + 4g + v%4 of vector j
  {
    float* part = reinterpret_cast<float*>(lds_w);
    const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
#pragma unroll
    for (int cb = 0; cb < kNCB; ++cb)
#pragma unroll
      for (int qd = 0; qd < 4; ++qd)
        *reinterpret_cast<float4*>(part + j * kPartStride + 32 * cb + 8 * qd + 4 * g) =
            make_float4(acc_o[cb][4 * qd], acc_o[cb][4 * qd + 1], acc_o[cb][4 * qd + 2], acc_o[cb][4 * qd + 3]);
    if (g == 0) {
      part[kMaxVectors * kPartStride + j] = m_run;
      part[kMaxVectors * kPartStride + kMaxVectors + j] = l_tot;
    }
  }
  __syncthreads();

  // One output element (vector v, channel c) per thread and step, the wavefronts merged in wavefront order.
  auto merged = [&](int v, int c, float& M, float& S, float& o) {
    M = kNegInf;
#pragma unroll
    for (int w = 0; w < NWV; ++w)
      M = fmaxf(M, reinterpret_cast<const float*>(lds + w * kWaveLds)[kMaxVectors * kPartStride + v]);
    S = 0.f;
    o = 0.f;
    if (M != kNegInf) {
#pragma unroll
      for (int w = 0; w < NWV; ++w) {
        const float* part = reinterpret_cast<const float*>(lds + w * kWaveLds);
        const float wgt = exp2_hw(part[kMaxVectors * kPartStride + v] - M);
        S = fmaf(part[kMaxVectors * kPartStride + kMaxVectors + v], wgt, S);
        o = fmaf(part[v * kPartStride + c], wgt, o);
      }
    }
  };
  auto out_row_of = [&](int v, int& i_out, int& h_out) -> int64_t {
    const int il = static_cast<int>(fast_div(static_cast<uint32_t>(v), div_G));
    i_out = row0 + il;
    h_out = kvh * G + (v - il * G);
    return static_cast<int64_t>(q0 + i_out) * H + h_out;
  };
  const int n_out = nv * kDH;

  if (nsplit == 1) {
    for (int e = tid; e < n_out; e += kThreads) {
      const int v = e / kDH, c = e % kDH;
      float M, S, o;
      merged(v, c, M, S, o);
      int i_out, h_out;
      const int64_t out_row = out_row_of(v, i_out, h_out);
      O[out_row * kDH + c] = static_cast<uint16_t>(f32_to_bf16_bits((S > 0.f) ? o / S : 0.f));
      if (lse != nullptr && c == 0) lse[out_row] = (S > 0.f) ? (M + __log2f(S)) * 0.6931471805599453f : kNegInf;
    }
    return;
  }

  // ---- several splits: partial records [m, s, o[0..DH)] per (sequence, row, head, split); the last split
  // waits for the others' flags and merges in split order (device-scope accesses, as in the split-K kernel) ----
  const int64_t b_row0 = static_cast<int64_t>(b) * max_q;
  if (split + 1 < nsplit) {
    for (int e = tid; e < n_out; e += kThreads) {
      const int v = e / kDH, c = e % kDH;
      float M, S, o;
      merged(v, c, M, S, o);
      int i_out, h_out;
      out_row_of(v, i_out, h_out);
      float* rec = ws + (((b_row0 + i_out) * H + h_out) * nsplit + split) * partial_floats<kDH>();
      if (c == 0) {
        __hip_atomic_store(rec + 0, M, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(rec + 1, S, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      __hip_atomic_store(rec + 2 + c, o, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // this thread's stores are acknowledged
    __syncthreads();
    if (tid < nv) {
      int i_out, h_out;
      out_row_of(tid, i_out, h_out);
      __hip_atomic_store(flags + ((b_row0 + i_out) * H + h_out) * nsplit + split, kPartialReady, __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
    }
    return;
  }
  // ---- the last split ----
  // (1) All flags are polled at once (one per thread and round: a device-scope load is a round trip past the
  // XCD's L2); the thread that sees the flag of (vector, split) fetches that record's m and s right away.  They go
  // to LDS behind the wavefronts' partials (room for 32 vectors x kMaxSplits - 1 splits in each of the first two regions).
  float* const st_m = reinterpret_cast<float*>(lds + kPartBytes);
  float* const st_s = reinterpret_cast<float*>(lds + kWaveLds + kPartBytes);
  float* const tot_s = st_m + kMaxVectors * (kMaxSplits - 1);  // per vector: the total sum and the weight of the own partial
  float* const own_w = tot_s + kMaxVectors;
  float* const tot_m = own_w + kMaxVectors;
  const int ns1 = nsplit - 1;
  const int n_flags = nv * ns1;
  auto row_slot = [&](int v) -> int64_t {
    int i_out, h_out;
    out_row_of(v, i_out, h_out);
    return ((b_row0 + i_out) * H + h_out) * nsplit;
  };
  int ok = 1;
  for (int f = tid; f < n_flags; f += kThreads) {
    const int v = f / ns1, sp = f - v * ns1;
    const int64_t slot = row_slot(v) + sp;
    int polls = 0;
    while (__hip_atomic_load(flags + slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != kPartialReady) {
      if (++polls > kMaxPolls) {
        ok = 0;
        break;
      }
      __builtin_amdgcn_s_sleep(16);
    }
    const float* rec = ws + slot * partial_floats<kDH>();
    st_m[f] = __hip_atomic_load(rec + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    st_s[f] = __hip_atomic_load(rec + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  const bool complete = __syncthreads_and(ok) != 0;
  // (2) One thread per vector: the total maximum, every partial's weight (kept where its maximum was) and the total
  // sum, added in split order with the own partial (the last split) last.
  if (tid < nv) {
    const int v = tid;
    float M_own, S_own, unused;
    merged(v, 0, M_own, S_own, unused);
    float M = M_own;
    for (int sp = 0; sp < ns1; ++sp) M = fmaxf(M, st_m[v * ns1 + sp]);
    float S = 0.f;
    for (int sp = 0; sp < ns1; ++sp) {
      const float w = (M == kNegInf) ? 0.f : exp2_hw(st_m[v * ns1 + sp] - M);
      st_m[v * ns1 + sp] = w;
      S = fmaf(st_s[v * ns1 + sp], w, S);
    }
    const float w_own = (M == kNegInf) ? 0.f : exp2_hw(M_own - M);
    tot_s[v] = fmaf(S_own, w_own, S);
    own_w[v] = w_own;
    tot_m[v] = M;
  }
  __syncthreads();
  // (3) Outputs: a thread takes two neighbouring channels of a vector per step; the records of four steps and up to
  // sixteen splits are requested before the first is used, so the merge costs a few round trips, not one per record.
  constexpr int kStepsAtOnce = 4, kBatch = 16;
  constexpr int kRecWords = partial_floats<kDH>() / 2;  // a record in 8-byte words
  const int n_pairs = nv * (kDH / 2);
  for (int e0 = tid; e0 < n_pairs; e0 += kStepsAtOnce * kThreads) {
    int vv[kStepsAtOnce], cc[kStepsAtOnce];
    const uint64_t* rec[kStepsAtOnce];
    float acc0[kStepsAtOnce], acc1[kStepsAtOnce];
#pragma unroll
    for (int k = 0; k < kStepsAtOnce; ++k) {
      const int e = e0 + k * kThreads;
      const int ee = e < n_pairs ? e : e0;  // spare steps repeat the first one; nothing of them is stored
      vv[k] = ee / (kDH / 2);
      cc[k] = 2 * (ee % (kDH / 2));
      rec[k] = reinterpret_cast<const uint64_t*>(ws + row_slot(vv[k]) * partial_floats<kDH>() + 2 + cc[k]);
      acc0[k] = 0.f;
      acc1[k] = 0.f;
    }
    for (int s0 = 0; s0 < ns1; s0 += kBatch) {
      uint64_t ld[kStepsAtOnce][kBatch];
#pragma unroll
      for (int k = 0; k < kStepsAtOnce; ++k)
#pragma unroll
        for (int u = 0; u < kBatch; ++u)
          ld[k][u] = __hip_atomic_load(rec[k] + static_cast<int64_t>(min(s0 + u, ns1 - 1)) * kRecWords, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
      for (int k = 0; k < kStepsAtOnce; ++k)
#pragma unroll
        for (int u = 0; u < kBatch; ++u)
          if (s0 + u < ns1) {
            const float w = st_m[vv[k] * ns1 + s0 + u];
            acc0[k] = fmaf(__uint_as_float(static_cast<uint32_t>(ld[k][u])), w, acc0[k]);
            acc1[k] = fmaf(__uint_as_float(static_cast<uint32_t>(ld[k][u] >> 32)), w, acc1[k]);
          }
    }
#pragma unroll
    for (int k = 0; k < kStepsAtOnce; ++k) {
      if (e0 + k * kThreads >= n_pairs) continue;
      const int v = vv[k], c = cc[k];
      float M_own, S_own, o0, o1;
      merged(v, c, M_own, S_own, o0);
      merged(v, c + 1, M_own, S_own, o1);
      const float w = own_w[v], S = tot_s[v];
      const float nan = __builtin_nanf("");
      const float r0 = fmaf(o0, w, acc0[k]), r1 = fmaf(o1, w, acc1[k]);
      const float val0 = !complete ? nan : (S > 0.f) ? r0 / S : 0.f;  // a partial never arrived: fail loudly
      const float val1 = !complete ? nan : (S > 0.f) ? r1 / S : 0.f;
      int i_out, h_out;
      const int64_t out_row = out_row_of(v, i_out, h_out);
      *reinterpret_cast<uint32_t*>(O + out_row * kDH + c) = f32_to_bf16_bits(val0) | (f32_to_bf16_bits(val1) << 16);
      if (lse != nullptr && c == 0)
        lse[out_row] = !complete ? nan : (S > 0.f) ? (tot_m[v] + __log2f(S)) * 0.6931471805599453f : kNegInf;
    }
  }
  // the flags are left cleared for the next call on this workspace
  for (int f = tid; f < n_flags; f += kThreads) {
    const int v = f / ns1, sp = f - v * ns1;
    __hip_atomic_store(flags + row_slot(v) + sp, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

template <int DH, int NWV>
int launch_nwv(const AttnParams& p, int row0, int rows_per, int nsplit, uint32_t* flags) {
  constexpr int kLds = NWV * GroupDims<DH>::kWaveLds;
  const void* kernel = reinterpret_cast<const void*>(&group_attention_kernel<DH, NWV>);
  const int rc = allow_dynamic_lds(kernel, kLds);
  if (rc != DODO_OK) return rc;
  const int G = p.H / p.H_kv;
  const dim3 grid(static_cast<unsigned>(p.H_kv), static_cast<unsigned>(p.B), static_cast<unsigned>(nsplit));
  hipLaunchKernelGGL((group_attention_kernel<DH, NWV>), grid, dim3(NWV * kWave), kLds, p.stream,
                     static_cast<const uint16_t*>(p.Q), static_cast<const uint16_t*>(p.Kn),
                     static_cast<const uint16_t*>(p.Vn), static_cast<const uint16_t*>(p.Kl),
                     static_cast<const uint16_t*>(p.Vl), p.cu_q, p.cu_nuggets, p.nug_len, p.cu_local, p.loc_len, p.H,
                     p.H_kv, G, make_fast_div(static_cast<uint32_t>(G)), p.max_q, row0, rows_per, nsplit, p.nug_tok_stride,
                     p.nug_head_stride, p.scale_log2e, static_cast<uint16_t*>(p.O), p.lse, static_cast<float*>(p.ws),
                     flags);
  return launch_status();
}

constexpr int kWantedWorkgroups = 512;  // two per compute unit of the 256

// Splits for these bounds: enough workgroups for two per compute unit (one of four wavefronts where that takes
// splitting), at least eight tiles per split, and no more than the caller's workspace has records for (none if it
// is not 8-byte aligned: records are read in 8-byte words).
int group_split_count(const AttnParams& p) {
  const int64_t pairs = static_cast<int64_t>(p.B) * p.H_kv;
  const int64_t rows = static_cast<int64_t>(p.max_k) + p.max_local;
  int64_t n = pairs >= kWantedWorkgroups / 2 ? (kWantedWorkgroups + pairs - 1) / pairs
                                             : (kWantedWorkgroups / 2 + pairs - 1) / pairs;
  const int64_t room = rows / (8 * kKeys);
  if (n > room) n = room;
  const int64_t most = p.d_h == 128 ? GroupDims<128>::kMaxSplits : GroupDims<64>::kMaxSplits;
  if (n > most) n = most;
  const int64_t records_per_split = static_cast<int64_t>(p.B) * p.max_q * p.H;
  int64_t fit;
  if (p.ws_flags != nullptr) {  // records and flags in separate regions of ws_slots entries each
    fit = p.ws_slots / records_per_split;
  } else {  // one region: records of d_h + 2 floats, then a flag each
    const bool usable = p.ws != nullptr && (reinterpret_cast<uintptr_t>(p.ws) & 7) == 0;
    fit = usable ? static_cast<int64_t>(p.ws_bytes / (records_per_split * (p.d_h + 3) * sizeof(float))) : 0;
  }
  if (n > fit) n = fit;
  return n < 1 ? 1 : static_cast<int>(n);
}

}  // namespace

size_t group_workspace_bytes(int32_t B, int32_t H, int32_t H_kv, int32_t d_h, int32_t max_q, int32_t max_k,
                             int32_t max_local) {
  AttnParams p{};
  p.B = B; p.H = H; p.H_kv = H_kv; p.d_h = d_h; p.max_q = max_q; p.max_k = max_k; p.max_local = max_local;
  p.ws = &p;  // any non-null address: the count is not limited by a workspace here
  p.ws_bytes = ~static_cast<size_t>(0);
  const int n = group_split_count(p);
  return n <= 1 ? 0 : static_cast<size_t>(B) * max_q * H * n * (d_h + 3) * sizeof(float);
}

// Launches that cover the query rows of a call: each takes as many rows as fit the 32 vectors of a tile with G
// heads per row.  0: the kernel does not take such a call (fewer than 4 vectors share a row, more than 32 heads
// per KV head, or more than four passes over the keys, where the K/V rows would be read too often).
int group_launches(int32_t H, int32_t H_kv, int32_t max_q) {
  const int64_t G = H / H_kv;
  if (G > kMaxVectors || G * max_q < 4) return 0;
  const int rows_per = static_cast<int>(kMaxVectors / G);
  const int launches = (max_q + rows_per - 1) / rows_per;
  return launches <= 4 ? launches : 0;
}

bool group_attention_applies(const AttnParams& p) {
  if (p.dtype != DODO_DTYPE_BF16 || (p.d_h != 128 && p.d_h != 64) || p.nug_idx != nullptr) return false;
  if (group_launches(p.H, p.H_kv, p.max_q) == 0) return false;
  if (p.B > 65535) return false;  // second grid dimension
  // a row number times a stride in bytes is kept in 32 bits
  if (p.nug_tok_stride * 2 * kKeys > 0xffffffffLL || static_cast<int64_t>(p.H_kv) * p.d_h * 2 * kKeys > 0xffffffffLL)
    return false;
  // at least a workgroup for every other compute unit: with fewer (a small batch and a workspace too small to
  // split further), the split-K kernel's wider workgroups keep more loads in flight
  return static_cast<int64_t>(p.B) * p.H_kv * group_split_count(p) * 2 >= compute_units();
}

int launch_group_attention(const AttnParams& p) {
  const int nsplit = group_split_count(p);
  uint32_t* flags = p.ws_flags != nullptr
                        ? static_cast<uint32_t*>(p.ws_flags)
                        : reinterpret_cast<uint32_t*>(static_cast<float*>(p.ws) +
                                                      static_cast<int64_t>(p.B) * p.max_q * p.H * nsplit * (p.d_h + 2));
  // two workgroups of two wavefronts per compute unit when there are that many; else one of four
  const bool two = static_cast<int64_t>(p.B) * p.H_kv * nsplit >= 2 * compute_units();
  const int rows_per = kMaxVectors / (p.H / p.H_kv);
  for (int row0 = 0; row0 < p.max_q; row0 += rows_per) {  // (records and flags of different rows are apart)
    int rc;
    if (p.d_h == 128) {
      rc = two ? launch_nwv<128, 2>(p, row0, rows_per, nsplit, flags) : launch_nwv<128, 4>(p, row0, rows_per, nsplit, flags);
    } else {
      rc = two ? launch_nwv<64, 2>(p, row0, rows_per, nsplit, flags) : launch_nwv<64, 4>(p, row0, rows_per, nsplit, flags);
    }
    if (rc != DODO_OK) return rc;
  }
  return DODO_OK;
}

}  // namespace dodo
