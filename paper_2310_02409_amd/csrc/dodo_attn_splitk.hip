// Bandwidth-bound nugget attention (Eq. 9 / Eq. 13 of the Dodo paper) for
// single-token decode and small query counts: every visible K and V row is
// read once with 16-byte loads, a group of lanes per row.
//
// One workgroup handles one (query row, head, split) -- or several query vectors: the GH query heads of one KV head
// (grouped-query attention) and / or QR consecutive query rows of a small query block, which read the same K/V rows,
// or two neighbouring heads of plain multi-head attention, whose rows lie side by side in memory.  Its lane groups
// are then split between those query vectors; where they read the same row, the row is requested by their groups
// in the same instructions and the compute unit's L1 turns that into one read, so it comes from HBM once per KV
// head and row group rather than once per query vector.  The workgroup's threads form threads / lanes-per-row
// lane groups; with one query vector, group g walks rows g, g+G, ... of the split, four rows per batch, two
// batches in flight, keeping an independent online-softmax state (running max, sum, d_h partial outputs spread
// over its lanes) in base 2.  Lane groups are merged across the lanes of a wavefront, then through LDS, in a
// fixed order.  With several splits every workgroup but the last of a row writes its partial (m, s, o) to the
// workspace and raises a flag; the workgroup of the last split waits for those flags (workgroups start in index
// order and the last split has the highest indices, so what it waits for is running or done; the wait is bounded
// anyway), merges the partials in split order, writes the row and clears the flags.  No float atomics anywhere,
// so results are run-to-run deterministic.
#include "dodo_attn.h"

namespace dodo {
namespace {

constexpr int kRowsInFlight = 4;  // rows a group loads before it starts the arithmetic
constexpr float kNegInf = -__builtin_inff();

template <int DTYPE>
struct Vec16;
// dot(q, k) of the 16 bytes a lane holds of each.  bf16: products of pairs are exact in fp32 and summed in fp32 by
// the packed dot instruction, straight from the packed values (no unpacking of K).
template <>
struct Vec16<DODO_DTYPE_BF16> {
  static constexpr int kElems = 8;
  __device__ static __forceinline__ void unpack(const uint4& v, float* f) {
    f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x); f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
    f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z); f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
  }
  __device__ static __forceinline__ float dot(const uint4& q, const uint4& k) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    float d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q.x), __builtin_bit_cast(bf16x2, k.x), 0.f, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q.y), __builtin_bit_cast(bf16x2, k.y), d, false);
    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q.z), __builtin_bit_cast(bf16x2, k.z), d, false);
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q.w), __builtin_bit_cast(bf16x2, k.w), d, false);
  }
};
template <>
struct Vec16<DODO_DTYPE_F32> {
  static constexpr int kElems = 4;
  __device__ static __forceinline__ void unpack(const uint4& v, float* f) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
  }
  __device__ static __forceinline__ float dot(const uint4& q, const uint4& k) {
    float d = __uint_as_float(q.x) * __uint_as_float(k.x);
    d = fmaf(__uint_as_float(q.y), __uint_as_float(k.y), d);
    d = fmaf(__uint_as_float(q.z), __uint_as_float(k.z), d);
    return fmaf(__uint_as_float(q.w), __uint_as_float(k.w), d);
  }
};

// Sum over the kLPR lanes that share a K/V row (kLPR = 8, 16 or 32 consecutive lanes), every lane getting the total.
template <int kLPR>
__device__ __forceinline__ float sum_over_row_lanes(float d) {
  d = lanes_sum<(kLPR >= 16 ? 16 : 8)>(d);
  if (kLPR >= 32) d += __shfl_xor(d, 16, kWave);
  return d;
}

__device__ __forceinline__ float exp2_guard(float x) { return __builtin_amdgcn_exp2f(x); }  // exp2(-inf) = 0

// INDEXED: Kn / Vn are the context's K / V ([N, H_kv, DH], nug_tok_stride between tokens) and nugget j of
// sequence b is token cu_ctx[b] + nug_idx[cu_nuggets[b] + j] of it (no packed cache has been made).
// GROUPED: the workgroup serves GH query heads of one KV head times QR query rows, more than one query vector in all
// (else both are 1 and everything about them folds away).
template <int DTYPE, int DH, int kThreads, bool INDEXED, bool GROUPED>
__global__ __launch_bounds__(kThreads) void splitk_attention_kernel(
    const void* __restrict__ Q, const void* __restrict__ Kn, const void* __restrict__ Vn,
    const void* __restrict__ Kl, const void* __restrict__ Vl, const int32_t* __restrict__ cu_q,
    const int32_t* __restrict__ cu_nuggets, const int32_t* __restrict__ nug_len,
    const int32_t* __restrict__ cu_local, const int32_t* __restrict__ loc_len, const int32_t* __restrict__ nug_idx,
    const int32_t* __restrict__ cu_ctx,
    int H, int H_kv, int G, int gh_log2, int qr_log2, int max_q, int nsplit, int64_t nug_tok_stride, int64_t nug_head_stride,
    float scale_log2e, void* __restrict__ O, float* __restrict__ lse, float* __restrict__ ws,
    uint32_t* __restrict__ flags) {
  // (powers of two, like the lane groups they are dealt to; G = H / H_kv query heads share a KV head)
  const int GH_L = GROUPED ? gh_log2 : 0, QR_L = GROUPED ? qr_log2 : 0, GV_L = GH_L + QR_L;
  const int GH = 1 << GH_L;  // query heads per workgroup
  const int QR = 1 << QR_L;  // query rows per workgroup
  const int GV = 1 << GV_L;  // query vectors per workgroup
  using VT = Vec16<DTYPE>;
  constexpr int kEPL = VT::kElems;          // elements per lane
  constexpr int kLPR = DH / kEPL;           // lanes per K/V row
  constexpr int kGroups = kThreads / kLPR;  // rows processed side by side
  constexpr size_t kEs = DTYPE == DODO_DTYPE_F32 ? 4 : 2;

  __shared__ float part_m[kGroups], part_s[kGroups];
  __shared__ float part_o[kGroups][DH];

  // The kernel lasts tens of microseconds and nothing overlaps its first instructions, so the scalar loads at
  // its start are kept to two dependent rounds: all arguments (the compiler would otherwise fetch them a few at a
  // time, right before their first use), then all of the sequence's boundaries.
  asm volatile("" ::"s"(Q), "s"(Kn), "s"(Vn), "s"(Kl), "s"(Vl), "s"(cu_q), "s"(cu_nuggets), "s"(nug_len), "s"(cu_local),
               "s"(loc_len), "s"(nug_tok_stride), "s"(nug_head_stride), "s"(O), "s"(lse), "s"(H), "s"(H_kv), "s"(G),
               "s"(gh_log2), "s"(qr_log2), "s"(max_q), "s"(nsplit), "s"(scale_log2e));
  // Grid: x = head (or group of GH heads), y = (sequence, row group), z = split.  Workgroups are started in index
  // order with x fastest and z slowest, so the workgroups of the last split, which wait for the others of their
  // row and combine, start after everything they wait for.  (The three indices come from the hardware: taking a
  // linear index apart would cost several integer divisions, each some thirty vector instructions that all
  // wavefronts of the workgroup execute before their first load.)
  const int split = blockIdx.z;
  // Grouped-query attention: the query heads that share a KV head read the same K/V rows.  Workgroups are handed
  // to the 8 XCDs round-robin and every XCD has an L2 of its own.  Where the heads of a group have a workgroup each
  // (GH == 1: few workgroups in all), they are placed a multiple of 8 workgroups apart, so that they run on one XCD
  // at about the same time and share the rows in its L2 as far as that holds them.  (Query rows of one head are H
  // workgroups apart, which does the same when H is a multiple of 8.)
  // GH > 1: this workgroup serves heads head0 .. head0 + GH - 1; else the one head head0
  int head0 = blockIdx.x;
  if (GV == 1) {
    if (G > 1 && (H_kv & 7) == 0) {
      head0 = ((head0 / (8 * G)) * 8 + (head0 & 7)) * G + (head0 >> 3) % G;  // KV head from the position mod 8, then the head in its group
    } else if (G > 1 && (H_kv == 1 || H_kv == 2 || H_kv == 4)) {
      head0 = (head0 % H_kv) * G + head0 / H_kv;
    }
  } else {
    head0 <<= GH_L;
  }
  const int IG = (max_q + QR - 1) >> QR_L;  // row groups per sequence
  int b = blockIdx.y, ig = 0;
  if (IG > 1) {
    b = blockIdx.y / IG;
    ig = blockIdx.y - b * IG;
  }
  const int i0 = ig << QR_L;  // first query row of this workgroup
  // Everything the addresses depend on is fetched at once, before the first branch: each dependent round of
  // scalar loads is a memory latency that nothing overlaps at the start of a kernel that lasts tens of them.
  const int32_t* k_end_p = nug_len != nullptr ? nug_len + b : cu_nuggets + b + 1;
  const int32_t* l_end_p = loc_len != nullptr ? loc_len + b : cu_local + b + 1;
  const int q0 = cu_q[b], q_end = cu_q[b + 1];
  const int k0 = cu_nuggets[b], k_end = *k_end_p;
  const int l0 = cu_local[b], l_end = *l_end_p;
  const int64_t ctx0 = INDEXED ? cu_ctx[b] : 0;
  asm volatile("" ::"s"(q0), "s"(q_end), "s"(k0), "s"(k_end), "s"(l0), "s"(l_end), "s"(ctx0));
  const int q_b = q_end - q0;
  const int k_b = nug_len != nullptr ? k_end : k_end - k0;
  const int m_b = loc_len != nullptr ? l_end : l_end - l0;
  if (i0 >= q_b) return;  // uniform over the workgroup
  const int g = threadIdx.x / kLPR;
  const int sub = threadIdx.x % kLPR;
  const int qv = g & (GV - 1);  // this lane group's query vector among the workgroup's: (row, head) = (qv / GH, qv % GH)
  const int rs = g >> GV_L;     // ... and its row stream: K/V rows rs, rs + R, ... of the split
  const int R = kGroups >> GV_L;
  const int i = i0 + (qv >> GH_L);
  const bool row_ok = i < q_b;  // (a row group may reach past the sequence's last query row)
  const int h = head0 + (qv & (GH - 1));
  const int kvh = G == 1 ? h : h / G;
  // causal rule, bottom-right aligned: row i sees the nuggets and local rows j <= m_b - q_b + i.  The split is cut
  // from what the workgroup's last row sees (the most); every lane group stops at what its own row sees.
  const int i_last = min(i0 + QR, q_b) - 1;
  const int n_vis_wg = k_b + max(0, min(m_b, m_b - q_b + i_last + 1));
  const int n_vis = row_ok ? k_b + max(0, min(m_b, m_b - q_b + i + 1)) : 0;
  const int chunk = nsplit == 1 ? n_vis_wg : (n_vis_wg + nsplit - 1) / nsplit;
  const int r0 = split * chunk;
  const int r1_wg = min(r0 + chunk, n_vis_wg);  // rows [r0, r1_wg) are loaded by the workgroup ...
  const int r1 = min(r0 + chunk, n_vis);        // ... of which this lane group's query vector sees [r0, r1)
  const int64_t row_id = static_cast<int64_t>(q0 + min(i, q_b - 1)) * H + h;

  uint4 q_raw = make_uint4(0, 0, 0, 0);  // this lane's 16 bytes of the query vector, as they are in memory
  // Row addresses without branches: a row is `row` strides (32 x 32 -> 64 bits; the host checks that a stride in
  // bytes fits in 32 bits) past the first row of its region (nuggets of this sequence or KV head, local rows),
  // and the region's base pointers are uniform over the workgroup.
  const uint32_t nug_stride_b = static_cast<uint32_t>(nug_tok_stride * static_cast<int64_t>(kEs));
  const uint32_t loc_stride_b = static_cast<uint32_t>(static_cast<int64_t>(H_kv) * DH * static_cast<int64_t>(kEs));
  const int64_t nug_first = ((INDEXED ? ctx0 : static_cast<int64_t>(k0)) * nug_tok_stride +
                             static_cast<int64_t>(kvh) * nug_head_stride) * static_cast<int64_t>(kEs);
  const int64_t loc_first = (static_cast<int64_t>(l0) * H_kv + kvh) * DH * static_cast<int64_t>(kEs);
  const char* const nugK = static_cast<const char*>(Kn) + nug_first;
  const char* const nugV = static_cast<const char*>(Vn) + nug_first;
  const char* const locK = static_cast<const char*>(Kl) + loc_first;
  const char* const locV = static_cast<const char*>(Vl) + loc_first;
  const uint64_t lane_off = static_cast<uint64_t>(sub * kEPL) * kEs;

  float m = kNegInf, ssum = 0.f;
  float o[kEPL];
#pragma unroll
  for (int e = 0; e < kEPL; ++e) o[e] = 0.f;

  // A batch = kRowsInFlight rows per group.  The loads of batch i+1 are issued before the arithmetic of batch i
  // (two register sets), so that the memory latency is paid once per workgroup, not once per batch.
  struct Batch {
    uint4 kv[kRowsInFlight], vv[kRowsInFlight];
    int j0;
  };
  auto load_batch = [&](Batch& bt, int j0) {
    bt.j0 = j0;
    int tok[kRowsInFlight];  // INDEXED: sequence-local token of a nugget row (all index loads go out before the rows')
    if (INDEXED) {
#pragma unroll
      for (int u = 0; u < kRowsInFlight; ++u) {
        const int jr = j0 + u * R + rs;
        const int j = jr < r1_wg ? jr : r1_wg - 1;
        tok[u] = j < k_b ? nug_idx[k0 + j] : 0;
      }
    }
#pragma unroll
    for (int u = 0; u < kRowsInFlight; ++u) {
      // loads are unconditional (rows past the end re-read the last row of the range and are
      // discarded): a branch around them would serialise the loads behind a full wait
      const int jr = j0 + u * R + rs;
      const int j = jr < r1_wg ? jr : r1_wg - 1;
      const bool nug = j < k_b;
      const uint32_t row = static_cast<uint32_t>(nug ? (INDEXED ? tok[u] : j) : j - k_b);
      const uint64_t off = static_cast<uint64_t>(row) * (nug ? nug_stride_b : loc_stride_b) + lane_off;
      bt.kv[u] = load16_stream((nug ? nugK : locK) + off);
      bt.vv[u] = load16_stream((nug ? nugV : locV) + off);
    }
  };
  auto use_batch = [&](const Batch& bt) {
    float logit[kRowsInFlight];
    float mx = m;
#pragma unroll
    for (int u = 0; u < kRowsInFlight; ++u) {
      const float d = sum_over_row_lanes<kLPR>(VT::dot(q_raw, bt.kv[u])) * scale_log2e;
      logit[u] = (bt.j0 + u * R + rs < r1) ? d : kNegInf;
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
        VT::unpack(bt.vv[u], vf);
        ssum += p;
#pragma unroll
        for (int e = 0; e < kEPL; ++e) o[e] = fmaf(p, vf[e], o[e]);
      }
      m = mx;
    }
  };
  {
    // Two register sets, two batches in flight.  The compiler keeps the count of outstanding loads that every
    // wait is based on, and where paths meet it must assume the fewest younger loads that any of them issued, so
    // a load under a condition turns the waits for everything older into waits for (nearly) all loads.  Hence
    // the shape of this loop: inside it every batch is loaded and used unconditionally (a batch past the end of
    // the split re-reads its last row and masks itself), the last pair of batches is used after the loop without
    // further loads, and the query vector, requested behind the first two batches, is waited for before the loop.
    const int kStep = R * kRowsInFlight;
    Batch ba, bb;
    if (r0 < r1_wg) {  // (uniform over the workgroup; false for an empty split)
      const int n_pairs = (r1_wg - r0 + 2 * kStep - 1) / (2 * kStep);
      int j0 = r0;
      load_batch(ba, j0);
      load_batch(bb, j0 + kStep);
      q_raw = *reinterpret_cast<const uint4*>(static_cast<const char*>(Q) + (row_id * DH + sub * kEPL) * kEs);
      asm volatile("" ::"v"(q_raw.x), "v"(q_raw.y), "v"(q_raw.z), "v"(q_raw.w));  // the query vector has arrived
      for (int it = 1; it < n_pairs; ++it) {
        use_batch(ba);
        load_batch(ba, j0 + 2 * kStep);
        use_batch(bb);
        load_batch(bb, j0 + 3 * kStep);
        j0 += 2 * kStep;
      }
      use_batch(ba);
      if (j0 + kStep < r1_wg) use_batch(bb);
    }
  }

  // ---- merge the lane groups of each query vector in group order ----
  // One query vector per workgroup: the lane groups of a wavefront are merged across lanes first (pairs, then
  // pairs of pairs; both partners evaluate the same expression, lower group first), so that LDS holds one
  // partial per wavefront and the loops below are short.  Several query vectors: one partial per lane group.
  constexpr int kParts = GROUPED ? kGroups : kThreads / kWave;
  if (!GROUPED) {
#pragma unroll
    for (int off = kLPR; off < kWave; off <<= 1) {
      const bool upper = (threadIdx.x & off) != 0;
      const float m_x = __shfl_xor(m, off, kWave), s_x = __shfl_xor(ssum, off, kWave);
      const float m_a = upper ? m_x : m, m_b2 = upper ? m : m_x;
      const float s_a = upper ? s_x : ssum, s_b2 = upper ? ssum : s_x;
      const float mb = fmaxf(m_a, m_b2);
      const float w_a = (mb == kNegInf) ? 0.f : exp2_guard(m_a - mb), w_b = (mb == kNegInf) ? 0.f : exp2_guard(m_b2 - mb);
      ssum = fmaf(s_b2, w_b, s_a * w_a);
#pragma unroll
      for (int e = 0; e < kEPL; ++e) {
        const float o_x = __shfl_xor(o[e], off, kWave);
        const float o_a = upper ? o_x : o[e], o_b = upper ? o[e] : o_x;
        o[e] = fmaf(o_b, w_b, o_a * w_a);
      }
      m = mb;
    }
  }
  const int part = GROUPED ? g : static_cast<int>(threadIdx.x) / kWave;
  if (GROUPED || (threadIdx.x & (kWave - 1)) < kLPR) {
    if (sub == 0) {
      part_m[part] = m;
      part_s[part] = ssum;
    }
#pragma unroll
    for (int e = 0; e < kEPL; ++e) part_o[part][sub * kEPL + e] = o[e];
  }
  __syncthreads();
  for (int hh = 0; hh < GV; ++hh) {  // one query vector of the workgroup after the other (uniform over the workgroup)
    const int i_out = i0 + (hh >> GH_L), h_out = head0 + (hh & (GH - 1));
    if (i_out >= q_b) continue;
    const int64_t out_row = static_cast<int64_t>(q0 + i_out) * H + h_out;
    float Mg = kNegInf, Sg = 0.f, og = 0.f;  // this workgroup's merged partial of the head (threads < DH: channel threadIdx.x)
    if (threadIdx.x < DH) {
      const int c = threadIdx.x;
      float M = kNegInf;
      for (int gg = hh; gg < kParts; gg += GV) M = fmaxf(M, part_m[gg]);
      float S = 0.f, oc = 0.f;
      if (M != kNegInf) {
        for (int gg = hh; gg < kParts; gg += GV) {
          const float wgt = exp2_guard(part_m[gg] - M);
          S = fmaf(part_s[gg], wgt, S);
          oc = fmaf(part_o[gg][c], wgt, oc);
        }
      }
      Mg = M;
      Sg = S;
      og = oc;
      if (nsplit == 1) {
        const float val = (S > 0.f) ? oc / S : 0.f;
        if (DTYPE == DODO_DTYPE_F32) {
          static_cast<float*>(O)[out_row * DH + c] = val;
        } else {
          static_cast<uint16_t*>(O)[out_row * DH + c] = static_cast<uint16_t>(f32_to_bf16_bits(val));
        }
        if (lse != nullptr && c == 0) lse[out_row] = (S > 0.f) ? (M + __log2f(S)) * 0.6931471805599453f : kNegInf;
      }
    }
    if (nsplit == 1) continue;

    // ---- several splits: the last one combines, in split order ----
    const int64_t slot0 = ((static_cast<int64_t>(b) * max_q + i_out) * H + h_out) * nsplit;
    if (split + 1 < nsplit) {
      // Records and flags are written and read with device-scope atomic accesses (plain stores and
      // loads that go to the level where all XCDs agree), so no cache has to be written back or
      // invalidated as a whole; the wait makes sure that the record has arrived there before the
      // flag is sent after it.
      if (threadIdx.x < DH) {
        float* rec = ws + (slot0 + split) * partial_floats<DH>();
        if (threadIdx.x == 0) {
          __hip_atomic_store(rec + 0, Mg, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_store(rec + 1, Sg, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __hip_atomic_store(rec + 2 + threadIdx.x, og, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this thread's stores are acknowledged
      }
      __syncthreads();
      if (threadIdx.x == 0)
        __hip_atomic_store(flags + slot0 + split, kPartialReady, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      continue;
    }
    // one thread per flag, all at once: a device-scope load is a round trip past the XCD's L2, and the splits of
    // a row finish at about the same time, so polling the flags one after the other would cost a trip each
    int ok = 1;
    if (static_cast<int>(threadIdx.x) + 1 < nsplit) {
      int polls = 0;
      while (__hip_atomic_load(flags + slot0 + threadIdx.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != kPartialReady) {
        if (++polls > kMaxPolls) {
          ok = 0;
          break;
        }
        __builtin_amdgcn_s_sleep(16);
      }
    }
    const int all_there = __syncthreads_and(ok);
    if (threadIdx.x < DH) {
      const int c = threadIdx.x;
      const float* rec0 = ws + slot0 * partial_floats<DH>();
      // splits in batches of 8 with all loads of a batch issued before the first use; the own
      // partial (the last split) comes last, so the order of the merge is the split order
      constexpr int kBatch = 8;
      float M = kNegInf, S = 0.f, oc = 0.f;
      auto merge = [&](float m1, float s1, float o1) {
        const float mb = fmaxf(M, m1);
        if (mb != kNegInf) {
          const float keep = exp2_guard(M - mb), wgt = exp2_guard(m1 - mb);
          S = fmaf(s1, wgt, S * keep);
          oc = fmaf(o1, wgt, oc * keep);
          M = mb;
        }
      };
      for (int s0 = 0; s0 + 1 < nsplit; s0 += kBatch) {
        float mm[kBatch], sv[kBatch], ov[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
          const float* r = rec0 + min(s0 + u, nsplit - 2) * partial_floats<DH>();
          mm[u] = __hip_atomic_load(r + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          sv[u] = __hip_atomic_load(r + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          ov[u] = __hip_atomic_load(r + 2 + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u)
          if (s0 + u + 1 < nsplit) merge(mm[u], sv[u], ov[u]);
      }
      merge(Mg, Sg, og);
      const bool complete = all_there != 0;
      const float nan = __builtin_nanf("");
      const float val = !complete ? nan : (S > 0.f) ? oc / S : 0.f;  // a partial never arrived: fail loudly
      if (DTYPE == DODO_DTYPE_F32) {
        static_cast<float*>(O)[out_row * DH + c] = val;
      } else {
        static_cast<uint16_t*>(O)[out_row * DH + c] = static_cast<uint16_t>(f32_to_bf16_bits(val));
      }
      if (lse != nullptr && c == 0)
        lse[out_row] = !complete ? nan : (S > 0.f) ? (M + __log2f(S)) * 0.6931471805599453f : kNegInf;
      // the flags are left cleared for the next call on this workspace
      for (int f = c; f + 1 < nsplit; f += DH)
        __hip_atomic_store(flags + slot0 + f, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

// Query vectors that a workgroup serves together because they read the same K/V rows: gh query heads of one KV
// head times qr consecutive query rows (powers of two, at most 8 vectors: the lane groups of the smallest
// workgroup), as long as that still leaves two workgroups per compute unit.  (The kernel takes any gh neighbouring
// query heads: each lane group derives its own KV head.)
void vectors_per_workgroup(const AttnParams& p, int nsplit, int* gh_out, int* qr_out) {
  const int G = p.H / p.H_kv;
  int gh = 1, qr = 1;
  while (gh < 8 && G % (2 * gh) == 0) gh *= 2;
  while (gh * qr < 8 && qr < p.max_q) qr *= 2;
  auto workgroups = [&](int gh_, int qr_) {
    return static_cast<int64_t>(p.B) * ((p.max_q + qr_ - 1) / qr_) * (p.H / gh_) * nsplit;
  };
  while (qr > 1 && workgroups(gh, qr) < 2 * compute_units()) qr /= 2;
  while (gh > 1 && workgroups(gh, qr) < 2 * compute_units()) gh /= 2;
  // Heads that share nothing can still share a workgroup: in the token-major layouts the rows of neighbouring KV
  // heads lie side by side, so two heads per workgroup read 2 * d_h contiguous elements of every token instead of
  // d_h (measured: 4% less time for a batch of 64 sequences with 32 heads; wider groups leave too few workgroups
  // to keep the loads of a compute unit in flight, so that is where it stops).
  const bool heads_side_by_side = p.nug_head_stride == p.d_h;
  if (G == 1 && gh == 1 && heads_side_by_side && p.H % 2 == 0 && 2 * qr <= 8 && workgroups(2, qr) >= 4 * compute_units())
    gh = 2;
  *gh_out = gh;
  *qr_out = qr;
}

template <int DTYPE, int DH, bool INDEXED>
int launch_t(const AttnParams& p, int nsplit) {
  int gh = 1, qr = 1;
  vectors_per_workgroup(p, nsplit, &gh, &qr);
  const int64_t row_groups = static_cast<int64_t>(p.B) * ((p.max_q + qr - 1) / qr);  // (sequence, row group) pairs
  if (row_groups > 65535 || nsplit > 65535) return DODO_ERR_UNSUPPORTED;              // second and third grid dimension
  const int64_t rows = row_groups * (p.H / gh);                                        // workgroups per split
  int gh_log2 = 0, qr_log2 = 0;
  while ((1 << gh_log2) < gh) ++gh_log2;
  while ((1 << qr_log2) < qr) ++qr_log2;
  // one flag word per record (one record per query row, head and split): right behind the records, unless the
  // caller keeps them elsewhere
  uint32_t* flags = p.ws_flags != nullptr
                        ? static_cast<uint32_t*>(p.ws_flags)
                        : reinterpret_cast<uint32_t*>(static_cast<float*>(p.ws) +
                                                      static_cast<int64_t>(p.B) * p.max_q * p.H * nsplit * partial_floats<DH>());
  // few workgroups (about one per CU) with many rows each: 16 wavefronts per workgroup keep enough
  // loads in flight; otherwise 4 wavefronts and several workgroups per CU
  const bool wide = rows * nsplit <= 512 && static_cast<int64_t>(p.max_k) + p.max_local >= 512;
  const dim3 grid(static_cast<unsigned>(p.H / gh), static_cast<unsigned>(row_groups), static_cast<unsigned>(nsplit));
#define DODO_LAUNCH_SPLITK(THREADS, GROUPED)                                                                               \
  hipLaunchKernelGGL((splitk_attention_kernel<DTYPE, DH, THREADS, INDEXED, GROUPED>), grid, dim3(THREADS), 0, p.stream, p.Q,  \
                     p.Kn, p.Vn, p.Kl, p.Vl, p.cu_q, p.cu_nuggets, p.nug_len, p.cu_local, p.loc_len, p.nug_idx, p.cu_ctx, p.H, \
                     p.H_kv, p.H / p.H_kv, gh_log2, qr_log2, p.max_q, nsplit, p.nug_tok_stride, p.nug_head_stride, p.scale_log2e, p.O, p.lse,         \
                     static_cast<float*>(p.ws), flags)
  if (wide) {
    if (gh * qr > 1) DODO_LAUNCH_SPLITK(1024, true); else DODO_LAUNCH_SPLITK(1024, false);
  } else {
    if (gh * qr > 1) DODO_LAUNCH_SPLITK(256, true); else DODO_LAUNCH_SPLITK(256, false);
  }
#undef DODO_LAUNCH_SPLITK
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
  return static_cast<size_t>(B) * max_q * H * nsplit * (d_h + 3) * sizeof(float);  // records, then one flag each
}

int launch_splitk_attention(const AttnParams& p) {
  const int nsplit = splitk_count(p.B, p.H, p.max_q, p.max_k, p.max_local);
  if (static_cast<int64_t>(p.B) * p.max_q * p.H * nsplit > 0x7fffffffLL) return DODO_ERR_UNSUPPORTED;
  // the kernel multiplies a row number by a stride in bytes kept in 32 bits
  if (p.nug_tok_stride * 4 > 0xffffffffLL || static_cast<int64_t>(p.H_kv) * p.d_h * 4 > 0xffffffffLL)
    return DODO_ERR_UNSUPPORTED;
  const bool indexed = p.nug_idx != nullptr;
  if (p.dtype == DODO_DTYPE_BF16) {
    if (p.d_h == 128) return indexed ? launch_t<DODO_DTYPE_BF16, 128, true>(p, nsplit) : launch_t<DODO_DTYPE_BF16, 128, false>(p, nsplit);
    if (p.d_h == 64) return indexed ? launch_t<DODO_DTYPE_BF16, 64, true>(p, nsplit) : launch_t<DODO_DTYPE_BF16, 64, false>(p, nsplit);
  } else {
    if (p.d_h == 128) return indexed ? launch_t<DODO_DTYPE_F32, 128, true>(p, nsplit) : launch_t<DODO_DTYPE_F32, 128, false>(p, nsplit);
    if (p.d_h == 64) return indexed ? launch_t<DODO_DTYPE_F32, 64, true>(p, nsplit) : launch_t<DODO_DTYPE_F32, 64, false>(p, nsplit);
  }
  return DODO_ERR_UNSUPPORTED;
}

}  // namespace dodo
