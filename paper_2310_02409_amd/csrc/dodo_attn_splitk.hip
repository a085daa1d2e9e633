// Bandwidth-bound nugget attention (Eq. 9 / Eq. 13 of the Dodo paper) for
// single-token decode and small query counts: every visible K and V row is
// read once with 16-byte loads, a group of lanes per row.
//
// One workgroup handles one (query row, head, split) -- or several query vectors that read the same K/V rows:
// the GH query heads of one KV head (grouped-query attention) and / or QR consecutive query rows of a small
// query block.  Its lane groups are then split between those query vectors, every K/V row is requested by
// their groups in the same instructions, and the compute unit's L1 turns that into one read of the row, so
// the row comes from HBM once per KV head and row group rather than once per query vector.  Its 256 threads form
// G = 256 / lanes-per-row groups; with one head, group g walks rows g, g+G, ... of the split,
// keeping an independent online-softmax state (running max, sum, d_h partial
// outputs spread over its lanes) in base 2.  Groups are merged through LDS in
// group order.  With several splits every workgroup but the last of a row
// writes its partial (m, s, o) to the workspace and raises a flag; the
// workgroup of the last split waits for those flags (workgroups start in index
// order and the last split has the highest indices, so what it waits for is
// running or done; the wait is bounded anyway), merges the partials in split
// order, writes the row and clears the flags.  No float atomics anywhere, so
// results are run-to-run deterministic.
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

// partial record of one split in the workspace: [m, s, o[0..DH)] floats; after all records, one
// 32-bit flag per record
template <int DH>
__host__ __device__ constexpr int partial_floats() { return DH + 2; }
constexpr uint32_t kPartialReady = 0x600DD0D0u;  // flag value of a record that has been written
constexpr int kMaxPolls = 1 << 17;               // bound of the combiner's wait (~0.1 s, never reached in a healthy run)

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
    int H, int H_kv, int GH_arg, int QR_arg, int max_q, int nsplit, int64_t nug_tok_stride, int64_t nug_head_stride,
    float scale_log2e, void* __restrict__ O, float* __restrict__ lse, float* __restrict__ ws,
    uint32_t* __restrict__ flags) {
  const int GH = GROUPED ? GH_arg : 1;  // query heads per workgroup
  const int QR = GROUPED ? QR_arg : 1;  // query rows per workgroup
  const int GV = GH * QR;               // query vectors per workgroup
  using VT = Vec16<DTYPE>;
  constexpr int kEPL = VT::kElems;          // elements per lane
  constexpr int kLPR = DH / kEPL;           // lanes per K/V row
  constexpr int kGroups = kThreads / kLPR;  // rows processed side by side
  constexpr size_t kEs = DTYPE == DODO_DTYPE_F32 ? 4 : 2;

  __shared__ float part_m[kGroups], part_s[kGroups];
  __shared__ float part_o[kGroups][DH];

  // Split-major order: workgroups are started in index order, so the workgroups of the last split,
  // which wait for the others of their row and combine, start after everything they wait for.
  const int rows_total = gridDim.x / nsplit;
  int t = blockIdx.x % rows_total;
  const int split = blockIdx.x / rows_total;
  // Grouped-query attention: the query heads that share a KV head read the same K/V rows.  Workgroups are handed
  // to the 8 XCDs round-robin and every XCD has an L2 of its own.  Where the heads of a group have a workgroup each
  // (GH == 1: few workgroups in all), they are placed a multiple of 8 workgroups apart, so that they run on one XCD
  // at about the same time and share the rows in its L2 as far as that holds them.  (Query rows of one head are H
  // workgroups apart, which does the same when H is a multiple of 8.)
  // GH > 1: this workgroup serves heads head0 .. head0 + GH - 1 (one KV head); else the one head head0
  const int HG = H / GH;
  int head0 = t % HG;
  t /= HG;
  if (GV == 1) {
    const int G = H / H_kv;
    if (G > 1 && (H_kv & 7) == 0) {
      head0 = ((head0 / (8 * G)) * 8 + (head0 & 7)) * G + (head0 >> 3) % G;  // KV head from the position mod 8, then the head in its group
    } else if (G > 1 && (H_kv == 1 || H_kv == 2 || H_kv == 4)) {
      head0 = (head0 % H_kv) * G + head0 / H_kv;
    }
  } else {
    head0 *= GH;
  }
  const int IG = (max_q + QR - 1) / QR;  // row groups per sequence
  const int i0 = (t % IG) * QR;          // first query row of this workgroup
  const int b = t / IG;
  const int q0 = cu_q[b];
  const int q_b = cu_q[b + 1] - q0;
  if (i0 >= q_b) return;  // uniform over the workgroup
  const int k0 = cu_nuggets[b], k_b = nug_len != nullptr ? nug_len[b] : cu_nuggets[b + 1] - k0;
  const int l0 = cu_local[b], m_b = loc_len != nullptr ? loc_len[b] : cu_local[b + 1] - l0;
  const int g = threadIdx.x / kLPR;
  const int sub = threadIdx.x % kLPR;
  const int qv = g % GV;      // this lane group's query vector among the workgroup's: (row, head) = (qv / GH, qv % GH)
  const int rs = g / GV;      // ... and its row stream: K/V rows rs, rs + R, ... of the split
  const int R = kGroups / GV;
  const int i = i0 + qv / GH;
  const bool row_ok = i < q_b;  // (a row group may reach past the sequence's last query row)
  const int h = head0 + qv % GH;
  const int kvh = h / (H / H_kv);  // the same for all heads of the workgroup
  // causal rule, bottom-right aligned: row i sees the nuggets and local rows j <= m_b - q_b + i.  The split is cut
  // from what the workgroup's last row sees (the most); every lane group stops at what its own row sees.
  const int i_last = min(i0 + QR, q_b) - 1;
  const int n_vis_wg = k_b + max(0, min(m_b, m_b - q_b + i_last + 1));
  const int n_vis = row_ok ? k_b + max(0, min(m_b, m_b - q_b + i + 1)) : 0;
  const int chunk = (n_vis_wg + nsplit - 1) / nsplit;
  const int r0 = split * chunk;
  const int r1_wg = min(r0 + chunk, n_vis_wg);  // rows [r0, r1_wg) are loaded by the workgroup ...
  const int r1 = min(r0 + chunk, n_vis);        // ... of which this lane group's query vector sees [r0, r1)
  const int64_t row_id = static_cast<int64_t>(q0 + min(i, q_b - 1)) * H + h;

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

  const int64_t ctx0 = INDEXED ? cu_ctx[b] : 0;
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
      const int64_t nug_row = INDEXED ? ctx0 + tok[u] : static_cast<int64_t>(k0 + j);
      const int64_t off = nug ? (nug_row * nug_tok_stride + nug_base) * kEs
                              : (static_cast<int64_t>(l0 + j - k_b) * H_kv * DH + loc_base) * kEs;
      bt.kv[u] = load16_stream(static_cast<const char*>(nug ? Kn : Kl) + off);
      bt.vv[u] = load16_stream(static_cast<const char*>(nug ? Vn : Vl) + off);
    }
  };
  auto use_batch = [&](const Batch& bt) {
    float logit[kRowsInFlight];
    float mx = m;
#pragma unroll
    for (int u = 0; u < kRowsInFlight; ++u) {
      float kf[kEPL];
      VT::unpack(bt.kv[u], kf);
      float d = q[0] * kf[0];
#pragma unroll
      for (int e = 1; e < kEPL; ++e) d = fmaf(q[e], kf[e], d);
#pragma unroll
      for (int off = kLPR / 2; off >= 1; off >>= 1) d += __shfl_xor(d, off, kWave);
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
    const int kStep = R * kRowsInFlight;
    Batch ba, bb;
    int j0 = r0;  // (uniform over the workgroup, like r1_wg)
    if (j0 < r1_wg) load_batch(ba, j0);
    while (j0 < r1_wg) {
      if (j0 + kStep < r1_wg) load_batch(bb, j0 + kStep);
      use_batch(ba);
      j0 += kStep;
      if (j0 >= r1_wg) break;
      if (j0 + kStep < r1_wg) load_batch(ba, j0 + kStep);
      use_batch(bb);
      j0 += kStep;
    }
  }

  // ---- merge the lane groups of each head in group order ----
  if (sub == 0) {
    part_m[g] = m;
    part_s[g] = ssum;
  }
#pragma unroll
  for (int e = 0; e < kEPL; ++e) part_o[g][sub * kEPL + e] = o[e];
  __syncthreads();
  __shared__ int all_there;
  for (int hh = 0; hh < GV; ++hh) {  // one query vector of the workgroup after the other (uniform over the workgroup)
    const int i_out = i0 + hh / GH, h_out = head0 + hh % GH;
    if (i_out >= q_b) continue;
    const int64_t out_row = static_cast<int64_t>(q0 + i_out) * H + h_out;
    float Mg = kNegInf, Sg = 0.f, og = 0.f;  // this workgroup's merged partial of the head (threads < DH: channel threadIdx.x)
    if (threadIdx.x < DH) {
      const int c = threadIdx.x;
      float M = kNegInf;
      for (int gg = hh; gg < kGroups; gg += GV) M = fmaxf(M, part_m[gg]);
      float S = 0.f, oc = 0.f;
      if (M != kNegInf) {
        for (int gg = hh; gg < kGroups; gg += GV) {
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
    if (threadIdx.x == 0) {
      int ok = 1;
      for (int s2 = 0; ok && s2 + 1 < nsplit; ++s2) {
        int polls = 0;
        while (__hip_atomic_load(flags + slot0 + s2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != kPartialReady) {
          if (++polls > kMaxPolls) {
            ok = 0;
            break;
          }
          __builtin_amdgcn_s_sleep(16);
        }
      }
      all_there = ok;
    }
    __syncthreads();
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
      const bool ok = all_there != 0;
      const float nan = __builtin_nanf("");
      const float val = !ok ? nan : (S > 0.f) ? oc / S : 0.f;  // a partial never arrived: fail loudly
      if (DTYPE == DODO_DTYPE_F32) {
        static_cast<float*>(O)[out_row * DH + c] = val;
      } else {
        static_cast<uint16_t*>(O)[out_row * DH + c] = static_cast<uint16_t>(f32_to_bf16_bits(val));
      }
      if (lse != nullptr && c == 0)
        lse[out_row] = !ok ? nan : (S > 0.f) ? (M + __log2f(S)) * 0.6931471805599453f : kNegInf;
      // the flags are left cleared for the next call on this workspace
      for (int f = c; f + 1 < nsplit; f += DH)
        __hip_atomic_store(flags + slot0 + f, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();  // all_there is reused by the next head
  }
}

// Query vectors that a workgroup serves together because they read the same K/V rows: gh query heads of one KV
// head times qr consecutive query rows (powers of two, at most 8 vectors: the lane groups of the smallest
// workgroup), as long as that still leaves two workgroups per compute unit.
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
  *gh_out = gh;
  *qr_out = qr;
}

template <int DTYPE, int DH, bool INDEXED>
int launch_t(const AttnParams& p, int nsplit) {
  int gh = 1, qr = 1;
  vectors_per_workgroup(p, nsplit, &gh, &qr);
  const int64_t rows = static_cast<int64_t>(p.B) * ((p.max_q + qr - 1) / qr) * (p.H / gh);  // workgroups per split
  // one flag word per record (one record per query row, head and split): right behind the records, unless the
  // caller keeps them elsewhere
  uint32_t* flags = p.ws_flags != nullptr
                        ? static_cast<uint32_t*>(p.ws_flags)
                        : reinterpret_cast<uint32_t*>(static_cast<float*>(p.ws) +
                                                      static_cast<int64_t>(p.B) * p.max_q * p.H * nsplit * partial_floats<DH>());
  // few workgroups (about one per CU) with many rows each: 16 wavefronts per workgroup keep enough
  // loads in flight; otherwise 4 wavefronts and several workgroups per CU
  const bool wide = rows * nsplit <= 512 && static_cast<int64_t>(p.max_k) + p.max_local >= 512;
  const dim3 grid(static_cast<unsigned>(rows * nsplit));
#define DODO_LAUNCH_SPLITK(THREADS, GROUPED)                                                                               \
  hipLaunchKernelGGL((splitk_attention_kernel<DTYPE, DH, THREADS, INDEXED, GROUPED>), grid, dim3(THREADS), 0, p.stream, p.Q,  \
                     p.Kn, p.Vn, p.Kl, p.Vl, p.cu_q, p.cu_nuggets, p.nug_len, p.cu_local, p.loc_len, p.nug_idx, p.cu_ctx, p.H, \
                     p.H_kv, gh, qr, p.max_q, nsplit, p.nug_tok_stride, p.nug_head_stride, p.scale_log2e, p.O, p.lse,         \
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
