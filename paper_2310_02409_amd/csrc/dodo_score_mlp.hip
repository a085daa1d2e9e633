// dodo_score_mlp: the scorer as the 2-layer feedforward network of the Dodo
// paper's appendix (Sec. 2.1, App. B: d -> d_hid -> 1, 16.8 M parameters for
// d = d_hid = 4096):
//     s[t] = sum_j w2[j] * act( sum_c W1[j,c] x[t,c] + b1[j] ) + b2.
// The paper does not name the activation; ReLU, GELU (erf form) and tanh are
// offered.  2 N d d_hid flop: a dense contraction, so it runs on the matrix cores.
//
// MFMA kernel (bf16, d % 64 == 0, d_hid % 256 == 0): a workgroup of 8 wavefronts
// owns 256 tokens and walks over 256-wide tiles of hidden units; for each it
// accumulates H^T = W1_tile X^T over d in steps of 64 channels with
// v_mfma_f32_32x32x16_bf16 (A = W1 rows, B = token rows, so that a token is a lane
// of the accumulators and the reduction over hidden units stays inside a lane),
// then applies bias, activation and w2 to the accumulators and adds them to the
// tokens' partial scores.  The N x d_hid intermediate never leaves the registers.
// X and W1 tiles stream global -> LDS with 16-byte direct loads of whole 128-byte
// rows into two 64 KiB stages; the 16-byte pieces of a row are XOR-swizzled so
// that the fragment reads are conflict-free (measured: no bank-conflict cycles).
// One barrier per step, after the third of its four 16-channel parts: by then a
// wavefront holds the last part's fragments in registers, so the stage can be
// refilled (for the step after next) right after the barrier, and the next
// step's first fragments are fetched under the last part's matrix instructions.
// The hidden tiles are split over (at least four) workgroups, and the workgroups
// resident on one XCD form a patch of token tiles x splits that share their
// panels through that XCD's L2; a second kernel adds the partial scores in split
// order.  All sums have a fixed order (no atomics): run-to-run deterministic.
//
// Everything else (fp32 inputs, other shapes) takes a plain kernel that keeps a
// few token rows in LDS and gives one wavefront a hidden unit at a time: correct
// for any shape, slow for large ones (W1 is re-read for every group of tokens).
#include "dodo_common.h"

namespace dodo {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef __attribute__((address_space(3))) void lds_void;

constexpr int kTokTile = 256;  // tokens per workgroup
constexpr int kHidTile = 256;  // hidden units per tile
constexpr int kBK = 64;        // channels per step
constexpr int kStagesG = 2;
constexpr int kOperandBytes = kTokTile * kBK * 2;  // 16 KiB: one operand tile of a stage (both tiles have 256 rows)
constexpr int kStageBytesG = 2 * kOperandBytes;
constexpr int kMlpThreads = 512;
constexpr int kLoadsPerStep = 8;  // direct loads per wavefront per step (4 of X, 4 of W1)

__device__ __forceinline__ float activation(float h, int act) {
  if (act == DODO_ACT_RELU) return fmaxf(h, 0.f);
  if (act == DODO_ACT_GELU) return 0.5f * h * (1.f + erff(h * 0.70710678118654752440f));
  return tanhf(h);
}

__global__ __launch_bounds__(kMlpThreads, 1) void score_mlp_mfma_kernel(
    const uint16_t* __restrict__ X, const uint16_t* __restrict__ W1, const float* __restrict__ b1,
    const uint16_t* __restrict__ w2, float b2, int act, int64_t N, int d, int d_hid, int64_t row_stride, int hsplit,
    float* __restrict__ out) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const uint32_t lds_base = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_void*)lds));
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int lane = tid % kWave;
  const int j32 = lane & 31, g = lane >> 5;
  const int tg = wave >> 1, hg = wave & 1;  // token group (64 tokens) and hidden group (128 units) of this wavefront

  // Workgroup -> (token tile, split).  Block i runs on XCD i % 8, and the workgroups resident on one XCD at a time
  // are consecutive slots i / 8: these cover a few token tiles times all the splits, so that their X panels and
  // W1 panels are shared through that XCD's L2 instead of every workgroup streaming panels of its own.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int split = slot % hsplit;
  const int64_t tok_tile = static_cast<int64_t>(slot / hsplit) * 8 + xcd;
  const int64_t tok0 = tok_tile * kTokTile;
  if (tok0 >= N) return;  // the grid is rounded up to whole groups of 8 token tiles
  const int tiles_total = d_hid / kHidTile;
  const int tiles_per_split = (tiles_total + hsplit - 1) / hsplit;
  const int tile0 = split * tiles_per_split;
  const int n_tiles = max(0, min(tiles_per_split, tiles_total - tile0));
  const int ksteps = d / kBK;
  const int n_steps = n_tiles * ksteps;

  // ---- loader: per step, wavefront w brings rows 32w .. 32w+31 of the X tile and of the W1 tile, 8 rows of 128
  // bytes (1 KiB, whole cache lines) per instruction; lane i sits at (row i/8, position i%8) and fetches the piece
  // that the swizzle stores there: piece = pos ^ ((row >> 1) & 7)
  const int l_row = lane >> 3, l_pos = lane & 7;
  uint32_t x_off[4], w_off[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int r = 32 * wave + 8 * u + l_row;
    const uint32_t piece_bytes = static_cast<uint32_t>((l_pos ^ ((r >> 1) & 7)) * 16);
    const int64_t tok = min(tok0 + r, N - 1);  // rows past the end re-read the last token; nothing of them is stored
    x_off[u] = static_cast<uint32_t>((tok - tok0) * row_stride * 2) + piece_bytes;
    w_off[u] = static_cast<uint32_t>(r) * static_cast<uint32_t>(d) * 2u + piece_bytes;
  }
  const uint16_t* x_base = X + tok0 * row_stride;
  auto issue_part = [&](int step, int q) {  // eighth q of a step's loads: (u = q / 2, operand = q % 2)
    const int st = min(step, n_steps - 1);  // past the end: re-read the last step into a stage nobody reads any more
    const int ht = tile0 + st / ksteps, ks = st % ksteps;
    const uint32_t stage = lds_base + (step % kStagesG) * kStageBytesG;
    const int u = q >> 1;
    if ((q & 1) == 0) {
      dma16_uniform(x_base + ks * kBK, x_off[u], __builtin_amdgcn_readfirstlane(stage + (32 * wave + 8 * u) * 128));
    } else {
      dma16_uniform(W1 + static_cast<int64_t>(ht) * kHidTile * d + ks * kBK, w_off[u],
            __builtin_amdgcn_readfirstlane(stage + kOperandBytes + (32 * wave + 8 * u) * 128));
    }
  };
  auto issue_step = [&](int step) {
#pragma unroll
    for (int q = 0; q < 8; ++q) issue_part(step, q);
  };

  // ---- fragment addresses: row r of a tile at r*128, piece p at (p ^ ((r >> 1) & 7)) * 16
  const int f_sw = (j32 >> 1) & 7;
  const int x_row_off = (64 * tg + j32) * 128;                    // token blocks tb = 0, 1: + 32*128*tb
  const int w_row_off = kOperandBytes + (128 * hg + j32) * 128;   // hidden blocks hb = 0..3: + 32*128*hb

  floatx16 acc[4][2];
  float part[2] = {0.f, 0.f};  // partial scores of tokens 64 tg + 32 tb + j32 (this lane's half of the hidden units)
  auto zero_acc = [&]() {
#pragma unroll
    for (int hb = 0; hb < 4; ++hb)
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[hb][tb][v] = 0.f;
  };
  zero_acc();

  bf16x8 xf[2][2], wf[2][4];  // two fragment sets, used alternately by the four 16-channel parts of a step
  auto read_frags = [&](int step, int ks, bf16x8* xo, bf16x8* wo) {
    const char* stg = lds + (step % kStagesG) * kStageBytesG;
    const int piece = ((2 * ks + g) ^ f_sw) << 4;
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) xo[tb] = *reinterpret_cast<const bf16x8*>(stg + x_row_off + tb * 4096 + piece);
#pragma unroll
    for (int hb = 0; hb < 4; ++hb) wo[hb] = *reinterpret_cast<const bf16x8*>(stg + w_row_off + hb * 4096 + piece);
  };
  auto mfma_set = [&](int set) {
#pragma unroll
    for (int hb = 0; hb < 4; ++hb)
#pragma unroll
      for (int tb = 0; tb < 2; ++tb)
        acc[hb][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[set][hb], xf[set][tb], acc[hb][tb], 0, 0, 0);
  };
  if (n_steps > 0) {
    issue_step(0);
    issue_step(1);
    __builtin_amdgcn_s_waitcnt(0x0f70 | kLoadsPerStep);  // step 0 has landed
    __syncthreads();
    read_frags(0, 0, xf[0], wf[0]);
  }
  for (int step = 0; step < n_steps; ++step) {
    // parts 0..2: the next part's fragments are requested, then the matrix cores work on the current part's
    read_frags(step, 1, xf[1], wf[1]);
    mfma_set(0);
    read_frags(step, 2, xf[0], wf[0]);
    mfma_set(1);
    read_frags(step, 3, xf[1], wf[1]);
    mfma_set(0);
    // this wavefront has read everything it needs of this step's stage, and its part of the next step has landed;
    // after the barrier that holds for every wavefront
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
    __syncthreads();
    read_frags(step + 1, 0, xf[0], wf[0]);  // (after the last step: a stage that holds old data; not used)
#pragma unroll
    for (int hb = 0; hb < 4; ++hb) {
#pragma unroll
      for (int tb = 0; tb < 2; ++tb) {
        acc[hb][tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[1][hb], xf[1][tb], acc[hb][tb], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        issue_part(step + kStagesG, 2 * hb + tb);  // refill this step's stage
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if ((step + 1) % ksteps == 0) {
      // a hidden tile is complete: accumulator v of block hb is hidden unit 32 hb + 8 (v/4) + 4 g + v%4
      const int ht = tile0 + step / ksteps;
      const int jbase = ht * kHidTile + 128 * hg + 4 * g;
#pragma unroll
      for (int hb = 0; hb < 4; ++hb)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          const int jj = jbase + 32 * hb + 8 * vq;
          const float4 bb = *reinterpret_cast<const float4*>(b1 + jj);
          const uint2 ww = *reinterpret_cast<const uint2*>(w2 + jj);
          const float wv[4] = {bf16_lo(ww.x), bf16_hi(ww.x), bf16_lo(ww.y), bf16_hi(ww.y)};
          const float bv[4] = {bb.x, bb.y, bb.z, bb.w};
#pragma unroll
          for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int e = 0; e < 4; ++e)
              part[tb] = fmaf(wv[e], activation(acc[hb][tb][4 * vq + e] + bv[e], act), part[tb]);
        }
      zero_acc();
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0f70);  // drain the look-ahead loads
  __syncthreads();                     // (the stages are about to be reused as a reduction buffer)

  // ---- the two halves of a token's hidden units sit in lanes j32 and j32 + 32; the two hidden groups in two
  // wavefronts: added in a fixed order through LDS
  float* red = reinterpret_cast<float*>(lds);  // [2 hidden groups][256 tokens]
#pragma unroll
  for (int tb = 0; tb < 2; ++tb) {
    const float both = part[tb] + __shfl_xor(part[tb], 32, kWave);
    if (g == 0) red[hg * kTokTile + 64 * tg + 32 * tb + j32] = both;
  }
  __syncthreads();
  if (tid < kTokTile) {
    const int64_t tok = tok0 + tid;
    if (tok < N) {
      float s = red[tid] + red[kTokTile + tid];
      if (hsplit == 1) {
        s += b2;
        out[tok] = (s == 0.f) ? 0.f : s;
      } else {
        out[static_cast<int64_t>(split) * N + tok] = s;
      }
    }
  }
}

// partial scores of the splits, added in split order, plus the output bias
__global__ void score_mlp_combine_kernel(const float* __restrict__ partial, int hsplit, int64_t N, float b2,
                                         float* __restrict__ scores) {
  const int64_t t = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (t >= N) return;
  float s = 0.f;
  for (int p = 0; p < hsplit; ++p) s += partial[static_cast<int64_t>(p) * N + t];
  s += b2;
  scores[t] = (s == 0.f) ? 0.f : s;
}

// ---- plain kernel: `kTok` token rows in LDS, one hidden unit per wavefront at a time
constexpr int kPlainThreads = 256;
template <int DTYPE>
__global__ __launch_bounds__(kPlainThreads) void score_mlp_plain_kernel(
    const void* __restrict__ X, const void* __restrict__ W1, const float* __restrict__ b1, const void* __restrict__ w2,
    float b2, int act, int64_t N, int d, int d_hid, int64_t row_stride, int tok_per_wg, float* __restrict__ scores) {
  extern __shared__ float xs[];  // [tok_per_wg][d] as fp32, then [waves][tok_per_wg] partial sums
  constexpr int kWaves = kPlainThreads / kWave;
  const int64_t tok0 = static_cast<int64_t>(blockIdx.x) * tok_per_wg;
  const int nt = static_cast<int>(min<int64_t>(tok_per_wg, N - tok0));
  for (int i = threadIdx.x; i < nt * d; i += kPlainThreads)
    xs[i] = load_elem<DTYPE>(X, (tok0 + i / d) * row_stride + i % d);
  __syncthreads();
  const int wave = threadIdx.x / kWave, lane = lane_id();
  float* red = xs + static_cast<size_t>(tok_per_wg) * d;
  for (int t = 0; t < nt; ++t) {
    float a = 0.f;
    for (int j = wave; j < d_hid; j += kWaves) {
      float h = 0.f;
      for (int c = lane; c < d; c += kWave) h = fmaf(load_elem<DTYPE>(W1, static_cast<int64_t>(j) * d + c), xs[t * d + c], h);
#pragma unroll
      for (int off = kWave / 2; off >= 1; off >>= 1) h += __shfl_xor(h, off, kWave);
      a = fmaf(load_elem<DTYPE>(w2, j), activation(h + b1[j], act), a);
    }
    if (lane == 0) red[wave * tok_per_wg + t] = a;
  }
  __syncthreads();
  if (threadIdx.x < nt) {
    float s = 0.f;
    for (int w = 0; w < kWaves; ++w) s += red[w * tok_per_wg + threadIdx.x];
    s += b2;
    scores[tok0 + threadIdx.x] = (s == 0.f) ? 0.f : s;
  }
}

bool mfma_path(int dtype, int64_t N, int32_t d, int32_t d_hid, int64_t row_stride, const void* X, const void* W1,
               const void* b1, const void* w2) {
  return dtype == DODO_DTYPE_BF16 && d % kBK == 0 && d_hid % kHidTile == 0 && row_stride % 8 == 0 && aligned16(X) &&
         aligned16(W1) && aligned16(b1) && (reinterpret_cast<uintptr_t>(w2) % 8 == 0) &&
         static_cast<int64_t>(kHidTile) * d * 2 < 0x7fffffffLL && static_cast<int64_t>(kTokTile) * row_stride * 2 < 0x7fffffffLL;
}

int hidden_splits(int64_t N, int32_t d_hid) {
  const int64_t blocks = (N + kTokTile - 1) / kTokTile;
  const int tiles = d_hid / kHidTile;
  // at least 4 splits (when there are that many tiles) so that an XCD's resident workgroups form a 2-D patch of
  // the (token tile, hidden tile) plane; more while the grid does not fill the chip
  int hs = 1;
  while (hs * 2 <= tiles && (hs < 4 || blocks * hs < compute_units())) hs *= 2;
  return hs;
}

}  // namespace
}  // namespace dodo

extern "C" size_t dodo_score_mlp_workspace_bytes(int dtype, int64_t N, int32_t d, int32_t d_hid) {
  using namespace dodo;
  if (N <= 0 || d <= 0 || d_hid <= 0) return 0;
  if (dtype != DODO_DTYPE_BF16 || d % kBK != 0 || d_hid % kHidTile != 0) return 0;
  const int hs = hidden_splits(N, d_hid);
  return hs > 1 ? static_cast<size_t>(hs) * N * sizeof(float) : 0;
}

extern "C" int dodo_score_mlp(const void* hidden, const void* W1, const float* b1, const void* w2, float b2, int act,
                              int dtype, int64_t N, int32_t d, int32_t d_hid, int64_t row_stride, float* scores,
                              void* ws, size_t ws_bytes, void* stream) {
  using namespace dodo;
  if (N < 0 || d <= 0 || d_hid <= 0 || row_stride < d) return DODO_ERR_INVALID_ARG;
  if (act != DODO_ACT_RELU && act != DODO_ACT_GELU && act != DODO_ACT_TANH) return DODO_ERR_INVALID_ARG;
  if (N == 0) return DODO_OK;
  if (!hidden || !W1 || !b1 || !w2 || !scores) return DODO_ERR_INVALID_ARG;
  if (!dtype_ok(dtype)) return DODO_ERR_UNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (mfma_path(dtype, N, d, d_hid, row_stride, hidden, W1, b1, w2)) {
    const int hs = hidden_splits(N, d_hid);
    const size_t need = hs > 1 ? static_cast<size_t>(hs) * N * sizeof(float) : 0;
    if (need > 0 && (!ws || ws_bytes < need)) return DODO_ERR_WORKSPACE_TOO_SMALL;
    const int64_t blocks = ((N + kTokTile - 1) / kTokTile + 7) / 8 * 8 * hs;
    if (blocks > 0x7fffffffLL) return DODO_ERR_UNSUPPORTED;
    constexpr int kLds = kStagesG * kStageBytesG;
    {
      const int rc_lds = allow_dynamic_lds(reinterpret_cast<const void*>(score_mlp_mfma_kernel), kLds);
      if (rc_lds != DODO_OK) return rc_lds;
    }
    hipLaunchKernelGGL(score_mlp_mfma_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kMlpThreads), kLds, s,
                       static_cast<const uint16_t*>(hidden), static_cast<const uint16_t*>(W1), b1,
                       static_cast<const uint16_t*>(w2), b2, act, N, d, d_hid, row_stride, hs,
                       hs > 1 ? static_cast<float*>(ws) : scores);
    int rc = launch_status();
    if (rc != DODO_OK || hs == 1) return rc;
    hipLaunchKernelGGL(score_mlp_combine_kernel, dim3(static_cast<unsigned>((N + 255) / 256)), dim3(256), 0, s,
                       static_cast<const float*>(ws), hs, N, b2, scores);
    return launch_status();
  }
  // plain kernel: as many token rows per workgroup as fit in 128 KiB of LDS (at most 8)
  const int64_t row_bytes = static_cast<int64_t>(d) * 4;
  int tok = static_cast<int>(128 * 1024 / row_bytes);
  if (tok < 1) return DODO_ERR_UNSUPPORTED;  // d > 32768
  if (tok > 8) tok = 8;
  const size_t lds = static_cast<size_t>(tok) * d * 4 + (kPlainThreads / kWave) * tok * 4;
  const int64_t blocks = (N + tok - 1) / tok;
  if (blocks > 0x7fffffffLL) return DODO_ERR_UNSUPPORTED;
  if (dtype == DODO_DTYPE_BF16) {
    {
      const int rc_lds = allow_dynamic_lds(reinterpret_cast<const void*>(score_mlp_plain_kernel<DODO_DTYPE_BF16>), static_cast<int>(lds));
      if (rc_lds != DODO_OK) return rc_lds;
    }
    hipLaunchKernelGGL(score_mlp_plain_kernel<DODO_DTYPE_BF16>, dim3(static_cast<unsigned>(blocks)), dim3(kPlainThreads),
                       lds, s, hidden, W1, b1, w2, b2, act, N, d, d_hid, row_stride, tok, scores);
  } else {
    {
      const int rc_lds = allow_dynamic_lds(reinterpret_cast<const void*>(score_mlp_plain_kernel<DODO_DTYPE_F32>), static_cast<int>(lds));
      if (rc_lds != DODO_OK) return rc_lds;
    }
    hipLaunchKernelGGL(score_mlp_plain_kernel<DODO_DTYPE_F32>, dim3(static_cast<unsigned>(blocks)), dim3(kPlainThreads),
                       lds, s, hidden, W1, b1, w2, b2, act, N, d, d_hid, row_stride, tok, scores);
  }
  return launch_status();
}
