// Dodo hot-path oracle: TEST INFRASTRUCTURE, not product code.
//
// A plain, single-threaded, double-precision CPU statement of what the Dodo
// compression path computes (arXiv 2310.02409): count -> Scorer -> TopK ->
// sub-selection of K/V -> attention over [nuggets ; local tokens].  Every
// function is the definition written out: no tiling, no online softmax, no
// radix tricks, no threads.  It shares no code, header or constant with the
// HIP library and must never be imported by it; only the tests, the smoke
// check and the benchmark's cpu_baseline leg may load it.
//
// Element types: 0 = IEEE fp32, 1 = bfloat16 stored as uint16 (upper half of
// an fp32).  Both widen to double exactly.
//
// Pins (see tests/test_oracle_*.py): every function below is pinned by closed
// forms, brute force and library cross-checks; none is "parity unpinned".
// sanitize_main.cpp runs all of them under AddressSanitizer and
// UndefinedBehaviorSanitizer (tests/test_sanitizers.py).
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <vector>

namespace {

constexpr int kF32 = 0;
constexpr int kBF16 = 1;
constexpr uint32_t kForceLast = 1u;
constexpr int kTokenMajor = 0;  // cache[token][head][channel]
constexpr int kHeadMajor = 1;   // cache[head][token][channel]

inline size_t elem_size(int dtype) { return dtype == kF32 ? 4 : 2; }

inline double load(const void* base, int dtype, int64_t i) {
  if (dtype == kF32) {
    return static_cast<double>(static_cast<const float*>(base)[i]);
  }
  uint32_t bits = static_cast<uint32_t>(static_cast<const uint16_t*>(base)[i]) << 16;
  float f;
  std::memcpy(&f, &bits, 4);
  return static_cast<double>(f);
}

// Rounds a double to the storage type (round to nearest even, once) and stores it.
inline void store(void* base, int dtype, int64_t i, double v) {
  const float f = static_cast<float>(v);
  if (dtype == kF32) {
    static_cast<float*>(base)[i] = f;
    return;
  }
  // double -> bf16 in one rounding: round the double's value at bf16 precision directly
  uint32_t bits;
  std::memcpy(&bits, &f, 4);
  if (std::isnan(v)) {
    static_cast<uint16_t*>(base)[i] = 0x7fc0;
    return;
  }
  // candidates: f truncated to bf16 and its neighbour away from zero; pick the nearer to v (ties to even)
  uint32_t lo = bits & 0xffff0000u;
  float flo;
  std::memcpy(&flo, &lo, 4);
  if (static_cast<double>(flo) == v) {
    static_cast<uint16_t*>(base)[i] = static_cast<uint16_t>(lo >> 16);
    return;
  }
  // f may itself have been rounded from v; compare against v, not f, using both bf16 neighbours of v
  const double av = std::fabs(v);
  uint32_t mag = lo & 0x7fff0000u;
  float fm;
  std::memcpy(&fm, &mag, 4);
  if (static_cast<double>(fm) > av) {  // rounding to float went up past a bf16 value: step down
    mag -= 0x10000u;
    std::memcpy(&fm, &mag, 4);
  }
  uint32_t up = mag + 0x10000u;
  float fu;
  std::memcpy(&fu, &up, 4);
  const double dl = av - static_cast<double>(fm), du = static_cast<double>(fu) - av;
  uint32_t pick = (dl < du) ? mag : (du < dl) ? up : ((mag >> 16) & 1u) ? up : mag;
  static_cast<uint16_t*>(base)[i] = static_cast<uint16_t>((pick | (lo & 0x80000000u)) >> 16);
}

// "a has a strictly higher score than b" with NaN placed below everything.
inline bool higher(float a, float b) {
  if (std::isnan(a)) return false;
  if (std::isnan(b)) return true;
  return a > b;  // -0.0f == +0.0f here, as required
}

struct AttnArgs {
  const void *Q, *Kn, *Vn, *Kl, *Vl;
  const int32_t *cu_q, *cu_nug, *cu_local;
  int32_t H, H_kv, d_h;
  double scale;
  int dtype, layout;
  int64_t Kt;  // total nugget rows (needed for the head-major cache)
};

inline int64_t cache_off(const AttnArgs& a, int64_t tok, int32_t kvh) {
  if (a.layout == kTokenMajor) return (tok * a.H_kv + kvh) * a.d_h;
  return (static_cast<int64_t>(kvh) * a.Kt + tok) * a.d_h;
}

// One query row of Eq. 13 (compressor mode) / Eq. 9 (mixed resolution):
// softmax over every nugget of the sequence followed by the local rows the
// causal rule admits, then the weighted mean of the matching V rows.
void attention_row(const AttnArgs& a, int32_t b, int32_t h, int32_t i, double* o, double* lse) {
  const int32_t dh = a.d_h;
  const int32_t kvh = h / (a.H / a.H_kv);
  const int64_t q_b = a.cu_q[b + 1] - a.cu_q[b];
  const int64_t k_b = a.cu_nug[b + 1] - a.cu_nug[b];
  const int64_t m_b = a.cu_local[b + 1] - a.cu_local[b];
  // bottom-right aligned causal rule: local row j is visible iff j <= m_b - q_b + i
  int64_t n_local = m_b - q_b + i + 1;
  if (n_local < 0) n_local = 0;
  if (n_local > m_b) n_local = m_b;
  const int64_t n_vis = k_b + n_local;
  for (int32_t c = 0; c < dh; ++c) o[c] = 0.0;
  if (n_vis == 0) {
    *lse = -std::numeric_limits<double>::infinity();
    return;
  }
  const int64_t qoff = ((a.cu_q[b] + static_cast<int64_t>(i)) * a.H + h) * dh;
  std::vector<double> logit(n_vis);
  std::vector<int64_t> koff(n_vis);
  std::vector<char> from_local(n_vis);
  for (int64_t j = 0; j < n_vis; ++j) {
    if (j < k_b) {
      koff[j] = cache_off(a, a.cu_nug[b] + j, kvh);
      from_local[j] = 0;
    } else {
      koff[j] = ((a.cu_local[b] + (j - k_b)) * a.H_kv + kvh) * dh;
      from_local[j] = 1;
    }
    const void* kbase = from_local[j] ? a.Kl : a.Kn;
    double dot = 0.0;
    for (int32_t c = 0; c < dh; ++c) dot += load(a.Q, a.dtype, qoff + c) * load(kbase, a.dtype, koff[j] + c);
    logit[j] = a.scale * dot;
  }
  double M = logit[0];
  for (int64_t j = 1; j < n_vis; ++j) M = std::max(M, logit[j]);
  double denom = 0.0;
  for (int64_t j = 0; j < n_vis; ++j) {
    const double p = std::exp(logit[j] - M);
    denom += p;
    const void* vbase = from_local[j] ? a.Vl : a.Vn;
    for (int32_t c = 0; c < dh; ++c) o[c] += p * load(vbase, a.dtype, koff[j] + c);
  }
  for (int32_t c = 0; c < dh; ++c) o[c] /= denom;
  *lse = M + std::log(denom);
}

}  // namespace

extern "C" {

// Nugget count for a context of n tokens at keep-fraction num/den, i.e. the
// paper's k = ceil(n / r) with r = den/num (Sec. 2.3), clamped to 1 <= k <= n
// (Eq. 7).  Integer arithmetic throughout.
int64_t oracle_nugget_count(int64_t n, int64_t num, int64_t den) {
  if (n <= 0) return 0;
  int64_t k = (n * num + den - 1) / den;
  if (k < 1) k = 1;
  if (k > n) k = n;
  return k;
}

// Scorer as a linear head (Eq. 6 / Eq. 15): s[t] = sum_c x[t,c] * w[c] + bias,
// summed left to right in double, rounded once to fp32; -0 is emitted as +0.
void oracle_score(const void* hidden, const void* w, float bias, int dtype, int64_t N, int64_t d,
                  int64_t row_stride, float* scores) {
  for (int64_t t = 0; t < N; ++t) {
    double acc = 0.0;
    for (int64_t c = 0; c < d; ++c) acc += load(hidden, dtype, t * row_stride + c) * load(w, dtype, c);
    acc += static_cast<double>(bias);
    float s = static_cast<float>(acc);
    if (s == 0.0f) s = 0.0f;  // canonical zero
    scores[t] = s;
  }
}

// Scorer as the 2-layer feedforward network of the paper's appendix (Sec. 2.1, App. B: d -> d_hid -> 1,
// 16.8 M parameters for d = d_hid = 4096): s[t] = sum_j w2[j] * act(sum_c W1[j,c] x[t,c] + b1[j]) + b2,
// W1 row-major [d_hid, d].  The paper does not name the activation; act is 0 = ReLU, 1 = GELU
// (x Phi(x), erf form), 2 = tanh.  Sums left to right in double, one rounding to fp32, -0 emitted as +0.
void oracle_score_mlp(const void* hidden, const void* W1, const float* b1, const void* w2, float b2, int act,
                      int dtype, int64_t N, int64_t d, int64_t d_hid, int64_t row_stride, float* scores) {
  for (int64_t t = 0; t < N; ++t) {
    double acc = 0.0;
    for (int64_t j = 0; j < d_hid; ++j) {
      double h = 0.0;
      for (int64_t c = 0; c < d; ++c) h += load(W1, dtype, j * d + c) * load(hidden, dtype, t * row_stride + c);
      h += static_cast<double>(b1[j]);
      double a;
      if (act == 0) {
        a = h > 0.0 ? h : 0.0;
      } else if (act == 1) {
        a = 0.5 * h * (1.0 + std::erf(h * 0.70710678118654752440));
      } else {
        a = std::tanh(h);
      }
      acc += load(w2, dtype, j) * a;
    }
    acc += static_cast<double>(b2);
    float s = static_cast<float>(acc);
    if (s == 0.0f) s = 0.0f;
    scores[t] = s;
  }
}

// TopK selection (Eq. 14): per sequence, the k_b tokens with the highest score,
// ties won by the lower index, emitted in ascending position order.  With the
// force-last flag (footnote to Eq. 14) the final token of the sequence is
// always one of the k_b and the remaining k_b - 1 are chosen among the others.
// Returns 0, or -1 if some k_b exceeds its n_b.
int oracle_select_topk(const float* scores, const int32_t* cu_seqlens, const int32_t* cu_nuggets, int32_t B,
                       uint32_t flags, int32_t* nugget_idx) {
  for (int32_t b = 0; b < B; ++b) {
    const int64_t n = cu_seqlens[b + 1] - cu_seqlens[b];
    const int64_t k = cu_nuggets[b + 1] - cu_nuggets[b];
    if (k > n || k < 0) return -1;
    if (k == 0) continue;
    const float* s = scores + cu_seqlens[b];
    int32_t* out = nugget_idx + cu_nuggets[b];
    const bool force = (flags & kForceLast) != 0;
    const int64_t n_free = force ? n - 1 : n;  // tokens competing on score
    const int64_t k_free = force ? k - 1 : k;
    std::vector<int32_t> order(n_free);
    for (int64_t i = 0; i < n_free; ++i) order[i] = static_cast<int32_t>(i);
    // stable: equal scores keep ascending index order
    std::stable_sort(order.begin(), order.end(), [s](int32_t x, int32_t y) { return higher(s[x], s[y]); });
    std::vector<int32_t> chosen(order.begin(), order.begin() + k_free);
    if (force) chosen.push_back(static_cast<int32_t>(n - 1));
    std::sort(chosen.begin(), chosen.end());
    for (int64_t j = 0; j < k; ++j) out[j] = chosen[j];
  }
  return 0;
}

// Threshold selection (Eq. 8): alpha_i = 1{s_i > Lambda}; writes the flags and
// returns through counts[b] how many tokens each sequence keeps.
void oracle_select_threshold(const float* scores, const int32_t* cu_seqlens, int32_t B, float lambda,
                             uint8_t* alpha, int32_t* counts) {
  for (int32_t b = 0; b < B; ++b) {
    int32_t c = 0;
    for (int64_t t = cu_seqlens[b]; t < cu_seqlens[b + 1]; ++t) {
      alpha[t] = scores[t] > lambda ? 1 : 0;
      c += alpha[t];
    }
    counts[b] = c;
  }
}

// Threshold calibration (Sec. 2.4: the threshold is estimated by running the scorer on sampled
// tokens so that about t/r of t tokens are kept): with k = nugget count of the n sampled scores,
// Lambda is the (k+1)-th highest score of the sample, so that exactly k of them exceed it when there
// are no ties.  Score order is that of the selection rule (NaN lowest).  If k >= n, or the
// (k+1)-th highest is NaN, everything that can be kept is kept: Lambda = -inf.
float oracle_threshold_from_sample(const float* sample, int64_t n, int64_t num, int64_t den) {
  const int64_t k = oracle_nugget_count(n, num, den);
  if (k >= n) return -std::numeric_limits<float>::infinity();
  std::vector<float> v(sample, sample + n);
  std::stable_sort(v.begin(), v.end(), [](float a, float b) { return higher(a, b); });
  const float lam = v[k];
  if (std::isnan(lam)) return -std::numeric_limits<float>::infinity();
  return lam == 0.0f ? 0.0f : lam;  // canonical zero
}

// Threshold selection as index lists: the kept tokens of every sequence in ascending position
// order, packed (sequence b at cu_nuggets_out[b] ...), with the counts and their running sum.
void oracle_select_threshold_indices(const float* scores, const int32_t* cu_seqlens, int32_t B, float lambda,
                                     int32_t* counts, int32_t* cu_nuggets_out, int32_t* nugget_idx) {
  cu_nuggets_out[0] = 0;
  for (int32_t b = 0; b < B; ++b) {
    int32_t c = 0;
    for (int64_t t = cu_seqlens[b]; t < cu_seqlens[b + 1]; ++t)
      if (scores[t] > lambda) nugget_idx[cu_nuggets_out[b] + c++] = static_cast<int32_t>(t - cu_seqlens[b]);
    counts[b] = c;
    cu_nuggets_out[b + 1] = cu_nuggets_out[b] + c;
  }
}

// One step of the autoregressive mode (Sec. 2.4 with the mixed resolution of Eq. 9): in every
// sequence one token leaves the window of uncompressed tokens; if its score exceeds Lambda its K and
// V rows are appended to that sequence's nugget cache (capacity `cap` rows per sequence, caches
// token-major [B, cap, H_kv, d_h]); a full cache drops the token and reports it through the return
// value (number of dropped tokens).  counts[b] is updated.
int32_t oracle_stream_append(const float* scores, float lambda, const void* K_rows, const void* V_rows, int dtype,
                             int32_t B, int32_t H_kv, int32_t d_h, int64_t row_stride, int32_t cap, int32_t* counts,
                             void* Kn, void* Vn) {
  const size_t es = elem_size(dtype);
  const size_t row_bytes = static_cast<size_t>(H_kv) * d_h * es;
  int32_t dropped = 0;
  for (int32_t b = 0; b < B; ++b) {
    if (!(scores[b] > lambda)) continue;
    if (counts[b] >= cap) {
      ++dropped;
      continue;
    }
    const size_t dst = (static_cast<size_t>(b) * cap + counts[b]) * row_bytes;
    const size_t src = static_cast<size_t>(b) * row_stride * es;
    std::memcpy(static_cast<char*>(Kn) + dst, static_cast<const char*>(K_rows) + src, row_bytes);
    std::memcpy(static_cast<char*>(Vn) + dst, static_cast<const char*>(V_rows) + src, row_bytes);
    ++counts[b];
  }
  return dropped;
}

// Compaction of the pooling baseline the paper compares with (Sec. 5.1: the text is chunked evenly
// into segments and each segment's states are mean-pooled into one vector, at the same compression
// ratio): sequence b of n_b tokens becomes k_b = cu_nuggets[b+1] - cu_nuggets[b] rows, row j being the
// mean of tokens floor(j n_b / k_b) .. floor((j+1) n_b / k_b) - 1, summed in double and rounded once.
void oracle_meanpool(const void* K, const void* V, int dtype, const int32_t* cu_seqlens, const int32_t* cu_nuggets,
                     int32_t B, int64_t Kt, int32_t H_kv, int32_t d_h, int64_t token_stride, void* Kn, void* Vn,
                     int layout) {
  for (int32_t b = 0; b < B; ++b) {
    const int64_t n = cu_seqlens[b + 1] - cu_seqlens[b];
    const int64_t k = cu_nuggets[b + 1] - cu_nuggets[b];
    for (int64_t j = 0; j < k; ++j) {
      const int64_t t0 = j * n / k, t1 = (j + 1) * n / k;
      const int64_t dst_tok = cu_nuggets[b] + j;
      for (int32_t h = 0; h < H_kv; ++h)
        for (int32_t c = 0; c < d_h; ++c) {
          double sk = 0.0, sv = 0.0;
          for (int64_t t = t0; t < t1; ++t) {
            const int64_t src = (cu_seqlens[b] + t) * token_stride + static_cast<int64_t>(h) * d_h + c;
            sk += load(K, dtype, src);
            sv += load(V, dtype, src);
          }
          const double inv = t1 > t0 ? 1.0 / static_cast<double>(t1 - t0) : 0.0;
          const int64_t dst = (layout == kTokenMajor) ? (dst_tok * H_kv + h) * d_h + c
                                                      : (static_cast<int64_t>(h) * Kt + dst_tok) * d_h + c;
          store(Kn, dtype, dst, sk * inv);
          store(Vn, dtype, dst, sv * inv);
        }
    }
  }
}

// Sub-selection (Eq. 5): nuggets are the chosen tokens' own K and V rows,
// copied bit for bit into the compact cache.
void oracle_gather(const void* K, const void* V, int dtype, const int32_t* nugget_idx, const int32_t* cu_seqlens,
                   const int32_t* cu_nuggets, int32_t B, int64_t Kt, int32_t H_kv, int32_t d_h,
                   int64_t token_stride, void* Kn, void* Vn, int layout) {
  const size_t es = elem_size(dtype);
  const size_t head_bytes = static_cast<size_t>(d_h) * es;
  for (int32_t b = 0; b < B; ++b) {
    const int64_t k = cu_nuggets[b + 1] - cu_nuggets[b];
    for (int64_t j = 0; j < k; ++j) {
      const int64_t src_tok = cu_seqlens[b] + nugget_idx[cu_nuggets[b] + j];
      const int64_t dst_tok = cu_nuggets[b] + j;
      for (int32_t h = 0; h < H_kv; ++h) {
        const size_t src = (static_cast<size_t>(src_tok) * token_stride + static_cast<size_t>(h) * d_h) * es;
        const size_t dst = (layout == kTokenMajor)
                               ? (static_cast<size_t>(dst_tok) * H_kv + h) * head_bytes
                               : (static_cast<size_t>(h) * Kt + dst_tok) * head_bytes;
        std::memcpy(static_cast<char*>(Kn) + dst, static_cast<const char*>(K) + src, head_bytes);
        std::memcpy(static_cast<char*>(Vn) + dst, static_cast<const char*>(V) + src, head_bytes);
      }
    }
  }
}

// Nugget attention for every query row of every sequence and head.
// O is [sum q_b, H, d_h] in double, lse is [sum q_b, H] in double.
void oracle_attention(const void* Q, const void* Kn, const void* Vn, const void* Kl, const void* Vl,
                      const int32_t* cu_q, const int32_t* cu_nuggets, const int32_t* cu_local, int32_t B, int32_t H,
                      int32_t H_kv, int32_t d_h, double scale, int dtype, int layout, int64_t Kt, double* O,
                      double* lse) {
  AttnArgs a{Q, Kn, Vn, Kl, Vl, cu_q, cu_nuggets, cu_local, H, H_kv, d_h, scale, dtype, layout, Kt};
  for (int32_t b = 0; b < B; ++b) {
    const int32_t q_b = cu_q[b + 1] - cu_q[b];
    for (int32_t i = 0; i < q_b; ++i) {
      for (int32_t h = 0; h < H; ++h) {
        const int64_t row = (static_cast<int64_t>(cu_q[b]) + i) * H + h;
        attention_row(a, b, h, i, O + row * d_h, lse + row);
      }
    }
  }
}

// The same definition for a list of sampled (sequence, head, query row)
// triples; O_rows is [nrows, d_h], lse_rows is [nrows].
void oracle_attention_rows(const void* Q, const void* Kn, const void* Vn, const void* Kl, const void* Vl,
                           const int32_t* cu_q, const int32_t* cu_nuggets, const int32_t* cu_local, int32_t H,
                           int32_t H_kv, int32_t d_h, double scale, int dtype, int layout, int64_t Kt,
                           int64_t nrows, const int32_t* row_b, const int32_t* row_h, const int32_t* row_i,
                           double* O_rows, double* lse_rows) {
  AttnArgs a{Q, Kn, Vn, Kl, Vl, cu_q, cu_nuggets, cu_local, H, H_kv, d_h, scale, dtype, layout, Kt};
  for (int64_t r = 0; r < nrows; ++r) attention_row(a, row_b[r], row_h[r], row_i[r], O_rows + r * d_h, lse_rows + r);
}

// Segment form of the autoregressive objective (Sec. 2.4, "Learning"): text b is cut into segments of seg_len
// tokens, and the tokens of segment c share the splitting index t = max(0, c * seg_len - tau).  One entry per
// segment, texts in order, segments in order: its first query row, the text's nugget range start, how many of
// the text's nuggets have an index below t, the first uncompressed token it sees and how many it sees up to
// its own end.  Returns the number of entries; arrays hold `capacity` entries (seg_cu_q one more).
int64_t oracle_segment_plan(const int32_t* nugget_idx, const int32_t* cu_seqlens, const int32_t* cu_nuggets, int32_t B,
                            int32_t seg_len, int32_t tau, int64_t capacity, int32_t* seg_cu_q, int32_t* nug_start,
                            int32_t* nug_len, int32_t* loc_start, int32_t* loc_len) {
  int64_t e = 0;
  for (int32_t b = 0; b < B; ++b) {
    const int32_t s0 = cu_seqlens[b], n = cu_seqlens[b + 1] - cu_seqlens[b];
    const int32_t k0 = cu_nuggets[b], k = cu_nuggets[b + 1] - cu_nuggets[b];
    for (int32_t c = 0; static_cast<int64_t>(c) * seg_len < n; ++c) {
      const int32_t start = c * seg_len;
      const int32_t t = std::max(0, start - tau);
      int32_t below = 0;
      for (int32_t j = 0; j < k; ++j) below += nugget_idx[k0 + j] < t ? 1 : 0;
      if (e < capacity) {
        seg_cu_q[e] = s0 + start;
        nug_start[e] = k0;
        nug_len[e] = below;
        loc_start[e] = s0 + t;
        loc_len[e] = std::min(start + seg_len, n) - t;
      }
      ++e;
    }
  }
  if (e <= capacity) seg_cu_q[e] = cu_seqlens[B];
  return e;
}

// Attention under that objective, one query token at a time (Eq. 9 with the splitting index shared by a
// segment): token i of a text, with t = max(0, (i / seg_len) * seg_len - tau), attends over the text's nuggets
// whose index is below t (rows of the packed token-major Kn / Vn) followed by the text's own tokens t .. i
// (rows of K / V).  Q, O: [N, H, d_h]; K, V: [N, H_kv, d_h]; O and lse in double.
void oracle_attention_segment_mask(const void* Q, const void* Kn, const void* Vn, const void* K, const void* V,
                                   const int32_t* nugget_idx, const int32_t* cu_seqlens, const int32_t* cu_nuggets,
                                   int32_t B, int32_t H, int32_t H_kv, int32_t d_h, int32_t seg_len, int32_t tau,
                                   double scale, int dtype, double* O, double* lse) {
  for (int32_t b = 0; b < B; ++b) {
    const int64_t s0 = cu_seqlens[b], n = cu_seqlens[b + 1] - cu_seqlens[b];
    const int64_t k0 = cu_nuggets[b], k = cu_nuggets[b + 1] - cu_nuggets[b];
    for (int64_t i = 0; i < n; ++i) {
      const int64_t t = std::max<int64_t>(0, (i / seg_len) * seg_len - tau);
      for (int32_t h = 0; h < H; ++h) {
        const int32_t kvh = h / (H / H_kv);
        const int64_t qoff = ((s0 + i) * H + h) * d_h;
        std::vector<double> logit;
        std::vector<int64_t> off;      // element offset of the key / value row
        std::vector<char> is_nugget;
        for (int64_t j = 0; j < k; ++j) {
          if (nugget_idx[k0 + j] < t) {
            off.push_back(((k0 + j) * H_kv + kvh) * d_h);
            is_nugget.push_back(1);
          }
        }
        for (int64_t u = t; u <= i; ++u) {
          off.push_back(((s0 + u) * H_kv + kvh) * d_h);
          is_nugget.push_back(0);
        }
        const size_t n_vis = off.size();  // never empty: token i sees itself
        logit.resize(n_vis);
        for (size_t j = 0; j < n_vis; ++j) {
          const void* kb = is_nugget[j] ? Kn : K;
          double dot = 0.0;
          for (int32_t c = 0; c < d_h; ++c) dot += load(Q, dtype, qoff + c) * load(kb, dtype, off[j] + c);
          logit[j] = scale * dot;
        }
        double M = logit[0];
        for (size_t j = 1; j < n_vis; ++j) M = std::max(M, logit[j]);
        double* o = O + qoff;
        for (int32_t c = 0; c < d_h; ++c) o[c] = 0.0;
        double denom = 0.0;
        for (size_t j = 0; j < n_vis; ++j) {
          const double p = std::exp(logit[j] - M);
          denom += p;
          const void* vb = is_nugget[j] ? Vn : V;
          for (int32_t c = 0; c < d_h; ++c) o[c] += p * load(vb, dtype, off[j] + c);
        }
        for (int32_t c = 0; c < d_h; ++c) o[c] /= denom;
        lse[(s0 + i) * H + h] = M + std::log(denom);
      }
    }
  }
}

// Gradient that the straight-through estimator hands to the scores (Sec. 2.5, Eq. 17-18) for one layer:
//   grad[i] = grad_scale * sum over heads h and query rows j of dl/dxi[j, i],
// where xi[j, i] is the input of the softmax of query row j at nugget i and dl/dxi = P (dP - D), with P the
// attention weights of Eq. 13 / Eq. 9 over nuggets and the causally visible local rows, dP[j, i] = dO[j] . v_i
// and D[j] = dO[j] . O[j].  Token-major nugget cache; grad is double [Kt], overwritten.
void oracle_ste_score_grad(const void* Q, const void* Kn, const void* Vn, const void* Kl, const void* Vl,
                           const void* dO, const int32_t* cu_q, const int32_t* cu_nuggets, const int32_t* cu_local,
                           int32_t B, int32_t H, int32_t H_kv, int32_t d_h, double scale, double grad_scale, int dtype,
                           int64_t Kt, double* grad) {
  for (int64_t i = 0; i < Kt; ++i) grad[i] = 0.0;
  for (int32_t b = 0; b < B; ++b) {
    const int64_t q0 = cu_q[b], q_b = cu_q[b + 1] - cu_q[b];
    const int64_t k0 = cu_nuggets[b], k_b = cu_nuggets[b + 1] - cu_nuggets[b];
    const int64_t l0 = cu_local[b], m_b = cu_local[b + 1] - cu_local[b];
    if (k_b == 0) continue;
    for (int32_t h = 0; h < H; ++h) {
      const int32_t kvh = h / (H / H_kv);
      for (int64_t j = 0; j < q_b; ++j) {
        int64_t n_loc = m_b - q_b + j + 1;
        n_loc = std::max<int64_t>(0, std::min(n_loc, m_b));
        const int64_t n_vis = k_b + n_loc;
        const int64_t qoff = ((q0 + j) * H + h) * d_h;
        auto row_off = [&](int64_t r) { return r < k_b ? ((k0 + r) * H_kv + kvh) * d_h : ((l0 + r - k_b) * H_kv + kvh) * d_h; };
        std::vector<double> p(n_vis);
        double M = -std::numeric_limits<double>::infinity();
        for (int64_t r = 0; r < n_vis; ++r) {
          const void* kb = r < k_b ? Kn : Kl;
          double dot = 0.0;
          for (int32_t c = 0; c < d_h; ++c) dot += load(Q, dtype, qoff + c) * load(kb, dtype, row_off(r) + c);
          p[r] = scale * dot;
          M = std::max(M, p[r]);
        }
        double denom = 0.0;
        for (int64_t r = 0; r < n_vis; ++r) {
          p[r] = std::exp(p[r] - M);
          denom += p[r];
        }
        std::vector<double> o(d_h, 0.0);
        for (int64_t r = 0; r < n_vis; ++r) {
          p[r] /= denom;
          const void* vb = r < k_b ? Vn : Vl;
          for (int32_t c = 0; c < d_h; ++c) o[c] += p[r] * load(vb, dtype, row_off(r) + c);
        }
        double big_d = 0.0;
        for (int32_t c = 0; c < d_h; ++c) big_d += load(dO, dtype, qoff + c) * o[c];
        for (int64_t r = 0; r < k_b; ++r) {
          double d_p = 0.0;
          for (int32_t c = 0; c < d_h; ++c) d_p += load(dO, dtype, qoff + c) * load(Vn, dtype, row_off(r) + c);
          grad[k0 + r] += grad_scale * p[r] * (d_p - big_d);
        }
      }
    }
  }
}

}  // extern "C"
