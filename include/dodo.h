/*
 * dodo.h -- C ABI of the Dodo hot path on MI355X (gfx950).
 *
 * Dodo (arXiv 2310.02409) compresses a context of n tokens into k << n
 * "nuggets": a Scorer rates every token (Eq. 6 / Eq. 15), TopK keeps the k best
 * per sequence (Eq. 14), the chosen tokens' own hidden states -- for attention,
 * their K and V rows -- are kept at every layer (Eq. 5, Eq. 7), and later
 * tokens attend over [nuggets ; recent uncompressed tokens] (Eq. 9, Eq. 13).
 * The calls below are those four steps.
 *
 * Conventions shared by every call
 *  - All tensor pointers are DEVICE pointers owned by the caller; the library
 *    never allocates, frees or keeps them.  Inputs are const and must not
 *    alias outputs.  Workspaces are caller-owned device memory too.
 *  - Ragged batches are packed: sequence b owns rows cu[b] .. cu[b+1]-1 of a
 *    [total, ...] tensor; cu_* are DEVICE int32 arrays of B+1 non-decreasing
 *    entries starting at 0 (their contents are trusted, not validated).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls only enqueue work on it and return; they never synchronise.
 *  - Return value: DODO_OK or a negative DODO_ERR_* code.  Everything that can
 *    be checked without touching the device is checked first, so invalid
 *    arguments are rejected before any launch (and on hosts with no GPU).
 *  - Data pointers must be 16-byte aligned; row strides must keep rows
 *    16-byte aligned.
 */
#ifndef DODO_H_
#define DODO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DODO_VERSION 100 /* major*10000 + minor*100 + patch */

/* status codes */
#define DODO_OK 0
#define DODO_ERR_INVALID_ARG (-1)         /* null pointer, negative size, k > n, H % H_kv != 0, bad flag/layout */
#define DODO_ERR_UNSUPPORTED (-2)         /* dtype / head_dim / alignment outside the supported set */
#define DODO_ERR_WORKSPACE_TOO_SMALL (-3) /* ws_bytes below what the *_workspace_bytes query returns */
#define DODO_ERR_HIP (-4)                 /* a HIP runtime call failed (launch error, no device) */
#define DODO_ERR_SCRATCH_LIMIT (-5)       /* the problem needs more than the library's static scratch buffer holds */

/* element types of hidden states / Q / K / V (scores are always fp32) */
#define DODO_DTYPE_F32 0
#define DODO_DTYPE_BF16 1

/* dodo_select_topk flags */
#define DODO_TOPK_FORCE_LAST 1u /* the last token of each sequence is always selected (footnote to Eq. 14) */

/* nugget-cache layouts (local K/V, Q and O are always token-major) */
#define DODO_LAYOUT_TOKEN_MAJOR 0 /* [Kt, H_kv, d_h] */
#define DODO_LAYOUT_HEAD_MAJOR 1  /* [H_kv, Kt, d_h] */

/* Library version (DODO_VERSION of the build). Host only. */
int dodo_version(void);

/* Static, human-readable text for a status code; for DODO_ERR_HIP the text of
 * the most recent HIP error seen by the calling thread. Host only. */
const char* dodo_status_string(int status);

/*
 * Nugget count of an n-token context at keep-fraction num/den, i.e. the
 * paper's k = ceil(n / r) with compression ratio r = den/num (Sec. 2.3),
 * clamped to 1 <= k <= n (Eq. 7); 0 when n <= 0.  Pure host integer arithmetic:
 * callers build cu_nuggets with it, so no device read-back is ever needed.
 * Returns -1 if num <= 0 or den <= 0.
 */
int64_t dodo_nugget_count(int64_t n, int64_t num, int64_t den);

/*
 * Scorer as a linear head (Eq. 6 / Eq. 15): scores[t] = sum_c hidden[t,c]*w[c] + bias
 * for t in [0, N).  hidden is [N, d] with `row_stride` elements between rows
 * (>= d), w is [d], both of `dtype`; products and sums are fp32; scores is
 * fp32 [N], with -0 written as +0.  d must be a multiple of 8.  The result is
 * run-to-run deterministic.  N == 0 is a no-op.
 */
int dodo_score(const void* hidden, const void* w, float bias, int dtype, int64_t N, int32_t d, int64_t row_stride,
               float* scores, void* stream);

/*
 * The same Scorer for L layers in one launch (Eq. 6 / Eq. 15 per layer; for per-layer selection, where every
 * layer rates its own hidden states): layer l reads hidden + l * hidden_layer_stride ([N, d] with row_stride)
 * and w + l * w_layer_stride ([d]), adds biases[l] (device fp32 [L], or NULL for no bias) and writes
 * scores + l * scores_layer_stride (fp32 [N]).  Strides in elements; hidden_layer_stride a multiple of
 * 16 bytes; scores_layer_stride >= N; strides may be 0 (the layers share the tensor).  L == 0 is a no-op,
 * L <= 65535.  Bit for bit what L calls of dodo_score produce.
 */
int dodo_score_layers(const void* hidden, const void* w, const float* biases, int dtype, int32_t L, int64_t N, int32_t d,
                      int64_t row_stride, int64_t hidden_layer_stride, int64_t w_layer_stride,
                      int64_t scores_layer_stride, float* scores, void* stream);

/* activations of dodo_score_mlp */
#define DODO_ACT_RELU 0
#define DODO_ACT_GELU 1 /* x * Phi(x), erf form */
#define DODO_ACT_TANH 2

/* Bytes of device workspace dodo_score_mlp needs (may be 0). */
size_t dodo_score_mlp_workspace_bytes(int dtype, int64_t N, int32_t d, int32_t d_hid);

/*
 * Scorer as the 2-layer feedforward network of the paper's appendix (Sec. 2.1, App. B:
 * d -> d_hid -> 1; 16.8 M parameters for d = d_hid = 4096):
 *   scores[t] = sum_j w2[j] * act( sum_c W1[j,c] * hidden[t,c] + b1[j] ) + b2
 * hidden [N, d] (row_stride elements between rows), W1 [d_hid, d] row-major and w2 [d_hid] of
 * `dtype`; b1 [d_hid] fp32; scores fp32 [N], -0 written as +0.  The paper does not name the
 * activation: `act` is one of DODO_ACT_*.  bf16 inputs with d % 64 == 0 and d_hid % 256 == 0 run on
 * the matrix cores (products bf16 x bf16, sums fp32, the N x d_hid intermediate stays in registers);
 * everything else takes a plain kernel that is correct for any shape with d <= 32768 but slow for
 * large ones.  Run-to-run deterministic.  N == 0 is a no-op.
 */
int dodo_score_mlp(const void* hidden, const void* W1, const float* b1, const void* w2, float b2, int act,
                   int dtype, int64_t N, int32_t d, int32_t d_hid, int64_t row_stride, float* scores, void* ws,
                   size_t ws_bytes, void* stream);

/* Bytes of device workspace dodo_select_topk can use for B sequences of at most max_n tokens (0 for short
 * sequences).  With it, long sequences are split over several workgroups that exchange histograms and counts
 * through it; without it (NULL or too small) one workgroup per sequence does the same work, more slowly.
 * The workspace must be zero-filled before its first use; a call leaves it zero-filled (apart from the status
 * word), so it can be reused by the next call as it is.  It must not be shared by calls that may overlap in time.
 * The workgroups of a sequence wait for each other (bounded: about 0.1 s), so they must be able to run at the
 * same time; the form is only chosen when they fit the GPU together, but work from other streams that keeps
 * compute units busy for longer than the bound, or a workspace that was not zero-filled, makes a wait run out.
 * The first 32-bit word of the workspace is a STATUS WORD that tells: the library only ever sets bits in it
 * (DODO_SELECT_WAIT_FAILED = 1: a wait ran out in some call since the word was last cleared; the index lists of
 * the sequences concerned are invalid -- filled with the last token's index, which is safe to gather -- and must
 * not be used).  A caller that uses the workspace form reads the word after the stream has drained, whenever it
 * needs to know, and clears it itself; the rest of the workspace heals by itself (it is zero-filled again
 * when the failed call's last workgroup ends). */
#define DODO_SELECT_WAIT_FAILED 1u
size_t dodo_select_topk_workspace_bytes(int32_t B, int32_t max_n);

/*
 * TopK selection (Eq. 14).  For each sequence b, with n_b = cu_seqlens[b+1] -
 * cu_seqlens[b] and k_b = cu_nuggets[b+1] - cu_nuggets[b] (0 <= k_b <= n_b),
 * writes to nugget_idx[cu_nuggets[b] ..] the sequence-local indices of the k_b
 * tokens with the highest score, in ascending order.  Equal scores: the lower
 * index wins.  NaN ranks below -inf; -0 equals +0.  With DODO_TOPK_FORCE_LAST
 * token n_b-1 is always selected and the other k_b-1 are the best of the rest.
 * Only integer comparisons on the score bits are used: the result is unique
 * and bit-exact.  max_n / max_k are host-side upper bounds on n_b / k_b
 * (0 < max_k <= max_n); a sequence longer than max_n is left unprocessed.
 * ws is optional (see dodo_select_topk_workspace_bytes); the result does not depend on it.  B == 0 is a no-op.
 */
int dodo_select_topk(const float* scores, const int32_t* cu_seqlens, const int32_t* cu_nuggets, int32_t B,
                     int32_t max_n, int32_t max_k, uint32_t flags, int32_t* nugget_idx, void* ws, size_t ws_bytes,
                     void* stream);

/*
 * Sub-selection (Eq. 5): packs the chosen tokens' K and V rows into the compact
 * nugget cache, bit for bit.  K, V are [N, H_kv, d_h] with `token_stride`
 * elements between tokens (>= H_kv*d_h); nugget_idx holds sequence-local
 * indices as written by dodo_select_topk, with room for Kt entries; Kt =
 * cu_nuggets[B] is the total nugget count (host value), or an upper bound of it
 * (rows from cu_nuggets[B] on are left untouched).  Output Kn, Vn: [Kt, H_kv, d_h] (token-major) or
 * [H_kv, Kt, d_h] (head-major), contiguous.  Kt == 0 is a no-op.
 */
int dodo_gather_nuggets(const void* K, const void* V, int dtype, const int32_t* nugget_idx,
                        const int32_t* cu_seqlens, const int32_t* cu_nuggets, int32_t B, int64_t Kt, int32_t H_kv,
                        int32_t d_h, int64_t token_stride, void* Kn, void* Vn, int layout, void* stream);

/*
 * Sub-selection (Eq. 5) for L layers in one launch.  The Scorer reads one fixed layer and the indices it
 * yields select the nuggets of every layer (Sec. 2.1), so the K/V of all layers are packed with the
 * same nugget_idx / cu_nuggets: layer l reads K + l * src_layer_stride, V + l * src_layer_stride
 * ([N, H_kv, d_h] with token_stride each) and writes Kn + l * dst_layer_stride, Vn + l * dst_layer_stride
 * (each as dodo_gather_nuggets writes it, in `layout` with Kt rows).  Strides in elements, multiples of
 * 16 bytes; dst_layer_stride >= Kt * H_kv * d_h; src_layer_stride may be 0 (every layer reads the same
 * rows).  L == 0 is a no-op; L <= 65535.  Bit for bit what L calls of dodo_gather_nuggets produce.
 */
int dodo_gather_nuggets_layers(const void* K, const void* V, int dtype, const int32_t* nugget_idx,
                               const int32_t* cu_seqlens, const int32_t* cu_nuggets, int32_t B, int64_t Kt, int32_t L,
                               int32_t H_kv, int32_t d_h, int64_t token_stride, int64_t src_layer_stride,
                               int64_t dst_layer_stride, void* Kn, void* Vn, int layout, void* stream);

/* Bytes of device workspace dodo_nugget_attention needs for these bounds (may be 0).  The workspace holds
 * the partial results of the split-K kernel and one flag word per partial.  Its contents need not be
 * initialised, with one exception: no flag word may hold the library's "ready" value 0x600DD0D0 on
 * entry -- the call clears the flags it used, so zero-filled memory and memory that was a workspace in a
 * completed call with the same arguments both qualify; fill it with zeros after a call that was aborted or
 * before a call with other sizes.
 * A workspace must not be shared by calls that may overlap in time. */
size_t dodo_nugget_attention_workspace_bytes(int32_t B, int32_t H, int32_t d_h, int32_t max_q, int32_t max_k,
                                             int32_t max_local, int dtype);

/* The same with the number of KV heads known: at least the size above, and more where the kernel for grouped
 * heads and small query blocks (see dodo_nugget_attention) would like to split the keys of a (sequence, KV head)
 * pair over more workgroups than that size has partial records for -- a small batch with few KV heads.  That
 * kernel takes whatever workspace it is given and splits as far as the records fit (not at all without one, or
 * with one that is not 8-byte aligned), so the smaller size is always sufficient and this one is the faster.
 * Same rules for the contents. */
size_t dodo_nugget_attention_workspace_bytes_grouped(int32_t B, int32_t H, int32_t H_kv, int32_t d_h, int32_t max_q,
                                                     int32_t max_k, int32_t max_local, int dtype);

/*
 * Nugget attention (Eq. 13 compressor mode; Eq. 9 mixed resolution).  For
 * sequence b with q_b query rows, k_b nuggets and m_b local rows, query row i
 * of head h attends, with softmax(softmax_scale * q.k) in natural base, over
 * all k_b nuggets followed by local rows j <= m_b - q_b + i (causal mask
 * aligned to the bottom right: the local buffer ends with the query block's
 * own K/V).  A row that sees nothing outputs 0 and lse = -inf.
 *   Q  [sum q_b, H, d_h]       Kl, Vl [sum m_b, H_kv, d_h]   (token-major)
 *   Kn, Vn nugget cache in `layout`, Kt = cu_nuggets[B] rows in total
 *   O  [sum q_b, H, d_h] of `dtype`;  lse (optional, may be NULL) fp32 [sum q_b, H]
 * Query head h reads KV head h / (H / H_kv).  max_q / max_k / max_local are
 * host-side upper bounds on q_b / k_b / m_b.  Arithmetic: bf16 inputs are
 * multiplied on the matrix cores with fp32 accumulation when max_q >= 16
 * (query-block kernel); smaller max_q and all fp32 inputs use the bandwidth-
 * bound split-K kernel, whose last split combines the partials in split order.  Both are deterministic.
 * Supported: d_h in {64, 128}, fp32 or bf16.  When 4 or more query vectors read the same K/V rows -- (H / H_kv) *
 * max_q of them: grouped-query heads, a small query block, or both -- and the inputs are bf16, a
 * third kernel reads every K/V row once for up to 32 of them and multiplies on the matrix cores (fp32 accumulation,
 * partial results merged in a fixed order: deterministic for a given workspace size); more vectors take up to four
 * passes over the keys, each for as many query rows as fill 32 vectors.  Otherwise the split-K kernel
 * serves the query heads of a KV head from one workgroup when there are enough (sequence, row, KV head) triples to
 * fill the GPU that way.
 * The split-K kernel takes at most 65535 (sequence, query-row group) pairs per call (B * max_q at most, fewer when
 * it groups query rows), and K/V token strides below 2^32 bytes; beyond that DODO_ERR_UNSUPPORTED.
 */
int dodo_nugget_attention(const void* Q, const void* Kn, const void* Vn, const void* Kl, const void* Vl,
                          const int32_t* cu_q, const int32_t* cu_nuggets, const int32_t* cu_local, int32_t B,
                          int32_t H, int32_t H_kv, int32_t d_h, int32_t max_q, int32_t max_k, int32_t max_local,
                          int64_t Kt, float softmax_scale, int dtype, int layout, void* O, float* lse, void* ws,
                          size_t ws_bytes, void* stream);

/*
 * dodo_nugget_attention for callers that cannot allocate or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  Same arguments, results and kernels
 * as dodo_nugget_attention without `ws` / `ws_bytes`: the split-K kernel's partial results and flags go
 * to a buffer inside the library (a static device array of about 2.1 MB that every GPU the library runs
 * on holds until the process ends); the call itself allocates and frees nothing.  The buffer has room for
 * DODO_NOALLOC_MAX_PARTIALS partial results, i.e. (sequence, query row, head, split) combinations of a
 * call that splits (dodo_nugget_attention_workspace_bytes / ((d_h + 3) * 4) gives the number for given
 * bounds; 0 means the call needs no buffer at all and always fits); beyond that the call returns
 * DODO_ERR_SCRATCH_LIMIT and launches nothing (the kernel for grouped heads and small query blocks never
 * does: it splits as far as the buffer has room).  All calls on one GPU share that GPU's buffer: calls that
 * may overlap in time on one GPU (different streams, different threads) race and must not be made; calls
 * on one stream are ordered and safe.  Each call leaves the buffer's flags cleared for the next.
 */
#define DODO_NOALLOC_MAX_PARTIALS 4096
int dodo_nugget_attention_noalloc(const void* Q, const void* Kn, const void* Vn, const void* Kl, const void* Vl,
                                  const int32_t* cu_q, const int32_t* cu_nuggets, const int32_t* cu_local, int32_t B,
                                  int32_t H, int32_t H_kv, int32_t d_h, int32_t max_q, int32_t max_k,
                                  int32_t max_local, int64_t Kt, float softmax_scale, int dtype, int layout, void* O,
                                  float* lse, void* stream);

/*
 * Compaction of the pooling baseline the paper compares with (Sec. 5.1: the text is chunked evenly
 * into segments whose states are mean-pooled, at the same compression ratio): sequence b becomes
 * k_b = cu_nuggets[b+1] - cu_nuggets[b] rows, row j the mean of the K (V) rows of tokens
 * floor(j n_b / k_b) .. floor((j+1) n_b / k_b) - 1.  Same shapes, layouts and restrictions as
 * dodo_gather_nuggets (without an index list), so the result feeds the same attention calls.
 * Sums and the division are done in double in token order and rounded once: bit-exact.
 */
int dodo_meanpool_nuggets(const void* K, const void* V, int dtype, const int32_t* cu_seqlens,
                          const int32_t* cu_nuggets, int32_t B, int64_t Kt, int32_t H_kv, int32_t d_h,
                          int64_t token_stride, void* Kn, void* Vn, int layout, void* stream);

/*
 * As dodo_nugget_attention, for nugget caches with room to grow (the autoregressive mode of
 * Sec. 2.4, where the number of nuggets depends on the data): the nuggets of sequence b are the
 * rows nugget_start[b] .. nugget_start[b] + nugget_len[b] of the cache (device int32 [B] each;
 * for the caches of dodo_stream_append: nugget_start[b] = b * cap, nugget_len = counts).
 * Kt is the number of rows of the whole cache (it only matters for the head-major layout) and
 * max_k a host-side upper bound on nugget_len (for instance cap).
 */
int dodo_nugget_attention_cached(const void* Q, const void* Kn, const void* Vn, const void* Kl, const void* Vl,
                                 const int32_t* cu_q, const int32_t* nugget_start, const int32_t* nugget_len,
                                 const int32_t* cu_local, int32_t B, int32_t H, int32_t H_kv, int32_t d_h,
                                 int32_t max_q, int32_t max_k, int32_t max_local, int64_t Kt, float softmax_scale,
                                 int dtype, int layout, void* O, float* lse, void* ws, size_t ws_bytes, void* stream);

/*
 * Nugget attention without a packed cache (Eq. 5 and Eq. 13 / Eq. 9 in one call): the nuggets of
 * sequence b are read where they are, as tokens cu_seqlens[b] + nugget_idx[cu_nuggets[b] + j] of the
 * context's K, V ([N, H_kv, d_h], token_stride elements between tokens, a multiple of 16 bytes).
 * The result is what dodo_gather_nuggets (token-major) followed by dodo_nugget_attention gives,
 * bit for bit; the other arguments are those of dodo_nugget_attention, and
 * dodo_nugget_attention_workspace_bytes gives the workspace for the same bounds.  max_n is a host-
 * side upper bound on the context length of a sequence.  Limits of the query-block kernel (bf16,
 * max_q >= 16): max_k <= 7680 (4096 when max_q <= 128), max_n * token_stride *
 * sizeof(element) < 2^31; beyond them DODO_ERR_UNSUPPORTED (pack the cache instead).
 * Meant for caches that are read once: a packed cache is cheaper to read again and lets the
 * context's K/V be freed, which is the point of the method.
 */
int dodo_nugget_attention_indexed(const void* Q, const void* K, const void* V, const int32_t* nugget_idx,
                                  const int32_t* cu_seqlens, const void* Kl, const void* Vl, const int32_t* cu_q,
                                  const int32_t* cu_nuggets, const int32_t* cu_local, int32_t B, int32_t H,
                                  int32_t H_kv, int32_t d_h, int32_t max_q, int32_t max_k, int32_t max_local,
                                  int32_t max_n, int64_t token_stride, float softmax_scale, int dtype, void* O,
                                  float* lse, void* ws, size_t ws_bytes, void* stream);

/*
 * Segment form of the autoregressive objective (Sec. 2.4, "Learning"): a text is chunked into
 * segments of seg_len tokens, and the tokens of segment c share the splitting index
 * t_c = max(0, c * seg_len - tau): they see the nuggets among the text's first t_c tokens and,
 * causally, its uncompressed tokens from t_c on.  dodo_segment_plan writes one entry per segment,
 * texts in order, segments in order (text b owns ceil(n_b / seg_len) entries):
 *   seg_cu_q[e]      first query row (= first token of the segment in the packed token arrays);
 *                    seg_cu_q[capacity] = N closes the cumulative array
 *   seg_nug_start[e] = cu_nuggets[b];  seg_nug_len[e] = number of the text's nuggets with index < t_c
 *   seg_loc_start[e] = cu_seqlens[b] + t_c;  seg_loc_len[e] = (end of the segment) - t_c
 * nugget_idx / cu_nuggets are the text's nuggets as dodo_select_topk or dodo_select_threshold write
 * them (ascending).  capacity >= the number of segments (a host value: the sum of ceil(n_b / seg_len));
 * entries beyond the last segment come out empty (no query rows); n_segments_out (device, optional)
 * receives the actual number, so that a capacity that was too small can be detected.  All arrays are
 * device int32: [capacity + 1] for seg_cu_q, [capacity] for the others.
 */
int dodo_segment_plan(const int32_t* nugget_idx, const int32_t* cu_seqlens, const int32_t* cu_nuggets, int32_t B,
                      int32_t seg_len, int32_t tau, int32_t capacity, int32_t* seg_cu_q, int32_t* seg_nug_start,
                      int32_t* seg_nug_len, int32_t* seg_loc_start, int32_t* seg_loc_len, int32_t* n_segments_out,
                      void* stream);

/*
 * Nugget attention over the entries of dodo_segment_plan (or any other ranges of that form): entry e
 * has query rows seg_cu_q[e] .. seg_cu_q[e+1] of Q, the nuggets seg_nug_start[e] .. + seg_nug_len[e]
 * of the cache Kn / Vn (`layout`, Kt rows), and the local rows seg_loc_start[e] .. + seg_loc_len[e] of
 * K / V ([N, H_kv, d_h] contiguous: the text's own uncompressed keys and values), under the same
 * bottom-right aligned causal rule as dodo_nugget_attention.  Ranges of different entries may overlap.
 * max_q / max_k / max_local bound the three lengths (for a plan: seg_len, the largest nugget count of
 * a text, seg_len + tau).  Everything else as in dodo_nugget_attention.
 */
int dodo_nugget_attention_segments(const void* Q, const void* Kn, const void* Vn, const void* K, const void* V,
                                   const int32_t* seg_cu_q, const int32_t* seg_nug_start, const int32_t* seg_nug_len,
                                   const int32_t* seg_loc_start, const int32_t* seg_loc_len, int32_t n_segments,
                                   int32_t H, int32_t H_kv, int32_t d_h, int32_t max_q, int32_t max_k,
                                   int32_t max_local, int64_t Kt, float softmax_scale, int dtype, int layout, void* O,
                                   float* lse, void* ws, size_t ws_bytes, void* stream);

/*
 * Score gradient of the straight-through estimator (Sec. 2.5, Eq. 17-18) for one layer.  The forward
 * pass adds s_i - stopgrad(s_i) to the attention logits of nugget i, so the gradient of the loss in
 * s_i is the sum over query rows j and heads h of its gradient in the softmax input xi[j, i]:
 *   grad[i] (+)= grad_scale * sum_h sum_j P[j,i] * (dO[j,h].v_i - dO[j,h].O[j,h]),
 *   P[j,i] = exp(softmax_scale * q_j.k_i - lse[j,h]).
 * Q, dO, O are [Sq, H, d_h] of `dtype` and lse fp32 [Sq, H] exactly as dodo_nugget_attention took and
 * returned them for this layer (lse is required there); Kn, Vn, cu_q, cu_nuggets, layout, Kt as in
 * that call (every nugget of a sequence is visible to all of its query rows, so the local rows enter
 * through O and lse only).  grad_scores is fp32 [Kt], packed like the nugget cache; accumulate != 0
 * adds to it (the sum over layers of Eq. 18: one call per layer), else it is overwritten.
 * grad_scale: softmax_scale if the score is added to the unscaled logit xi of Eq. 17, 1 if it is
 * added to the softmax input.  Sq = total query rows (host value); max_q / max_k bound q_b / k_b.
 * ws: dodo_ste_score_grad_workspace_bytes(Sq, H, Kt) bytes, contents irrelevant.
 * d_h % 8 == 0; bf16 with d_h = 128 runs on the matrix cores, everything else in a plain kernel.
 * Deterministic (fixed summation order, no atomics).
 */
size_t dodo_ste_score_grad_workspace_bytes(int64_t Sq, int32_t H, int64_t Kt);
int dodo_ste_score_grad(const void* Q, const void* Kn, const void* Vn, const void* dO, const void* O, const float* lse,
                        const int32_t* cu_q, const int32_t* cu_nuggets, int32_t B, int32_t H, int32_t H_kv,
                        int32_t d_h, int32_t max_q, int32_t max_k, int64_t Sq, int64_t Kt, float softmax_scale,
                        float grad_scale, int accumulate, int dtype, int layout, float* grad_scores, void* ws,
                        size_t ws_bytes, void* stream);

/*
 * Threshold of the autoregressive mode from sampled scores (Sec. 2.4: Lambda is set so that about
 * t/r of t tokens are kept, and is estimated by running the scorer on sampled tokens).  With
 * k = dodo_nugget_count(n, num, den), writes to *lambda_out (device, fp32) the (k+1)-th highest
 * of the n sampled scores (device, fp32), so that exactly k of them exceed it when there are no
 * ties; NaN ranks lowest, -0 counts as +0.  If k >= n, or that score is NaN, the threshold is
 * -inf (keep everything).  Integer comparisons on the score bits only: bit-exact.  n >= 1.
 * ws is optional (dodo_threshold_from_sample_workspace_bytes(n) bytes, contents irrelevant; 0 for small samples):
 * with it a large sample is histogrammed by many workgroups, one launch per radix pass; without it (NULL or too
 * small) one workgroup does the same work, more slowly.  The result does not depend on it.
 */
size_t dodo_threshold_from_sample_workspace_bytes(int64_t n);
int dodo_threshold_from_sample(const float* sample, int64_t n, int64_t num, int64_t den, float* lambda_out, void* ws,
                               size_t ws_bytes, void* stream);

/*
 * Threshold selection (Eq. 8): token i of a sequence is kept iff scores[i] > *lambda (device fp32;
 * strict, false for NaN), which does not depend on later tokens.  Writes, without any host
 * read-back: counts[b] (int32 [B]), their running sum cu_nuggets (int32 [B+1]) and the kept tokens'
 * sequence-local indices in ascending order, packed, to nugget_idx[cu_nuggets[b] ..] (room for
 * cu_seqlens[B] entries) -- the format dodo_gather_nuggets and dodo_nugget_attention take.  The
 * total cu_nuggets[B] is only known on the device: pass dodo_gather_nuggets an upper bound as Kt
 * (token-major layout; rows past cu_nuggets[B] are skipped).  B == 0 is a no-op.
 */
int dodo_select_threshold(const float* scores, const int32_t* cu_seqlens, int32_t B, const float* lambda,
                          int32_t* counts, int32_t* cu_nuggets, int32_t* nugget_idx, void* stream);

/*
 * One decode step of the autoregressive mode (Sec. 2.4 with the mixed resolution of Eq. 9): in each
 * of B sequences one token leaves the window of uncompressed tokens.  scores[b] is its score
 * (device fp32 [B]), K_rows / V_rows its key and value rows ([B, H_kv, d_h] of `dtype`, row_stride
 * elements between sequences).  If scores[b] > *lambda the rows are appended to sequence b's nugget
 * cache at row b * cap + counts[b] of Kn / Vn ([B * cap, H_kv, d_h], token-major) and counts[b]
 * (device int32, in/out) grows by one; a full cache drops the token and adds one to *dropped
 * (device int32, may be NULL).  H_kv * d_h * element size and the row stride must be multiples
 * of 16 bytes.
 */
int dodo_stream_append(const float* scores, const float* lambda, const void* K_rows, const void* V_rows, int dtype,
                       int32_t B, int32_t H_kv, int32_t d_h, int64_t row_stride, int32_t cap, int32_t* counts,
                       int32_t* dropped, void* Kn, void* Vn, void* stream);

/*
 * Measurement aids (no step of the paper's method): a read-only pass over `bytes` of src, and a plain copy of
 * `bytes` from src to dst, written like the library's bandwidth-bound kernels.  A benchmark times them in the
 * same run as the path's kernels, as what this device's memory system gives such code, next to the nominal
 * peak.  Device pointers, 16-byte aligned, bytes a multiple of 16, src and dst disjoint; sink is a device word
 * that is (practically never) written, it only keeps the loads alive.
 */
int dodo_probe_read(const void* src, size_t bytes, uint32_t* sink, void* stream);
int dodo_probe_copy(const void* src, void* dst, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DODO_H_ */
