// Internal interface between the dodo_nugget_attention entry point and its two kernels.
#pragma once
#include "dodo_common.h"

namespace dodo {

struct AttnParams {
  const void *Q, *Kn, *Vn, *Kl, *Vl;
  const int32_t *cu_q, *cu_nuggets, *cu_local;
  const int32_t* nug_len;  // null: nuggets of sequence b are rows cu_nuggets[b] .. cu_nuggets[b+1]; else cu_nuggets[b] .. + nug_len[b]
  const int32_t* loc_len;  // null: local rows of sequence b are rows cu_local[b] .. cu_local[b+1]; else cu_local[b] .. + loc_len[b]
  // gather-free form (both null otherwise): Kn / Vn are the context's K / V, nugget j of sequence b is its token
  // cu_ctx[b] + nug_idx[cu_nuggets[b] + j]
  const int32_t *nug_idx, *cu_ctx;
  int heavy_last;  // != 0: later entries of the batch cost more (segment plans); the query-block kernel starts with them
  int32_t max_n;  // gather-free form: host-side upper bound on the context length of a sequence
  int32_t B, H, H_kv, d_h, max_q, max_k, max_local;
  int64_t nug_tok_stride, nug_head_stride;  // elements between tokens / KV heads of the nugget cache
  float scale_log2e;                        // softmax_scale * log2(e): logits are kept in base 2
  int dtype;
  void* O;
  float* lse;
  void* ws;        // split-K kernel: partial records, followed by one flag word per record ...
  void* ws_flags;  // ... unless this is set: then the flag words live here
  hipStream_t stream;
};

// Split count of the bandwidth-bound kernel for these bounds (>= 1), shared by
// the launch and the workspace query.
int splitk_count(int32_t B, int32_t H, int32_t max_q, int32_t max_k, int32_t max_local);
size_t splitk_workspace_bytes(int32_t B, int32_t H, int32_t d_h, int32_t max_q, int nsplit);

// fp32 or bf16, d_h in {64,128}, any max_q: one workgroup per (query row, head, split).
int launch_splitk_attention(const AttnParams& p);
// bf16, d_h in {64,128}: MFMA kernel over 128- or 256-row query blocks.
int launch_block_attention(const AttnParams& p);

}  // namespace dodo
