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
  void* ws;         // bandwidth-bound kernels: partial records, followed by one flag word per record ...
  size_t ws_bytes;  //   (bytes at ws)
  void* ws_flags;   // ... unless this is set: then the flag words live here, and both regions hold ws_slots entries
  int64_t ws_slots;
  hipStream_t stream;
};

// Workspace format of the bandwidth-bound kernels: one partial record [m, s, o[0..DH)] of floats per (sequence,
// query row, head, split); after all records (or where ws_flags points), one 32-bit flag per record.
template <int DH>
__host__ __device__ constexpr int partial_floats() { return DH + 2; }
constexpr uint32_t kPartialReady = 0x600DD0D0u;  // flag value of a record that has been written
constexpr int kMaxPolls = 1 << 17;               // bound of the combiner's wait (~0.1 s, never reached in a healthy run)

// Split count of the bandwidth-bound kernels for these bounds (>= 1), shared by
// the launches and the workspace query.
int splitk_count(int32_t B, int32_t H, int32_t max_q, int32_t max_k, int32_t max_local);
size_t splitk_workspace_bytes(int32_t B, int32_t H, int32_t d_h, int32_t max_q, int nsplit);

// fp32 or bf16, d_h in {64,128}, any max_q: one workgroup per (query row, head, split).
int launch_splitk_attention(const AttnParams& p);
// bf16, d_h in {64,128}, at least 4 query vectors per KV head and sequence ((H / H_kv) * max_q): MFMA kernel that reads
// every K/V row once for up to 32 of them (more: up to four passes).  group_attention_applies says whether it takes the call.
// It splits the keys of a (sequence, KV head) pair as far as the caller's workspace has room for records;
// group_workspace_bytes is the size that lets it split as far as it would like to (0: no split wanted).
bool group_attention_applies(const AttnParams& p);
int group_launches(int32_t H, int32_t H_kv, int32_t max_q);  // 0: not for these head counts and this max_q
size_t group_workspace_bytes(int32_t B, int32_t H, int32_t H_kv, int32_t d_h, int32_t max_q, int32_t max_k,
                             int32_t max_local);
int launch_group_attention(const AttnParams& p);
// bf16, d_h in {64,128}: MFMA kernel over 128- or 256-row query blocks.
int launch_block_attention(const AttnParams& p);

}  // namespace dodo
