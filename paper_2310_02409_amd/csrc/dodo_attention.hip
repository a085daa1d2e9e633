// dodo_nugget_attention: argument checks and dispatch between the MFMA
// query-block kernel and the two bandwidth-bound kernels (one query vector per K/V row read: split-K kernel on
// the vector pipe; several: grouped kernel on the matrix cores).
#include <mutex>

#include "dodo_attn.h"

namespace dodo {
namespace {

constexpr int kBlockKernelMinQ = 16;

bool use_block_kernel(int dtype, int32_t d_h, int32_t max_q) {
  return dtype == DODO_DTYPE_BF16 && (d_h == 128 || d_h == 64) && max_q >= kBlockKernelMinQ;
}

}  // namespace
}  // namespace dodo

extern "C" size_t dodo_nugget_attention_workspace_bytes(int32_t B, int32_t H, int32_t d_h, int32_t max_q, int32_t max_k,
                                                        int32_t max_local, int dtype) {
  using namespace dodo;
  if (B <= 0 || H <= 0 || d_h <= 0 || max_q <= 0 || max_k < 0 || max_local < 0) return 0;
  if (use_block_kernel(dtype, d_h, max_q)) return 0;
  return splitk_workspace_bytes(B, H, d_h, max_q, splitk_count(B, H, max_q, max_k, max_local));
}

extern "C" size_t dodo_nugget_attention_workspace_bytes_grouped(int32_t B, int32_t H, int32_t H_kv, int32_t d_h,
                                                                int32_t max_q, int32_t max_k, int32_t max_local,
                                                                int dtype) {
  using namespace dodo;
  const size_t plain = dodo_nugget_attention_workspace_bytes(B, H, d_h, max_q, max_k, max_local, dtype);
  if (B <= 0 || H <= 0 || H_kv <= 0 || H % H_kv != 0 || max_q <= 0 || max_k < 0 || max_local < 0) return plain;
  if (use_block_kernel(dtype, d_h, max_q) || dtype != DODO_DTYPE_BF16 || (d_h != 128 && d_h != 64)) return plain;
  if (group_launches(H, H_kv, max_q) == 0) return plain;  // too few query vectors share their K/V rows, or too many
  const size_t grouped = group_workspace_bytes(B, H, H_kv, d_h, max_q, max_k, max_local);
  return grouped > plain ? grouped : plain;
}

// ---- the entry point that allocates nothing: the split-K kernel's partial records and flags live in a
// file-scope device array.  Its name is only a host-side handle: the device address is looked up once per
// device and kept, and that pointer is what the kernels get.
namespace dodo {
namespace {

constexpr int kScratchSlots = DODO_NOALLOC_MAX_PARTIALS;            // (query row, head, split) records
constexpr size_t kScratchFlagBytes = kScratchSlots * sizeof(uint32_t);
constexpr size_t kScratchRecordBytes = static_cast<size_t>(kScratchSlots) * (128 + 2) * sizeof(float);
constexpr size_t kScratchBytes = kScratchFlagBytes + kScratchRecordBytes;

// flags first (zero when the library is loaded; every call leaves the flags it used at zero), records after
// them, so that no record of an earlier call with another shape is ever read as a flag
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (each GPU has its own copy at its own address).
int scratch_address(void** out) {
  int dev = 0;
  DODO_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return DODO_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    DODO_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (ptr == nullptr) return DODO_ERR_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return DODO_OK;
}

}  // namespace
}  // namespace dodo

namespace dodo {
namespace {

// What the variants of the call add to the plain one (all null / 0 there).
struct Variant {
  const int32_t* nug_len = nullptr;  // nuggets of b: rows cu_nuggets[b] .. + nug_len[b]
  const int32_t* loc_len = nullptr;  // local rows of b: rows cu_local[b] .. + loc_len[b]
  const int32_t* nug_idx = nullptr;  // gather-free form: Kn / Vn are the context's K / V with ctx_stride
  const int32_t* cu_ctx = nullptr;   //   elements between tokens, sequences of at most max_n tokens
  int64_t ctx_stride = 0;
  int32_t max_n = 0;
  int heavy_last = 0;                // later entries cost more: start with them
  bool library_scratch = false;      // partial records and flags go to the library's own static buffer
};

int attention_entry(const void* Q, const void* Kn, const void* Vn, const void* Kl, const void* Vl, const int32_t* cu_q,
                    const int32_t* cu_nuggets, const int32_t* cu_local, const Variant& v, int32_t B, int32_t H,
                    int32_t H_kv, int32_t d_h, int32_t max_q, int32_t max_k, int32_t max_local, int64_t Kt,
                    float softmax_scale, int dtype, int layout, void* O, float* lse, void* ws, size_t ws_bytes,
                    void* stream) {
  if (B < 0 || H <= 0 || H_kv <= 0 || d_h <= 0 || max_q < 0 || max_k < 0 || max_local < 0 || Kt < 0)
    return DODO_ERR_INVALID_ARG;
  if (H % H_kv != 0) return DODO_ERR_INVALID_ARG;
  if (layout != DODO_LAYOUT_TOKEN_MAJOR && layout != DODO_LAYOUT_HEAD_MAJOR) return DODO_ERR_INVALID_ARG;
  if (!(softmax_scale == softmax_scale)) return DODO_ERR_INVALID_ARG;
  if (B == 0 || max_q == 0) return DODO_OK;
  if (!Q || !O || !cu_q || !cu_nuggets || !cu_local) return DODO_ERR_INVALID_ARG;
  if (max_k > 0 && (!Kn || !Vn)) return DODO_ERR_INVALID_ARG;
  if (max_local > 0 && (!Kl || !Vl)) return DODO_ERR_INVALID_ARG;
  if (!dtype_ok(dtype)) return DODO_ERR_UNSUPPORTED;
  if (d_h != 64 && d_h != 128) return DODO_ERR_UNSUPPORTED;
  if (!aligned16(Q) || !aligned16(O) || !aligned16(Kn) || !aligned16(Vn) || !aligned16(Kl) || !aligned16(Vl))
    return DODO_ERR_UNSUPPORTED;
  AttnParams p;
  p.Q = Q; p.Kn = Kn; p.Vn = Vn; p.Kl = Kl; p.Vl = Vl;
  p.cu_q = cu_q; p.cu_nuggets = cu_nuggets; p.nug_len = v.nug_len; p.cu_local = cu_local; p.loc_len = v.loc_len;
  p.nug_idx = v.nug_idx; p.cu_ctx = v.cu_ctx; p.max_n = v.max_n; p.heavy_last = v.heavy_last;
  p.B = B; p.H = H; p.H_kv = H_kv; p.d_h = d_h; p.max_q = max_q; p.max_k = max_k; p.max_local = max_local;
  if (v.nug_idx != nullptr) {
    p.nug_tok_stride = v.ctx_stride;
    p.nug_head_stride = d_h;
  } else if (layout == DODO_LAYOUT_TOKEN_MAJOR) {
    p.nug_tok_stride = static_cast<int64_t>(H_kv) * d_h;
    p.nug_head_stride = d_h;
  } else {
    p.nug_tok_stride = d_h;
    p.nug_head_stride = Kt * d_h;
  }
  p.scale_log2e = softmax_scale * 1.4426950408889634f;
  p.dtype = dtype;
  p.O = O; p.lse = lse; p.ws = ws; p.ws_bytes = ws_bytes; p.ws_flags = nullptr; p.ws_slots = 0;
  p.stream = static_cast<hipStream_t>(stream);
  if (use_block_kernel(dtype, d_h, max_q)) return launch_block_attention(p);
  if (v.library_scratch) {
    // flags in the first part of the buffer, records (of up to 128 channels) after them
    void* base = nullptr;
    const int rc = scratch_address(&base);
    if (rc != DODO_OK) return rc;
    p.ws_flags = base;
    p.ws_slots = kScratchSlots;
    p.ws = static_cast<unsigned char*>(base) + kScratchFlagBytes;
    p.ws_bytes = kScratchRecordBytes;
  }
  // (the grouped kernel splits only as far as the workspace it is given has room: it needs none)
  if (group_attention_applies(p)) return launch_group_attention(p);
  const size_t need = dodo_nugget_attention_workspace_bytes(B, H, d_h, max_q, max_k, max_local, dtype);
  if (v.library_scratch) {  // need = records * (d_h + 3) * 4 bytes: the limit is on the records
    if (need / ((static_cast<size_t>(d_h) + 3) * sizeof(float)) > static_cast<size_t>(kScratchSlots)) return DODO_ERR_SCRATCH_LIMIT;
  } else if (need > 0 && (!ws || ws_bytes < need)) {
    return DODO_ERR_WORKSPACE_TOO_SMALL;
  }
  return launch_splitk_attention(p);
}

}  // namespace
}  // namespace dodo

extern "C" int dodo_nugget_attention(const void* Q, const void* Kn, const void* Vn, const void* Kl, const void* Vl,
                                     const int32_t* cu_q, const int32_t* cu_nuggets, const int32_t* cu_local,
                                     int32_t B, int32_t H, int32_t H_kv, int32_t d_h, int32_t max_q, int32_t max_k,
                                     int32_t max_local, int64_t Kt, float softmax_scale, int dtype, int layout,
                                     void* O, float* lse, void* ws, size_t ws_bytes, void* stream) {
  return dodo::attention_entry(Q, Kn, Vn, Kl, Vl, cu_q, cu_nuggets, cu_local, dodo::Variant{}, B, H, H_kv, d_h, max_q,
                               max_k, max_local, Kt, softmax_scale, dtype, layout, O, lse, ws, ws_bytes, stream);
}

extern "C" int dodo_nugget_attention_noalloc(const void* Q, const void* Kn, const void* Vn, const void* Kl,
                                             const void* Vl, const int32_t* cu_q, const int32_t* cu_nuggets,
                                             const int32_t* cu_local, int32_t B, int32_t H, int32_t H_kv, int32_t d_h,
                                             int32_t max_q, int32_t max_k, int32_t max_local, int64_t Kt,
                                             float softmax_scale, int dtype, int layout, void* O, float* lse,
                                             void* stream) {
  dodo::Variant v;
  v.library_scratch = true;
  return dodo::attention_entry(Q, Kn, Vn, Kl, Vl, cu_q, cu_nuggets, cu_local, v, B, H, H_kv, d_h, max_q, max_k,
                               max_local, Kt, softmax_scale, dtype, layout, O, lse, nullptr, 0, stream);
}

extern "C" int dodo_nugget_attention_cached(const void* Q, const void* Kn, const void* Vn, const void* Kl,
                                            const void* Vl, const int32_t* cu_q, const int32_t* nugget_start,
                                            const int32_t* nugget_len, const int32_t* cu_local, int32_t B, int32_t H,
                                            int32_t H_kv, int32_t d_h, int32_t max_q, int32_t max_k, int32_t max_local,
                                            int64_t Kt, float softmax_scale, int dtype, int layout, void* O, float* lse,
                                            void* ws, size_t ws_bytes, void* stream) {
  if (B > 0 && max_q > 0 && !nugget_len) return DODO_ERR_INVALID_ARG;
  dodo::Variant v;
  v.nug_len = nugget_len;
  return dodo::attention_entry(Q, Kn, Vn, Kl, Vl, cu_q, nugget_start, cu_local, v, B, H, H_kv, d_h, max_q, max_k,
                               max_local, Kt, softmax_scale, dtype, layout, O, lse, ws, ws_bytes, stream);
}

extern "C" int dodo_nugget_attention_indexed(const void* Q, const void* K, const void* V, const int32_t* nugget_idx,
                                             const int32_t* cu_seqlens, const void* Kl, const void* Vl,
                                             const int32_t* cu_q, const int32_t* cu_nuggets, const int32_t* cu_local,
                                             int32_t B, int32_t H, int32_t H_kv, int32_t d_h, int32_t max_q,
                                             int32_t max_k, int32_t max_local, int32_t max_n, int64_t token_stride,
                                             float softmax_scale, int dtype, void* O, float* lse, void* ws,
                                             size_t ws_bytes, void* stream) {
  if (max_n < 0 || max_k > max_n) return DODO_ERR_INVALID_ARG;
  if (H_kv > 0 && d_h > 0 && token_stride < static_cast<int64_t>(H_kv) * d_h) return DODO_ERR_INVALID_ARG;
  if (B > 0 && max_q > 0 && max_k > 0 && (!nugget_idx || !cu_seqlens)) return DODO_ERR_INVALID_ARG;
  if (dodo::dtype_ok(dtype) && (token_stride * dodo::elem_bytes(dtype)) % 16 != 0) return DODO_ERR_UNSUPPORTED;
  dodo::Variant v;
  if (max_k > 0) {  // without nuggets the call is the plain one (nothing is read through the index list)
    v.nug_idx = nugget_idx;
    v.cu_ctx = cu_seqlens;
    v.ctx_stride = token_stride;
    v.max_n = max_n;
  }
  return dodo::attention_entry(Q, K, V, Kl, Vl, cu_q, cu_nuggets, cu_local, v, B, H, H_kv, d_h, max_q, max_k, max_local,
                               0, softmax_scale, dtype, DODO_LAYOUT_TOKEN_MAJOR, O, lse, ws, ws_bytes, stream);
}

extern "C" int dodo_nugget_attention_segments(const void* Q, const void* Kn, const void* Vn, const void* K, const void* V,
                                              const int32_t* seg_cu_q, const int32_t* seg_nug_start,
                                              const int32_t* seg_nug_len, const int32_t* seg_loc_start,
                                              const int32_t* seg_loc_len, int32_t n_segments, int32_t H, int32_t H_kv,
                                              int32_t d_h, int32_t max_q, int32_t max_k, int32_t max_local, int64_t Kt,
                                              float softmax_scale, int dtype, int layout, void* O, float* lse, void* ws,
                                              size_t ws_bytes, void* stream) {
  if (n_segments > 0 && max_q > 0 && (!seg_nug_len || !seg_loc_len)) return DODO_ERR_INVALID_ARG;
  dodo::Variant v;
  v.nug_len = seg_nug_len;
  v.loc_len = seg_loc_len;
  v.heavy_last = 1;
  return dodo::attention_entry(Q, Kn, Vn, K, V, seg_cu_q, seg_nug_start, seg_loc_start, v, n_segments, H, H_kv, d_h,
                               max_q, max_k, max_local, Kt, softmax_scale, dtype, layout, O, lse, ws, ws_bytes, stream);
}
