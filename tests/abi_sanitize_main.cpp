// Host-only driver for a build of the library's host code with AddressSanitizer and UndefinedBehaviorSanitizer:
// every entry point is called with arguments that its validation must reject (or accept as a no-op) before any
// device work, as on a host without a GPU.  Exit status 0 = every status as expected and no sanitizer report.
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "dodo.h"

#define EXPECT(call, want)                                                            \
  do {                                                                                \
    const long long got_ = static_cast<long long>(call);                              \
    if (got_ != static_cast<long long>(want)) {                                       \
      std::fprintf(stderr, "%s = %lld, expected %lld\n", #call, got_, (long long)(want)); \
      std::exit(1);                                                                   \
    }                                                                                 \
  } while (0)

int main() {
  alignas(16) static char buf[64];
  void* P = buf;
  const int32_t* PI = reinterpret_cast<const int32_t*>(buf);
  int32_t* PO = reinterpret_cast<int32_t*>(buf);
  float* PF = reinterpret_cast<float*>(buf);
  EXPECT(dodo_version(), DODO_VERSION);
  for (int s = -7; s <= 1; ++s)
    if (std::strlen(dodo_status_string(s)) == 0) return 1;
  EXPECT(dodo_nugget_count(320, 1, 10), 32);
  EXPECT(dodo_nugget_count(0, 1, 10), 0);
  EXPECT(dodo_nugget_count(INT64_MAX, INT64_MAX, 1), INT64_MAX);
  EXPECT(dodo_nugget_count(5, 0, 1), -1);
  EXPECT(dodo_score(nullptr, P, 0.f, DODO_DTYPE_BF16, 4, 64, 64, PF, nullptr), DODO_ERR_INVALID_ARG);
  EXPECT(dodo_score(P, P, 0.f, 7, 4, 64, 64, PF, nullptr), DODO_ERR_UNSUPPORTED);
  EXPECT(dodo_score(P, P, 0.f, DODO_DTYPE_BF16, 0, 64, 64, PF, nullptr), DODO_OK);
  EXPECT(dodo_score(P, P, 0.f, DODO_DTYPE_BF16, 4, 64, 8, PF, nullptr), DODO_ERR_INVALID_ARG);
  EXPECT(dodo_score_mlp(P, P, PF, P, 0.f, 9, DODO_DTYPE_BF16, 4, 64, 256, 64, PF, nullptr, 0, nullptr), DODO_ERR_INVALID_ARG);
  EXPECT(dodo_select_topk(PF, PI, PI, 2, 10, 11, 0, PO, nullptr, 0, nullptr), DODO_ERR_INVALID_ARG);
  EXPECT(dodo_select_topk(PF, PI, PI, 2, 10, 5, 8, PO, nullptr, 0, nullptr), DODO_ERR_INVALID_ARG);
  EXPECT(dodo_select_topk(nullptr, nullptr, nullptr, 0, 10, 5, 0, nullptr, nullptr, 0, nullptr), DODO_OK);
  EXPECT(dodo_select_topk_workspace_bytes(8, 4096), 0);
  EXPECT(dodo_gather_nuggets(P, P, DODO_DTYPE_BF16, PI, PI, PI, 2, 5, 4, 64, 8, P, P, 0, nullptr), DODO_ERR_INVALID_ARG);
  EXPECT(dodo_gather_nuggets(P, P, DODO_DTYPE_BF16, PI, PI, PI, 2, 5, 4, 64, 256, P, P, 3, nullptr), DODO_ERR_INVALID_ARG);
  EXPECT(dodo_gather_nuggets(P, P, DODO_DTYPE_BF16, PI, PI, PI, 2, 0, 4, 64, 256, P, P, 0, nullptr), DODO_OK);
  EXPECT(dodo_gather_nuggets_layers(P, P, DODO_DTYPE_BF16, PI, PI, PI, 2, 5, 70000, 4, 64, 256, 0, 5 * 256, P, P, 0, nullptr),
         DODO_ERR_UNSUPPORTED);
  EXPECT(dodo_meanpool_nuggets(P, P, 5, PI, PI, 2, 5, 4, 64, 256, P, P, 0, nullptr), DODO_ERR_UNSUPPORTED);
  EXPECT(dodo_nugget_attention(P, P, P, P, P, PI, PI, PI, 2, 8, 3, 128, 16, 10, 20, 10, 0.1f, DODO_DTYPE_BF16, 0, P, nullptr,
                               nullptr, 0, nullptr),
         DODO_ERR_INVALID_ARG);  // H % H_kv != 0
  EXPECT(dodo_nugget_attention(P, P, P, P, P, PI, PI, PI, 2, 8, 8, 96, 16, 10, 20, 10, 0.1f, DODO_DTYPE_BF16, 0, P, nullptr,
                               nullptr, 0, nullptr),
         DODO_ERR_UNSUPPORTED);  // head size
  EXPECT(dodo_nugget_attention(P, P, P, P, P, PI, PI, PI, 1, 2, 2, 128, 1, 3000, 1000, 3000, 0.1f, DODO_DTYPE_BF16, 0, P,
                               nullptr, nullptr, 0, nullptr),
         DODO_ERR_WORKSPACE_TOO_SMALL);
  EXPECT(dodo_nugget_attention(P, P, P, P, P, PI, PI, PI, 0, 2, 2, 128, 1, 3000, 1000, 3000, 0.1f, DODO_DTYPE_BF16, 0, P,
                               nullptr, nullptr, 0, nullptr),
         DODO_OK);
  EXPECT(dodo_nugget_attention_noalloc(P, P, P, P, P, PI, PI, PI, 2, 8, 3, 128, 16, 10, 20, 10, 0.1f, DODO_DTYPE_BF16, 0, P,
                                       nullptr, nullptr),
         DODO_ERR_INVALID_ARG);
  EXPECT(dodo_nugget_attention_cached(P, P, P, P, P, PI, PI, nullptr, PI, 2, 8, 8, 128, 16, 10, 20, 10, 0.1f, DODO_DTYPE_BF16, 0,
                                      P, nullptr, nullptr, 0, nullptr),
         DODO_ERR_INVALID_ARG);
  EXPECT(dodo_nugget_attention_indexed(P, P, P, PI, PI, P, P, PI, PI, PI, 2, 8, 8, 128, 16, 30, 20, 10, 1024, 0.1f,
                                       DODO_DTYPE_BF16, P, nullptr, nullptr, 0, nullptr),
         DODO_ERR_INVALID_ARG);  // max_k > max_n
  EXPECT(dodo_nugget_attention_segments(P, P, P, P, P, PI, PI, nullptr, PI, PI, 3, 8, 8, 128, 16, 10, 20, 10, 0.1f,
                                        DODO_DTYPE_BF16, 0, P, nullptr, nullptr, 0, nullptr),
         DODO_ERR_INVALID_ARG);
  EXPECT(dodo_segment_plan(PI, PI, PI, 2, 0, 1, 4, PO, PO, PO, PO, PO, PO, nullptr), DODO_ERR_INVALID_ARG);
  EXPECT(dodo_ste_score_grad(P, P, P, P, P, nullptr, PI, PI, 2, 8, 8, 128, 16, 10, 32, 20, 0.1f, 0.1f, 0, DODO_DTYPE_BF16, 0, PF,
                             nullptr, 0, nullptr),
         DODO_ERR_INVALID_ARG);
  EXPECT(dodo_threshold_from_sample(PF, 0, 1, 10, PF, nullptr, 0, nullptr), DODO_ERR_INVALID_ARG);
  EXPECT(dodo_select_threshold(PF, PI, -1, PF, PO, PO, PO, nullptr), DODO_ERR_INVALID_ARG);
  EXPECT(dodo_stream_append(PF, PF, P, P, DODO_DTYPE_BF16, 2, 4, 64, 8, 16, PO, nullptr, P, P, nullptr), DODO_ERR_INVALID_ARG);
  EXPECT(dodo_probe_read(P, 24, reinterpret_cast<uint32_t*>(buf), nullptr), DODO_ERR_UNSUPPORTED);
  EXPECT(dodo_probe_copy(P, nullptr, 32, nullptr), DODO_ERR_INVALID_ARG);
  std::puts("abi sanitizer driver: ok");
  return 0;
}
