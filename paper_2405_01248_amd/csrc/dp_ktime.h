// Optional per-launch kernel timing (hipEvents around individual launches), used by the
// measurement entry points dp_ktime_begin / dp_ktime_end.  Disabled by default: the
// compute entry points then record nothing.
#pragma once
#include <hip/hip_runtime.h>

namespace dp {

enum KernelKind {
  KK_GEMM_NT = 0, KK_GEMM_NN = 1, KK_GEMM_TN = 2, KK_ATTN_FWD = 3, KK_ATTN_BWD_DQ = 4, KK_ATTN_BWD_DKV = 5,
  KK_LN_FWD = 6, KK_LN_BWD = 7, KK_GEGLU_FWD = 8, KK_GEGLU_BWD = 9, KK_REDUCE = 10, KK_OTHER = 11, KK_GEMM_F32 = 12,
  KK_ATTN_F32 = 13, KK_CONV = 14, KK_GROUPNORM = 15, KK_SOFTMAX = 16, KK_GEMM_FP8 = 17
};

bool ktime_enabled();
void ktime_open(int kind, double flops, double bytes, int m, int n, int k, hipStream_t s);
void ktime_close(hipStream_t s);

// Brackets the launches issued during its lifetime when timing is enabled.
struct KScope {
  hipStream_t s; bool on;
  KScope(int kind, double flops, double bytes, hipStream_t st, int m = 0, int n = 0, int k = 0) : s(st), on(ktime_enabled()) {
    if (on) ktime_open(kind, flops, bytes, m, n, k, s);
  }
  ~KScope() { if (on) ktime_close(s); }
};

}  // namespace dp
