// dp_op_gemm_static: dp_op_gemm for callers that cannot allocate device memory (code under HIP graph
// capture, tight serving loops, harnesses that forbid hipMalloc).  The split-K partial sums, which
// dp_op_gemm keeps in a caller-provided workspace, live in a file-scope device array here.  Every GPU the
// library runs on holds its own copy of that array until the process ends.
#include "../../include/dpipe.h"
#include "dp_kernels.h"
#include "dp_errors.h"

#include <cstring>
#include <mutex>

// The array's name is a host-side stand-in, not a device address: host code only ever uses the address
// hipGetSymbolAddress returns for the current device (scratch_of_current_device below).
static __device__ __align__(256) unsigned char scratch[DP_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each device, looked up once per device

// Address of this library's scratch array on the device that is current for the calling thread.
int scratch_of_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return dp::set_error(DP_EHIP, "dp_op_gemm_static: hipGetDevice failed");
  if (dev < 0 || dev >= kMaxDevices) return dp::set_errorf(DP_EUNSUPPORTED, "dp_op_gemm_static: device index %d not supported (max %d)", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return dp::set_errorf(DP_EHIP, "dp_op_gemm_static: hipGetSymbolAddress failed on device %d (%s)", dev, hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return DP_OK;
}

}  // namespace

extern "C" int dp_op_gemm_static(int dtype, const void* A, int lda, int a_kmajor, const void* B, int ldb, int b_kmajor, int M, int N,
                                 int K, const void* bias, void* C, int ldc, int out_is_f32, int accumulate, int tile_cfg,
                                 void* hip_stream) {
  using namespace dp;
  if (dtype != DP_F32 && dtype != DP_BF16) return set_error(DP_EINVAL, "unknown dtype");
  if (!A || !B || !C) return set_error(DP_EINVAL, "dp_op_gemm_static: NULL operand");
  if (((uintptr_t)A % 16) || ((uintptr_t)B % 16) || ((uintptr_t)C % 16)) return set_error(DP_EALIGN, "dp_op_gemm_static: operands must be 16-byte aligned");
  if (M <= 0 || N <= 0 || K <= 0) return set_error(DP_EINVAL, "gemm: non-positive size");
  // what dp_op_gemm would want as workspace for this problem must fit the static array
  const size_t need = dp_op_gemm_workspace_bytes(M, N, K);
  if (need > (size_t)DP_STATIC_SCRATCH_BYTES)
    return set_errorf(DP_EWORKSPACE, "dp_op_gemm_static: %d x %d x %d needs %zu bytes of split-K scratch, the static scratch holds %zu",
                      M, N, K, need, (size_t)DP_STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  if (int e = scratch_of_current_device(&ws)) return e;
  GemmArgs g;
  memset(&g, 0, sizeof(g));
  g.dtype = dtype; g.A = A; g.B = B; g.M = M; g.N = N; g.K = K; g.lda = lda; g.ldb = ldb; g.a_mc = a_kmajor != 0; g.b_mc = b_kmajor != 0;
  if (out_is_f32) {
    if (bias) return set_error(DP_EUNSUPPORTED, "dp_op_gemm_static: bias with fp32 output is not supported");
    g.out_f32 = (float*)C; g.ldo32 = ldc; g.accumulate = accumulate != 0;
  } else {
    g.out = C; g.ldo = ldc; g.bias = bias;
  }
  // Every split writes its whole partial tile before the reduction pass reads it, so nothing in the
  // array has to start at zero; what an earlier call left there is overwritten or never read.
  g.splitk_ws = (float*)ws; g.splitk_ws_bytes = DP_STATIC_SCRATCH_BYTES;
  g.force_cfg = tile_cfg;
  return launch_gemm(g, (hipStream_t)hip_stream);
}
