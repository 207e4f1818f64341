// pd_linear_fwd_bf16_static: the Linear forward product of pd_linear_fwd_bf16 for callers that cannot allocate
// device memory (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  The split-K
// kernels need scratch for their fp32 partial sums; here it is a file-scope device array that every GPU the library
// runs on holds from load time until the process ends, instead of a workspace argument.
#include <hip/hip_runtime.h>

#include <mutex>

#include "../../include/pd.h"
#include "pd_error.h"
#include "pd_kernels.h"

// 32 MiB: room for the 32 partial sums (the most the split-K kernels ever form) of a 64 x 4096 output.
#define PD_STATIC_SCRATCH_BYTES (32u << 20)
static __device__ __align__(256) unsigned char scratch[PD_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
constexpr int kMaxSplits = 32;  // upper limit of pick_splits / launch_skinny_dma in gemm_bf16.hip
std::mutex g_mu;
float* g_scratch_of_device[kMaxDevices] = {};  // device address of `scratch` on each GPU (every GPU has its own copy)

// The array's name is only a host-side stand-in; its device address on the CURRENT device comes from the runtime,
// once per device.
int scratch_ptr(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return pd::fail(PD_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return pd::fail(PD_EINVAL, "device ordinal %d out of range (max %d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_scratch_of_device[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return pd::fail(PD_EHIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    g_scratch_of_device[dev] = static_cast<float*>(p);
  }
  *out = g_scratch_of_device[dev];
  return PD_OK;
}

}  // namespace

extern "C" {

size_t pd_linear_fwd_bf16_static_max_bytes(void) { return PD_STATIC_SCRATCH_BYTES; }

int pd_linear_fwd_bf16_static(void* stream, const void* x, const void* w, const void* b, void* y, int32_t M, int32_t N,
                              int32_t K, int32_t relu) {
  if (!x || !w || !y) return pd::fail(PD_EINVAL, "null pointer");
  if (M < 1 || N < 1 || K < 1 || (N % 8) || (K % 8)) return pd::fail(PD_EINVAL, "need M,N,K >= 1 and N,K divisible by 8");
  // Sized for the worst case, whatever number of partial sums the kernels then choose: the limit depends on the
  // output shape only, so a caller knows in advance which shapes are served.
  const size_t need = (size_t)kMaxSplits * (size_t)M * (size_t)N * sizeof(float);
  if (need > PD_STATIC_SCRATCH_BYTES)
    return pd::fail(PD_ENOMEM, "pd_linear_fwd_bf16_static serves outputs of at most %zu elements (M * N); %d x %d has %zu: "
                    "use pd_linear_fwd_bf16 with a workspace", (size_t)PD_STATIC_SCRATCH_BYTES / (kMaxSplits * sizeof(float)), M, N,
                    (size_t)M * N);
  float* ws = nullptr;
  const int rc = scratch_ptr(&ws);
  if (rc != PD_OK) return rc;
  // Nothing in the scratch has to start at zero: every partial sum the reducing kernel reads is written by the
  // product kernel of the same call.  (Calls that overlap on one GPU share the array and race.)
  const hipError_t e = pd::linear_fwd_bf16(static_cast<hipStream_t>(stream), static_cast<const pd::bf16_t*>(x),
                                           static_cast<const pd::bf16_t*>(w), static_cast<const pd::bf16_t*>(b),
                                           static_cast<pd::bf16_t*>(y), nullptr, M, N, K, relu != 0, ws, need);
  if (e != hipSuccess) return pd::fail(PD_EHIP, "linear_fwd_bf16: %s", hipGetErrorString(e));
  return PD_OK;
}

}  // extern "C"
