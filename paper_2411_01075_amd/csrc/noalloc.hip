// The one entry point of the library that neither allocates nor asks its caller for a work area: the weight gradient
// of a linear layer with its split-contraction partial sums in a fixed device array.  For callers that cannot
// allocate: code under HIP graph capture, tight serving loops, harnesses that forbid allocation.
#include "layer_impl.h"
#include <mutex>

using namespace cephalo;

// Partial sums of a split token axis: `splits` fp32 images of the [N, K] gradient, written by the first pass of a call
// and read back by its second pass.  One copy per GPU, held from the moment the library is loaded on that GPU until
// the process ends.  In host code this name is only a handle for hipGetSymbolAddress: it is not a device address.
static __device__ __align__(256) unsigned char scratch[CEPHALO_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void* scratch_of_device[kMaxDevices];      // device address of `scratch` on each GPU, asked for once per GPU

// The current device's copy of `scratch`.  Each GPU has its own copy at its own address, so the address is looked up
// with that GPU current and kept per GPU.
int current_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(CEPHALO_EHIP, "linear_wgrad_static: hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(CEPHALO_EUNSUPPORTED, "linear_wgrad_static: device index %d is outside [0, %d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_of_device[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p)
      return fail(CEPHALO_EHIP, "linear_wgrad_static: hipGetSymbolAddress on device %d: %s", dev, hipGetErrorString(e));
    scratch_of_device[dev] = p;
  }
  *out = scratch_of_device[dev];
  return CEPHALO_OK;
}
}  // namespace

extern "C" int cephalo_op_linear_wgrad_static(int32_t dtype, const void* dY, const void* X, int32_t T, int32_t N, int32_t K,
                                              float* G, float scale, int32_t accumulate, void* stream) {
  if (T <= 0 || N <= 0 || K <= 0) return fail(CEPHALO_EINVAL, "linear_wgrad_static: sizes %d x %d x %d must be positive", T, N, K);
  if (!dY || !X || !G) return fail(CEPHALO_EINVAL, "linear_wgrad_static: null buffer");
  if (accumulate != 0 && accumulate != 1) return fail(CEPHALO_EINVAL, "linear_wgrad_static: accumulate must be 0 or 1");
  if (dtype != CEPHALO_F32 && dtype != CEPHALO_BF16) return fail(CEPHALO_EINVAL, "linear_wgrad_static: unknown dtype %d", dtype);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dtype == CEPHALO_F32)      // the fp32 kernel does not split the contraction: no scratch at all
    return wgrad<float>(static_cast<const float*>(dY), static_cast<const float*>(X), T, N, K, G, scale, accumulate, nullptr, s);
  const int splits = gemm_grad_splits(N, K, T);
  const size_t need = splits > 1 ? (size_t)splits * N * K * sizeof(float) : 0;
  if (need > (size_t)CEPHALO_NOALLOC_SCRATCH_BYTES)
    return fail(CEPHALO_EWORKSPACE, "linear_wgrad_static: a %d x %d gradient over %d tokens is summed in %d pieces and needs %zu B of partial "
                "sums; the fixed area holds %zu B (use cephalo_op_linear_wgrad with a work area of its own)",
                N, K, T, splits, need, (size_t)CEPHALO_NOALLOC_SCRATCH_BYTES);
  void* part = nullptr;
  if (need) TRY(current_scratch(&part));
  // Nothing in the area has to start at zero: every partial tile the second pass reads was written by the first pass
  // of this same call.
  return wgrad<bf16>(static_cast<const bf16*>(dY), static_cast<const bf16*>(X), T, N, K, G, scale, accumulate, static_cast<float*>(part), s);
}
