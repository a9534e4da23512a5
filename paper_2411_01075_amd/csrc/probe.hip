// Measurement probes: what the matrix cores and the memory system of the device at hand sustain, for the benchmark to
// quote beside the published peaks.  Not used by any computation.
#include "common.h"

using namespace cephalo;

namespace {

typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// A stream of v_mfma_f32_16x16x32_bf16 on operands held in registers: the wavefront tile of the GEMM kernel (4 row
// fragments x 8 column fragments, 32 accumulators of 4 registers), no LDS and no memory traffic inside the loop.  The
// operands come from `seed` (the caller fills it with random bf16 values: the rate depends on the data, zeros run
// faster than the chip can sustain on real operands).
// (Eight wavefronts per block as in the GEMM kernel, so that the accumulators stay in the ordinary register file; the
// loop is kept rolled and closed by a scheduling barrier, otherwise the compiler rotates the accumulators through copies
// that throttle the stream.)
__global__ void __launch_bounds__(512) mfma_stream_kernel(const bf16x8* __restrict__ seed, int iters, float* __restrict__ sink) {
  bf16x8 fa[4], fb[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) fa[i] = seed[(i * 512 + threadIdx.x) & 4095];
#pragma unroll
  for (int j = 0; j < 8; ++j) fb[j] = seed[((4 + j) * 512 + threadIdx.x + 64 * (blockIdx.x & 3)) & 4095];
  f32x4 acc[4][8];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
  f32x4 t = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) t += acc[i][j];
  if (t[0] + t[1] + t[2] + t[3] == 1.2345678f) sink[0] = t[0];      // keeps the products alive
}

// mode 0: read n16 16-byte vectors of src (summed), 1: write them to dst, 2: copy src to dst.  Streaming accesses,
// 256 threads x 4 vectors per block, one pass.
template <int MODE>
__global__ void __launch_bounds__(256) stream_kernel(f32x4* __restrict__ dst, const f32x4* __restrict__ src, int64_t n16, float* __restrict__ sink) {
  const int64_t base = (int64_t)blockIdx.x * 1024;
  f32x4 x[4], acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int64_t i = base + u * 256 + threadIdx.x;
    if (i < n16) x[u] = MODE == 1 ? f32x4{1.f, 2.f, 3.f, 4.f} : __builtin_nontemporal_load(src + i);
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int64_t i = base + u * 256 + threadIdx.x;
    if (i < n16) { if (MODE == 0) acc += x[u]; else __builtin_nontemporal_store(x[u], dst + i); }
  }
  if (MODE == 0 && acc[0] + acc[1] + acc[2] + acc[3] == 1.2345678f) sink[0] = acc[0];
}

}  // namespace

extern "C" int cephalo_probe_mfma(const void* seed_bf16, int32_t blocks, int32_t iters, float* sink, double* flops_out, void* stream) {
  if (!seed_bf16 || !sink || blocks <= 0 || iters <= 0) return fail(CEPHALO_EINVAL, "probe_mfma: bad arguments");
  if (!aligned16(seed_bf16)) return fail(CEPHALO_EINVAL, "probe_mfma: seed must be 16-byte aligned");
  mfma_stream_kernel<<<blocks, 512, 0, static_cast<hipStream_t>(stream)>>>(static_cast<const bf16x8*>(seed_bf16), iters, sink);
  CEPHALO_CHECK_LAUNCH("probe_mfma");
  if (flops_out) *flops_out = (double)blocks * 8.0 * iters * 32.0 * (2.0 * 16 * 16 * 32);      // wavefronts x products x flops
  return CEPHALO_OK;
}

extern "C" int cephalo_probe_stream(int32_t mode, void* dst, const void* src, int64_t bytes, float* sink, void* stream) {
  if (mode < 0 || mode > 2 || bytes <= 0 || bytes % 16 != 0 || !sink) return fail(CEPHALO_EINVAL, "probe_stream: bad arguments");
  if ((mode != 1 && !src) || (mode != 0 && !dst) || !aligned16(dst) || !aligned16(src)) return fail(CEPHALO_EINVAL, "probe_stream: bad buffers");
  const int64_t n16 = bytes / 16;
  const int64_t blocks = (n16 + 1023) / 1024;
  if (blocks > 0x7fffffff) return fail(CEPHALO_EUNSUPPORTED, "probe_stream: too many bytes");
  hipStream_t s = static_cast<hipStream_t>(stream);
  f32x4* d = static_cast<f32x4*>(dst);
  const f32x4* r = static_cast<const f32x4*>(src);
  if (mode == 0) stream_kernel<0><<<(int)blocks, 256, 0, s>>>(d, r, n16, sink);
  else if (mode == 1) stream_kernel<1><<<(int)blocks, 256, 0, s>>>(d, r, n16, sink);
  else stream_kernel<2><<<(int)blocks, 256, 0, s>>>(d, r, n16, sink);
  CEPHALO_CHECK_LAUNCH("probe_stream");
  return CEPHALO_OK;
}
