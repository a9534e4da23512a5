// Flat training-state kernels: slice Adam, gradient accumulation, bf16 parameter copy.
// All three are streaming passes bound by HBM bandwidth: 16-byte vector body, scalar
// head/tail around it, coalesced grid-stride order.
#include "common.h"
#include <cmath>

// Every element must see the same instruction sequence whether it sits in the vector
// body or in the scalar head/tail, so fused multiply-add contraction is switched off here.
#pragma clang fp contract(off)

namespace cephalo {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

struct AdamHyper {
  float lr, beta1, beta2, one_minus_beta1, one_minus_beta2, inv_bc1, inv_bc2, eps, weight_decay;
};

// One element's update.  kDecay: the decay term weight_decay * p joins the gradient before the moments are formed.
template <bool kDecay>
__device__ __forceinline__ void adam_element(float& p, float g, float& m, float& v, const AdamHyper& h) {
  if (kDecay) g = g + h.weight_decay * p;
  m = h.beta1 * m + h.one_minus_beta1 * g;
  v = h.beta2 * v + h.one_minus_beta2 * (g * g);
  const float m_hat = m * h.inv_bc1;
  const float v_hat = v * h.inv_bc2;
  p = p - h.lr * (m_hat / (__fsqrt_rn(v_hat) + h.eps));
}

// One wavefront per block, one 16-byte group per lane and buffer: a block's seven accesses are each one 1 KiB run.
// Measured on the 381.6 M-element slice of the largest workload: 5.86 TB/s in this shape, 5.69 with 256 threads,
// 5.50 with 256 threads x 4 groups and a grid-stride loop, 4.8 - 5.1 with persistent blocks over contiguous ranges.
constexpr int kAdamThreads = 64;
// The body starts where p's address is a multiple of this many bytes.  A wavefront's 1 KiB store that starts inside
// a 128-byte line leaves two partly written lines behind, and streaming stores are not merged afterwards: the same
// slice starting 32 bytes into a line runs at 4.5 TB/s instead of 5.5.  256 rather than 128, so that the bf16 copy's
// 512-byte stores (half as many bytes per element) start on a line as well.
constexpr int kAdamAlignBytes = 256;

// Slice = head (scalar, up to 63 elements, until p's address is a multiple of 256 bytes; with all four base pointers
//               congruent modulo 256 that holds for every buffer)
//       + body (nvec groups of 4, 16-byte aligned in every buffer) + tail (scalar, up to 3).
template <bool kLowp, bool kDecay>
__global__ void __launch_bounds__(kAdamThreads)
shard_adam_kernel(float* __restrict__ p, const float* __restrict__ g, float* __restrict__ m,
                  float* __restrict__ v, bf16* __restrict__ p_lowp,
                  int64_t offset, int64_t len, int64_t head, int64_t nvec, AdamHyper h) {
  const int64_t body0 = offset + head;
  f32x4* p4 = reinterpret_cast<f32x4*>(p + body0);
  const f32x4* g4 = reinterpret_cast<const f32x4*>(g + body0);
  f32x4* m4 = reinterpret_cast<f32x4*>(m + body0);
  f32x4* v4 = reinterpret_cast<f32x4*>(v + body0);
  for (int64_t i = (int64_t)blockIdx.x * kAdamThreads + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * kAdamThreads) {
    const f32x4 gg = __builtin_nontemporal_load(g4 + i);
    f32x4 pp = __builtin_nontemporal_load(p4 + i);
    f32x4 mm = __builtin_nontemporal_load(m4 + i);
    f32x4 vv = __builtin_nontemporal_load(v4 + i);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      float pc = pp[c], mc = mm[c], vc = vv[c];
      adam_element<kDecay>(pc, gg[c], mc, vc, h);
      pp[c] = pc; mm[c] = mc; vv[c] = vc;
    }
    __builtin_nontemporal_store(pp, p4 + i);
    __builtin_nontemporal_store(mm, m4 + i);
    __builtin_nontemporal_store(vv, v4 + i);
    if (kLowp) {
      typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
      bf16x4 q;
      q[0] = (bf16)pp[0]; q[1] = (bf16)pp[1]; q[2] = (bf16)pp[2]; q[3] = (bf16)pp[3];
      __builtin_nontemporal_store(q, reinterpret_cast<bf16x4*>(p_lowp + body0) + i);
    }
  }
  // Scalar head and tail: at most 63 + 3 elements, taken by the lanes of block 0.
  if (blockIdx.x == 0) {
    const int64_t tail0 = head + 4 * nvec;  // slice-relative start of the tail
    const int64_t ntail = len - tail0;
    for (int64_t r = threadIdx.x; r < head + ntail; r += kAdamThreads) {
      const int64_t i = offset + (r < head ? r : tail0 + (r - head));
      float pi = p[i], mi = m[i], vi = v[i];
      adam_element<kDecay>(pi, g[i], mi, vi, h);
      p[i] = pi; m[i] = mi; v[i] = vi;
      if (kLowp) p_lowp[i] = (bf16)pi;
    }
  }
}

constexpr int kStreamThreads = 256;
constexpr int kStreamUnroll = 4;

__global__ void __launch_bounds__(kStreamThreads)
grad_accum_kernel(float* __restrict__ acc, const float* __restrict__ g, float scale, int64_t n) {
  const int64_t nvec = n / 4;
  f32x4* a4 = reinterpret_cast<f32x4*>(acc);
  const f32x4* g4 = reinterpret_cast<const f32x4*>(g);
  const int64_t chunk = (int64_t)kStreamThreads * kStreamUnroll;
  for (int64_t base = (int64_t)blockIdx.x * chunk; base < nvec; base += (int64_t)gridDim.x * chunk) {
    f32x4 aa[kStreamUnroll], gg[kStreamUnroll];
#pragma unroll
    for (int u = 0; u < kStreamUnroll; ++u) {
      const int64_t i = base + u * kStreamThreads + threadIdx.x;
      if (i < nvec) { aa[u] = a4[i]; gg[u] = __builtin_nontemporal_load(g4 + i); }
    }
#pragma unroll
    for (int u = 0; u < kStreamUnroll; ++u) {
      const int64_t i = base + u * kStreamThreads + threadIdx.x;
      if (i < nvec) {
        aa[u][0] = aa[u][0] + scale * gg[u][0];
        aa[u][1] = aa[u][1] + scale * gg[u][1];
        aa[u][2] = aa[u][2] + scale * gg[u][2];
        aa[u][3] = aa[u][3] + scale * gg[u][3];
        a4[i] = aa[u];
      }
    }
  }
  if (blockIdx.x == 0 && (int64_t)threadIdx.x < n - 4 * nvec) {
    const int64_t i = 4 * nvec + threadIdx.x;
    acc[i] = acc[i] + scale * g[i];
  }
}

__global__ void __launch_bounds__(kStreamThreads)
cast_bf16_kernel(bf16* __restrict__ dst, const float* __restrict__ src, int64_t n) {
  typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
  const int64_t nvec = n / 4;
  const f32x4* s4 = reinterpret_cast<const f32x4*>(src);
  bf16x4* d4 = reinterpret_cast<bf16x4*>(dst);
  for (int64_t i = (int64_t)blockIdx.x * kStreamThreads + threadIdx.x; i < nvec;
       i += (int64_t)gridDim.x * kStreamThreads) {
    const f32x4 s = s4[i];
    bf16x4 q;
    q[0] = (bf16)s[0]; q[1] = (bf16)s[1]; q[2] = (bf16)s[2]; q[3] = (bf16)s[3];
    d4[i] = q;
  }
  if (blockIdx.x == 0 && (int64_t)threadIdx.x < n - 4 * nvec) {
    const int64_t i = 4 * nvec + threadIdx.x;
    dst[i] = (bf16)src[i];
  }
}

int grid_for(int64_t work_items, int per_block) {
  int64_t blocks = (work_items + per_block - 1) / per_block;
  if (blocks < 1) blocks = 1;
  const int64_t cap = (int64_t)1 << 30;      // (a grid-stride loop takes what lies beyond)
  return (int)(blocks < cap ? blocks : cap);
}

}  // namespace
}  // namespace cephalo

using namespace cephalo;

extern "C" int cephalo_shard_adam(float* p, const float* g, float* m, float* v, void* p_lowp,
                                  int64_t P, int64_t offset, int64_t len,
                                  float lr, float beta1, float beta2, float eps, float weight_decay, int64_t step,
                                  void* stream) {
  if (P < 0 || offset < 0 || len < 0 || offset > P || len > P - offset)
    return fail(CEPHALO_EINVAL, "shard_adam: slice [%lld, %lld+%lld) is not inside [0, %lld)",
                (long long)offset, (long long)offset, (long long)len, (long long)P);
  if (step < 1) return fail(CEPHALO_EINVAL, "shard_adam: step is 1-based, got %lld", (long long)step);
  if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f) || !std::isfinite(lr) ||
      !(weight_decay >= 0.f) || !std::isfinite(weight_decay))
    return fail(CEPHALO_EINVAL, "shard_adam: hyper-parameters out of range (beta1 %g beta2 %g eps %g lr %g weight_decay %g)",
                beta1, beta2, eps, lr, weight_decay);
  if (len == 0) return CEPHALO_OK;
  if (!p || !g || !m || !v) return fail(CEPHALO_EINVAL, "shard_adam: null buffer");
  if (!aligned16(p) || !aligned16(g) || !aligned16(m) || !aligned16(v) || !aligned16(p_lowp))
    return fail(CEPHALO_EINVAL, "shard_adam: base pointers must be 16-byte aligned");
  AdamHyper h;
  h.lr = lr; h.beta1 = beta1; h.beta2 = beta2; h.eps = eps; h.weight_decay = weight_decay;
  h.one_minus_beta1 = 1.0f - beta1;
  h.one_minus_beta2 = 1.0f - beta2;
  h.inv_bc1 = (float)(1.0 / (1.0 - std::pow((double)beta1, (double)step)));
  h.inv_bc2 = (float)(1.0 / (1.0 - std::pow((double)beta2, (double)step)));
  // elements before p's address reaches a multiple of kAdamAlignBytes (p is 16-byte aligned, so the count is whole
  // and the body is 16-byte aligned in all four buffers)
  const uintptr_t first = reinterpret_cast<uintptr_t>(p) + (uintptr_t)offset * 4;
  int64_t head = (int64_t)((kAdamAlignBytes - first % kAdamAlignBytes) % kAdamAlignBytes) / 4;
  if (head > len) head = len;
  const int64_t nvec = (len - head) / 4;
  const int grid = grid_for(nvec, kAdamThreads);
  hipStream_t s = static_cast<hipStream_t>(stream);
  bf16* lp = static_cast<bf16*>(p_lowp);
  const bool decay = weight_decay != 0.f;
  if (lp && decay) shard_adam_kernel<true, true><<<grid, kAdamThreads, 0, s>>>(p, g, m, v, lp, offset, len, head, nvec, h);
  else if (lp) shard_adam_kernel<true, false><<<grid, kAdamThreads, 0, s>>>(p, g, m, v, lp, offset, len, head, nvec, h);
  else if (decay) shard_adam_kernel<false, true><<<grid, kAdamThreads, 0, s>>>(p, g, m, v, nullptr, offset, len, head, nvec, h);
  else shard_adam_kernel<false, false><<<grid, kAdamThreads, 0, s>>>(p, g, m, v, nullptr, offset, len, head, nvec, h);
  CEPHALO_CHECK_LAUNCH("shard_adam");
  return CEPHALO_OK;
}

extern "C" int cephalo_grad_accum(float* acc, const float* g, float scale, int64_t n, void* stream) {
  if (n < 0) return fail(CEPHALO_EINVAL, "grad_accum: n = %lld < 0", (long long)n);
  if (n == 0) return CEPHALO_OK;
  if (!acc || !g) return fail(CEPHALO_EINVAL, "grad_accum: null buffer");
  if (!aligned16(acc) || !aligned16(g)) return fail(CEPHALO_EINVAL, "grad_accum: pointers must be 16-byte aligned");
  const int grid = grid_for(n / 4, kStreamThreads * kStreamUnroll);
  grad_accum_kernel<<<grid, kStreamThreads, 0, static_cast<hipStream_t>(stream)>>>(acc, g, scale, n);
  CEPHALO_CHECK_LAUNCH("grad_accum");
  return CEPHALO_OK;
}

namespace cephalo {
int launch_cast_bf16(bf16* dst, const float* src, int64_t n, hipStream_t s) {
  if (n <= 0) return CEPHALO_OK;
  const int grid = grid_for(n / 4, kStreamThreads);
  cast_bf16_kernel<<<grid, kStreamThreads, 0, s>>>(dst, src, n);
  CEPHALO_CHECK_LAUNCH("cast_bf16");
  return CEPHALO_OK;
}
}  // namespace cephalo

extern "C" int cephalo_cast_bf16(void* dst, const float* src, int64_t n, void* stream) {
  if (n < 0) return fail(CEPHALO_EINVAL, "cast_bf16: n = %lld < 0", (long long)n);
  if (n == 0) return CEPHALO_OK;
  if (!dst || !src) return fail(CEPHALO_EINVAL, "cast_bf16: null buffer");
  if (!aligned16(dst) || !aligned16(src)) return fail(CEPHALO_EINVAL, "cast_bf16: pointers must be 16-byte aligned");
  const int grid = grid_for(n / 4, kStreamThreads);
  cast_bf16_kernel<<<grid, kStreamThreads, 0, static_cast<hipStream_t>(stream)>>>(static_cast<bf16*>(dst), src, n);
  CEPHALO_CHECK_LAUNCH("cast_bf16");
  return CEPHALO_OK;
}
