// Plain attention forward/backward with fp32 arithmetic: one wavefront per (row, head, sample),
// scores of the whole row held in LDS.  It serves the fp32 workload and is the in-library
// cross-check for the MFMA attention; cost is O(S^2 d) per head with no operand reuse.
#include "kernels.h"

namespace cephalo {
namespace {

constexpr int kMaxHeadDim = 128;

// dynamic LDS: float row[S]  (+ a second float row[S] in the key-side backward)
template <typename T>
__global__ void __launch_bounds__(64)
attn_fwd_kernel(const T* __restrict__ qkv, T* __restrict__ O, float* __restrict__ lse,
                int S, int H, int A, int causal) {
  extern __shared__ float smem[];
  __shared__ float qs[kMaxHeadDim];
  float* p = smem;
  const int s = blockIdx.x, a = blockIdx.y, n = blockIdx.z, lane = threadIdx.x;
  const int d = H / A;
  const float scale = 1.0f / sqrtf((float)d);
  const int64_t ld = 3 * (int64_t)H;
  const T* base = qkv + (int64_t)n * S * ld + a * d;
  for (int e = lane; e < d; e += 64) qs[e] = (float)base[(int64_t)s * ld + e];
  __syncthreads();
  const int last = causal ? s : S - 1;
  float mx = -INFINITY;
  for (int t = lane; t <= last; t += 64) {
    const T* kr = base + (int64_t)t * ld + H;
    float z = 0.f;
    for (int e = 0; e < d; ++e) z += qs[e] * (float)kr[e];
    z *= scale;
    p[t] = z;
    mx = fmaxf(mx, z);
  }
  mx = wave_max(mx);
  float sum = 0.f;
  for (int t = lane; t <= last; t += 64) {
    const float e = expf(p[t] - mx);
    p[t] = e;
    sum += e;
  }
  sum = wave_sum(sum);
  __syncthreads();
  const float inv = 1.0f / sum;
  for (int e = lane; e < d; e += 64) {
    float o = 0.f;
    for (int t = 0; t <= last; ++t) o += p[t] * (float)base[(int64_t)t * ld + 2 * H + e];
    O[((int64_t)n * S + s) * H + a * d + e] = (T)(o * inv);
  }
  if (lane == 0) lse[((int64_t)n * A + a) * S + s] = mx + logf(sum);
}

// dvec[n,a,s] = sum_e dO[s, a*d+e] * O[s, a*d+e]
template <typename T>
__global__ void __launch_bounds__(64)
attn_dvec_kernel(const T* __restrict__ O, const T* __restrict__ dO, float* __restrict__ dvec, int S, int H, int A) {
  const int s = blockIdx.x, a = blockIdx.y, n = blockIdx.z, lane = threadIdx.x;
  const int d = H / A;
  const int64_t o = ((int64_t)n * S + s) * H + a * d;
  float acc = 0.f;
  for (int e = lane; e < d; e += 64) acc += (float)dO[o + e] * (float)O[o + e];
  acc = wave_sum(acc);
  if (lane == 0) dvec[((int64_t)n * A + a) * S + s] = acc;
}

// dQ[s] = scale * sum_t dZ[s,t] K[t],  dZ = P * (dP - dvec[s]),  dP[s,t] = dO[s] . V[t]
template <typename T>
__global__ void __launch_bounds__(64)
attn_dq_kernel(const T* __restrict__ qkv, const T* __restrict__ dO, const float* __restrict__ lse,
               const float* __restrict__ dvec, T* __restrict__ dqkv, int S, int H, int A, int causal) {
  extern __shared__ float smem[];
  __shared__ float qs[kMaxHeadDim], dos[kMaxHeadDim];
  float* dz = smem;
  const int s = blockIdx.x, a = blockIdx.y, n = blockIdx.z, lane = threadIdx.x;
  const int d = H / A;
  const float scale = 1.0f / sqrtf((float)d);
  const int64_t ld = 3 * (int64_t)H;
  const T* base = qkv + (int64_t)n * S * ld + a * d;
  for (int e = lane; e < d; e += 64) {
    qs[e] = (float)base[(int64_t)s * ld + e];
    dos[e] = (float)dO[((int64_t)n * S + s) * H + a * d + e];
  }
  __syncthreads();
  const int last = causal ? s : S - 1;
  const float l = lse[((int64_t)n * A + a) * S + s], dv = dvec[((int64_t)n * A + a) * S + s];
  for (int t = lane; t <= last; t += 64) {
    const T* kr = base + (int64_t)t * ld + H;
    const T* vr = base + (int64_t)t * ld + 2 * H;
    float z = 0.f, dp = 0.f;
    for (int e = 0; e < d; ++e) { z += qs[e] * (float)kr[e]; dp += dos[e] * (float)vr[e]; }
    dz[t] = expf(z * scale - l) * (dp - dv);
  }
  __syncthreads();
  for (int e = lane; e < d; e += 64) {
    float acc = 0.f;
    for (int t = 0; t <= last; ++t) acc += dz[t] * (float)base[(int64_t)t * ld + H + e];
    dqkv[((int64_t)n * S + s) * ld + a * d + e] = (T)(acc * scale);
  }
}

// dV[t] = sum_s P[s,t] dO[s],  dK[t] = scale * sum_s dZ[s,t] Q[s]
template <typename T>
__global__ void __launch_bounds__(64)
attn_dkv_kernel(const T* __restrict__ qkv, const T* __restrict__ dO, const float* __restrict__ lse,
                const float* __restrict__ dvec, T* __restrict__ dqkv, int S, int H, int A, int causal) {
  extern __shared__ float smem[];
  __shared__ float ks[kMaxHeadDim], vs[kMaxHeadDim];
  float* ps = smem;
  float* dz = smem + S;
  const int t = blockIdx.x, a = blockIdx.y, n = blockIdx.z, lane = threadIdx.x;
  const int d = H / A;
  const float scale = 1.0f / sqrtf((float)d);
  const int64_t ld = 3 * (int64_t)H;
  const T* base = qkv + (int64_t)n * S * ld + a * d;
  for (int e = lane; e < d; e += 64) {
    ks[e] = (float)base[(int64_t)t * ld + H + e];
    vs[e] = (float)base[(int64_t)t * ld + 2 * H + e];
  }
  __syncthreads();
  const int first = causal ? t : 0;
  for (int s = first + lane; s < S; s += 64) {
    const T* qr = base + (int64_t)s * ld;
    const T* dor = dO + ((int64_t)n * S + s) * H + a * d;
    float z = 0.f, dp = 0.f;
    for (int e = 0; e < d; ++e) { z += (float)qr[e] * ks[e]; dp += (float)dor[e] * vs[e]; }
    const float pr = expf(z * scale - lse[((int64_t)n * A + a) * S + s]);
    ps[s] = pr;
    dz[s] = pr * (dp - dvec[((int64_t)n * A + a) * S + s]);
  }
  __syncthreads();
  for (int e = lane; e < d; e += 64) {
    float av = 0.f, ak = 0.f;
    for (int s = first; s < S; ++s) {
      av += ps[s] * (float)dO[((int64_t)n * S + s) * H + a * d + e];
      ak += dz[s] * (float)base[(int64_t)s * ld + e];
    }
    dqkv[((int64_t)n * S + t) * ld + 2 * H + a * d + e] = (T)av;
    dqkv[((int64_t)n * S + t) * ld + H + a * d + e] = (T)(ak * scale);
  }
}

}  // namespace

template <typename T>
int launch_attn_fwd_simple(const T* qkv, T* O, float* lse, int m, int S, int H, int A, int causal, hipStream_t s) {
  if (H / A > kMaxHeadDim) return fail(CEPHALO_EUNSUPPORTED, "attention: head dim %d > %d", H / A, kMaxHeadDim);
  if ((size_t)S * 2 * sizeof(float) > 60000) return fail(CEPHALO_EUNSUPPORTED, "attention (plain kernel): seq %d too long", S);
  dim3 grid(S, A, m);
  attn_fwd_kernel<T><<<grid, 64, S * sizeof(float), s>>>(qkv, O, lse, S, H, A, causal);
  CEPHALO_CHECK_LAUNCH("attn_fwd");
  return CEPHALO_OK;
}

template <typename T>
int launch_attn_bwd_simple(const T* qkv, const T* O, const T* dO, const float* lse, float* dvec, T* dqkv,
                           int m, int S, int H, int A, int causal, hipStream_t s) {
  if (H / A > kMaxHeadDim) return fail(CEPHALO_EUNSUPPORTED, "attention: head dim %d > %d", H / A, kMaxHeadDim);
  if ((size_t)S * 2 * sizeof(float) > 60000) return fail(CEPHALO_EUNSUPPORTED, "attention (plain kernel): seq %d too long", S);
  dim3 grid(S, A, m);
  attn_dvec_kernel<T><<<grid, 64, 0, s>>>(O, dO, dvec, S, H, A);
  attn_dq_kernel<T><<<grid, 64, S * sizeof(float), s>>>(qkv, dO, lse, dvec, dqkv, S, H, A, causal);
  attn_dkv_kernel<T><<<grid, 64, 2 * S * sizeof(float), s>>>(qkv, dO, lse, dvec, dqkv, S, H, A, causal);
  CEPHALO_CHECK_LAUNCH("attn_bwd");
  return CEPHALO_OK;
}

template int launch_attn_fwd_simple<float>(const float*, float*, float*, int, int, int, int, int, hipStream_t);
template int launch_attn_fwd_simple<bf16>(const bf16*, bf16*, float*, int, int, int, int, int, hipStream_t);
template int launch_attn_bwd_simple<float>(const float*, const float*, const float*, const float*, float*, float*,
                                           int, int, int, int, int, hipStream_t);
template int launch_attn_bwd_simple<bf16>(const bf16*, const bf16*, const bf16*, const float*, float*, bf16*,
                                          int, int, int, int, int, hipStream_t);

}  // namespace cephalo
