// Plain LDS-tiled GEMM with fp32 FMA arithmetic, any operand strides, ragged edges allowed.
// It serves the fp32 workload (whose sizes are launch-bound, not throughput-bound) and
// shapes the MFMA kernel does not take.  64x64 output tile, 16-deep k-slab, 4x4 per thread.
#include "kernels.h"

namespace cephalo {
namespace {

constexpr int TM = 64, TN = 64, TK = 16, kThreads = 256;

template <typename T>
__global__ void __launch_bounds__(kThreads) gemm_simple_kernel(GemmArgs<T> a) {
  __shared__ float As[TK][TM + 4];
  __shared__ float Bs[TK][TN + 4];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  const bool a_kfast = (a.a_cs == 1), b_kfast = (a.b_cs == 1);
  for (int k0 = 0; k0 < a.K; k0 += TK) {
#pragma unroll
    for (int i = 0; i < (TM * TK) / kThreads; ++i) {
      const int idx = tid + kThreads * i;
      const int k = a_kfast ? (idx % TK) : (idx / TM);
      const int m = a_kfast ? (idx / TK) : (idx % TM);
      float val = 0.f;
      if (m0 + m < a.M && k0 + k < a.K) val = (float)a.A[(int64_t)(m0 + m) * a.a_rs + (int64_t)(k0 + k) * a.a_cs];
      As[k][m] = val;
    }
#pragma unroll
    for (int i = 0; i < (TN * TK) / kThreads; ++i) {
      const int idx = tid + kThreads * i;
      const int k = b_kfast ? (idx % TK) : (idx / TN);
      const int n = b_kfast ? (idx / TK) : (idx % TN);
      float val = 0.f;
      if (n0 + n < a.N && k0 + k < a.K) val = (float)a.B[(int64_t)(n0 + n) * a.b_rs + (int64_t)(k0 + k) * a.b_cs];
      Bs[k][n] = val;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < TK; ++k) {
      float av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) av[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) bv[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += av[i] * bv[j];
    }
    __syncthreads();
  }

#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= a.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= a.N) continue;
      const int64_t o = a.epi == EPI_GRAD ? (int64_t)m * a.N + n : (int64_t)m * (a.ldc ? a.ldc : a.N) + n;
      float v = acc[i][j];
      auto put = [&](float r) { if (a.Cf) a.Cf[o] = r; else a.C[o] = (T)r; };   // fp32 output if Cf is set
      switch (a.epi) {
        case EPI_NONE: case EPI_NONE_HEAD: put(v); break;
        case EPI_BIAS: put(v + (float)a.bias[n]); break;
        case EPI_BIAS_RESID: put(v + (a.bias ? (float)a.bias[n] : 0.f) + (a.Rf ? a.Rf[o] : (float)a.R[o])); break;
        case EPI_BIAS_GELU: {
          const float z = v + (float)a.bias[n];
          a.Z[o] = (T)z;
          a.C[o] = (T)gelu_f(z);
        } break;
        case EPI_DGELU: a.C[o] = (T)(v * gelu_grad_f((float)a.Z[o])); break;
        case EPI_BIAS_GELU_DERIV: {
          const float z = v + (float)a.bias[n];
          reinterpret_cast<typename FactorOf<T>::type*>(a.Z)[o] = (typename FactorOf<T>::type)gelu_grad_f(z);
          a.C[o] = (T)gelu_f(z);
        } break;
        case EPI_MUL: a.C[o] = (T)(v * (float)reinterpret_cast<const typename FactorOf<T>::type*>(a.Z)[o]); break;
        case EPI_ROPE: {
          // the partner column's product sits in the same thread (columns come in aligned groups of four)
          float r = v;
          if (n < a.rot_cols) {
            const float* cs = a.rot + ((int64_t)(m % a.rot_S) * (a.rot_d / 2) + (n % a.rot_d) / 2) * 2;
            r = (j & 1) ? acc[i][j ^ 1] * cs[1] + v * cs[0] : v * cs[0] - acc[i][j ^ 1] * cs[1];
          }
          put(r);
        } break;
        case EPI_DSWIGLU: {
          float dg, du;
          swiglu_grad((float)a.Z[o], (float)a.Z[o + a.N], v, dg, du);
          a.C[o] = (T)dg;
          a.C[o + a.N] = (T)du;
        } break;
        case EPI_GRAD: a.G[o] = (a.accumulate ? a.G[o] : 0.f) + a.scale * v; break;
      }
    }
  }
}

}  // namespace

template <typename T>
int launch_gemm_simple(const GemmArgs<T>& a, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return fail(CEPHALO_EINVAL, "gemm: empty problem %dx%dx%d", a.M, a.N, a.K);
  dim3 grid((a.N + TN - 1) / TN, (a.M + TM - 1) / TM);
  gemm_simple_kernel<T><<<grid, kThreads, 0, s>>>(a);
  CEPHALO_CHECK_LAUNCH("gemm_simple");
  return CEPHALO_OK;
}

template int launch_gemm_simple<float>(const GemmArgs<float>&, hipStream_t);
template int launch_gemm_simple<bf16>(const GemmArgs<bf16>&, hipStream_t);

}  // namespace cephalo
