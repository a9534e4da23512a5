// Internal launch interface between the layer driver and the kernel files.
// Every function enqueues on `s` and returns; shapes were validated by the caller.
#pragma once
#include "common.h"

namespace cephalo {

// ---------------------------------------------------------------------------------------
// Element type helpers: 16-byte vectors of the activation type, widened to float.
template <typename T> struct Vec;
template <> struct Vec<float> {
  static constexpr int N = 4;
  typedef float raw __attribute__((ext_vector_type(4)));
};
template <> struct Vec<bf16> {
  static constexpr int N = 8;
  typedef bf16 raw __attribute__((ext_vector_type(8)));
};

// A saved epilogue factor (the GELU derivative kept by the forward for the backward) multiplies an fp32 accumulator;
// it is never a matrix operand.  In the bf16 mode it is therefore stored as an IEEE half: the same two bytes, three
// more significand bits (it lies in [-0.13, 1.13], far inside the half range), one bf16 rounding less on the way to
// every gradient upstream of the feed-forward block.
typedef _Float16 f16;
template <> struct Vec<f16> {
  static constexpr int N = 8;
  typedef f16 raw __attribute__((ext_vector_type(8)));
};
template <typename T> struct FactorOf { typedef T type; };
template <> struct FactorOf<bf16> { typedef f16 type; };

template <typename T>
__device__ __forceinline__ void load_vec(const T* p, float (&out)[Vec<T>::N]) {
  typename Vec<T>::raw r = *reinterpret_cast<const typename Vec<T>::raw*>(p);
#pragma unroll
  for (int i = 0; i < Vec<T>::N; ++i) out[i] = (float)r[i];
}
template <typename T>
__device__ __forceinline__ void store_vec(T* p, const float (&in)[Vec<T>::N]) {
  typename Vec<T>::raw r;
#pragma unroll
  for (int i = 0; i < Vec<T>::N; ++i) r[i] = (T)in[i];
  *reinterpret_cast<typename Vec<T>::raw*>(p) = r;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// exact GELU and its derivative, fp32
__device__ __forceinline__ float gelu_f(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752440f)); }
__device__ __forceinline__ float gelu_grad_f(float z) {
  const float cdf = 0.5f * (1.0f + erff(z * 0.70710678118654752440f));
  const float pdf = 0.39894228040143267794f * __expf(-0.5f * z * z);
  return cdf + z * pdf;
}


// Branch-free exact-form GELU for the bf16 epilogues.  erf(|x|) = 1 - (a1 t + ... + a5 t^5) exp(-x^2),
// t = 1/(1 + p|x|)  (Abramowitz & Stegun 7.1.26, absolute error <= 1.5e-7: three orders of magnitude
// below one bf16 rounding of the result).  With x = z/sqrt(2) the exponential exp(-z^2/2) is shared
// between Phi(z) and the density phi(z) of the derivative.
__device__ __forceinline__ void gelu_terms_fast(float z, float& cdf, float& pdf_unnorm) {
  const float ax = fabsf(z) * 0.70710678118654752440f;
  const float t = __builtin_amdgcn_rcpf(1.0f + 0.3275911f * ax);
  const float e = __expf(-ax * ax);                   // exp(-z^2/2)
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  const float erf_abs = 1.0f - poly * e;
  cdf = 0.5f * (1.0f + copysignf(erf_abs, z));
  pdf_unnorm = e;
}
__device__ __forceinline__ float gelu_fast(float z) {
  float cdf, e;
  gelu_terms_fast(z, cdf, e);
  return z * cdf;
}
__device__ __forceinline__ float gelu_grad_fast(float z) {
  float cdf, e;
  gelu_terms_fast(z, cdf, e);
  return cdf + z * (0.39894228040143267794f * e);
}
// both at once: gelu(z) and gelu'(z)
__device__ __forceinline__ void gelu_and_grad_fast(float z, float& y, float& dy) {
  float cdf, e;
  gelu_terms_fast(z, cdf, e);
  y = z * cdf;
  dy = cdf + z * (0.39894228040143267794f * e);
}

// ---------------------------------------------------------------------------------------
// GEMM:  C[M,N] = sum_k A(m,k) * B(n,k)  followed by an epilogue.
// Operand element (m,k) of A sits at A[m*a_rs + k*a_cs]; one of the two strides is 1.
// Likewise B(n,k) at B[n*b_rs + k*b_cs].
enum Epilogue {
  EPI_NONE = 0,        // C = acc
  EPI_BIAS = 1,        // C = acc + bias[n]
  EPI_BIAS_RESID = 2,  // C = acc + bias[n] + R[m,n]
  EPI_BIAS_GELU = 3,   // Z = acc + bias[n] ; C = gelu(Z)          (Z and C both stored)
  EPI_DGELU = 4,       // C = acc * gelu'(Z[m,n])
  EPI_GRAD = 5,        // G[m,n] = (accumulate ? G[m,n] : 0) + scale * acc     (G fp32)
  EPI_ROPE = 7,        // C = acc with each pair of columns (2i, 2i+1) below rot_cols turned by the rotary angle of its
                       //   row's position m % rot_S and of its place in the head: (e, o) -> (e cos - o sin, e sin + o cos)
  EPI_BIAS_GELU_DERIV = 9,  // z = acc + bias[n];  C = gelu(z);  Z = gelu'(z)   (the derivative is saved in place of the pre-activation:
                            //   Phi(z) and exp(-z^2/2) are at hand in the forward, and the backward becomes EPI_MUL)
  EPI_NONE_HEAD = 11,       // as EPI_NONE; the vocabulary projections of a stack's head use it, so that they are kernels of their own
                            //   in a profile and do not mix into the figures of the layers' projections
  EPI_MUL = 10,             // C = acc * Z[m,n]
  EPI_DSWIGLU = 8,     // gated SiLU backward, acc = dh[m,n], n < N = F; Z and C are [M, 2N] = [gate | up] (pitch ldc >= 2N):
                       //   C[m,n] = acc * Z[m,N+n] * silu'(Z[m,n]);  C[m,N+n] = acc * silu(Z[m,n])
};

// gated SiLU feed-forward h = silu(g) * u: gradients with respect to g and u given d = dL/dh
__device__ __forceinline__ void swiglu_grad(float g, float u, float d, float& dg, float& du) {
  const float sg = 1.0f / (1.0f + __expf(-g));
  dg = d * u * sg * (1.0f + g * (1.0f - sg));
  du = d * g * sg;
}

template <typename T>
struct GemmArgs {
  const T* A; int64_t a_rs, a_cs;
  const T* B; int64_t b_rs, b_cs;
  int M, N, K;
  int epi;
  T* C;            // [M,N] row-major with row pitch ldc (unused for EPI_GRAD)
  int ldc;         // row pitch of C, R and Z in elements; 0 means N.  If N is not a multiple of 8 the pitch must cover N
                   // rounded up to 8; the padding columns are then written too (with the products of zero B rows)
  const T* bias;   // [N]
  const T* R;      // [M,N] residual
  const float* Rf; // if set, EPI_BIAS_RESID reads its residual from here in fp32 (pitch ldc) instead of R
  float* Cf;       // if set, EPI_NONE / EPI_BIAS / EPI_BIAS_RESID write their result here in fp32 (pitch ldc) instead of C
  T* Z;            // [M,N] pre-activation: written by EPI_BIAS_GELU, read by EPI_DGELU ([M,2N], read by EPI_DSWIGLU);
                   // EPI_BIAS_GELU_DERIV writes gelu'(z) here and EPI_MUL reads it as a factor
  float* G;        // [M,N] fp32 gradient (EPI_GRAD)
  float scale;
  int accumulate;
  const float* rot;   // EPI_ROPE: [rot_S, rot_d/2, 2] = (cos, sin); rot_d: head width (divides rot_cols, multiple of 8)
  int rot_S, rot_d, rot_cols;
  // EPI_GRAD with the contraction split over `splits` > 1 blocks per tile (long token axes, few output tiles): each
  // block writes its partial tile to part[split][M][N] and a second pass adds the partials in split order (fixed
  // order: reproducible) and applies scale / accumulate.  part holds splits*M*N floats.
  int splits;
  float* part;
  // EPI_GRAD, optional: the sums of A's rows over the contracted axis as well (beside a weight gradient dW = dY^T X these
  // are the column sums of dY, the bias gradient), rowsum[m] = (accumulate ? rowsum[m] : 0) + scale * sum_k A[m][k].
  // The row fragments pass through the registers anyway; each k-slab of a tile row is summed by exactly one wavefront
  // among the blocks of that row, with one extra MFMA per fragment, into rowsum_part (gemm_rowsum_part_bytes(M, N)
  // bytes), and a second pass adds the pieces in a fixed order.  Only the MFMA path takes it: ask gemm_mfma_takes first.
  float* rowsum;
  float* rowsum_part;
  size_t rowsum_part_bytes;
};
size_t gemm_rowsum_part_bytes(int M, int N);            // upper bound over tile shapes and splits
bool gemm_mfma_takes(const GemmArgs<bf16>& a);          // whether launch_gemm_mfma runs this problem on its MFMA kernels

// Number of pieces the weight-gradient GEMM G[M,N] = sum over K tokens would like the token axis cut into (1: none).
int gemm_grad_splits(int M, int N, int K);

template <typename T> int launch_gemm_simple(const GemmArgs<T>& a, hipStream_t s);
int launch_gemm_mfma(const GemmArgs<bf16>& a, hipStream_t s);  // bf16 operands, MFMA, fp32 accumulate
// While one of these is alive on a thread, that thread's GEMM launches choose their tiles for 256 / `kernels` compute
// units: the caller runs that many kernels side by side on different streams (results do not depend on the choice).
struct GemmSideBySide {
  explicit GemmSideBySide(int kernels);
  ~GemmSideBySide();
  void now(int kernels);       // change the number for the launches that follow
  int before;
};
int gemm_set_side_by_side(int kernels);   // the same number, set for good; returns the previous value
int64_t gemm_general_count();   // calls of launch_gemm_mfma that ended in launch_gemm_simple

// ---------------------------------------------------------------------------------------
// LayerNorm over the last axis of x[rows, H].  The residual stream x is fp32; the output u is in the activation type.
// rms: root-mean-square norm instead, u = gamma * x / sqrt(mean(x^2) + eps) (beta is not read; the mean written is 0).
template <typename T>
int launch_ln_fwd(const float* x, const T* gamma, const T* beta, T* u, float* mean, float* rstd,
                  int rows, int H, float eps, hipStream_t s, bool rms = false);

// out = resid + LN-backward(du), all fp32 (resid may be null: no residual); out_lowp, if not null, receives the same
// values in the activation type (the copy a following GEMM reads).  Each block of rows also writes its partial sums
// of dgamma (du * xhat) and dbeta (du) to part_g / part_b ([ln_bwd_blocks(rows)][H] fp32 each);
// launch_reduce_partials folds any number of such partial rows into a flat-gradient slice:
//   g = (accumulate ? g : 0) + scale * sum over chunks.
// part_s, if not null (LayerNorm form only): the blocks' column sums of `out`, laid out like part_g.
template <typename T>
int launch_ln_bwd(const float* du, const float* x, const float* mean, const float* rstd, const T* gamma,
                  const float* resid, float* out, T* out_lowp, float* part_g, float* part_b, int rows, int H, hipStream_t s,
                  bool rms = false, float* part_s = nullptr);
int ln_bwd_blocks(int rows);

// Rotary position embedding in place on the Q and K thirds of qkv [rows, 3H] (row % S = position, pairs (2i, 2i+1) of
// each head rotated by position * base^(-2i/d)); inverse: by the negative angle (the backward of the rotation).
// Rotary embedding: tab [S, d/2, 2] = (cos, sin) of position * base^(-2i/d); launch_rotary turns the Q and K thirds of
// qkv [rows, 3H] in place (inverse: by the negative angle).
int launch_rotary_table(float* tab, int S, int d, float base, hipStream_t s);
template <typename T> int launch_rotary(T* qkv, const float* tab, int rows, int S, int H, int heads, int inverse, hipStream_t s);
// Gated SiLU: gu [rows, 2F] = [gate | up], h [rows, F] = silu(gate) * up; backward dgu from dh and gu.
template <typename T> int launch_swiglu_fwd(const T* gu, T* h, int64_t rows, int F, hipStream_t s);
// tmp (reduce_tmp_bytes(nchunks, N) bytes, may be null) lets a long reduction run in two parallel stages.
int launch_reduce_partials(const float* partials, int nchunks, int N, float* g, float scale, int accumulate,
                           float* tmp, size_t tmp_bytes, hipStream_t s);
size_t reduce_tmp_bytes(int nchunks, int N);

// g[n] = (accumulate ? g[n] : 0) + scale * sum_t dY[t][n]   (bias gradient), dY [rows, N]
template <typename T>
int launch_colsum(const T* dY, float* partials, size_t partial_bytes, float* g, float scale,
                  int accumulate, int rows, int N, hipStream_t s);
size_t colsum_partial_bytes(int rows, int N);

// dst[i] = bf16(src[i]), i in [0, n)
int launch_cast_bf16(bf16* dst, const float* src, int64_t n, hipStream_t s);

// out[c][r] = in[r][c] for a row-major bf16 matrix [rows, cols]; out has row pitch out_pitch (0: rows) and its
// columns [rows, out_pitch) are zero-filled; cols and the pitch are multiples of 8
int launch_transpose_bf16(const bf16* in, bf16* out, int rows, int cols, hipStream_t s, int out_pitch = 0);

// ---------------------------------------------------------------------------------------
// Attention on the packed projection qkv [m*S, 3H] (Q | K | V column blocks, head a in
// columns [a*d,(a+1)*d) of each block).  O [m*S, H], lse [m, A, S] fp32 (log-sum-exp of the
// scaled, masked scores of each query row).
template <typename T>
int launch_attn_fwd_simple(const T* qkv, T* O, float* lse, int m, int S, int H, int A, int causal, hipStream_t s);
// dqkv [m*S, 3H]; dvec [m, A, S] fp32 scratch for rowsum(dO*O)
template <typename T>
int launch_attn_bwd_simple(const T* qkv, const T* O, const T* dO, const float* lse, float* dvec, T* dqkv,
                           int m, int S, int H, int A, int causal, hipStream_t s);

int launch_attn_fwd_mfma(const bf16* qkv, bf16* O, float* lse, int m, int S, int H, int A, int causal, hipStream_t s);
// rot: if not null, a rotary table [S, d/2, 2] by which the stored dq and dk are turned back (q and k were rotated)
int launch_attn_bwd_mfma(const bf16* qkv, const bf16* O, const bf16* dO, const float* lse, float* dvec, bf16* dqkv,
                         int m, int S, int H, int A, int causal, hipStream_t s, const float* rot = nullptr);

}  // namespace cephalo
