// Internals of the layer driver, shared by the single-layer entry points and the stack driver:
// flat layout, workspace carving, kernel selection and the launch sequences of one micro-batch's
// forward, its backward data path, and the parameter-gradient pass over a run of tokens.
#pragma once
#include "kernels.h"
#include <initializer_list>
#include <type_traits>
#include <algorithm>

#define TRY(expr) do { int rc__ = (expr); if (rc__ != CEPHALO_OK) return rc__; } while (0)

namespace cephalo {
namespace {   // internal linkage in each translation unit that includes this header

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

// Llama-style layers (kind 1): no biases, no beta, and the first feed-forward projection produces gate and up values,
// 2F columns.
inline bool is_llama(const cephalo_layer_desc& d) { return d.kind == CEPHALO_LAYER_LLAMA; }
inline int64_t ff1_width(const cephalo_layer_desc& d) { return is_llama(d) ? 2 * (int64_t)d.mlp : d.mlp; }

// Offsets (elements) of the 12 tensors of the flat layer layout.
struct ParamOffsets {
  int64_t ln1_g, ln1_b, w_qkv, b_qkv, w_o, b_o, ln2_g, ln2_b, w_fc1, b_fc1, w_fc2, b_fc2, total;
};

ParamOffsets param_offsets(const cephalo_layer_desc& d) {
  const int64_t H = d.hidden, F = d.mlp;
  ParamOffsets o;
  int64_t p = 0;
  const int64_t vec = is_llama(d) ? 0 : 1;               // beta and bias vectors exist in the GPT-style layer only
  o.ln1_g = p; p += H;
  o.ln1_b = p; p += vec * H;
  o.w_qkv = p; p += 3 * H * H;
  o.b_qkv = p; p += vec * 3 * H;
  o.w_o = p;   p += H * H;
  o.b_o = p;   p += vec * H;
  o.ln2_g = p; p += H;
  o.ln2_b = p; p += vec * H;
  o.w_fc1 = p; p += ff1_width(d) * H;
  o.b_fc1 = p; p += vec * F;
  o.w_fc2 = p; p += H * F;
  o.b_fc2 = p; p += vec * H;
  o.total = p;
  return o;
}

int check_desc(const cephalo_layer_desc* d) {
  if (!d) return fail(CEPHALO_EINVAL, "layer desc is null");
  if (d->hidden <= 0 || d->heads <= 0 || d->mlp <= 0 || d->seq <= 0)
    return fail(CEPHALO_EINVAL, "layer desc: hidden %d heads %d mlp %d seq %d must all be positive",
                d->hidden, d->heads, d->mlp, d->seq);
  if (d->hidden % d->heads != 0)
    return fail(CEPHALO_EINVAL, "layer desc: hidden %d is not a multiple of heads %d", d->hidden, d->heads);
  if (d->dtype != CEPHALO_F32 && d->dtype != CEPHALO_BF16) return fail(CEPHALO_EINVAL, "layer desc: unknown dtype %d", d->dtype);
  if (d->causal != 0 && d->causal != 1) return fail(CEPHALO_EINVAL, "layer desc: causal must be 0 or 1");
  if (d->kind != CEPHALO_LAYER_GPT && d->kind != CEPHALO_LAYER_LLAMA) return fail(CEPHALO_EINVAL, "layer desc: unknown kind %d", d->kind);
  if (d->kind == CEPHALO_LAYER_LLAMA && (d->hidden / d->heads) % 8 != 0)
    return fail(CEPHALO_EUNSUPPORTED, "layer desc: the rotary embedding needs a head dim that is a multiple of 8, got %d", d->hidden / d->heads);
  if (!(d->ln_eps >= 0.f)) return fail(CEPHALO_EINVAL, "layer desc: ln_eps %g < 0", d->ln_eps);
  if (d->hidden % 8 != 0 || d->mlp % 8 != 0)
    return fail(CEPHALO_EUNSUPPORTED, "layer desc: hidden %d and mlp %d must be multiples of 8 (16-byte rows)", d->hidden, d->mlp);
  const int hd = d->hidden / d->heads;
  if (hd > 128) return fail(CEPHALO_EUNSUPPORTED, "layer desc: head dim %d > 128", hd);
  if (d->dtype == CEPHALO_BF16 && hd % 8 != 0)
    return fail(CEPHALO_EUNSUPPORTED, "layer desc: bf16 attention needs a head dim that is a multiple of 8, got %d", hd);
  // a wavefront of the norm kernels holds one row in registers: 64 lanes x 16 vectors of 16 bytes of the activation type
  const int widest = d->dtype == CEPHALO_F32 ? 4096 : 8192;
  if (d->hidden > widest) return fail(CEPHALO_EUNSUPPORTED, "layer desc: hidden %d > %d (the limit for this dtype)", d->hidden, widest);
  return CEPHALO_OK;
}

// The residual stream (x, x1, y and the gradients dy, dx1, dx) is fp32 in both modes; everything a GEMM or
// the attention reads is in the activation type T (float, or bf16 with fp32 accumulation).  Where a
// residual-stream gradient is also a GEMM operand, the kernel that produces it writes a second copy in T
// ("lowp"); in fp32 mode the two are the same buffer.
//
// Saved activations of `n` samples, tensor-major: each tensor is one [n*S, width] matrix, so the
// slice of a micro-batch is a row range and the whole share is one contiguous operand.
struct SaveLayout {
  size_t mean1, rstd1, u, qkv, lse, O, x1, mean2, rstd2, u2, z, h, rot, total;
};
// Backward work area.  dz, dx1 and dqkv (the dY operands of the weight gradients) and the copy of dy in the
// activation type are kept for `span` samples; the rest is per micro-batch of m samples.
struct ScratchLayout {
  size_t dz, dx1, dx1l, dyl, dqkv, du2, dO, du, dvec, wT, wg_part, rs_part, rs_part_bytes, ln_part, col_part, col_part_bytes, total;
  size_t slot_each; // bytes of one slot's du2, dO, du, dvec (slot k's copies lie k * slot_each further on)
  size_t ln_rows;   // rows of each of the four LayerNorm partial arrays (ln2.gamma, ln2.beta, ln1.gamma, ln1.beta)
};

SaveLayout save_layout(const cephalo_layer_desc& d, int n) {
  const size_t es = d.dtype == CEPHALO_F32 ? 4 : 2;
  const size_t T = (size_t)n * d.seq, H = d.hidden, F = d.mlp;
  SaveLayout L;
  size_t p = 0;
  auto take = [&](size_t bytes) { size_t at = p; p += align_up(bytes); return at; };
  L.mean1 = take(T * 4); L.rstd1 = take(T * 4);
  L.u = take(T * H * es);
  L.qkv = take(T * 3 * H * es);
  L.lse = take((size_t)n * d.heads * d.seq * 4);
  L.O = take(T * H * es);
  L.x1 = take(T * H * 4);
  L.mean2 = take(T * 4); L.rstd2 = take(T * 4);
  L.u2 = take(T * H * es);
  L.z = take(T * (size_t)ff1_width(d) * es);      // derivative of the activation at the pre-activation (GPT-style) or gate | up (Llama-style)
  L.h = take(T * F * es);
  L.rot = is_llama(d) ? take((size_t)d.seq * (H / d.heads) * sizeof(float)) : 0;   // rotary table [S, d/2] of (cos, sin), shared by all samples
  L.total = p;
  return L;
}

// slots: how many micro-batches may be in their backward at once (each needs its own per-micro-batch buffers)
ScratchLayout scratch_layout(const cephalo_layer_desc& d, int m, int span, int slots = 1) {
  const size_t es = d.dtype == CEPHALO_F32 ? 4 : 2;
  const size_t Tm = (size_t)m * d.seq, Ts = (size_t)span * d.seq, H = d.hidden, F = d.mlp;
  ScratchLayout L;
  size_t p = 0;
  auto take = [&](size_t bytes) { size_t at = p; p += align_up(bytes); return at; };
  const size_t F1 = (size_t)ff1_width(d);
  L.dz = take(Ts * F1 * es);
  L.dx1 = take(Ts * H * 4);
  L.dx1l = es == 4 ? L.dx1 : take(Ts * H * es);
  L.dyl = es == 4 ? 0 : take(Ts * H * es);
  L.dqkv = take(Ts * 3 * H * es);
  L.slot_each = align_up(Tm * H * 4) + align_up(Tm * H * es) + align_up(Tm * H * 4) + align_up((size_t)m * d.heads * d.seq * 4);
  L.du2 = take(Tm * H * 4);        // gradients entering the LayerNorm backward: fp32
  L.dO = take(Tm * H * es);
  L.du = take(Tm * H * 4);
  L.dvec = take((size_t)m * d.heads * d.seq * 4);
  if (slots > 1) take((size_t)(slots - 1) * L.slot_each);      // the same four again per further slot
  L.wT = es == 4 ? 0 : take((size_t)param_offsets(d).total * es);   // the four weight matrices transposed, at their flat-layout offsets
  L.wg_part = p;                    // partial weight gradients of a split token axis (largest of the four projections)
  if (es != 4) {
    size_t need = 0;
    const int dims[4][2] = {{(int)(3 * H), (int)H}, {(int)H, (int)H}, {(int)F1, (int)H}, {(int)H, (int)F}};
    for (auto& nk : dims) {
      const int sp = gemm_grad_splits(nk[0], nk[1], (int)Ts);
      if (sp > 1) need = std::max(need, (size_t)sp * nk[0] * nk[1] * sizeof(float));
    }
    take(need);
  }
  // pieces of the bias gradients that the weight-gradient GEMMs of the two bf16-fed projections sum on the way
  L.rs_part_bytes = (es != 4 && !is_llama(d)) ? std::max(gemm_rowsum_part_bytes((int)(3 * H), (int)H), gemm_rowsum_part_bytes((int)F1, (int)H)) : 0;
  L.rs_part = take(L.rs_part_bytes);
  L.ln_rows = (size_t)(span / m) * ln_bwd_blocks((int)Tm);
  L.ln_part = take(6 * L.ln_rows * H * sizeof(float));      // d gamma and d beta of both norms, and the column sums of the two LayerNorm backwards' results
  const int widest = (int)(3 * H > F1 ? 3 * H : F1);
  L.col_part_bytes = colsum_partial_bytes((int)Ts, widest);
  L.col_part = take(L.col_part_bytes);
  L.total = p;
  return L;
}

constexpr float kRopeBase = 10000.0f;   // rotary embedding: angle of pair i at position t is t * base^(-2i/d)

// ---- kernel selection ------------------------------------------------------------------
template <typename T> int gemm(const GemmArgs<T>& a, hipStream_t s);
template <> int gemm<float>(const GemmArgs<float>& a, hipStream_t s) { return launch_gemm_simple<float>(a, s); }
template <> int gemm<bf16>(const GemmArgs<bf16>& a, hipStream_t s) { return launch_gemm_mfma(a, s); }

template <typename T> int attn_fwd(const T* qkv, T* O, float* lse, int m, int S, int H, int A, int causal, hipStream_t s);
template <> int attn_fwd<float>(const float* qkv, float* O, float* lse, int m, int S, int H, int A, int causal, hipStream_t s) {
  return launch_attn_fwd_simple<float>(qkv, O, lse, m, S, H, A, causal, s);
}
template <> int attn_fwd<bf16>(const bf16* qkv, bf16* O, float* lse, int m, int S, int H, int A, int causal, hipStream_t s) {
  return launch_attn_fwd_mfma(qkv, O, lse, m, S, H, A, causal, s);
}
// rot: if not null, the rotary table of a layer whose q and k were rotated; dq and dk then come back through the rotation
template <typename T>
int attn_bwd(const T* qkv, const T* O, const T* dO, const float* lse, float* dvec, T* dqkv, int m, int S, int H, int A, int causal, hipStream_t s,
             const float* rot = nullptr);
template <> int attn_bwd<float>(const float* qkv, const float* O, const float* dO, const float* lse, float* dvec, float* dqkv,
                                int m, int S, int H, int A, int causal, hipStream_t s, const float* rot) {
  int rc = launch_attn_bwd_simple<float>(qkv, O, dO, lse, dvec, dqkv, m, S, H, A, causal, s);
  if (rc == CEPHALO_OK && rot) rc = launch_rotary<float>(dqkv, rot, m * S, S, H, A, 1, s);
  return rc;
}
template <> int attn_bwd<bf16>(const bf16* qkv, const bf16* O, const bf16* dO, const float* lse, float* dvec, bf16* dqkv,
                               int m, int S, int H, int A, int causal, hipStream_t s, const float* rot) {
  return launch_attn_bwd_mfma(qkv, O, dO, lse, dvec, dqkv, m, S, H, A, causal, s, rot);   // fused into the stores of dq and dk
}

template <typename T> T* at(void* base, size_t off) { return reinterpret_cast<T*>(static_cast<char*>(base) + off); }
template <typename T> const T* at(const void* base, size_t off) { return reinterpret_cast<const T*>(static_cast<const char*>(base) + off); }

// Y[T,N] = X[T,K] W[N,K]^T (+ epilogue): both operands k-contiguous
template <typename T>
GemmArgs<T> linear_fwd(const T* X, const T* W, int Tn, int N, int K) {
  GemmArgs<T> a = {};
  a.A = X; a.a_rs = K; a.a_cs = 1;
  a.B = W; a.b_rs = K; a.b_cs = 1;
  a.M = Tn; a.N = N; a.K = K;
  return a;
}
// dX[T,K] = dY[T,N] W[N,K]: contraction over N; B(n'=k, k'=n) = W[n*K + k]
template <typename T>
GemmArgs<T> linear_dgrad(const T* dY, const T* W, int Tn, int N, int K) {
  GemmArgs<T> a = {};
  a.A = dY; a.a_rs = N; a.a_cs = 1;
  a.B = W; a.b_rs = 1; a.b_cs = K;
  a.M = Tn; a.N = K; a.K = N;
  return a;
}
// the same with the transposed weight WT[K,N] at hand: both operands contiguous along the contracted axis
template <typename T>
GemmArgs<T> linear_dgrad_wt(const T* dY, const T* WT, int Tn, int N, int K) {
  GemmArgs<T> a = {};
  a.A = dY; a.a_rs = N; a.a_cs = 1;
  a.B = WT; a.b_rs = N; a.b_cs = 1;
  a.M = Tn; a.N = K; a.K = N;
  return a;
}
// dW[N,K] = dY[T,N]^T X[T,K]: contraction over T; both operands strided along it
template <typename T>
GemmArgs<T> linear_wgrad(const T* dY, const T* X, int Tn, int N, int K, float* G, float scale, int accumulate) {
  GemmArgs<T> a = {};
  a.A = dY; a.a_rs = 1; a.a_cs = N;
  a.B = X; a.b_rs = 1; a.b_cs = K;
  a.M = N; a.N = K; a.K = Tn;
  a.epi = EPI_GRAD; a.G = G; a.scale = scale; a.accumulate = accumulate;
  return a;
}

// Parameter gradient of a linear layer over Tn tokens: G[N, K] (+)= scale * dY^T X, dY [Tn, ldy >= N], X [Tn, K].
// Both operands are read as they lie, token-major (the contraction runs over their rows: the GEMM reads such
// operands with transposing LDS reads at the rate of k-contiguous ones, so no transposed copy is made).
// `part`: room for the pieces of a split contraction (sized by gemm_grad_splits for the whole token axis), or null.
// `colsums` (optional): where the column sums of dY, the bias gradient of the same projection, are wanted with the same
// scale / acc.  The bf16 GEMM sums them beside the products when it can (one piece, operands that fit its MFMA kernels)
// and then sets colsums->done; otherwise the caller runs the column-sum kernel.
struct ColsumsBeside { float* g; float* part; size_t part_bytes; bool done; };
template <typename T>
int wgrad(const T* dY, const T* X, int Tn, int N, int K, float* G, float scale, int acc, float* part, hipStream_t s, int ldy = 0,
          ColsumsBeside* colsums = nullptr);
template <>
int wgrad<float>(const float* dY, const float* X, int Tn, int N, int K, float* G, float scale, int acc, float*, hipStream_t s, int ldy,
                 ColsumsBeside*) {
  GemmArgs<float> a = linear_wgrad<float>(dY, X, Tn, N, K, G, scale, acc);
  if (ldy) a.a_cs = ldy;
  return gemm<float>(a, s);
}
template <>
int wgrad<bf16>(const bf16* dY, const bf16* X, int Tn, int N, int K, float* G, float scale, int acc, float* part, hipStream_t s, int ldy,
                ColsumsBeside* colsums) {
  if (!ldy) ldy = N;
  // the GEMM addresses its operands through 32-bit buffer descriptors: contract over the tokens in pieces below 2 GiB
  const int64_t widest = ldy > K ? ldy : K;
  int64_t piece = ((int64_t)0x7ff00000 / (2 * widest)) / 64 * 64;
  if (piece <= 0) return fail(CEPHALO_EUNSUPPORTED, "wgrad: a row of %lld elements is too wide", (long long)widest);
  for (int64_t t0 = 0; t0 < Tn; t0 += piece) {
    const int tc = (int)(Tn - t0 < piece ? Tn - t0 : piece);
    GemmArgs<bf16> a = linear_wgrad<bf16>(dY + t0 * ldy, X + t0 * K, tc, N, K, G, scale, t0 > 0 ? 1 : acc);
    a.a_cs = ldy;
    a.splits = part ? gemm_grad_splits(N, K, tc) : 1;     // `part` was sized with the same rule for the whole token axis
    a.part = part;
    if (tc != Tn) a.splits = 1;
    if (colsums && tc == Tn && colsums->part && colsums->part_bytes >= gemm_rowsum_part_bytes(N, K) && gemm_mfma_takes(a)) {
      a.rowsum = colsums->g; a.rowsum_part = colsums->part; a.rowsum_part_bytes = colsums->part_bytes;
      colsums->done = true;
    }
    TRY(gemm<bf16>(a, s));
  }
  return CEPHALO_OK;
}

template <typename T> struct Saved {
  float *mean1, *rstd1, *lse, *mean2, *rstd2, *x1, *rot;
  T *u, *qkv, *O, *u2, *z, *h;
};
// pointers to the saved tensors of the samples starting at `sample0` inside a save area laid out by L
template <typename T>
Saved<T> saved_at(void* base, const SaveLayout& L, const cephalo_layer_desc& d, int sample0) {
  const size_t t0 = (size_t)sample0 * d.seq, H = d.hidden, F = d.mlp;
  Saved<T> s;
  s.mean1 = at<float>(base, L.mean1) + t0; s.rstd1 = at<float>(base, L.rstd1) + t0;
  s.mean2 = at<float>(base, L.mean2) + t0; s.rstd2 = at<float>(base, L.rstd2) + t0;
  s.lse = at<float>(base, L.lse) + (size_t)sample0 * d.heads * d.seq;
  s.u = at<T>(base, L.u) + t0 * H; s.qkv = at<T>(base, L.qkv) + t0 * 3 * H; s.O = at<T>(base, L.O) + t0 * H;
  s.x1 = at<float>(base, L.x1) + t0 * H; s.u2 = at<T>(base, L.u2) + t0 * H;
  s.z = at<T>(base, L.z) + t0 * (size_t)ff1_width(d); s.h = at<T>(base, L.h) + t0 * F;
  s.rot = at<float>(base, L.rot);
  return s;
}

template <typename T> struct Work {
  T *dz, *dx1l, *dyl, *dqkv;   // at the token offset of the current micro-batch (or of the span for the parameter pass)
  float *dx1;                  // likewise; dx1l is its copy in T (the same buffer in fp32 mode), dyl the caller's dy in T
  T *dO, *wT;
  float *du2, *du, *dvec;
  float *ln2_g, *ln2_b, *ln1_g, *ln1_b;   // LayerNorm partial sums, at the row offset of the current micro-batch
  float *ln2_s, *ln1_s;                   // column sums of dx1 and of dx, block by block like the above (GPT-style layer)
  float *col_part; size_t col_part_bytes;
  float *wg_part;
  float *rs_part; size_t rs_part_bytes;
};
template <typename T>
Work<T> work_at(void* base, const ScratchLayout& W, const cephalo_layer_desc& d, int sample0, int mb_index, int m, int slot = 0) {
  const size_t t0 = (size_t)sample0 * d.seq, H = d.hidden, F = d.mlp;
  Work<T> w;
  w.dz = at<T>(base, W.dz) + t0 * (size_t)ff1_width(d); w.dx1 = at<float>(base, W.dx1) + t0 * H; w.dx1l = at<T>(base, W.dx1l) + t0 * H;
  w.dyl = at<T>(base, W.dyl) + t0 * H; w.dqkv = at<T>(base, W.dqkv) + t0 * 3 * H;
  const size_t so = (size_t)slot * W.slot_each;
  w.du2 = at<float>(base, W.du2 + so); w.dO = at<T>(base, W.dO + so); w.du = at<float>(base, W.du + so); w.wT = at<T>(base, W.wT);
  w.dvec = at<float>(base, W.dvec + so);
  float* ln = at<float>(base, W.ln_part);
  const size_t r0 = (size_t)mb_index * ln_bwd_blocks(m * d.seq) * H, arr = W.ln_rows * H;
  w.ln2_g = ln + r0; w.ln2_b = ln + arr + r0; w.ln1_g = ln + 2 * arr + r0; w.ln1_b = ln + 3 * arr + r0;
  w.ln2_s = ln + 4 * arr + r0; w.ln1_s = ln + 5 * arr + r0;
  w.col_part = at<float>(base, W.col_part); w.col_part_bytes = W.col_part_bytes;
  w.wg_part = at<float>(base, W.wg_part);
  w.rs_part = at<float>(base, W.rs_part); w.rs_part_bytes = W.rs_part_bytes;
  return w;
}

// ---- forward of one micro-batch ----------------------------------------------------------------
template <typename T>
int layer_fwd_t(const cephalo_layer_desc& d, const T* P, const float* x, float* y, int m, const Saved<T>& sv, hipStream_t s) {
  const ParamOffsets o = param_offsets(d);
  const int Tn = m * d.seq, H = d.hidden, F = d.mlp;
  if (is_llama(d)) {
    // u = RMS1(x); qkv = u Wqkv^T; rotary on q, k; attention; x1 = x + O Wo^T; u2 = RMS2(x1); [g | up] = u2 Wgu^T;
    // h = silu(g) up; y = x1 + h Wdown^T
    TRY(launch_ln_fwd<T>(x, P + o.ln1_g, (const T*)nullptr, sv.u, sv.mean1, sv.rstd1, Tn, H, d.ln_eps, s, true));
    TRY(launch_rotary_table(sv.rot, d.seq, H / d.heads, kRopeBase, s));   // (every micro-batch writes the same values)
    {
      GemmArgs<T> a = linear_fwd<T>(sv.u, P + o.w_qkv, Tn, 3 * H, H);
      a.epi = EPI_ROPE; a.C = sv.qkv;       // q and k leave the GEMM already rotated (one rounding, of the rotated value)
      a.rot = sv.rot; a.rot_S = d.seq; a.rot_d = H / d.heads; a.rot_cols = 2 * H;
      TRY(gemm<T>(a, s));
    }
    TRY(attn_fwd<T>(sv.qkv, sv.O, sv.lse, m, d.seq, H, d.heads, d.causal, s));
    {
      GemmArgs<T> a = linear_fwd<T>(sv.O, P + o.w_o, Tn, H, H);
      a.epi = EPI_BIAS_RESID; a.bias = nullptr; a.Rf = x; a.Cf = sv.x1;
      TRY(gemm<T>(a, s));
    }
    TRY(launch_ln_fwd<T>(sv.x1, P + o.ln2_g, (const T*)nullptr, sv.u2, sv.mean2, sv.rstd2, Tn, H, d.ln_eps, s, true));
    {
      GemmArgs<T> a = linear_fwd<T>(sv.u2, P + o.w_fc1, Tn, 2 * F, H);
      a.epi = EPI_NONE; a.C = sv.z;
      TRY(gemm<T>(a, s));
    }
    TRY(launch_swiglu_fwd<T>(sv.z, sv.h, Tn, F, s));
    {
      GemmArgs<T> a = linear_fwd<T>(sv.h, P + o.w_fc2, Tn, H, F);
      a.epi = EPI_BIAS_RESID; a.bias = nullptr; a.Rf = sv.x1; a.Cf = y;
      TRY(gemm<T>(a, s));
    }
    return CEPHALO_OK;
  }
  TRY(launch_ln_fwd<T>(x, P + o.ln1_g, P + o.ln1_b, sv.u, sv.mean1, sv.rstd1, Tn, H, d.ln_eps, s));
  {
    GemmArgs<T> a = linear_fwd<T>(sv.u, P + o.w_qkv, Tn, 3 * H, H);
    a.epi = EPI_BIAS; a.bias = P + o.b_qkv; a.C = sv.qkv;
    TRY(gemm<T>(a, s));
  }
  TRY(attn_fwd<T>(sv.qkv, sv.O, sv.lse, m, d.seq, H, d.heads, d.causal, s));
  {
    GemmArgs<T> a = linear_fwd<T>(sv.O, P + o.w_o, Tn, H, H);
    a.epi = EPI_BIAS_RESID; a.bias = P + o.b_o; a.Rf = x; a.Cf = sv.x1;
    TRY(gemm<T>(a, s));
  }
  TRY(launch_ln_fwd<T>(sv.x1, P + o.ln2_g, P + o.ln2_b, sv.u2, sv.mean2, sv.rstd2, Tn, H, d.ln_eps, s));
  {
    GemmArgs<T> a = linear_fwd<T>(sv.u2, P + o.w_fc1, Tn, F, H);
    a.epi = EPI_BIAS_GELU_DERIV; a.bias = P + o.b_fc1; a.Z = sv.z; a.C = sv.h;      // saved: gelu'(z), the factor the backward needs
    TRY(gemm<T>(a, s));
  }
  {
    GemmArgs<T> a = linear_fwd<T>(sv.h, P + o.w_fc2, Tn, H, F);
    a.epi = EPI_BIAS_RESID; a.bias = P + o.b_fc2; a.Rf = sv.x1; a.Cf = y;
    TRY(gemm<T>(a, s));
  }
  return CEPHALO_OK;
}

// The copy of a residual-stream gradient in the activation type: the buffer itself in fp32 mode.
template <typename T> const T* lowp_of(const float* f, const T* l);
template <> inline const float* lowp_of<float>(const float* f, const float*) { return f; }
template <> inline const bf16* lowp_of<bf16>(const float*, const bf16* l) { return l; }
template <typename T> T* lowp_out(T* l) { return std::is_same<T, float>::value ? nullptr : l; }   // nothing extra to write in fp32 mode

// dst = T(src) for n elements when T is not float (used where the caller hands dy in fp32)
template <typename T> int make_lowp(T* dst, const float* src, int64_t n, hipStream_t s);
template <> inline int make_lowp<float>(float*, const float*, int64_t, hipStream_t) { return CEPHALO_OK; }
template <> inline int make_lowp<bf16>(bf16* dst, const float* src, int64_t n, hipStream_t s) { return launch_cast_bf16(dst, src, n, s); }

// Input-gradient contraction dX = dY W of the linear layer whose weight sits at flat offset `off`.  In bf16 mode it
// reads the transposed copy made by prepare_dgrad_weights (so both MFMA operands come from 16-byte LDS reads, the
// same kernel as the forward); the fp32 path reads W in place.
template <typename T> GemmArgs<T> dgrad_args(const T* dY, const T* P, const T* wT, int64_t off, int Tn, int N, int K);
template <> inline GemmArgs<float> dgrad_args<float>(const float* dY, const float* P, const float*, int64_t off, int Tn, int N, int K) {
  return linear_dgrad<float>(dY, P + off, Tn, N, K);
}
template <> inline GemmArgs<bf16> dgrad_args<bf16>(const bf16* dY, const bf16*, const bf16* wT, int64_t off, int Tn, int N, int K) {
  return linear_dgrad_wt<bf16>(dY, wT + off, Tn, N, K);
}
// Once per layer and step (the weights do not change between micro-batches): W^T of the four projections.
template <typename T> int prepare_dgrad_weights(const cephalo_layer_desc& d, const T* P, T* wT, hipStream_t s);
template <> inline int prepare_dgrad_weights<float>(const cephalo_layer_desc&, const float*, float*, hipStream_t) { return CEPHALO_OK; }
template <> inline int prepare_dgrad_weights<bf16>(const cephalo_layer_desc& d, const bf16* P, bf16* wT, hipStream_t s) {
  const ParamOffsets o = param_offsets(d);
  const int H = d.hidden, F = d.mlp;
  TRY(launch_transpose_bf16(P + o.w_qkv, wT + o.w_qkv, 3 * H, H, s));
  TRY(launch_transpose_bf16(P + o.w_o, wT + o.w_o, H, H, s));
  TRY(launch_transpose_bf16(P + o.w_fc1, wT + o.w_fc1, (int)ff1_width(d), H, s));
  TRY(launch_transpose_bf16(P + o.w_fc2, wT + o.w_fc2, H, F, s));
  return CEPHALO_OK;
}

// ---- backward, data path of one micro-batch: dx and the dY operands (dz, dx1, dqkv) of the weight gradients --------
// dyl is dy in the activation type (same rows); dxl, if not null, receives dx in the activation type as well.
template <typename T>
int layer_bwd_data_t(const cephalo_layer_desc& d, const T* P, const float* x, const float* dy, const T* dyl, float* dx, T* dxl, int m,
                     const Saved<T>& sv, const Work<T>& w, hipStream_t s) {
  const ParamOffsets o = param_offsets(d);
  const int Tn = m * d.seq, H = d.hidden, F = d.mlp;
  if (is_llama(d)) {
    {
      GemmArgs<T> a = dgrad_args<T>(dyl, P, w.wT, o.w_fc2, Tn, H, F);   // dh = dy Wdown, then d[gate | up] from the fp32 products
      a.epi = EPI_DSWIGLU; a.Z = sv.z; a.C = w.dz; a.ldc = 2 * F;
      TRY(gemm<T>(a, s));
    }
    {
      GemmArgs<T> a = dgrad_args<T>(w.dz, P, w.wT, o.w_fc1, Tn, 2 * F, H);
      a.epi = EPI_NONE; a.Cf = w.du2;
      TRY(gemm<T>(a, s));
    }
    TRY(launch_ln_bwd<T>(w.du2, sv.x1, sv.mean2, sv.rstd2, P + o.ln2_g, dy, w.dx1, lowp_out<T>(w.dx1l), w.ln2_g, w.ln2_b, Tn, H, s, true));
    {
      GemmArgs<T> a = dgrad_args<T>(lowp_of<T>(w.dx1, w.dx1l), P, w.wT, o.w_o, Tn, H, H);
      a.epi = EPI_NONE; a.C = w.dO;
      TRY(gemm<T>(a, s));
    }
    TRY(attn_bwd<T>(sv.qkv, sv.O, w.dO, sv.lse, w.dvec, w.dqkv, m, d.seq, H, d.heads, d.causal, s, sv.rot));   // dq, dk: turned back by the angle
    {
      GemmArgs<T> a = dgrad_args<T>(w.dqkv, P, w.wT, o.w_qkv, Tn, 3 * H, H);
      a.epi = EPI_NONE; a.Cf = w.du;
      TRY(gemm<T>(a, s));
    }
    TRY(launch_ln_bwd<T>(w.du, x, sv.mean1, sv.rstd1, P + o.ln1_g, w.dx1, dx, lowp_out<T>(dxl), w.ln1_g, w.ln1_b, Tn, H, s, true));
    return CEPHALO_OK;
  }
  {
    GemmArgs<T> a = dgrad_args<T>(dyl, P, w.wT, o.w_fc2, Tn, H, F);   // dh = dy W2, then dz = dh * gelu'(z), the factor saved by the forward
    a.epi = EPI_MUL; a.Z = sv.z; a.C = w.dz;
    TRY(gemm<T>(a, s));
  }
  {
    GemmArgs<T> a = dgrad_args<T>(w.dz, P, w.wT, o.w_fc1, Tn, F, H);
    a.epi = EPI_NONE; a.Cf = w.du2;
    TRY(gemm<T>(a, s));
  }
  // u2 = LN2(x1); dx1 = dy + LN2-backward(du2)
  TRY(launch_ln_bwd<T>(w.du2, sv.x1, sv.mean2, sv.rstd2, P + o.ln2_g, dy, w.dx1, lowp_out<T>(w.dx1l), w.ln2_g, w.ln2_b, Tn, H, s, false, w.ln2_s));
  {
    GemmArgs<T> a = dgrad_args<T>(lowp_of<T>(w.dx1, w.dx1l), P, w.wT, o.w_o, Tn, H, H);
    a.epi = EPI_NONE; a.C = w.dO;
    TRY(gemm<T>(a, s));
  }
  TRY(attn_bwd<T>(sv.qkv, sv.O, w.dO, sv.lse, w.dvec, w.dqkv, m, d.seq, H, d.heads, d.causal, s));
  {
    GemmArgs<T> a = dgrad_args<T>(w.dqkv, P, w.wT, o.w_qkv, Tn, 3 * H, H);
    a.epi = EPI_NONE; a.Cf = w.du;
    TRY(gemm<T>(a, s));
  }
  // u = LN1(x); dx = dx1 + LN1-backward(du)
  TRY(launch_ln_bwd<T>(w.du, x, sv.mean1, sv.rstd1, P + o.ln1_g, w.dx1, dx, lowp_out<T>(dxl), w.ln1_g, w.ln1_b, Tn, H, s, false, w.ln1_s));
  return CEPHALO_OK;
}

// ---- backward, parameter path over `tokens` tokens (one micro-batch, or the whole share at once) ---------------------
// G <- (acc ? G : 0) + scale * (gradient summed over those tokens).  Over the whole share the sum over micro-batches
// happens inside the fp32 MFMA accumulators and each gradient element is written exactly once.  Bias gradients of the
// two residual-stream projections are column sums of the fp32 gradients of the stream: of dx1 (out-projection), which
// the backward of the second LayerNorm has summed block by block as it wrote it, and of dy (second feed-forward
// projection), summed here unless the caller passes none.  A caller whose dy was the dx of the layer above (a stack)
// passes null and gives that layer `b_fc2_below` instead: where the sums of its dx go, with the same scale / acc.
template <typename T>
int layer_bwd_params_t(const cephalo_layer_desc& d, const float* dy, const T* dyl, int tokens, int ln_chunks,
                       const Saved<T>& sv, const Work<T>& w, float* G, float scale, int acc, hipStream_t s, hipStream_t s2 = nullptr,
                       float* b_fc2_below = nullptr) {
  if (!s2) s2 = s;      // s2: where the bandwidth-bound reductions (bias column sums, norm-parameter partials) run, beside the GEMMs on s
  const ParamOffsets o = param_offsets(d);
  const int H = d.hidden, F = d.mlp;
  if (is_llama(d)) {
    TRY(wgrad<T>(dyl, sv.h, tokens, H, F, G + o.w_fc2, scale, acc, w.wg_part, s));
    TRY(wgrad<T>(w.dz, sv.u2, tokens, 2 * F, H, G + o.w_fc1, scale, acc, w.wg_part, s));
    TRY(launch_reduce_partials(w.ln2_g, ln_chunks, H, G + o.ln2_g, scale, acc, w.col_part, w.col_part_bytes, s2));
    TRY(wgrad<T>(lowp_of<T>(w.dx1, w.dx1l), sv.O, tokens, H, H, G + o.w_o, scale, acc, w.wg_part, s));
    TRY(wgrad<T>(w.dqkv, sv.u, tokens, 3 * H, H, G + o.w_qkv, scale, acc, w.wg_part, s));
    TRY(launch_reduce_partials(w.ln1_g, ln_chunks, H, G + o.ln1_g, scale, acc, w.col_part, w.col_part_bytes, s2));
    return CEPHALO_OK;
  }
  // (the other two bias gradients are sums of the very bf16 values their weight-gradient GEMMs read, and the GEMMs form
  // them on the way)
  if (b_fc2_below) TRY(launch_reduce_partials(w.ln1_s, ln_chunks, H, b_fc2_below, scale, acc, w.col_part, w.col_part_bytes, s2));
  if (dy) TRY(launch_colsum<float>(dy, w.col_part, w.col_part_bytes, G + o.b_fc2, scale, acc, tokens, H, s2));   // (null: the caller has summed it already)
  TRY(wgrad<T>(dyl, sv.h, tokens, H, F, G + o.w_fc2, scale, acc, w.wg_part, s));
  {
    ColsumsBeside cb = {G + o.b_fc1, w.rs_part, w.rs_part_bytes, false};
    TRY(wgrad<T>(w.dz, sv.u2, tokens, F, H, G + o.w_fc1, scale, acc, w.wg_part, s, 0, &cb));
    if (!cb.done) TRY(launch_colsum<T>(w.dz, w.col_part, w.col_part_bytes, G + o.b_fc1, scale, acc, tokens, F, s2));
  }
  TRY(launch_reduce_partials(w.ln2_g, ln_chunks, H, G + o.ln2_g, scale, acc, w.col_part, w.col_part_bytes, s2));
  TRY(launch_reduce_partials(w.ln2_b, ln_chunks, H, G + o.ln2_b, scale, acc, w.col_part, w.col_part_bytes, s2));
  TRY(launch_reduce_partials(w.ln2_s, ln_chunks, H, G + o.b_o, scale, acc, w.col_part, w.col_part_bytes, s2));
  TRY(wgrad<T>(lowp_of<T>(w.dx1, w.dx1l), sv.O, tokens, H, H, G + o.w_o, scale, acc, w.wg_part, s));
  {
    ColsumsBeside cb = {G + o.b_qkv, w.rs_part, w.rs_part_bytes, false};
    TRY(wgrad<T>(w.dqkv, sv.u, tokens, 3 * H, H, G + o.w_qkv, scale, acc, w.wg_part, s, 0, &cb));
    if (!cb.done) TRY(launch_colsum<T>(w.dqkv, w.col_part, w.col_part_bytes, G + o.b_qkv, scale, acc, tokens, 3 * H, s2));
  }
  TRY(launch_reduce_partials(w.ln1_g, ln_chunks, H, G + o.ln1_g, scale, acc, w.col_part, w.col_part_bytes, s2));
  TRY(launch_reduce_partials(w.ln1_b, ln_chunks, H, G + o.ln1_b, scale, acc, w.col_part, w.col_part_bytes, s2));
  return CEPHALO_OK;
}

template <typename T>
int run_fwd(const cephalo_layer_desc& d, const void* P, const float* x, float* y, int m, void* save, hipStream_t s) {
  const SaveLayout L = save_layout(d, m);
  return layer_fwd_t<T>(d, static_cast<const T*>(P), x, y, m, saved_at<T>(save, L, d, 0), s);
}

template <typename T>
int run_bwd(const cephalo_layer_desc& d, const void* P, const float* x, const float* dy, float* dx, int m, void* save,
            float* G, float scale, int acc, void* scratch, hipStream_t s) {
  const SaveLayout L = save_layout(d, m);
  const ScratchLayout W = scratch_layout(d, m, m);
  const Saved<T> sv = saved_at<T>(save, L, d, 0);
  const Work<T> w = work_at<T>(scratch, W, d, 0, 0, m);
  const int64_t act = (int64_t)m * d.seq * d.hidden;
  TRY(make_lowp<T>(w.dyl, dy, act, s));
  const T* dyl = lowp_of<T>(dy, w.dyl);
  TRY(prepare_dgrad_weights<T>(d, static_cast<const T*>(P), w.wT, s));
  TRY(layer_bwd_data_t<T>(d, static_cast<const T*>(P), x, dy, dyl, dx, (T*)nullptr, m, sv, w, s));
  return layer_bwd_params_t<T>(d, dy, dyl, m * d.seq, ln_bwd_blocks(m * d.seq), sv, w, G, scale, acc, s);
}

// The two compute streams of an interleaved step.  fork: the side stream continues from where the main stream is;
// join: the main stream continues only after the side stream's work so far.  Without interleave both do nothing.
struct Streams {
  hipStream_t main = nullptr, side = nullptr;
  bool on = false;
  hipEvent_t forked, joined;
  int err = CEPHALO_OK;
  void check(hipError_t e, const char* what) {
    if (e != hipSuccess && err == CEPHALO_OK) err = fail(CEPHALO_EHIP, "interleaved step: %s: %s", what, hipGetErrorString(e));
  }
  int open() {
    if (!on) return CEPHALO_OK;
    check(hipEventCreateWithFlags(&forked, hipEventDisableTiming), "event");
    check(hipEventCreateWithFlags(&joined, hipEventDisableTiming), "event");
    return err;
  }
  void fork() {
    if (!on) return;
    check(hipEventRecord(forked, main), "record");
    check(hipStreamWaitEvent(side, forked, 0), "wait");
  }
  void join() {
    if (!on) return;
    check(hipEventRecord(joined, side), "record");
    check(hipStreamWaitEvent(main, joined, 0), "wait");
  }
  int close() {          // the call ends joined: whoever waits for the main stream has waited for everything
    if (!on) return CEPHALO_OK;
    join();
    check(hipEventDestroy(forked), "event");
    check(hipEventDestroy(joined), "event");
    return err;
  }
};

// Whole share: forward of every micro-batch, data-path backward of every micro-batch, then ONE parameter pass over
// all b*S tokens (the dY operands and the saved activations of all micro-batches are contiguous by construction).
template <typename T>
int run_share(const cephalo_layer_desc& d, const void* Pv, const float* x, float* y, const float* dy, float* dx,
              int b, int m, void* save, float* G, float scale, void* scratch, hipStream_t s, hipStream_t side = nullptr) {
  const T* P = static_cast<const T*>(Pv);
  const SaveLayout L = save_layout(d, b);
  const ScratchLayout W = scratch_layout(d, m, b, 2);
  const int l = b / m;
  const size_t act = (size_t)m * d.seq * d.hidden;   // elements of one micro-batch of x / y / dy / dx
  // side: micro-batch j runs on stream j % 2 (two in flight, see Streams); what the micro-batches share is made first
  const int nst = side ? 2 : 1;
  hipStream_t st[2] = {s, side ? side : s};
  Streams J;
  J.main = s; J.side = side; J.on = side != nullptr;
  TRY(J.open());
  struct JCloser { Streams& j; bool done = false; ~JCloser() { if (!done) (void)j.close(); } } jcloser{J};   // early exits still join
  const Work<T> w0 = work_at<T>(scratch, W, d, 0, 0, m);
  TRY(make_lowp<T>(w0.dyl, dy, (int64_t)l * act, s));
  const T* dyl = lowp_of<T>(dy, w0.dyl);
  TRY(prepare_dgrad_weights<T>(d, P, w0.wT, s));
  J.fork();
  {
    GemmSideBySide hint(nst);
    for (int j = 0; j < l; ++j)
      TRY(layer_fwd_t<T>(d, P, x + j * act, y + j * act, m, saved_at<T>(save, L, d, j * m), st[j % nst]));
    for (int j = 0; j < l; ++j)
      TRY(layer_bwd_data_t<T>(d, P, x + j * act, dy + j * act, dyl + j * act, dx + j * act, (T*)nullptr, m,
                              saved_at<T>(save, L, d, j * m), work_at<T>(scratch, W, d, j * m, j, m, j % nst), st[j % nst]));
  }
  J.join();
  J.fork();      // the parameter pass's reductions beside its GEMMs
  TRY(layer_bwd_params_t<T>(d, dy, dyl, b * d.seq, l * ln_bwd_blocks(m * d.seq), saved_at<T>(save, L, d, 0), w0, G, scale, 0, s, st[1]));
  jcloser.done = true;
  return J.close();      // joins the streams; an error of the join or of the event release is the call's result
}

int check_io(const char* who, const cephalo_layer_desc* d, int m, std::initializer_list<const void*> ptrs) {
  TRY(check_desc(d));
  if (m <= 0) return fail(CEPHALO_EINVAL, "%s: micro-batch size m = %d must be positive", who, m);
  if ((int64_t)m * d->seq > (1 << 24)) return fail(CEPHALO_EUNSUPPORTED, "%s: m*S = %lld tokens per micro-batch is too many", who, (long long)m * d->seq);
  for (const void* p : ptrs) {
    if (!p) return fail(CEPHALO_EINVAL, "%s: null pointer argument", who);
    if (!aligned16(p)) return fail(CEPHALO_EINVAL, "%s: pointer %p is not 16-byte aligned", who, p);
  }
  return CEPHALO_OK;
}

}  // namespace
}  // namespace cephalo
