// Host driver of one transformer layer on one micro-batch, and of a whole batch share:
// argument checks in the paper's terms (batch share b, micro-batch size m, b = l*m),
// workspace carving, and the launch sequence on the caller's stream.
#include "kernels.h"
#include <type_traits>

namespace cephalo {
namespace {

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

// Offsets (elements) of the 12 tensors of the flat layer layout.
struct ParamOffsets {
  int64_t ln1_g, ln1_b, w_qkv, b_qkv, w_o, b_o, ln2_g, ln2_b, w_fc1, b_fc1, w_fc2, b_fc2, total;
};

ParamOffsets param_offsets(const cephalo_layer_desc& d) {
  const int64_t H = d.hidden, F = d.mlp;
  ParamOffsets o;
  int64_t p = 0;
  o.ln1_g = p; p += H;
  o.ln1_b = p; p += H;
  o.w_qkv = p; p += 3 * H * H;
  o.b_qkv = p; p += 3 * H;
  o.w_o = p;   p += H * H;
  o.b_o = p;   p += H;
  o.ln2_g = p; p += H;
  o.ln2_b = p; p += H;
  o.w_fc1 = p; p += F * H;
  o.b_fc1 = p; p += F;
  o.w_fc2 = p; p += H * F;
  o.b_fc2 = p; p += H;
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
  if (!(d->ln_eps >= 0.f)) return fail(CEPHALO_EINVAL, "layer desc: ln_eps %g < 0", d->ln_eps);
  if (d->hidden % 8 != 0 || d->mlp % 8 != 0)
    return fail(CEPHALO_EUNSUPPORTED, "layer desc: hidden %d and mlp %d must be multiples of 8 (16-byte rows)", d->hidden, d->mlp);
  const int hd = d->hidden / d->heads;
  if (hd > 128) return fail(CEPHALO_EUNSUPPORTED, "layer desc: head dim %d > 128", hd);
  if (d->dtype == CEPHALO_BF16 && hd != 64 && hd != 128)
    return fail(CEPHALO_EUNSUPPORTED, "layer desc: bf16 attention needs head dim 64 or 128, got %d", hd);
  if (d->hidden > 8192) return fail(CEPHALO_EUNSUPPORTED, "layer desc: hidden %d > 8192", d->hidden);
  return CEPHALO_OK;
}

struct SaveLayout {
  size_t mean1, rstd1, u, qkv, lse, O, x1, mean2, rstd2, u2, z, h, total;
};
struct ScratchLayout {
  size_t dz, du2, dx1, dO, dqkv, du, dvec, partials, partial_bytes, total;
};

SaveLayout save_layout(const cephalo_layer_desc& d, int m) {
  const size_t es = d.dtype == CEPHALO_F32 ? 4 : 2;
  const size_t T = (size_t)m * d.seq, H = d.hidden, F = d.mlp;
  SaveLayout L;
  size_t p = 0;
  auto take = [&](size_t bytes) { size_t at = p; p += align_up(bytes); return at; };
  L.mean1 = take(T * 4); L.rstd1 = take(T * 4);
  L.u = take(T * H * es);
  L.qkv = take(T * 3 * H * es);
  L.lse = take((size_t)m * d.heads * d.seq * 4);
  L.O = take(T * H * es);
  L.x1 = take(T * H * es);
  L.mean2 = take(T * 4); L.rstd2 = take(T * 4);
  L.u2 = take(T * H * es);
  L.z = take(T * F * es);
  L.h = take(T * F * es);
  L.total = p;
  return L;
}

ScratchLayout scratch_layout(const cephalo_layer_desc& d, int m) {
  const size_t es = d.dtype == CEPHALO_F32 ? 4 : 2;
  const size_t T = (size_t)m * d.seq, H = d.hidden, F = d.mlp;
  ScratchLayout L;
  size_t p = 0;
  auto take = [&](size_t bytes) { size_t at = p; p += align_up(bytes); return at; };
  L.dz = take(T * F * es);
  L.du2 = take(T * H * es);
  L.dx1 = take(T * H * es);
  L.dO = take(T * H * es);
  L.dqkv = take(T * 3 * H * es);
  L.du = take(T * H * es);
  L.dvec = take((size_t)m * d.heads * d.seq * 4);
  const int widest = (int)(3 * H > F ? 3 * H : F);
  size_t pb = ln_bwd_partial_bytes((int)T, (int)H);
  const size_t cb = colsum_partial_bytes((int)T, widest);
  if (cb > pb) pb = cb;
  L.partial_bytes = pb;
  L.partials = take(pb);
  L.total = p;
  return L;
}

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
template <typename T>
int attn_bwd(const T* qkv, const T* O, const T* dO, const float* lse, float* dvec, T* dqkv, int m, int S, int H, int A, int causal, hipStream_t s);
template <> int attn_bwd<float>(const float* qkv, const float* O, const float* dO, const float* lse, float* dvec, float* dqkv,
                                int m, int S, int H, int A, int causal, hipStream_t s) {
  return launch_attn_bwd_simple<float>(qkv, O, dO, lse, dvec, dqkv, m, S, H, A, causal, s);
}
template <> int attn_bwd<bf16>(const bf16* qkv, const bf16* O, const bf16* dO, const float* lse, float* dvec, bf16* dqkv,
                               int m, int S, int H, int A, int causal, hipStream_t s) {
  return launch_attn_bwd_mfma(qkv, O, dO, lse, dvec, dqkv, m, S, H, A, causal, s);
}

#define TRY(expr) do { int rc__ = (expr); if (rc__ != CEPHALO_OK) return rc__; } while (0)

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

template <typename T>
int layer_fwd_t(const cephalo_layer_desc& d, const T* P, const T* x, T* y, int m, void* save, hipStream_t s) {
  const ParamOffsets o = param_offsets(d);
  const SaveLayout L = save_layout(d, m);
  const int Tn = m * d.seq, H = d.hidden, F = d.mlp;
  T* u = at<T>(save, L.u); T* qkv = at<T>(save, L.qkv); T* O = at<T>(save, L.O); T* x1 = at<T>(save, L.x1);
  T* u2 = at<T>(save, L.u2); T* z = at<T>(save, L.z); T* h = at<T>(save, L.h);

  TRY(launch_ln_fwd<T>(x, P + o.ln1_g, P + o.ln1_b, u, at<float>(save, L.mean1), at<float>(save, L.rstd1), Tn, H, d.ln_eps, s));
  {
    GemmArgs<T> a = linear_fwd<T>(u, P + o.w_qkv, Tn, 3 * H, H);
    a.epi = EPI_BIAS; a.bias = P + o.b_qkv; a.C = qkv;
    TRY(gemm<T>(a, s));
  }
  TRY(attn_fwd<T>(qkv, O, at<float>(save, L.lse), m, d.seq, H, d.heads, d.causal, s));
  {
    GemmArgs<T> a = linear_fwd<T>(O, P + o.w_o, Tn, H, H);
    a.epi = EPI_BIAS_RESID; a.bias = P + o.b_o; a.R = x; a.C = x1;
    TRY(gemm<T>(a, s));
  }
  TRY(launch_ln_fwd<T>(x1, P + o.ln2_g, P + o.ln2_b, u2, at<float>(save, L.mean2), at<float>(save, L.rstd2), Tn, H, d.ln_eps, s));
  {
    GemmArgs<T> a = linear_fwd<T>(u2, P + o.w_fc1, Tn, F, H);
    a.epi = EPI_BIAS_GELU; a.bias = P + o.b_fc1; a.Z = z; a.C = h;
    TRY(gemm<T>(a, s));
  }
  {
    GemmArgs<T> a = linear_fwd<T>(h, P + o.w_fc2, Tn, H, F);
    a.epi = EPI_BIAS_RESID; a.bias = P + o.b_fc2; a.R = x1; a.C = y;
    TRY(gemm<T>(a, s));
  }
  return CEPHALO_OK;
}

template <typename T>
int layer_bwd_t(const cephalo_layer_desc& d, const T* P, const T* x, const T* dy, T* dx, int m, const void* save,
                float* G, float scale, int acc, void* scratch, hipStream_t s) {
  const ParamOffsets o = param_offsets(d);
  const SaveLayout L = save_layout(d, m);
  const ScratchLayout W = scratch_layout(d, m);
  const int Tn = m * d.seq, H = d.hidden, F = d.mlp;
  const T* u = at<T>(save, L.u); const T* qkv = at<T>(save, L.qkv); const T* O = at<T>(save, L.O);
  const T* x1 = at<T>(save, L.x1); const T* u2 = at<T>(save, L.u2); const T* z = at<T>(save, L.z); const T* h = at<T>(save, L.h);
  T* dz = at<T>(scratch, W.dz); T* du2 = at<T>(scratch, W.du2); T* dx1 = at<T>(scratch, W.dx1);
  T* dO = at<T>(scratch, W.dO); T* dqkv = at<T>(scratch, W.dqkv); T* du = at<T>(scratch, W.du);
  float* dvec = at<float>(scratch, W.dvec);
  float* part = at<float>(scratch, W.partials);

  // y = x1 + h W2^T + b2
  TRY(launch_colsum<T>(dy, part, W.partial_bytes, G + o.b_fc2, scale, acc, Tn, H, s));
  TRY(gemm<T>(linear_wgrad<T>(dy, h, Tn, H, F, G + o.w_fc2, scale, acc), s));
  {
    GemmArgs<T> a = linear_dgrad<T>(dy, P + o.w_fc2, Tn, H, F);   // dh, then dz = dh * gelu'(z)
    a.epi = EPI_DGELU; a.Z = const_cast<T*>(z); a.C = dz;
    TRY(gemm<T>(a, s));
  }
  // z = u2 W1^T + b1
  TRY(launch_colsum<T>(dz, part, W.partial_bytes, G + o.b_fc1, scale, acc, Tn, F, s));
  TRY(gemm<T>(linear_wgrad<T>(dz, u2, Tn, F, H, G + o.w_fc1, scale, acc), s));
  {
    GemmArgs<T> a = linear_dgrad<T>(dz, P + o.w_fc1, Tn, F, H);
    a.epi = EPI_NONE; a.C = du2;
    TRY(gemm<T>(a, s));
  }
  // u2 = LN2(x1); dx1 = dy + LN2-backward(du2)
  TRY(launch_ln_bwd<T>(du2, x1, at<float>(save, L.mean2), at<float>(save, L.rstd2), P + o.ln2_g, dy, dx1,
                       part, W.partial_bytes, G + o.ln2_g, G + o.ln2_b, scale, acc, Tn, H, s));
  // x1 = x + O Wo^T + bo
  TRY(launch_colsum<T>(dx1, part, W.partial_bytes, G + o.b_o, scale, acc, Tn, H, s));
  TRY(gemm<T>(linear_wgrad<T>(dx1, O, Tn, H, H, G + o.w_o, scale, acc), s));
  {
    GemmArgs<T> a = linear_dgrad<T>(dx1, P + o.w_o, Tn, H, H);
    a.epi = EPI_NONE; a.C = dO;
    TRY(gemm<T>(a, s));
  }
  TRY(attn_bwd<T>(qkv, O, dO, at<float>(save, L.lse), dvec, dqkv, m, d.seq, H, d.heads, d.causal, s));
  // qkv = u Wqkv^T + bqkv
  TRY(launch_colsum<T>(dqkv, part, W.partial_bytes, G + o.b_qkv, scale, acc, Tn, 3 * H, s));
  TRY(gemm<T>(linear_wgrad<T>(dqkv, u, Tn, 3 * H, H, G + o.w_qkv, scale, acc), s));
  {
    GemmArgs<T> a = linear_dgrad<T>(dqkv, P + o.w_qkv, Tn, 3 * H, H);
    a.epi = EPI_NONE; a.C = du;
    TRY(gemm<T>(a, s));
  }
  // u = LN1(x); dx = dx1 + LN1-backward(du)
  TRY(launch_ln_bwd<T>(du, x, at<float>(save, L.mean1), at<float>(save, L.rstd1), P + o.ln1_g, dx1, dx,
                       part, W.partial_bytes, G + o.ln1_g, G + o.ln1_b, scale, acc, Tn, H, s));
  return CEPHALO_OK;
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

using namespace cephalo;

extern "C" int64_t cephalo_layer_param_count(const cephalo_layer_desc* desc) {
  const int rc = check_desc(desc);
  if (rc != CEPHALO_OK) return rc;
  return param_offsets(*desc).total;
}

extern "C" int cephalo_layer_param_offsets(const cephalo_layer_desc* desc, int64_t* offsets) {
  TRY(check_desc(desc));
  if (!offsets) return fail(CEPHALO_EINVAL, "param_offsets: null output");
  const ParamOffsets o = param_offsets(*desc);
  const int64_t v[12] = {o.ln1_g, o.ln1_b, o.w_qkv, o.b_qkv, o.w_o, o.b_o, o.ln2_g, o.ln2_b, o.w_fc1, o.b_fc1, o.w_fc2, o.b_fc2};
  for (int i = 0; i < 12; ++i) offsets[i] = v[i];
  return CEPHALO_OK;
}

extern "C" int cephalo_layer_workspace_bytes(const cephalo_layer_desc* desc, int32_t micro_batch,
                                             size_t* save_bytes, size_t* scratch_bytes) {
  TRY(check_desc(desc));
  if (micro_batch <= 0) return fail(CEPHALO_EINVAL, "workspace_bytes: micro-batch size m = %d must be positive", micro_batch);
  if (!save_bytes || !scratch_bytes) return fail(CEPHALO_EINVAL, "workspace_bytes: null output");
  *save_bytes = save_layout(*desc, micro_batch).total;
  *scratch_bytes = scratch_layout(*desc, micro_batch).total;
  return CEPHALO_OK;
}

extern "C" int cephalo_layer_fwd(const cephalo_layer_desc* desc, const void* flat_param,
                                 const void* x, void* y, int32_t micro_batch,
                                 void* save, size_t save_bytes,
                                 void* scratch, size_t scratch_bytes, void* stream) {
  TRY(check_io("layer_fwd", desc, micro_batch, {flat_param, x, y, save}));
  if (x == y) return fail(CEPHALO_EINVAL, "layer_fwd: y may not alias x");
  if (save_bytes < save_layout(*desc, micro_batch).total)
    return fail(CEPHALO_EWORKSPACE, "layer_fwd: save area %zu B < %zu B", save_bytes, save_layout(*desc, micro_batch).total);
  (void)scratch; (void)scratch_bytes;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (desc->dtype == CEPHALO_F32)
    return layer_fwd_t<float>(*desc, static_cast<const float*>(flat_param), static_cast<const float*>(x),
                              static_cast<float*>(y), micro_batch, save, s);
  return layer_fwd_t<bf16>(*desc, static_cast<const bf16*>(flat_param), static_cast<const bf16*>(x),
                           static_cast<bf16*>(y), micro_batch, save, s);
}

extern "C" int cephalo_layer_bwd(const cephalo_layer_desc* desc, const void* flat_param,
                                 const void* x, const void* dy, void* dx, int32_t micro_batch,
                                 const void* save, size_t save_bytes,
                                 float* flat_grad, float grad_scale, int32_t accumulate,
                                 void* scratch, size_t scratch_bytes, void* stream) {
  TRY(check_io("layer_bwd", desc, micro_batch, {flat_param, x, dy, dx, save, flat_grad, scratch}));
  if (dx == dy) return fail(CEPHALO_EINVAL, "layer_bwd: dx may not alias dy");
  if (accumulate != 0 && accumulate != 1) return fail(CEPHALO_EINVAL, "layer_bwd: accumulate must be 0 or 1");
  if (save_bytes < save_layout(*desc, micro_batch).total)
    return fail(CEPHALO_EWORKSPACE, "layer_bwd: save area %zu B < %zu B", save_bytes, save_layout(*desc, micro_batch).total);
  if (scratch_bytes < scratch_layout(*desc, micro_batch).total)
    return fail(CEPHALO_EWORKSPACE, "layer_bwd: scratch %zu B < %zu B", scratch_bytes, scratch_layout(*desc, micro_batch).total);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (desc->dtype == CEPHALO_F32)
    return layer_bwd_t<float>(*desc, static_cast<const float*>(flat_param), static_cast<const float*>(x),
                              static_cast<const float*>(dy), static_cast<float*>(dx), micro_batch, save,
                              flat_grad, grad_scale, accumulate, scratch, s);
  return layer_bwd_t<bf16>(*desc, static_cast<const bf16*>(flat_param), static_cast<const bf16*>(x),
                           static_cast<const bf16*>(dy), static_cast<bf16*>(dx), micro_batch, save,
                           flat_grad, grad_scale, accumulate, scratch, s);
}

extern "C" int cephalo_share_layer_step(const cephalo_layer_desc* desc, const void* flat_param,
                                        const void* x, void* y, const void* dy, void* dx,
                                        int32_t batch_share, int32_t micro_batch,
                                        void* save, size_t save_bytes_total,
                                        float* flat_grad, float grad_scale,
                                        void* scratch, size_t scratch_bytes, void* stream) {
  TRY(check_io("share_layer_step", desc, micro_batch, {flat_param, x, y, dy, dx, save, flat_grad, scratch}));
  if (batch_share <= 0 || batch_share % micro_batch != 0)
    return fail(CEPHALO_EINVAL, "share_layer_step: batch share b = %d is not a positive multiple of micro-batch size m = %d",
                batch_share, micro_batch);
  const int l = batch_share / micro_batch;
  const size_t per = save_layout(*desc, micro_batch).total;
  if (save_bytes_total < per * (size_t)l)
    return fail(CEPHALO_EWORKSPACE, "share_layer_step: save area %zu B < %d micro-batches x %zu B", save_bytes_total, l, per);
  const size_t es = desc->dtype == CEPHALO_F32 ? 4 : 2;
  const size_t act = (size_t)micro_batch * desc->seq * desc->hidden * es;  // bytes of one micro-batch of x / y
  for (int j = 0; j < l; ++j)
    TRY(cephalo_layer_fwd(desc, flat_param, static_cast<const char*>(x) + j * act, static_cast<char*>(y) + j * act,
                          micro_batch, static_cast<char*>(save) + j * per, per, scratch, scratch_bytes, stream));
  for (int j = 0; j < l; ++j)
    TRY(cephalo_layer_bwd(desc, flat_param, static_cast<const char*>(x) + j * act, static_cast<const char*>(dy) + j * act,
                          static_cast<char*>(dx) + j * act, micro_batch, static_cast<char*>(save) + j * per, per,
                          flat_grad, grad_scale, j > 0, scratch, scratch_bytes, stream));
  return CEPHALO_OK;
}
