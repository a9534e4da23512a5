// C-ABI entry points of the individual building blocks (GEMM family, attention).
#include "layer_impl.h"

using namespace cephalo;

namespace {
template <typename T>
int op_gemm_t(const void* A, int64_t a_rs, int64_t a_cs, const void* B, int64_t b_rs, int64_t b_cs,
              int M, int N, int K, int epi, void* C, const void* bias, const void* R, void* Z,
              float* G, float scale, int accumulate, GemmArgs<T>* out) {
  GemmArgs<T>& a = *out;
  a.A = static_cast<const T*>(A); a.a_rs = a_rs; a.a_cs = a_cs;
  a.B = static_cast<const T*>(B); a.b_rs = b_rs; a.b_cs = b_cs;
  a.M = M; a.N = N; a.K = K; a.epi = epi;
  a.C = static_cast<T*>(C); a.bias = static_cast<const T*>(bias); a.R = static_cast<const T*>(R);
  a.Z = static_cast<T*>(Z); a.G = G; a.scale = scale; a.accumulate = accumulate;
  return CEPHALO_OK;
}

int check_attn(const cephalo_layer_desc* d, int m) {
  if (!d) return fail(CEPHALO_EINVAL, "attention: null desc");
  if (d->hidden <= 0 || d->heads <= 0 || d->seq <= 0 || d->hidden % d->heads != 0 || m <= 0)
    return fail(CEPHALO_EINVAL, "attention: bad sizes hidden %d heads %d seq %d m %d", d->hidden, d->heads, d->seq, m);
  const int hd = d->hidden / d->heads;
  if (hd > 128) return fail(CEPHALO_EUNSUPPORTED, "attention: head dim %d > 128", hd);
  if (d->dtype == CEPHALO_BF16 && hd % 8 != 0)
    return fail(CEPHALO_EUNSUPPORTED, "attention: bf16 needs a head dim that is a multiple of 8, got %d", hd);
  if (d->dtype != CEPHALO_F32 && d->dtype != CEPHALO_BF16) return fail(CEPHALO_EINVAL, "attention: unknown dtype %d", d->dtype);
  return CEPHALO_OK;
}
}  // namespace

extern "C" int32_t cephalo_gemm_side_by_side(int32_t kernels) { return cephalo::gemm_set_side_by_side(kernels); }
extern "C" int64_t cephalo_gemm_general_count(void) { return cephalo::gemm_general_count(); }

extern "C" int cephalo_op_gemm(int32_t dtype, const void* A, int64_t a_rs, int64_t a_cs,
                               const void* B, int64_t b_rs, int64_t b_cs, int32_t M, int32_t N, int32_t K,
                               int32_t epilogue, void* C, const void* bias, const void* R, void* Z,
                               float* G, float scale, int32_t accumulate, void* stream) {
  if (M <= 0 || N <= 0 || K <= 0) return fail(CEPHALO_EINVAL, "op_gemm: sizes %d x %d x %d must be positive", M, N, K);
  if (!A || !B) return fail(CEPHALO_EINVAL, "op_gemm: null operand");
  if ((a_rs != 1 && a_cs != 1) || (b_rs != 1 && b_cs != 1)) return fail(CEPHALO_EINVAL, "op_gemm: one stride of each operand must be 1");
  if (a_rs <= 0 || a_cs <= 0 || b_rs <= 0 || b_cs <= 0) return fail(CEPHALO_EINVAL, "op_gemm: strides must be positive");
  bool need_c = epilogue != EPI_GRAD, need_bias = false, need_r = false, need_z = false;
  const bool f32_out = epilogue == CEPHALO_EPI_NONE_F32 || epilogue == CEPHALO_EPI_BIAS_RESID_F32;
  if (epilogue == CEPHALO_EPI_NONE_F32) epilogue = EPI_NONE;
  if (epilogue == CEPHALO_EPI_BIAS_RESID_F32) epilogue = EPI_BIAS_RESID;
  if (epilogue == CEPHALO_EPI_BIAS_GELU_DERIV) epilogue = EPI_BIAS_GELU_DERIV;      // (public and internal numbers differ)
  else if (epilogue == CEPHALO_EPI_MUL) epilogue = EPI_MUL;
  else if (epilogue == EPI_BIAS_GELU_DERIV || epilogue == EPI_MUL) epilogue = -1;
  switch (epilogue) {
    case EPI_NONE: break;
    case EPI_BIAS: need_bias = true; break;
    case EPI_BIAS_RESID: need_bias = need_r = true; break;
    case EPI_BIAS_GELU: need_bias = need_z = true; break;
    case EPI_DGELU: need_z = true; break;
    case EPI_BIAS_GELU_DERIV: need_bias = need_z = true; break;
    case EPI_MUL: need_z = true; break;
    case EPI_GRAD: if (!G) return fail(CEPHALO_EINVAL, "op_gemm: EPI_GRAD needs G"); break;
    default: return fail(CEPHALO_EINVAL, "op_gemm: unknown epilogue %d", epilogue);
  }
  if ((need_c && !C) || (need_bias && !bias) || (need_r && !R) || (need_z && !Z))
    return fail(CEPHALO_EINVAL, "op_gemm: epilogue %d lacks a buffer", epilogue);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dtype == CEPHALO_F32) {
    GemmArgs<float> a = {};
    op_gemm_t<float>(A, a_rs, a_cs, B, b_rs, b_cs, M, N, K, epilogue, C, bias, R, Z, G, scale, accumulate, &a);
    return launch_gemm_simple<float>(a, s);     // fp32 mode: C and R are fp32 anyway
  }
  if (dtype == CEPHALO_BF16) {
    GemmArgs<bf16> a = {};
    op_gemm_t<bf16>(A, a_rs, a_cs, B, b_rs, b_cs, M, N, K, epilogue, C, bias, R, Z, G, scale, accumulate, &a);
    if (f32_out) { a.Cf = static_cast<float*>(C); a.Rf = static_cast<const float*>(R); a.C = nullptr; a.R = nullptr; }
    return launch_gemm_mfma(a, s);
  }
  return fail(CEPHALO_EINVAL, "op_gemm: unknown dtype %d", dtype);
}

namespace {
// workspace of linear_wgrad: the partial sums of a split token axis
size_t wgrad_part_bytes(int dtype, int T, int N, int K) {
  if (dtype != CEPHALO_BF16) return 0;
  const int sp = gemm_grad_splits(N, K, T);
  return sp > 1 ? (size_t)sp * N * K * sizeof(float) : 0;
}
}  // namespace

extern "C" size_t cephalo_op_linear_wgrad_workspace(int32_t dtype, int32_t T, int32_t N, int32_t K) {
  if (T <= 0 || N <= 0 || K <= 0) return 0;
  return wgrad_part_bytes(dtype, T, N, K) + 256;
}

extern "C" int cephalo_op_linear_wgrad(int32_t dtype, const void* dY, const void* X, int32_t T, int32_t N, int32_t K,
                                       float* G, float scale, int32_t accumulate, void* workspace, size_t workspace_bytes, void* stream) {
  if (T <= 0 || N <= 0 || K <= 0) return fail(CEPHALO_EINVAL, "linear_wgrad: sizes %d x %d x %d must be positive", T, N, K);
  if (!dY || !X || !G) return fail(CEPHALO_EINVAL, "linear_wgrad: null buffer");
  if (accumulate != 0 && accumulate != 1) return fail(CEPHALO_EINVAL, "linear_wgrad: accumulate must be 0 or 1");
  if (dtype != CEPHALO_F32 && dtype != CEPHALO_BF16) return fail(CEPHALO_EINVAL, "linear_wgrad: unknown dtype %d", dtype);
  if (workspace_bytes < cephalo_op_linear_wgrad_workspace(dtype, T, N, K) || (dtype == CEPHALO_BF16 && !workspace))
    return fail(CEPHALO_EWORKSPACE, "linear_wgrad: workspace %zu B < %zu B", workspace_bytes, cephalo_op_linear_wgrad_workspace(dtype, T, N, K));
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dtype == CEPHALO_F32)
    return wgrad<float>(static_cast<const float*>(dY), static_cast<const float*>(X), T, N, K, G, scale, accumulate, nullptr, s);
  float* part = wgrad_part_bytes(dtype, T, N, K) ? static_cast<float*>(workspace) : nullptr;
  return wgrad<bf16>(static_cast<const bf16*>(dY), static_cast<const bf16*>(X), T, N, K, G, scale, accumulate, part, s);
}

// work area of linear_wgrad_bias: [pieces of a split token axis | pieces of the column sums | the column-sum kernel's partials]
extern "C" size_t cephalo_op_linear_wgrad_bias_workspace(int32_t dtype, int32_t T, int32_t N, int32_t K) {
  if (T <= 0 || N <= 0 || K <= 0) return 0;
  const size_t rs = dtype == CEPHALO_BF16 ? gemm_rowsum_part_bytes(N, K) : 0;
  return align_up(wgrad_part_bytes(dtype, T, N, K)) + align_up(rs) + colsum_partial_bytes(T, N) + 256;
}

extern "C" int cephalo_op_linear_wgrad_bias(int32_t dtype, const void* dY, const void* X, int32_t T, int32_t N, int32_t K,
                                            float* G, float* gb, float scale, int32_t accumulate, void* workspace,
                                            size_t workspace_bytes, void* stream) {
  if (T <= 0 || N <= 0 || K <= 0) return fail(CEPHALO_EINVAL, "linear_wgrad_bias: sizes %d x %d x %d must be positive", T, N, K);
  if (!dY || !X || !G || !gb || !workspace) return fail(CEPHALO_EINVAL, "linear_wgrad_bias: null buffer");
  if (accumulate != 0 && accumulate != 1) return fail(CEPHALO_EINVAL, "linear_wgrad_bias: accumulate must be 0 or 1");
  if (dtype != CEPHALO_F32 && dtype != CEPHALO_BF16) return fail(CEPHALO_EINVAL, "linear_wgrad_bias: unknown dtype %d", dtype);
  if (N % 8 != 0) return fail(CEPHALO_EUNSUPPORTED, "linear_wgrad_bias: the output width %d must be a multiple of 8", N);
  for (const void* p : {dY, X, (const void*)G, (const void*)gb, (const void*)workspace})
    if (reinterpret_cast<uintptr_t>(p) % 16 != 0) return fail(CEPHALO_EINVAL, "linear_wgrad_bias: buffers must be 16-byte aligned");
  if (workspace_bytes < cephalo_op_linear_wgrad_bias_workspace(dtype, T, N, K))
    return fail(CEPHALO_EWORKSPACE, "linear_wgrad_bias: workspace %zu B < %zu B", workspace_bytes, cephalo_op_linear_wgrad_bias_workspace(dtype, T, N, K));
  hipStream_t s = static_cast<hipStream_t>(stream);
  char* w = static_cast<char*>(workspace);
  const size_t part_bytes = wgrad_part_bytes(dtype, T, N, K), rs_bytes = dtype == CEPHALO_BF16 ? gemm_rowsum_part_bytes(N, K) : 0;
  float* col_part = reinterpret_cast<float*>(w + align_up(part_bytes) + align_up(rs_bytes));
  const size_t col_bytes = colsum_partial_bytes(T, N);
  if (dtype == CEPHALO_F32) {
    TRY(wgrad<float>(static_cast<const float*>(dY), static_cast<const float*>(X), T, N, K, G, scale, accumulate, nullptr, s));
    return launch_colsum<float>(static_cast<const float*>(dY), col_part, col_bytes, gb, scale, accumulate, T, N, s);
  }
  ColsumsBeside cb = {gb, reinterpret_cast<float*>(w + align_up(part_bytes)), rs_bytes, false};
  TRY(wgrad<bf16>(static_cast<const bf16*>(dY), static_cast<const bf16*>(X), T, N, K, G, scale, accumulate,
                  part_bytes ? reinterpret_cast<float*>(w) : nullptr, s, 0, &cb));
  if (cb.done) return CEPHALO_OK;
  return launch_colsum<bf16>(static_cast<const bf16*>(dY), col_part, col_bytes, gb, scale, accumulate, T, N, s);
}

extern "C" int cephalo_op_attention_fwd(const cephalo_layer_desc* d, const void* qkv, void* O, float* lse,
                                        int32_t m, void* stream) {
  int rc = check_attn(d, m);
  if (rc != CEPHALO_OK) return rc;
  if (!qkv || !O || !lse) return fail(CEPHALO_EINVAL, "attention_fwd: null buffer");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (d->dtype == CEPHALO_F32)
    return launch_attn_fwd_simple<float>(static_cast<const float*>(qkv), static_cast<float*>(O), lse, m, d->seq, d->hidden, d->heads, d->causal, s);
  return launch_attn_fwd_mfma(static_cast<const bf16*>(qkv), static_cast<bf16*>(O), lse, m, d->seq, d->hidden, d->heads, d->causal, s);
}

extern "C" int cephalo_op_attention_bwd(const cephalo_layer_desc* d, const void* qkv, const void* O, const void* dO,
                                        const float* lse, float* dvec, void* dqkv, int32_t m, void* stream) {
  int rc = check_attn(d, m);
  if (rc != CEPHALO_OK) return rc;
  if (!qkv || !O || !dO || !lse || !dvec || !dqkv) return fail(CEPHALO_EINVAL, "attention_bwd: null buffer");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (d->dtype == CEPHALO_F32)
    return launch_attn_bwd_simple<float>(static_cast<const float*>(qkv), static_cast<const float*>(O), static_cast<const float*>(dO),
                                         lse, dvec, static_cast<float*>(dqkv), m, d->seq, d->hidden, d->heads, d->causal, s);
  return launch_attn_bwd_mfma(static_cast<const bf16*>(qkv), static_cast<const bf16*>(O), static_cast<const bf16*>(dO),
                              lse, dvec, static_cast<bf16*>(dqkv), m, d->seq, d->hidden, d->heads, d->causal, s);
}
