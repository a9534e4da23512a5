// C-ABI entry points of the individual building blocks (GEMM family, attention).
#include "kernels.h"

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
  if (d->dtype == CEPHALO_BF16 && hd != 64 && hd != 128)
    return fail(CEPHALO_EUNSUPPORTED, "attention: bf16 needs head dim 64 or 128, got %d", hd);
  if (d->dtype != CEPHALO_F32 && d->dtype != CEPHALO_BF16) return fail(CEPHALO_EINVAL, "attention: unknown dtype %d", d->dtype);
  return CEPHALO_OK;
}
}  // namespace

extern "C" int cephalo_op_gemm(int32_t dtype, const void* A, int64_t a_rs, int64_t a_cs,
                               const void* B, int64_t b_rs, int64_t b_cs, int32_t M, int32_t N, int32_t K,
                               int32_t epilogue, void* C, const void* bias, const void* R, void* Z,
                               float* G, float scale, int32_t accumulate, void* stream) {
  if (M <= 0 || N <= 0 || K <= 0) return fail(CEPHALO_EINVAL, "op_gemm: sizes %d x %d x %d must be positive", M, N, K);
  if (!A || !B) return fail(CEPHALO_EINVAL, "op_gemm: null operand");
  if ((a_rs != 1 && a_cs != 1) || (b_rs != 1 && b_cs != 1)) return fail(CEPHALO_EINVAL, "op_gemm: one stride of each operand must be 1");
  if (a_rs <= 0 || a_cs <= 0 || b_rs <= 0 || b_cs <= 0) return fail(CEPHALO_EINVAL, "op_gemm: strides must be positive");
  bool need_c = epilogue != EPI_GRAD, need_bias = false, need_r = false, need_z = false;
  switch (epilogue) {
    case EPI_NONE: break;
    case EPI_BIAS: need_bias = true; break;
    case EPI_BIAS_RESID: need_bias = need_r = true; break;
    case EPI_BIAS_GELU: need_bias = need_z = true; break;
    case EPI_DGELU: need_z = true; break;
    case EPI_GRAD: if (!G) return fail(CEPHALO_EINVAL, "op_gemm: EPI_GRAD needs G"); break;
    default: return fail(CEPHALO_EINVAL, "op_gemm: unknown epilogue %d", epilogue);
  }
  if ((need_c && !C) || (need_bias && !bias) || (need_r && !R) || (need_z && !Z))
    return fail(CEPHALO_EINVAL, "op_gemm: epilogue %d lacks a buffer", epilogue);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dtype == CEPHALO_F32) {
    GemmArgs<float> a = {};
    op_gemm_t<float>(A, a_rs, a_cs, B, b_rs, b_cs, M, N, K, epilogue, C, bias, R, Z, G, scale, accumulate, &a);
    return launch_gemm_simple<float>(a, s);
  }
  if (dtype == CEPHALO_BF16) {
    GemmArgs<bf16> a = {};
    op_gemm_t<bf16>(A, a_rs, a_cs, B, b_rs, b_cs, M, N, K, epilogue, C, bias, R, Z, G, scale, accumulate, &a);
    return launch_gemm_mfma(a, s);
  }
  return fail(CEPHALO_EINVAL, "op_gemm: unknown dtype %d", dtype);
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
