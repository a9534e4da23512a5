#include "kernels.h"
namespace cephalo {
int launch_attn_fwd_mfma(const bf16* qkv, bf16* O, float* lse, int m, int S, int H, int A, int causal, hipStream_t s) {
  return launch_attn_fwd_simple<bf16>(qkv, O, lse, m, S, H, A, causal, s);
}
int launch_attn_bwd_mfma(const bf16* qkv, const bf16* O, const bf16* dO, const float* lse, float* dvec, bf16* dqkv,
                         int m, int S, int H, int A, int causal, hipStream_t s) {
  return launch_attn_bwd_simple<bf16>(qkv, O, dO, lse, dvec, dqkv, m, S, H, A, causal, s);
}
}
