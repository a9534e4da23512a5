#include "kernels.h"
namespace cephalo {
int launch_gemm_mfma(const GemmArgs<bf16>& a, hipStream_t s) { return launch_gemm_simple<bf16>(a, s); }
}
