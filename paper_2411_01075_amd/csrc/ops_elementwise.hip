// C-ABI entry points of the bandwidth-bound building blocks (norm forward / backward, bias column sum), so that each
// can be checked against the oracle and timed on its own.
#include "layer_impl.h"

using namespace cephalo;

namespace {
int check_norm(const char* who, int dtype, int rows, int H) {
  if (dtype != CEPHALO_F32 && dtype != CEPHALO_BF16) return fail(CEPHALO_EINVAL, "%s: unknown dtype %d", who, dtype);
  if (rows <= 0 || H <= 0) return fail(CEPHALO_EINVAL, "%s: %d rows of %d must be positive", who, rows, H);
  if (H % 8 != 0) return fail(CEPHALO_EUNSUPPORTED, "%s: the row width %d must be a multiple of 8", who, H);
  const int widest = dtype == CEPHALO_F32 ? 4096 : 8192;      // one row per wavefront, held in registers
  if (H > widest) return fail(CEPHALO_EUNSUPPORTED, "%s: row width %d > %d (the limit for this dtype)", who, H, widest);
  return CEPHALO_OK;
}
bool all_aligned(std::initializer_list<const void*> ptrs) {
  for (const void* p : ptrs)
    if (!aligned16(p)) return false;
  return true;
}
size_t norm_bwd_part_floats(int rows, int H) { return (size_t)ln_bwd_blocks(rows) * H; }
}  // namespace

extern "C" int cephalo_op_norm_fwd(int32_t dtype, int32_t rms, const float* x, const void* gamma, const void* beta, void* u,
                                   float* mean, float* rstd, int32_t rows, int32_t H, float eps, void* stream) {
  TRY(check_norm("norm_fwd", dtype, rows, H));
  if (!x || !gamma || !u || !mean || !rstd || (!rms && !beta)) return fail(CEPHALO_EINVAL, "norm_fwd: null buffer");
  if (!all_aligned({x, gamma, beta, u})) return fail(CEPHALO_EINVAL, "norm_fwd: buffers must be 16-byte aligned");
  if (!(eps >= 0.f)) return fail(CEPHALO_EINVAL, "norm_fwd: eps %g < 0", eps);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dtype == CEPHALO_F32)
    return launch_ln_fwd<float>(x, static_cast<const float*>(gamma), static_cast<const float*>(beta), static_cast<float*>(u), mean, rstd, rows, H, eps, s, rms != 0);
  return launch_ln_fwd<bf16>(x, static_cast<const bf16*>(gamma), static_cast<const bf16*>(beta), static_cast<bf16*>(u), mean, rstd, rows, H, eps, s, rms != 0);
}

extern "C" size_t cephalo_op_norm_bwd_workspace(int32_t rows, int32_t H) {
  if (rows <= 0 || H <= 0) return 0;
  return (2 * norm_bwd_part_floats(rows, H)) * sizeof(float) + reduce_tmp_bytes(ln_bwd_blocks(rows), H) + 256;
}

extern "C" int cephalo_op_norm_bwd(int32_t dtype, int32_t rms, const float* du, const float* x, const float* mean, const float* rstd,
                                   const void* gamma, const float* resid, float* dx, void* dx_lowp, float* dgamma, float* dbeta,
                                   int32_t rows, int32_t H, void* workspace, size_t workspace_bytes, void* stream) {
  TRY(check_norm("norm_bwd", dtype, rows, H));
  if (!du || !x || !mean || !rstd || !gamma || !dx || !dgamma || (!rms && !dbeta) || !workspace) return fail(CEPHALO_EINVAL, "norm_bwd: null buffer");
  if (!all_aligned({du, x, gamma, resid, dx, dx_lowp, dgamma, dbeta, workspace})) return fail(CEPHALO_EINVAL, "norm_bwd: buffers must be 16-byte aligned");
  if (workspace_bytes < cephalo_op_norm_bwd_workspace(rows, H))
    return fail(CEPHALO_EWORKSPACE, "norm_bwd: workspace %zu B < %zu B", workspace_bytes, cephalo_op_norm_bwd_workspace(rows, H));
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int nb = ln_bwd_blocks(rows);
  float* part_g = static_cast<float*>(workspace);
  float* part_b = part_g + norm_bwd_part_floats(rows, H);
  float* tmp = part_b + norm_bwd_part_floats(rows, H);
  const size_t tmp_bytes = reduce_tmp_bytes(nb, H);
  if (dtype == CEPHALO_F32)
    TRY(launch_ln_bwd<float>(du, x, mean, rstd, static_cast<const float*>(gamma), resid, dx, static_cast<float*>(nullptr), part_g, part_b, rows, H, s, rms != 0));
  else
    TRY(launch_ln_bwd<bf16>(du, x, mean, rstd, static_cast<const bf16*>(gamma), resid, dx, static_cast<bf16*>(dx_lowp), part_g, part_b, rows, H, s, rms != 0));
  TRY(launch_reduce_partials(part_g, nb, H, dgamma, 1.0f, 0, tmp, tmp_bytes, s));
  if (!rms) TRY(launch_reduce_partials(part_b, nb, H, dbeta, 1.0f, 0, tmp, tmp_bytes, s));
  return CEPHALO_OK;
}

// norm_bwd in the LayerNorm form with the column sums of its result as a third reduction
extern "C" size_t cephalo_op_norm_bwd_sums_workspace(int32_t rows, int32_t H) {
  if (rows <= 0 || H <= 0) return 0;
  return (3 * norm_bwd_part_floats(rows, H)) * sizeof(float) + reduce_tmp_bytes(ln_bwd_blocks(rows), H) + 256;
}

extern "C" int cephalo_op_norm_bwd_sums(int32_t dtype, const float* du, const float* x, const float* mean, const float* rstd,
                                        const void* gamma, const float* resid, float* dx, void* dx_lowp, float* dgamma, float* dbeta,
                                        float* dx_colsum, int32_t rows, int32_t H, void* workspace, size_t workspace_bytes, void* stream) {
  TRY(check_norm("norm_bwd_sums", dtype, rows, H));
  if (!du || !x || !mean || !rstd || !gamma || !dx || !dgamma || !dbeta || !dx_colsum || !workspace) return fail(CEPHALO_EINVAL, "norm_bwd_sums: null buffer");
  if (!all_aligned({du, x, gamma, resid, dx, dx_lowp, dgamma, dbeta, dx_colsum, workspace})) return fail(CEPHALO_EINVAL, "norm_bwd_sums: buffers must be 16-byte aligned");
  if (workspace_bytes < cephalo_op_norm_bwd_sums_workspace(rows, H))
    return fail(CEPHALO_EWORKSPACE, "norm_bwd_sums: workspace %zu B < %zu B", workspace_bytes, cephalo_op_norm_bwd_sums_workspace(rows, H));
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int nb = ln_bwd_blocks(rows);
  const size_t each = norm_bwd_part_floats(rows, H);
  float* part_g = static_cast<float*>(workspace);
  float* part_b = part_g + each;
  float* part_s = part_b + each;
  float* tmp = part_s + each;
  const size_t tmp_bytes = reduce_tmp_bytes(nb, H);
  if (dtype == CEPHALO_F32)
    TRY(launch_ln_bwd<float>(du, x, mean, rstd, static_cast<const float*>(gamma), resid, dx, static_cast<float*>(nullptr), part_g, part_b, rows, H, s, false, part_s));
  else
    TRY(launch_ln_bwd<bf16>(du, x, mean, rstd, static_cast<const bf16*>(gamma), resid, dx, static_cast<bf16*>(dx_lowp), part_g, part_b, rows, H, s, false, part_s));
  TRY(launch_reduce_partials(part_g, nb, H, dgamma, 1.0f, 0, tmp, tmp_bytes, s));
  TRY(launch_reduce_partials(part_b, nb, H, dbeta, 1.0f, 0, tmp, tmp_bytes, s));
  TRY(launch_reduce_partials(part_s, nb, H, dx_colsum, 1.0f, 0, tmp, tmp_bytes, s));
  return CEPHALO_OK;
}

extern "C" size_t cephalo_op_colsum_workspace(int32_t rows, int32_t N) {
  if (rows <= 0 || N <= 0) return 0;
  return colsum_partial_bytes(rows, N) + 256;
}

extern "C" int cephalo_op_colsum(int32_t dtype, const void* X, int32_t rows, int32_t N, float* g, float scale, int32_t accumulate,
                                 void* workspace, size_t workspace_bytes, void* stream) {
  if (dtype != CEPHALO_F32 && dtype != CEPHALO_BF16) return fail(CEPHALO_EINVAL, "colsum: unknown dtype %d", dtype);
  if (rows <= 0 || N <= 0) return fail(CEPHALO_EINVAL, "colsum: %d rows of %d must be positive", rows, N);
  if (N % 8 != 0) return fail(CEPHALO_EUNSUPPORTED, "colsum: the row width %d must be a multiple of 8", N);
  if (!X || !g || !workspace) return fail(CEPHALO_EINVAL, "colsum: null buffer");
  if (accumulate != 0 && accumulate != 1) return fail(CEPHALO_EINVAL, "colsum: accumulate must be 0 or 1");
  if (!all_aligned({X, g, workspace})) return fail(CEPHALO_EINVAL, "colsum: buffers must be 16-byte aligned");
  if (workspace_bytes < cephalo_op_colsum_workspace(rows, N))
    return fail(CEPHALO_EWORKSPACE, "colsum: workspace %zu B < %zu B", workspace_bytes, cephalo_op_colsum_workspace(rows, N));
  hipStream_t s = static_cast<hipStream_t>(stream);
  float* part = static_cast<float*>(workspace);
  if (dtype == CEPHALO_F32) return launch_colsum<float>(static_cast<const float*>(X), part, workspace_bytes, g, scale, accumulate, rows, N, s);
  return launch_colsum<bf16>(static_cast<const bf16*>(X), part, workspace_bytes, g, scale, accumulate, rows, N, s);
}
