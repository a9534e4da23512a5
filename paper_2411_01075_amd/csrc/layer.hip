// C-ABI entry points of one transformer layer on one micro-batch and on a whole batch share:
// argument checks in the paper's terms (batch share b, micro-batch size m, b = l*m), then the
// launch sequences of layer_impl.h on the caller's stream.
#include "layer_impl.h"

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
  *scratch_bytes = scratch_layout(*desc, micro_batch, micro_batch).total;
  return CEPHALO_OK;
}

extern "C" int cephalo_share_workspace_bytes(const cephalo_layer_desc* desc, int32_t batch_share, int32_t micro_batch,
                                             size_t* save_bytes_total, size_t* scratch_bytes) {
  TRY(check_desc(desc));
  if (micro_batch <= 0 || batch_share <= 0 || batch_share % micro_batch != 0)
    return fail(CEPHALO_EINVAL, "share_workspace_bytes: batch share b = %d is not a positive multiple of micro-batch size m = %d",
                batch_share, micro_batch);
  if (!save_bytes_total || !scratch_bytes) return fail(CEPHALO_EINVAL, "share_workspace_bytes: null output");
  *save_bytes_total = save_layout(*desc, batch_share).total;
  *scratch_bytes = scratch_layout(*desc, micro_batch, batch_share, 2).total;
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
  const float* xf = static_cast<const float*>(x);
  float* yf = static_cast<float*>(y);
  if (desc->dtype == CEPHALO_F32) return run_fwd<float>(*desc, flat_param, xf, yf, micro_batch, save, s);
  return run_fwd<bf16>(*desc, flat_param, xf, yf, micro_batch, save, s);
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
  const size_t need = scratch_layout(*desc, micro_batch, micro_batch).total;
  if (scratch_bytes < need) return fail(CEPHALO_EWORKSPACE, "layer_bwd: scratch %zu B < %zu B", scratch_bytes, need);
  hipStream_t s = static_cast<hipStream_t>(stream);
  void* sv = const_cast<void*>(save);
  const float* xf = static_cast<const float*>(x);
  const float* dyf = static_cast<const float*>(dy);
  float* dxf = static_cast<float*>(dx);
  if (desc->dtype == CEPHALO_F32)
    return run_bwd<float>(*desc, flat_param, xf, dyf, dxf, micro_batch, sv, flat_grad, grad_scale, accumulate, scratch, s);
  return run_bwd<bf16>(*desc, flat_param, xf, dyf, dxf, micro_batch, sv, flat_grad, grad_scale, accumulate, scratch, s);
}

namespace {
int share_step_checked(const cephalo_layer_desc* desc, const void* flat_param,
                       const void* x, void* y, const void* dy, void* dx,
                       int32_t batch_share, int32_t micro_batch,
                       void* save, size_t save_bytes_total,
                       float* flat_grad, float grad_scale,
                       void* scratch, size_t scratch_bytes, void* stream, void* side_stream) {
  TRY(check_io("share_layer_step", desc, micro_batch, {flat_param, x, y, dy, dx, save, flat_grad, scratch}));
  if (batch_share <= 0 || batch_share % micro_batch != 0)
    return fail(CEPHALO_EINVAL, "share_layer_step: batch share b = %d is not a positive multiple of micro-batch size m = %d",
                batch_share, micro_batch);
  if ((int64_t)batch_share * desc->seq > (1 << 24))
    return fail(CEPHALO_EUNSUPPORTED, "share_layer_step: b*S = %lld tokens is too many", (long long)batch_share * desc->seq);
  if (x == y || dx == dy) return fail(CEPHALO_EINVAL, "share_layer_step: outputs may not alias inputs");
  const size_t need_save = save_layout(*desc, batch_share).total;
  if (save_bytes_total < need_save)
    return fail(CEPHALO_EWORKSPACE, "share_layer_step: save area %zu B < %zu B", save_bytes_total, need_save);
  const size_t need = scratch_layout(*desc, micro_batch, batch_share, 2).total;
  if (scratch_bytes < need) return fail(CEPHALO_EWORKSPACE, "share_layer_step: scratch %zu B < %zu B", scratch_bytes, need);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const float* xf = static_cast<const float*>(x);
  float* yf = static_cast<float*>(y);
  const float* dyf = static_cast<const float*>(dy);
  float* dxf = static_cast<float*>(dx);
  hipStream_t s2 = static_cast<hipStream_t>(side_stream);
  if (desc->dtype == CEPHALO_F32)
    return run_share<float>(*desc, flat_param, xf, yf, dyf, dxf, batch_share, micro_batch, save, flat_grad, grad_scale, scratch, s, s2);
  return run_share<bf16>(*desc, flat_param, xf, yf, dyf, dxf, batch_share, micro_batch, save, flat_grad, grad_scale, scratch, s, s2);
}
}  // namespace

extern "C" int cephalo_share_layer_step(const cephalo_layer_desc* desc, const void* flat_param,
                                        const void* x, void* y, const void* dy, void* dx,
                                        int32_t batch_share, int32_t micro_batch,
                                        void* save, size_t save_bytes_total,
                                        float* flat_grad, float grad_scale,
                                        void* scratch, size_t scratch_bytes, void* stream) {
  return share_step_checked(desc, flat_param, x, y, dy, dx, batch_share, micro_batch, save, save_bytes_total, flat_grad, grad_scale,
                            scratch, scratch_bytes, stream, nullptr);
}

extern "C" int cephalo_share_layer_step_interleaved(const cephalo_layer_desc* desc, const void* flat_param,
                                                    const void* x, void* y, const void* dy, void* dx,
                                                    int32_t batch_share, int32_t micro_batch,
                                                    void* save, size_t save_bytes_total,
                                                    float* flat_grad, float grad_scale,
                                                    void* scratch, size_t scratch_bytes, void* stream, void* side_stream) {
  if (!side_stream || side_stream == stream)
    return fail(CEPHALO_EINVAL, "share_layer_step_interleaved: needs a side stream other than the compute stream");
  return share_step_checked(desc, flat_param, x, y, dy, dx, batch_share, micro_batch, save, save_bytes_total, flat_grad, grad_scale,
                            scratch, scratch_bytes, stream, side_stream);
}
