"""ctypes binding of libcephalo.so: same names as include/cephalo.h, argument marshalling only.

Tensors are torch CUDA(HIP) tensors used as plain device memory; every step of the path runs
in the library's kernels.  There is no fallback: a missing library raises at first use.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcephalo.so")

F32 = 0
BF16 = 1

_lib = None


class CephaloError(RuntimeError):
    pass


class LayerDesc(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_int32), ("heads", ctypes.c_int32), ("mlp", ctypes.c_int32),
                ("seq", ctypes.c_int32), ("causal", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("ln_eps", ctypes.c_float), ("kind", ctypes.c_int32)]


LAYER_GPT, LAYER_LLAMA = 0, 1


def layer_desc(hidden, heads, mlp, seq, causal, dtype, ln_eps=1e-5, kind=LAYER_GPT):
    return LayerDesc(int(hidden), int(heads), int(mlp), int(seq), int(bool(causal)), int(dtype), float(ln_eps), int(kind))


def desc_from_config(cfg):
    kind = LAYER_LLAMA if getattr(cfg, "kind", "gpt") == "llama" else LAYER_GPT
    return layer_desc(cfg.hidden, cfg.heads, cfg.mlp, cfg.seq, cfg.causal, F32 if cfg.dtype == "f32" else BF16, kind=kind)


class StackDesc(ctypes.Structure):
    _fields_ = [("layer", LayerDesc), ("layers", ctypes.c_int32), ("vocab", ctypes.c_int32), ("checkpoint", ctypes.c_int32),
                ("offload", ctypes.c_int32), ("interleave", ctypes.c_int32)]


def stack_desc_from_config(cfg, checkpoint=False, offload=False, interleave=False):
    return StackDesc(desc_from_config(cfg), int(cfg.layers), int(cfg.vocab), int(bool(checkpoint)), int(offload),
                     int(bool(interleave)))


class GpuPerf(ctypes.Structure):
    _fields_ = [("t_fwd", ctypes.POINTER(ctypes.c_double)), ("t_bwd", ctypes.POINTER(ctypes.c_double)),
                ("max_m", ctypes.c_int32), ("mem_cap", ctypes.c_double)]


class ClusterModel(ctypes.Structure):
    _fields_ = [("allgather", ctypes.c_double), ("reducescatter", ctypes.c_double),
                ("allgather_uneven", ctypes.c_double), ("reducescatter_uneven", ctypes.c_double),
                ("mem_base", ctypes.c_double), ("mem_per_sample", ctypes.c_double), ("state_bytes", ctypes.c_double)]


_vp, _i32, _i64, _f32, _sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
_dp = ctypes.POINTER(LayerDesc)

# name -> (restype, argtypes); must list every symbol include/cephalo.h declares
SIGNATURES = {
    "cephalo_last_error": (ctypes.c_char_p, []),
    "cephalo_gemm_general_count": (ctypes.c_int64, []),
    "cephalo_gemm_side_by_side": (ctypes.c_int32, [ctypes.c_int32]),
    "cephalo_layer_param_count": (_i64, [_dp]),
    "cephalo_layer_param_offsets": (ctypes.c_int, [_dp, ctypes.POINTER(_i64)]),
    "cephalo_layer_workspace_bytes": (ctypes.c_int, [_dp, _i32, ctypes.POINTER(_sz), ctypes.POINTER(_sz)]),
    "cephalo_share_workspace_bytes": (ctypes.c_int, [_dp, _i32, _i32, ctypes.POINTER(_sz), ctypes.POINTER(_sz)]),
    "cephalo_layer_fwd": (ctypes.c_int, [_dp, _vp, _vp, _vp, _i32, _vp, _sz, _vp, _sz, _vp]),
    "cephalo_layer_bwd": (ctypes.c_int, [_dp, _vp, _vp, _vp, _vp, _i32, _vp, _sz, _vp, _f32, _i32, _vp, _sz, _vp]),
    "cephalo_share_layer_step": (ctypes.c_int, [_dp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _sz, _vp, _f32,
                                                _vp, _sz, _vp]),
    "cephalo_share_layer_step_interleaved": (ctypes.c_int, [_dp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _sz, _vp, _f32,
                                                _vp, _sz, _vp, _vp]),
    "cephalo_grad_accum": (ctypes.c_int, [_vp, _vp, _f32, _i64, _vp]),
    "cephalo_shard_adam": (ctypes.c_int, [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _f32, _f32, _f32, _f32, _f32, _i64, _vp]),
    "cephalo_cast_bf16": (ctypes.c_int, [_vp, _vp, _i64, _vp]),
    "cephalo_stack_param_count": (_i64, [ctypes.POINTER(StackDesc)]),
    "cephalo_stack_param_offsets": (ctypes.c_int, [ctypes.POINTER(StackDesc), ctypes.POINTER(_i64)]),
    "cephalo_stack_workspace_bytes": (ctypes.c_int, [ctypes.POINTER(StackDesc), _i32, _i32, ctypes.POINTER(_sz)]),
    "cephalo_stack_workspace_regions": (ctypes.c_int, [ctypes.POINTER(StackDesc), _i32, _i32, ctypes.POINTER(_sz)]),
    "cephalo_stack_step": (ctypes.c_int, [ctypes.POINTER(StackDesc), _vp, _vp, _vp, _i32, _i32, _vp, _f32, _vp, _vp, _sz, _vp]),
    "cephalo_stack_step_interleaved": (ctypes.c_int, [ctypes.POINTER(StackDesc), _vp, _vp, _vp, _i32, _i32, _vp, _f32, _vp, _vp, _sz, _vp, _vp]),
    "cephalo_stack_host_bytes": (ctypes.c_int, [ctypes.POINTER(StackDesc), _i32, _i32, ctypes.POINTER(_sz)]),
    "cephalo_stack_step_offload": (ctypes.c_int, [ctypes.POINTER(StackDesc), _vp, _vp, _vp, _i32, _i32, _vp, _f32, _vp, _vp, _sz,
                                                  _vp, _sz, _vp, _vp, _vp]),
    "cephalo_op_gemm": (ctypes.c_int, [_i32, _vp, _i64, _i64, _vp, _i64, _i64, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp,
                                       _vp, _f32, _i32, _vp]),
    "cephalo_op_linear_wgrad_workspace": (_sz, [_i32, _i32, _i32, _i32]),
    "cephalo_op_linear_wgrad": (ctypes.c_int, [_i32, _vp, _vp, _i32, _i32, _i32, _vp, _f32, _i32, _vp, _sz, _vp]),
    "cephalo_op_linear_wgrad_bias_workspace": (_sz, [_i32, _i32, _i32, _i32]),
    "cephalo_op_linear_wgrad_bias": (ctypes.c_int, [_i32, _vp, _vp, _i32, _i32, _i32, _vp, _vp, _f32, _i32, _vp, _sz, _vp]),
    "cephalo_op_linear_wgrad_static": (ctypes.c_int, [_i32, _vp, _vp, _i32, _i32, _i32, _vp, _f32, _i32, _vp]),
    "cephalo_op_norm_fwd": (ctypes.c_int, [_i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _f32, _vp]),
    "cephalo_op_norm_bwd_workspace": (_sz, [_i32, _i32]),
    "cephalo_op_norm_bwd_sums_workspace": (_sz, [_i32, _i32]),
    "cephalo_op_norm_bwd_sums": (ctypes.c_int, [_i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _sz, _vp]),
    "cephalo_op_norm_bwd": (ctypes.c_int, [_i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _sz, _vp]),
    "cephalo_op_colsum_workspace": (_sz, [_i32, _i32]),
    "cephalo_op_colsum": (ctypes.c_int, [_i32, _vp, _i32, _i32, _vp, _f32, _i32, _vp, _sz, _vp]),
    "cephalo_op_cross_entropy": (ctypes.c_int, [_i32, _vp, _i32, _vp, _vp, _vp, _i32, _i32, _f32, _vp]),
    "cephalo_probe_mfma": (ctypes.c_int, [_vp, _i32, _i32, _vp, ctypes.POINTER(ctypes.c_double), _vp]),
    "cephalo_probe_stream": (ctypes.c_int, [_i32, _vp, _vp, _i64, _vp, _vp]),
    "cephalo_plan_compute": (ctypes.c_int, [_i32, ctypes.POINTER(GpuPerf), _i32, ctypes.POINTER(ClusterModel),
                                            ctypes.POINTER(_i32), ctypes.POINTER(_i32), ctypes.POINTER(ctypes.c_double)]),
    "cephalo_plan_state": (ctypes.c_int, [_i32, ctypes.POINTER(GpuPerf), ctypes.POINTER(_i32), ctypes.POINTER(ClusterModel),
                                          ctypes.POINTER(ctypes.c_double)]),
    "cephalo_plan_units": (ctypes.c_int, [_i32, ctypes.POINTER(ctypes.c_double), _i32, ctypes.c_int64, ctypes.POINTER(ctypes.c_int64),
                                          ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(_i32)]),
    "cephalo_op_attention_fwd": (ctypes.c_int, [_dp, _vp, _vp, _vp, _i32, _vp]),
    "cephalo_op_attention_bwd": (ctypes.c_int, [_dp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp]),
}


def lib():
    """The loaded library; raises if it has not been built (python -m paper_2411_01075_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise CephaloError("libcephalo.so is missing at %s: build it with "
                               "`python -m paper_2411_01075_amd.build`" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise CephaloError("cephalo error %d: %s" % (rc, lib().cephalo_last_error().decode()))


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise CephaloError("expected a device tensor")
    if not t.is_contiguous():
        raise CephaloError("expected a contiguous tensor")
    return t.data_ptr()


def _pinned_ptr(t):
    if t.is_cuda or not t.is_pinned():
        raise CephaloError("expected a pinned host tensor")
    if not t.is_contiguous():
        raise CephaloError("expected a contiguous tensor")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream


def cephalo_last_error():
    return lib().cephalo_last_error().decode()


def cephalo_gemm_general_count():
    return int(lib().cephalo_gemm_general_count())


def cephalo_gemm_side_by_side(kernels):
    return int(lib().cephalo_gemm_side_by_side(int(kernels)))


def cephalo_layer_param_count(desc):
    n = lib().cephalo_layer_param_count(ctypes.byref(desc))
    if n < 0:
        _check(int(n))
    return int(n)


def cephalo_layer_param_offsets(desc):
    out = (_i64 * 12)()
    _check(lib().cephalo_layer_param_offsets(ctypes.byref(desc), out))
    return list(out)


def cephalo_layer_workspace_bytes(desc, micro_batch):
    a, b = _sz(0), _sz(0)
    _check(lib().cephalo_layer_workspace_bytes(ctypes.byref(desc), micro_batch, ctypes.byref(a), ctypes.byref(b)))
    return a.value, b.value


def cephalo_share_workspace_bytes(desc, batch_share, micro_batch):
    a, b = _sz(0), _sz(0)
    _check(lib().cephalo_share_workspace_bytes(ctypes.byref(desc), batch_share, micro_batch, ctypes.byref(a), ctypes.byref(b)))
    return a.value, b.value


def cephalo_layer_fwd(desc, flat_param, x, y, micro_batch, save, scratch, stream=None):
    _check(lib().cephalo_layer_fwd(ctypes.byref(desc), _ptr(flat_param), _ptr(x), _ptr(y), micro_batch,
                                   _ptr(save), save.numel() * save.element_size(),
                                   _ptr(scratch), scratch.numel() * scratch.element_size(), _stream(stream)))


def cephalo_layer_bwd(desc, flat_param, x, dy, dx, micro_batch, save, flat_grad, grad_scale, accumulate,
                      scratch, stream=None):
    _check(lib().cephalo_layer_bwd(ctypes.byref(desc), _ptr(flat_param), _ptr(x), _ptr(dy), _ptr(dx), micro_batch,
                                   _ptr(save), save.numel() * save.element_size(),
                                   _ptr(flat_grad), grad_scale, int(accumulate),
                                   _ptr(scratch), scratch.numel() * scratch.element_size(), _stream(stream)))


def cephalo_share_layer_step(desc, flat_param, x, y, dy, dx, batch_share, micro_batch, save, flat_grad,
                             grad_scale, scratch, stream=None):
    _check(lib().cephalo_share_layer_step(ctypes.byref(desc), _ptr(flat_param), _ptr(x), _ptr(y), _ptr(dy), _ptr(dx),
                                          batch_share, micro_batch,
                                          _ptr(save), save.numel() * save.element_size(),
                                          _ptr(flat_grad), grad_scale,
                                          _ptr(scratch), scratch.numel() * scratch.element_size(), _stream(stream)))

def cephalo_share_layer_step_interleaved(desc, flat_param, x, y, dy, dx, batch_share, micro_batch, save, flat_grad,
                                         grad_scale, scratch, side_stream, stream=None):
    _check(lib().cephalo_share_layer_step_interleaved(ctypes.byref(desc), _ptr(flat_param), _ptr(x), _ptr(y), _ptr(dy), _ptr(dx),
                                                      batch_share, micro_batch,
                                                      _ptr(save), save.numel() * save.element_size(),
                                                      _ptr(flat_grad), grad_scale,
                                                      _ptr(scratch), scratch.numel() * scratch.element_size(), _stream(stream),
                                                      _stream(side_stream)))


def cephalo_grad_accum(acc, g, scale, n=None, stream=None):
    n = acc.numel() if n is None else n
    _check(lib().cephalo_grad_accum(_ptr(acc), _ptr(g), scale, n, _stream(stream)))


def cephalo_shard_adam(p, g, m, v, p_lowp, P, offset, length, lr, beta1, beta2, eps, weight_decay, step, stream=None):
    _check(lib().cephalo_shard_adam(_ptr(p), _ptr(g), _ptr(m), _ptr(v), _ptr(p_lowp), P, offset, length,
                                    lr, beta1, beta2, eps, weight_decay, step, _stream(stream)))


def cephalo_cast_bf16(dst, src, n=None, stream=None):
    n = src.numel() if n is None else n
    _check(lib().cephalo_cast_bf16(_ptr(dst), _ptr(src), n, _stream(stream)))


EPI_NONE, EPI_BIAS, EPI_BIAS_RESID, EPI_BIAS_GELU, EPI_DGELU, EPI_GRAD, EPI_NONE_F32, EPI_BIAS_RESID_F32, EPI_BIAS_GELU_DERIV, EPI_MUL = range(10)


def cephalo_op_gemm(dtype, A, a_rs, a_cs, B, b_rs, b_cs, M, N, K, epilogue, C=None, bias=None, R=None, Z=None,
                    G=None, scale=1.0, accumulate=0, stream=None):
    _check(lib().cephalo_op_gemm(dtype, _ptr(A), a_rs, a_cs, _ptr(B), b_rs, b_cs, M, N, K, epilogue,
                                 _ptr(C), _ptr(bias), _ptr(R), _ptr(Z), _ptr(G), scale, int(accumulate), _stream(stream)))


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def cephalo_op_norm_fwd(dtype, rms, x, gamma, beta, u, mean, rstd, rows, H, eps, stream=None):
    _check(lib().cephalo_op_norm_fwd(dtype, int(rms), _ptr(x), _ptr(gamma), _ptr(beta), _ptr(u), _ptr(mean), _ptr(rstd), rows, H, eps, _stream(stream)))


def cephalo_op_norm_bwd_workspace(rows, H):
    return int(lib().cephalo_op_norm_bwd_workspace(rows, H))


def cephalo_op_norm_bwd_sums_workspace(rows, H):
    return int(lib().cephalo_op_norm_bwd_sums_workspace(rows, H))


def cephalo_op_norm_bwd_sums(dtype, du, x, mean, rstd, gamma, resid, dx, dx_lowp, dgamma, dbeta, dx_colsum, rows, H, workspace, stream=None):
    _check(lib().cephalo_op_norm_bwd_sums(dtype, _ptr(du), _ptr(x), _ptr(mean), _ptr(rstd), _ptr(gamma), _ptr(resid), _ptr(dx),
                                          _ptr(dx_lowp), _ptr(dgamma), _ptr(dbeta), _ptr(dx_colsum), rows, H, _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _stream(stream)))


def cephalo_op_norm_bwd(dtype, rms, du, x, mean, rstd, gamma, resid, dx, dx_lowp, dgamma, dbeta, rows, H, workspace, stream=None):
    _check(lib().cephalo_op_norm_bwd(dtype, int(rms), _ptr(du), _ptr(x), _ptr(mean), _ptr(rstd), _ptr(gamma), _ptr(resid), _ptr(dx),
                                     _ptr(dx_lowp), _ptr(dgamma), _ptr(dbeta), rows, H, _ptr(workspace), _nbytes(workspace), _stream(stream)))


def cephalo_op_colsum_workspace(rows, N):
    return int(lib().cephalo_op_colsum_workspace(rows, N))


def cephalo_op_colsum(dtype, X, rows, N, g, scale, accumulate, workspace, stream=None):
    _check(lib().cephalo_op_colsum(dtype, _ptr(X), rows, N, _ptr(g), scale, int(accumulate), _ptr(workspace), _nbytes(workspace), _stream(stream)))


def cephalo_op_cross_entropy(dtype, logits, ld, targets, dlogits, loss_rows, rows, V, coef, stream=None):
    _check(lib().cephalo_op_cross_entropy(dtype, _ptr(logits), ld, _ptr(targets), _ptr(dlogits), _ptr(loss_rows), rows, V, coef, _stream(stream)))


def cephalo_probe_mfma(seed, blocks, iters, sink, stream=None):
    """Returns the flops of the launch."""
    fl = ctypes.c_double(0.0)
    _check(lib().cephalo_probe_mfma(_ptr(seed), blocks, iters, _ptr(sink), ctypes.byref(fl), _stream(stream)))
    return fl.value


def cephalo_probe_stream(mode, dst, src, nbytes, sink, stream=None):
    _check(lib().cephalo_probe_stream(mode, _ptr(dst), _ptr(src), nbytes, _ptr(sink), _stream(stream)))


def cephalo_op_linear_wgrad_static(dtype, dY, X, T, N, K, G, scale, accumulate, stream=None):
    _check(lib().cephalo_op_linear_wgrad_static(dtype, _ptr(dY), _ptr(X), T, N, K, _ptr(G), scale, int(accumulate), _stream(stream)))


def cephalo_op_linear_wgrad_workspace(dtype, T, N, K):
    return int(lib().cephalo_op_linear_wgrad_workspace(dtype, T, N, K))


def cephalo_op_linear_wgrad(dtype, dY, X, T, N, K, G, scale, accumulate, workspace, stream=None):
    _check(lib().cephalo_op_linear_wgrad(dtype, _ptr(dY), _ptr(X), T, N, K, _ptr(G), scale, int(accumulate), _ptr(workspace),
                                         0 if workspace is None else workspace.numel() * workspace.element_size(), _stream(stream)))


def cephalo_op_linear_wgrad_bias_workspace(dtype, T, N, K):
    return int(lib().cephalo_op_linear_wgrad_bias_workspace(dtype, T, N, K))


def cephalo_op_linear_wgrad_bias(dtype, dY, X, T, N, K, G, gb, scale, accumulate, workspace, stream=None):
    _check(lib().cephalo_op_linear_wgrad_bias(dtype, _ptr(dY), _ptr(X), T, N, K, _ptr(G), _ptr(gb), scale, int(accumulate),
                                              _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def cephalo_op_attention_fwd(desc, qkv, O, lse, micro_batch, stream=None):
    _check(lib().cephalo_op_attention_fwd(ctypes.byref(desc), _ptr(qkv), _ptr(O), _ptr(lse), micro_batch, _stream(stream)))


def cephalo_op_attention_bwd(desc, qkv, O, dO, lse, dvec, dqkv, micro_batch, stream=None):
    _check(lib().cephalo_op_attention_bwd(ctypes.byref(desc), _ptr(qkv), _ptr(O), _ptr(dO), _ptr(lse), _ptr(dvec),
                                          _ptr(dqkv), micro_batch, _stream(stream)))


# Names of the 12 tensors of a layer in flat-layout order (see include/cephalo.h).
LAYER_TENSOR_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


# The Llama-style layer uses six of the twelve slots (the beta and bias slots are empty).
LLAMA_TENSOR_NAMES = ("rms1_g", None, "w_qkv", None, "w_o", None, "rms2_g", None, "w_gu", None, "w_down", None)


def flatten_layer_params(desc, tensors):
    """Host-side marshalling: dict name -> float32 array to the fp32 flat vector, at the offsets the library reports."""
    import numpy as np
    P = cephalo_layer_param_count(desc)
    offs = cephalo_layer_param_offsets(desc)
    flat = np.empty(P, dtype=np.float32)
    names = LLAMA_TENSOR_NAMES if desc.kind == LAYER_LLAMA else LAYER_TENSOR_NAMES
    for name, o in zip(names, offs):
        if name is None:
            continue
        t = tensors[name]
        flat[o:o + t.size] = t.reshape(-1)
    return flat


def cephalo_stack_param_count(sdesc):
    n = lib().cephalo_stack_param_count(ctypes.byref(sdesc))
    if n < 0:
        _check(int(n))
    return int(n)


def cephalo_stack_param_offsets(sdesc):
    """Offsets of (token embedding, learned positions, layer 0, final norm, head) in the stack's flat buffer."""
    out = (_i64 * 5)()
    _check(lib().cephalo_stack_param_offsets(ctypes.byref(sdesc), out))
    return list(out)


def cephalo_stack_workspace_bytes(sdesc, batch_share, micro_batch):
    a = _sz(0)
    _check(lib().cephalo_stack_workspace_bytes(ctypes.byref(sdesc), batch_share, micro_batch, ctypes.byref(a)))
    return a.value


def cephalo_stack_workspace_regions(sdesc, batch_share, micro_batch):
    a = (_sz * 3)()
    _check(lib().cephalo_stack_workspace_regions(ctypes.byref(sdesc), batch_share, micro_batch, a))
    return list(a)


def cephalo_stack_step(sdesc, flat_param, ids, targets, batch_share, micro_batch, flat_grad, grad_scale, loss, workspace,
                       stream=None):
    _check(lib().cephalo_stack_step(ctypes.byref(sdesc), _ptr(flat_param), _ptr(ids), _ptr(targets), batch_share, micro_batch,
                                    _ptr(flat_grad), grad_scale, _ptr(loss), _ptr(workspace),
                                    workspace.numel() * workspace.element_size(), _stream(stream)))


def cephalo_stack_step_interleaved(sdesc, flat_param, ids, targets, batch_share, micro_batch, flat_grad, grad_scale, loss, workspace,
                                   side_stream, stream=None):
    _check(lib().cephalo_stack_step_interleaved(ctypes.byref(sdesc), _ptr(flat_param), _ptr(ids), _ptr(targets), batch_share, micro_batch,
                                                _ptr(flat_grad), grad_scale, _ptr(loss), _ptr(workspace),
                                                workspace.numel() * workspace.element_size(), _stream(stream), _stream(side_stream)))


def cephalo_stack_host_bytes(sdesc, batch_share, micro_batch):
    out = _sz(0)
    _check(lib().cephalo_stack_host_bytes(ctypes.byref(sdesc), batch_share, micro_batch, ctypes.byref(out)))
    return int(out.value)


def cephalo_stack_step_offload(sdesc, flat_param, ids, targets, batch_share, micro_batch, flat_grad, grad_scale, loss, workspace,
                               host_area, copy_in_stream, copy_out_stream=None, stream=None):
    """host_area: a pinned CPU tensor; copy_*_stream: torch.cuda.Stream objects other than the compute stream (one for the
    copies to the device, one for the copies to the host; the second defaults to the first)."""
    if copy_out_stream is None:
        copy_out_stream = copy_in_stream
    _check(lib().cephalo_stack_step_offload(ctypes.byref(sdesc), _ptr(flat_param), _ptr(ids), _ptr(targets), batch_share, micro_batch,
                                            _ptr(flat_grad), grad_scale, _ptr(loss), _ptr(workspace),
                                            workspace.numel() * workspace.element_size(), _pinned_ptr(host_area),
                                            host_area.numel() * host_area.element_size(), _stream(stream), _stream(copy_in_stream),
                                            _stream(copy_out_stream)))


def flatten_stack_params(sdesc, params):
    """Host-side marshalling of a stack's parameters to the fp32 flat vector.  GPT-style: wte, wpe, layers, lnf_g, lnf_b;
    Llama-style: wte, layers, normf_g, w_head."""
    import numpy as np
    P = cephalo_stack_param_count(sdesc)
    PL = cephalo_layer_param_count(sdesc.layer)
    o_wte, o_wpe, o_layers, o_norm, o_head = cephalo_stack_param_offsets(sdesc)
    flat = np.full(P, np.nan, dtype=np.float32)

    def put(pos, t):
        flat[pos:pos + t.size] = t.reshape(-1)
        return pos + t.size
    put(o_wte, params["wte"])
    for i, lp in enumerate(params["layers"]):
        put(o_layers + i * PL, flatten_layer_params(sdesc.layer, lp))
    if sdesc.layer.kind == LAYER_LLAMA:
        put(o_norm, params["normf_g"])
        assert put(o_head, params["w_head"]) == P
    else:
        put(o_wpe, params["wpe"])
        assert put(put(o_norm, params["lnf_g"]), params["lnf_b"]) == P
    assert not np.isnan(flat).any()
    return flat


def _gpu_perf_array(gpus):
    """gpus: list of (t_fwd list indexed by m with [0] unused, t_bwd likewise, mem_cap).  Returns the ctypes array and
    the buffers that must stay alive while it is in use."""
    arr = (GpuPerf * len(gpus))()
    keep = []
    for i, (tf, tb, cap) in enumerate(gpus):
        a = (ctypes.c_double * len(tf))(*tf)
        b = (ctypes.c_double * len(tb))(*tb)
        keep += [a, b]
        arr[i] = GpuPerf(a, b, len(tf) - 1, float(cap))
    return arr, keep


def cluster_model(allgather, reducescatter, mem_base, mem_per_sample, state_bytes, uneven_factor=1.15):
    """Sec. 3.3 "Communication Latency": uneven collectives are taken to be 15 % slower than even ones."""
    return ClusterModel(allgather, reducescatter, allgather * uneven_factor, reducescatter * uneven_factor,
                        mem_base, mem_per_sample, state_bytes)


def cephalo_plan_compute(gpus, batch, cluster):
    """Returns (m list, l list, layer latency)."""
    arr, keep = _gpu_perf_array(gpus)
    n = len(gpus)
    m, l, lat = (_i32 * n)(), (_i32 * n)(), ctypes.c_double(0)
    _check(lib().cephalo_plan_compute(n, arr, batch, ctypes.byref(cluster), m, l, ctypes.byref(lat)))
    return list(m), list(l), lat.value


def cephalo_plan_state(gpus, m, cluster):
    """Returns the training-state ratios r_i."""
    arr, keep = _gpu_perf_array(gpus)
    n = len(gpus)
    mm = (_i32 * n)(*m)
    r = (ctypes.c_double * n)()
    _check(lib().cephalo_plan_state(n, arr, mm, ctypes.byref(cluster), r))
    return list(r)


def cephalo_plan_units(ratio, n_units, unit_len):
    """Returns (offsets, lens, n_even): offsets[u][i], lens[u][i] = GPU i's slice of unit u."""
    n = len(ratio)
    r = (ctypes.c_double * n)(*ratio)
    off = (ctypes.c_int64 * (n * n_units))()
    ln = (ctypes.c_int64 * (n * n_units))()
    ne = _i32(0)
    _check(lib().cephalo_plan_units(n, r, n_units, unit_len, off, ln, ctypes.byref(ne)))
    offs = [[off[u * n + i] for i in range(n)] for u in range(n_units)]
    lens = [[ln[u * n + i] for i in range(n)] for u in range(n_units)]
    return offs, lens, ne.value
