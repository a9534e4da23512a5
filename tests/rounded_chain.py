"""A control for the bf16 parity tests: the oracle's own layer, with the tensors that the bf16 mode keeps in bf16
rounded at the point where they are stored, and nothing else changed.

The oracle proper rounds only the parameters and then computes in fp64.  Every matrix-core operand of the bf16 mode
is a bf16 value, so a result that lies behind a chain of projections carries one rounding per link; on wide random
layers, whose branches are larger than the residual stream they join, the distance between *any* such chain and the
unrounded oracle passes the stated 5e-3 mean-relative budget.  This module lets a test tell the two causes apart:
the kernels are held to the stated tolerance against this chain (same roundings, fp64 arithmetic), and the chain's
own distance from the unrounded oracle is printed beside the kernels'.

Built from the oracle's functions (numpy fp64); test infrastructure only.  Stored in bf16: u, qkv, the attention
probabilities as they enter P V and P^T dO, O, u2, h; in the backward the copies of dy and dx1 that feed the
projections, dz, dO, dS, dqkv.  Stored as IEEE half: the saved GELU derivative (a factor, not an operand).  fp32 on
the GPU and therefore left unrounded here: the residual stream, LayerNorm statistics, softmax statistics, the
gradients entering LayerNorm's backward, every parameter gradient.
"""
import numpy as np

from oracle import layer as ol
from oracle import layout as olayout
from oracle.precision import round_to_bf16


def rb(a):
    return round_to_bf16(np.asarray(a, dtype=np.float32))


def rh(a):
    return np.asarray(a, dtype=np.float64).astype(np.float16).astype(np.float64)


def layer_fwd_bwd(p, x, dy, heads, causal, eps=1e-5):
    """p: bf16-valued fp64 parameter tensors; x, dy: [m, S, H] fp64.  Returns y, dx, parameter gradients."""
    H = x.shape[-1]
    rows = lambda t: t.reshape(-1, t.shape[-1])
    u, xhat1, rstd1 = ol.layer_norm_fwd(x, p["ln1_g"], p["ln1_b"], eps)
    u = rb(u)
    qkv = rb(u @ p["w_qkv"].T + p["b_qkv"])
    q, k, v = (ol.split_heads(qkv[..., i * H:(i + 1) * H], heads) for i in range(3))
    d, S = q.shape[-1], q.shape[-2]
    Z = (q @ k.transpose(0, 1, 3, 2)) / np.sqrt(d)
    if causal:
        Z = np.where(np.triu(np.ones((S, S), dtype=bool), k=1), -np.inf, Z)
    mx = Z.max(axis=-1, keepdims=True)
    E = np.exp(Z - mx)
    den = E.sum(axis=-1, keepdims=True)
    lse = mx + np.log(den)
    O = rb(ol.merge_heads((rb(E) @ v) / den))                  # exponentials enter P V in bf16, the row sum is fp32
    x1 = x + O @ p["w_o"].T + p["b_o"]
    u2, xhat2, rstd2 = ol.layer_norm_fwd(x1, p["ln2_g"], p["ln2_b"], eps)
    u2 = rb(u2)
    z = u2 @ p["w_fc1"].T + p["b_fc1"]
    gd = rh(ol.gelu_grad(z))
    h = rb(ol.gelu(z))
    y = x1 + h @ p["w_fc2"].T + p["b_fc2"]

    g = {}
    dy16 = rb(dy)
    g["w_fc2"] = rows(dy16).T @ rows(h)
    g["b_fc2"] = rows(dy).sum(axis=0)
    dz = rb((dy16 @ p["w_fc2"]) * gd)
    du2 = dz @ p["w_fc1"]
    g["w_fc1"] = rows(dz).T @ rows(u2)
    g["b_fc1"] = rows(dz).sum(axis=0)
    dx1_ln, g["ln2_g"], g["ln2_b"] = ol.layer_norm_bwd(du2, xhat2, rstd2, p["ln2_g"])
    dx1 = dy + dx1_ln
    dx1_16 = rb(dx1)
    dO = rb(dx1_16 @ p["w_o"])
    g["w_o"] = rows(dx1_16).T @ rows(O)
    g["b_o"] = rows(dx1).sum(axis=0)
    dOh = ol.split_heads(dO, heads)
    P = np.exp(Z - lse)
    dV = rb(P).transpose(0, 1, 3, 2) @ dOh
    dP = dOh @ v.transpose(0, 1, 3, 2)
    delta = (dOh * ol.split_heads(O, heads)).sum(axis=-1, keepdims=True)
    dS = rb(P * (dP - delta))
    dQ = (dS @ k) / np.sqrt(d)
    dK = (dS.transpose(0, 1, 3, 2) @ q) / np.sqrt(d)
    dqkv = rb(np.concatenate([ol.merge_heads(dQ), ol.merge_heads(dK), ol.merge_heads(dV)], axis=-1))
    du = dqkv @ p["w_qkv"]
    g["w_qkv"] = rows(dqkv).T @ rows(u)
    g["b_qkv"] = rows(dqkv).sum(axis=0)
    dx_ln, g["ln1_g"], g["ln1_b"] = ol.layer_norm_bwd(du, xhat1, rstd1, p["ln1_g"])
    return y, dx1 + dx_ln, g


def share_layer_step(flat_param, x, dy, H, F, heads, causal, m, scale=1.0):
    """The counterpart of oracle.share.share_layer_step on the rounded chain: y, dx, flat G over the whole share."""
    p = olayout.unflatten_layer(flat_param, H, F)
    y, dx = np.empty_like(x), np.empty_like(x)
    G = np.zeros_like(flat_param)
    for lo in range(0, x.shape[0], m):
        y[lo:lo + m], dx[lo:lo + m], g = layer_fwd_bwd(p, x[lo:lo + m], dy[lo:lo + m], heads, causal)
        G = G + scale * olayout.flatten_layer(g, H, F)
    return y, dx, G
