"""One transformer layer, forward and backward, for one micro-batch -- the plain definition.

The paper treats the layer as a given module made of self-attention and a feed-forward
network (Sec. 2.1) and measures its latency per micro-batch (Sec. 3.3, compute latency
model).  The form used here (the paper leaves it open): pre-LayerNorm residual blocks,
biased variance with eps inside the square root, scores scaled by 1/sqrt(d), causal mask
= strict upper triangle removed, exact (erf) GELU, biases on every projection, no dropout.

    u  = LN1(x)                 qkv = u W_qkv^T + b_qkv       (rows of W_qkv: Q | K | V)
    O  = concat_heads softmax(mask(Q_a K_a^T / sqrt(d))) V_a
    x1 = x + O W_o^T + b_o
    u2 = LN2(x1)                z = u2 W_fc1^T + b_fc1        h = GELU(z)
    y  = x1 + h W_fc2^T + b_fc2

Everything is fp64 numpy; `@` (a library matmul) is the only primitive.  Tensors carry a
leading sample axis: x is [m, S, H].  No blocking, fusion or reordering.
"""
import numpy as np
from scipy.special import erf


# ----------------------------------------------------------------------------- pieces
def layer_norm_fwd(x, gamma, beta, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)          # biased
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return gamma * xhat + beta, xhat, rstd


def layer_norm_bwd(du, xhat, rstd, gamma):
    """Returns dx, dgamma, dbeta for u = gamma * xhat + beta."""
    g = du * gamma
    dx = rstd * (g - g.mean(axis=-1, keepdims=True) - xhat * (g * xhat).mean(axis=-1, keepdims=True))
    H = du.shape[-1]
    dgamma = (du * xhat).reshape(-1, H).sum(axis=0)
    dbeta = du.reshape(-1, H).sum(axis=0)
    return dx, dgamma, dbeta


def gelu(z):
    return 0.5 * z * (1.0 + erf(z / np.sqrt(2.0)))


def gelu_grad(z):
    cdf = 0.5 * (1.0 + erf(z / np.sqrt(2.0)))
    pdf = np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi)
    return cdf + z * pdf


def split_heads(t, A):
    """[m, S, H] -> [m, A, S, d]; head a takes columns [a*d, (a+1)*d)."""
    m, S, H = t.shape
    return t.reshape(m, S, A, H // A).transpose(0, 2, 1, 3)


def merge_heads(t):
    """[m, A, S, d] -> [m, S, H]."""
    m, A, S, d = t.shape
    return t.transpose(0, 2, 1, 3).reshape(m, S, A * d)


def attention_fwd(q, k, v, causal):
    """q, k, v: [m, A, S, d].  Returns O [m, A, S, d] and the probabilities P [m, A, S, S]."""
    d = q.shape[-1]
    S = q.shape[-2]
    Z = (q @ k.transpose(0, 1, 3, 2)) / np.sqrt(d)
    if causal:
        future = np.triu(np.ones((S, S), dtype=bool), k=1)      # key index > query index
        Z = np.where(future, -np.inf, Z)
    Z = Z - Z.max(axis=-1, keepdims=True)
    E = np.exp(Z)
    P = E / E.sum(axis=-1, keepdims=True)
    return P @ v, P


def attention_bwd(dO, q, k, v, P):
    d = q.shape[-1]
    dV = P.transpose(0, 1, 3, 2) @ dO
    dP = dO @ v.transpose(0, 1, 3, 2)
    dZ = P * (dP - (dP * P).sum(axis=-1, keepdims=True))
    dQ = (dZ @ k) / np.sqrt(d)
    dK = (dZ.transpose(0, 1, 3, 2) @ q) / np.sqrt(d)
    return dQ, dK, dV


# ----------------------------------------------------------------------------- layer
def layer_fwd(p, x, heads, causal, eps=1e-5):
    """p: dict of fp64 tensors (names as in oracle.layout).  x: [m, S, H].  Returns y, cache."""
    H = x.shape[-1]
    u, xhat1, rstd1 = layer_norm_fwd(x, p["ln1_g"], p["ln1_b"], eps)
    qkv = u @ p["w_qkv"].T + p["b_qkv"]
    q = split_heads(qkv[..., 0:H], heads)
    k = split_heads(qkv[..., H:2 * H], heads)
    v = split_heads(qkv[..., 2 * H:3 * H], heads)
    Oh, P = attention_fwd(q, k, v, causal)
    O = merge_heads(Oh)
    x1 = x + O @ p["w_o"].T + p["b_o"]
    u2, xhat2, rstd2 = layer_norm_fwd(x1, p["ln2_g"], p["ln2_b"], eps)
    z = u2 @ p["w_fc1"].T + p["b_fc1"]
    h = gelu(z)
    y = x1 + h @ p["w_fc2"].T + p["b_fc2"]
    cache = dict(xhat1=xhat1, rstd1=rstd1, u=u, q=q, k=k, v=v, P=P, O=O,
                 xhat2=xhat2, rstd2=rstd2, u2=u2, z=z, h=h)
    return y, cache


def layer_bwd(p, cache, dy, heads):
    """Gradient of sum(dy * y) with respect to x and to every parameter tensor.

    Returns dx [m, S, H] and a dict of parameter gradients summed over the micro-batch's
    tokens (no averaging: any 1/B factor is the caller's, see oracle.accumulate)."""
    c = cache
    H = dy.shape[-1]
    F = c["z"].shape[-1]
    rows = lambda t: t.reshape(-1, t.shape[-1])                 # [m, S, n] -> [m*S, n]
    g = {}
    # y = x1 + h W2^T + b2
    dh = dy @ p["w_fc2"]
    g["w_fc2"] = rows(dy).T @ rows(c["h"])
    g["b_fc2"] = rows(dy).sum(axis=0)
    # h = GELU(z), z = u2 W1^T + b1
    dz = dh * gelu_grad(c["z"])
    du2 = dz @ p["w_fc1"]
    g["w_fc1"] = rows(dz).T @ rows(c["u2"])
    g["b_fc1"] = rows(dz).sum(axis=0)
    # u2 = LN2(x1); x1 also feeds the residual
    dx1_ln, g["ln2_g"], g["ln2_b"] = layer_norm_bwd(du2, c["xhat2"], c["rstd2"], p["ln2_g"])
    dx1 = dy + dx1_ln
    # x1 = x + O Wo^T + bo
    dO = dx1 @ p["w_o"]
    g["w_o"] = rows(dx1).T @ rows(c["O"])
    g["b_o"] = rows(dx1).sum(axis=0)
    # attention
    dQ, dK, dV = attention_bwd(split_heads(dO, heads), c["q"], c["k"], c["v"], c["P"])
    dqkv = np.concatenate([merge_heads(dQ), merge_heads(dK), merge_heads(dV)], axis=-1)
    # qkv = u Wqkv^T + bqkv
    du = dqkv @ p["w_qkv"]
    g["w_qkv"] = rows(dqkv).T @ rows(c["u"])
    g["b_qkv"] = rows(dqkv).sum(axis=0)
    # u = LN1(x); x also feeds the residual
    dx_ln, g["ln1_g"], g["ln1_b"] = layer_norm_bwd(du, c["xhat1"], c["rstd1"], p["ln1_g"])
    dx = dx1 + dx_ln
    return dx, g
