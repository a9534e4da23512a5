"""A Llama-style transformer layer, forward and backward, for one micro-batch -- the plain definition.

Five of the nine models the paper trains (Sec. 5.1, model table) are of this family; the paper treats the layer as a
given module (Sec. 2.1).  The form used here: pre-RMSNorm residual blocks, no biases, rotary position embedding on
queries and keys, causal attention with scores scaled by 1/sqrt(d), gated feed-forward with SiLU:

    u  = RMS1(x)               qkv = u W_qkv^T                 (rows of W_qkv: Q | K | V)
    q, k <- rotary(q), rotary(k)     O = concat_heads softmax(mask(Q_a K_a^T / sqrt(d))) V_a
    x1 = x + O W_o^T
    u2 = RMS2(x1)              [g | up] = u2 W_gu^T            (rows of W_gu: gate | up)
    h  = silu(g) * up          y = x1 + h W_down^T

RMS(x) = gamma * x / sqrt(mean(x^2) + eps).  Rotary: within each head, the pair of coordinates (2i, 2i+1) of the
token at position t (its index within the sample) is rotated by the angle t * base^(-2i/d), base = 10000.

Test infrastructure only: fp64 numpy, `@` the only primitive, no blocking, fusion or reordering.
"""
import numpy as np

from .layer import split_heads, merge_heads, attention_fwd, attention_bwd

NAMES = ("rms1_g", "w_qkv", "w_o", "rms2_g", "w_gu", "w_down")


def shapes(H, F):
    return {"rms1_g": (H,), "w_qkv": (3 * H, H), "w_o": (H, H), "rms2_g": (H,), "w_gu": (2 * F, H), "w_down": (H, F)}


def rms_norm_fwd(x, gamma, eps):
    rstd = 1.0 / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps)
    xhat = x * rstd
    return gamma * xhat, xhat, rstd


def rms_norm_bwd(du, xhat, rstd, gamma):
    """Returns dx, dgamma for u = gamma * xhat, xhat = x * rstd(x)."""
    g = du * gamma
    dx = rstd * (g - xhat * (g * xhat).mean(axis=-1, keepdims=True))
    H = du.shape[-1]
    return dx, (du * xhat).reshape(-1, H).sum(axis=0)


def rotary_angles(S, d, base=10000.0):
    """[S, d/2]: angle of pair i at position t."""
    inv = base ** (-2.0 * np.arange(d // 2) / d)
    return np.arange(S)[:, None] * inv[None, :]


def rotary(t, sign=1.0, base=10000.0):
    """t: [m, A, S, d].  Rotates every pair (2i, 2i+1) by sign * angle(position, i)."""
    S, d = t.shape[-2], t.shape[-1]
    ang = sign * rotary_angles(S, d, base)
    c, s = np.cos(ang), np.sin(ang)
    even, odd = t[..., 0::2], t[..., 1::2]
    out = np.empty_like(t)
    out[..., 0::2] = even * c - odd * s
    out[..., 1::2] = even * s + odd * c
    return out


def silu(z):
    return z / (1.0 + np.exp(-z))


def silu_grad(z):
    sg = 1.0 / (1.0 + np.exp(-z))
    return sg * (1.0 + z * (1.0 - sg))


def layer_fwd(p, x, heads, causal=True, eps=1e-5):
    H = x.shape[-1]
    F = p["w_down"].shape[1]
    u, xhat1, rstd1 = rms_norm_fwd(x, p["rms1_g"], eps)
    qkv = u @ p["w_qkv"].T
    q = rotary(split_heads(qkv[..., 0:H], heads))
    k = rotary(split_heads(qkv[..., H:2 * H], heads))
    v = split_heads(qkv[..., 2 * H:3 * H], heads)
    Oh, P = attention_fwd(q, k, v, causal)
    O = merge_heads(Oh)
    x1 = x + O @ p["w_o"].T
    u2, xhat2, rstd2 = rms_norm_fwd(x1, p["rms2_g"], eps)
    gu = u2 @ p["w_gu"].T
    g, up = gu[..., :F], gu[..., F:]
    h = silu(g) * up
    y = x1 + h @ p["w_down"].T
    cache = dict(xhat1=xhat1, rstd1=rstd1, u=u, q=q, k=k, v=v, P=P, O=O, xhat2=xhat2, rstd2=rstd2, u2=u2, g=g, up=up, h=h)
    return y, cache


def layer_bwd(p, cache, dy, heads):
    """Gradient of sum(dy * y) with respect to x and to every parameter tensor (summed over the tokens)."""
    c = cache
    rows = lambda t: t.reshape(-1, t.shape[-1])
    gr = {}
    dh = dy @ p["w_down"]
    gr["w_down"] = rows(dy).T @ rows(c["h"])
    dg = dh * c["up"] * silu_grad(c["g"])
    dup = dh * silu(c["g"])
    dgu = np.concatenate([dg, dup], axis=-1)
    du2 = dgu @ p["w_gu"]
    gr["w_gu"] = rows(dgu).T @ rows(c["u2"])
    dx1_n, gr["rms2_g"] = rms_norm_bwd(du2, c["xhat2"], c["rstd2"], p["rms2_g"])
    dx1 = dy + dx1_n
    dO = dx1 @ p["w_o"]
    gr["w_o"] = rows(dx1).T @ rows(c["O"])
    dQ, dK, dV = attention_bwd(split_heads(dO, heads), c["q"], c["k"], c["v"], c["P"])
    dQ, dK = rotary(dQ, -1.0), rotary(dK, -1.0)            # the rotation is orthogonal: its transpose is the inverse
    dqkv = np.concatenate([merge_heads(dQ), merge_heads(dK), merge_heads(dV)], axis=-1)
    du = dqkv @ p["w_qkv"]
    gr["w_qkv"] = rows(dqkv).T @ rows(c["u"])
    dx_n, gr["rms1_g"] = rms_norm_bwd(du, c["xhat1"], c["rstd1"], p["rms1_g"])
    return dx1 + dx_n, gr


def share_step(p, x, dy, heads, micro_batch, causal=True, eps=1e-5, scale=1.0):
    """Layered gradient accumulation over a batch share (Sec. 3.2): micro-batches of `micro_batch` samples in order,
    gradients summed in that order and scaled once.  Returns y, dx, gradient dict."""
    b = x.shape[0]
    assert b % micro_batch == 0
    ys, dxs, total = [], [], None
    for j in range(0, b, micro_batch):
        y, cache = layer_fwd(p, x[j:j + micro_batch], heads, causal, eps)
        dx, g = layer_bwd(p, cache, dy[j:j + micro_batch], heads)
        ys.append(y); dxs.append(dx)
        total = g if total is None else {k: total[k] + g[k] for k in g}
    return np.concatenate(ys), np.concatenate(dxs), {k: scale * v for k, v in total.items()}


def stack_step(params, ids, targets, heads, causal, m, scale=1.0, eps=1e-5):
    """A whole Llama-style stack on one GPU's batch share, in the layered order of Sec. 3.2 (every micro-batch through a
    layer before the next layer, forward and backward).  The paper names the models (Sec. 5.1, model table) and gives
    none of their pieces; the form here: x0 = wte[id] (the positions enter through the rotation inside each layer),
    L layers as above, a final RMSNorm, logits = normf(x) w_head^T with a head of its own (not tied to wte), loss =
    mean over all b*S tokens of the cross-entropy against the target ids.

    params: dict with 'wte' [V,H], 'layers' (list of layer dicts), 'normf_g' [H], 'w_head' [V,H] (fp64).
    ids, targets: [b, S] ints.  Returns (mean loss, scale * gradient in the same structure)."""
    from .stack import cross_entropy
    b, S = ids.shape
    H = params["wte"].shape[1]
    L = len(params["layers"])
    assert b % m == 0
    micro = [(lo, lo + m) for lo in range(0, b, m)]
    n_tok = b * S
    xs = [[params["wte"][ids[lo:hi]] for lo, hi in micro]]
    caches = []
    for li in range(L):
        outs, cs = [], []
        for j in range(len(micro)):
            y, c = layer_fwd(params["layers"][li], xs[li][j], heads, causal, eps)
            outs.append(y)
            cs.append(c)
        xs.append(outs)
        caches.append(cs)
    g = {"wte": np.zeros_like(params["wte"]), "normf_g": np.zeros(H), "w_head": np.zeros_like(params["w_head"]),
         "layers": [{k: np.zeros_like(v) for k, v in lp.items()} for lp in params["layers"]]}
    total = 0.0
    dxs = []
    for j, (lo, hi) in enumerate(micro):
        u, xhat, rstd = rms_norm_fwd(xs[L][j], params["normf_g"], eps)
        u2 = u.reshape(-1, H)
        logits = u2 @ params["w_head"].T
        tgt = targets[lo:hi].reshape(-1)
        loss, prob = cross_entropy(logits, tgt)
        total += loss.sum()
        dlogits = prob
        dlogits[np.arange(tgt.size), tgt] -= 1.0
        dlogits *= scale / n_tok
        g["w_head"] += dlogits.T @ u2
        du = (dlogits @ params["w_head"]).reshape(u.shape)
        dx, dgam = rms_norm_bwd(du, xhat, rstd, params["normf_g"])
        g["normf_g"] += dgam
        dxs.append(dx)
    for li in reversed(range(L)):
        for j in range(len(micro)):
            dxs[j], gl = layer_bwd(params["layers"][li], caches[li][j], dxs[j], heads)
            for k, v in gl.items():
                g["layers"][li][k] += v
    for j, (lo, hi) in enumerate(micro):
        np.add.at(g["wte"], ids[lo:hi].reshape(-1), dxs[j].reshape(-1, H))      # a token id met twice collects both gradients
    return total / n_tok, g
