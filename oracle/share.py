"""A GPU's batch share: micro-batch split, gradient accumulation, Eq. 1 scale.

Sec. 3.2: the share b is processed as l micro-batches of m samples, b = l * m, and the
gradients of the micro-batches are accumulated.  Sec. 3.1, Eq. 1: GPU i multiplies its
local (mean over b_i) gradient by N * b_i / B so that the plain average over the N GPUs
equals (1/B) * sum over all samples.
"""
import numpy as np
from . import layer as _layer
from . import layout as _layout


def split_share(b, m):
    """Sample ranges [j*m, (j+1)*m) of the l = b / m micro-batches; b must equal l * m."""
    if m <= 0 or b <= 0 or b % m != 0:
        raise ValueError("batch share b=%d is not a positive multiple of micro-batch size m=%d" % (b, m))
    return [(j * m, (j + 1) * m) for j in range(b // m)]


def eq1_scale(n_gpus, b_i, B):
    """Factor GPU i applies to its local mean gradient (Eq. 1)."""
    return n_gpus * b_i / B


def grad_accum(G, g, s):
    """G <- G + s * g, element-wise over a flat gradient buffer."""
    return G + s * g


def share_layer_step(flat_param, x, dy, H, F, heads, causal, m, scale=1.0, eps=1e-5):
    """Forward and backward of one layer over every micro-batch of the share, in order
    j = 0 .. l-1, accumulating the flat parameter gradient G = sum_j scale * g_j.

    flat_param: [P] fp64, x and dy: [b, S, H] fp64.  Returns y [b,S,H], dx [b,S,H], G [P]."""
    p = _layout.unflatten_layer(flat_param, H, F)
    y = np.empty_like(x)
    dx = np.empty_like(x)
    G = np.zeros_like(flat_param)
    for lo, hi in split_share(x.shape[0], m):
        y[lo:hi], cache = _layer.layer_fwd(p, x[lo:hi], heads, causal, eps)
        dx[lo:hi], g = _layer.layer_bwd(p, cache, dy[lo:hi], heads)
        G = grad_accum(G, _layout.flatten_layer(g, H, F), scale)
    return y, dx, G
