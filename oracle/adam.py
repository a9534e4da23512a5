"""Adam restricted to one GPU's slice of the flat training state.

Sec. 3.1 "Training State Partitioning": GPU i manages a ratio r_i of the parameters and of
the matching optimizer state; the ratio may be anything from none to all of it (Sec. 1).
Sec. 3.3: the optimizer is Adam with fp32 parameter, gradient and two moments.  The paper
gives no hyper-parameters; the usual ones are used (beta1 0.9, beta2 0.999, eps 1e-8 added
after the bias-corrected square root, bias correction on, 1-based step t).  Weight decay,
where asked for, is the form that goes with the name "Adam": the decay term weight_decay * p
joins the gradient before the moments are formed (an L2 penalty), not the decoupled form that
shrinks p beside the update; 0 switches it off and every workload here uses 0.

All four buffers are indexed globally: element i of p, g, m, v belongs together, and the
slice is i in [offset, offset + length).
"""
import numpy as np


def shard_adam(p, g, m, v, offset, length, lr, beta1, beta2, eps, t, weight_decay=0.0):
    """Returns new (p, m, v); elements outside [offset, offset+length) are untouched copies."""
    P = p.shape[0]
    if offset < 0 or length < 0 or offset + length > P:
        raise ValueError("slice [%d, %d) outside [0, %d)" % (offset, offset + length, P))
    if t < 1:
        raise ValueError("step count t is 1-based")
    p, m, v = p.copy(), m.copy(), v.copy()
    for i in (slice(offset, offset + length),):
        gi = g[i] + weight_decay * p[i]
        m[i] = beta1 * m[i] + (1.0 - beta1) * gi
        v[i] = beta2 * v[i] + (1.0 - beta2) * gi * gi
        m_hat = m[i] / (1.0 - beta1 ** t)
        v_hat = v[i] / (1.0 - beta2 ** t)
        p[i] = p[i] - lr * m_hat / (np.sqrt(v_hat) + eps)
    return p, m, v
