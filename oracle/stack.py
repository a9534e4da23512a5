"""A whole GPT-style stack on one GPU's batch share, in the layered order of Sec. 3.2
("Layered Gradient Accumulation": all micro-batches pass through a layer before the next layer).

The paper trains such stacks (Table 2) but describes none of their pieces; the form used here:
learned token and position embeddings, x0 = wte[id] + wpe[pos]; L pre-LN layers (oracle.layer);
final LayerNorm; logits = lnf(x) wte^T (tied, no bias); loss = mean over all b*S tokens of the
cross-entropy against the target ids.  The gradient of that mean loss (times `scale`, the factor of
Eq. 1) is accumulated over the micro-batches.  fp64 numpy throughout.

The loss value has no printed counterpart in the paper; it is pinned by finite differences and by
torch autograd on a tiny stack (tests/test_oracle_stack.py).
"""
import numpy as np
from . import layer as _layer
from . import share as _share


def cross_entropy(logits, targets):
    """Per-token loss and softmax probabilities.  logits [T, V], targets [T] ints."""
    z = logits - logits.max(axis=-1, keepdims=True)
    lse = np.log(np.exp(z).sum(axis=-1, keepdims=True))
    logp = z - lse
    loss = -logp[np.arange(logits.shape[0]), targets]
    return loss, np.exp(logp)


def stack_step(params, ids, targets, heads, causal, m, scale=1.0, eps=1e-5):
    """params: dict with 'wte' [V,H], 'wpe' [S,H], 'layers' (list of layer dicts), 'lnf_g', 'lnf_b' (fp64).
    ids, targets: [b, S] ints.  Returns (mean loss, grads in the same structure as params)."""
    b, S = ids.shape
    H = params["wte"].shape[1]
    L = len(params["layers"])
    micro = _share.split_share(b, m)
    n_tok = b * S
    # ---- forward, layer by layer, every micro-batch through a layer before the next layer
    xs = [[params["wte"][ids[lo:hi]] + params["wpe"][None, :S, :] for lo, hi in micro]]
    caches = []
    for li in range(L):
        outs, cs = [], []
        for j in range(len(micro)):
            y, c = _layer.layer_fwd(params["layers"][li], xs[li][j], heads, causal, eps)
            outs.append(y)
            cs.append(c)
        xs.append(outs)
        caches.append(cs)
    # ---- head: final LN, tied logits, mean cross-entropy; and its backward
    g = {"wte": np.zeros_like(params["wte"]), "wpe": np.zeros_like(params["wpe"]),
         "lnf_g": np.zeros(H), "lnf_b": np.zeros(H),
         "layers": [{k: np.zeros_like(v) for k, v in lp.items()} for lp in params["layers"]]}
    total = 0.0
    dxs = []
    for j, (lo, hi) in enumerate(micro):
        u, xhat, rstd = _layer.layer_norm_fwd(xs[L][j], params["lnf_g"], params["lnf_b"], eps)
        u2 = u.reshape(-1, H)
        logits = u2 @ params["wte"].T
        tgt = targets[lo:hi].reshape(-1)
        loss, prob = cross_entropy(logits, tgt)
        total += loss.sum()
        dlogits = prob
        dlogits[np.arange(tgt.size), tgt] -= 1.0
        dlogits *= scale / n_tok
        g["wte"] = _share.grad_accum(g["wte"], dlogits.T @ u2, 1.0)
        du = (dlogits @ params["wte"]).reshape(u.shape)
        dx, dgam, dbet = _layer.layer_norm_bwd(du, xhat, rstd, params["lnf_g"])
        g["lnf_g"] += dgam
        g["lnf_b"] += dbet
        dxs.append(dx)
    # ---- backward through the layers, again all micro-batches per layer
    for li in reversed(range(L)):
        for j in range(len(micro)):
            dxs[j], gl = _layer.layer_bwd(params["layers"][li], caches[li][j], dxs[j], heads)
            for k, v in gl.items():
                g["layers"][li][k] = _share.grad_accum(g["layers"][li][k], v, 1.0)
    # ---- embeddings: token rows gather their gradients, positions sum over samples
    for j, (lo, hi) in enumerate(micro):
        np.add.at(g["wte"], ids[lo:hi].reshape(-1), dxs[j].reshape(-1, H))
        g["wpe"][:S] += dxs[j].sum(axis=0)
    return total / n_tok, g
