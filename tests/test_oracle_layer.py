"""Pins for oracle.layer: the oracle is checked against things other than itself.

Brute force in pure Python, closed forms, invariants, central finite differences, and an
independent torch-autograd build of the same layer from library routines.
"""
import math
import numpy as np
import pytest
import torch

from oracle import layer as L
from oracle import layout
from tests import bruteforce as BF


def tiny_params(rng, H, F, scale=0.3):
    shapes = layout.layer_shapes(H, F)
    p = {k: rng.standard_normal(s) * scale for k, s in shapes.items()}
    p["ln1_g"] = 1.0 + p["ln1_g"]
    p["ln2_g"] = 1.0 + p["ln2_g"]
    return p


# ------------------------------------------------------------------ forward vs brute force
@pytest.mark.parametrize("causal", [True, False])
def test_layer_fwd_matches_python_loops(causal):
    rng = np.random.default_rng(1)
    m, S, H, F, A = 2, 5, 8, 12, 2
    p = tiny_params(rng, H, F)
    x = rng.standard_normal((m, S, H))
    y, _ = L.layer_fwd(p, x, A, causal, 1e-5)
    pl = {k: v.tolist() for k, v in p.items()}
    y_bf = np.array(BF.layer_fwd(pl, x.reshape(m * S, H).tolist(), S, H, F, A, causal, 1e-5)).reshape(m, S, H)
    assert np.max(np.abs(y - y_bf)) < 1e-12


# ------------------------------------------------------------------ LayerNorm
def test_layer_norm_closed_forms():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((3, 4, 16)) * 3 + 1.5
    eps = 1e-5
    u, xhat, rstd = L.layer_norm_fwd(x, np.ones(16), np.zeros(16), eps)
    assert np.max(np.abs(u.mean(-1))) < 1e-13
    var = x.var(-1)
    assert np.allclose(u.var(-1), var / (var + eps), rtol=1e-12)
    # a constant row maps to beta
    beta = rng.standard_normal(16)
    uc, _, _ = L.layer_norm_fwd(np.full((1, 1, 16), 7.25), rng.standard_normal(16), beta, eps)
    assert np.allclose(uc[0, 0], beta, atol=1e-12)


def test_layer_norm_bwd_invariants():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, 3, 16))
    gamma = 1 + 0.1 * rng.standard_normal(16)
    # dx is orthogonal to the constant direction always, and to xhat when eps = 0
    # (with eps > 0, mean(xhat^2) = var/(var+eps) < 1 leaves a residue of order eps)
    _, xhat, rstd = L.layer_norm_fwd(x, gamma, np.zeros(16), 0.0)
    dx, dg, db = L.layer_norm_bwd(rng.standard_normal((2, 3, 16)), xhat, rstd, gamma)
    assert np.max(np.abs(dx.sum(-1))) < 1e-12
    assert np.max(np.abs((dx * xhat).sum(-1))) < 1e-12


# ------------------------------------------------------------------ GELU
def test_gelu_closed_forms():
    assert L.gelu(np.array(0.0)) == 0.0
    assert L.gelu_grad(np.array(0.0)) == 0.5
    z = np.linspace(-6, 6, 49)
    assert np.allclose(L.gelu(z) - L.gelu(-z), z, atol=1e-14)
    assert abs(L.gelu(np.array(12.0)) - 12.0) < 1e-12
    # x * Phi(x) with Phi from the complementary error function
    ref = np.array([zi * 0.5 * math.erfc(-zi / math.sqrt(2)) for zi in z])
    assert np.allclose(L.gelu(z), ref, atol=1e-14)
    h = 1e-6
    fd = (L.gelu(z + h) - L.gelu(z - h)) / (2 * h)
    assert np.max(np.abs(fd - L.gelu_grad(z))) < 1e-9


# ------------------------------------------------------------------ attention
def test_attention_special_cases():
    rng = np.random.default_rng(4)
    m, A, S, d = 2, 3, 7, 4
    q, k, v = (rng.standard_normal((m, A, S, d)) for _ in range(3))
    O, P = L.attention_fwd(q, k, v, True)
    assert np.allclose(P.sum(-1), 1.0, atol=1e-14)
    assert np.all(np.triu(P[0, 0], 1) == 0.0)
    assert np.allclose(O[:, :, 0], v[:, :, 0], atol=1e-14)           # first causal row sees only itself
    O0, _ = L.attention_fwd(np.zeros_like(q), k, v, True)            # uniform weights -> running mean
    run_mean = np.cumsum(v, axis=2) / np.arange(1, S + 1)[None, None, :, None]
    assert np.allclose(O0, run_mean, atol=1e-13)
    O1, _ = L.attention_fwd(q[:, :, :1], k[:, :, :1], v[:, :, :1], False)   # S = 1
    assert np.allclose(O1, v[:, :, :1])
    # non-causal output is invariant under a joint permutation of key/value positions
    perm = rng.permutation(S)
    Op, _ = L.attention_fwd(q, k[:, :, perm], v[:, :, perm], False)
    On, _ = L.attention_fwd(q, k, v, False)
    assert np.allclose(Op, On, atol=1e-13)


def test_attention_bwd_row_sums_and_fd():
    rng = np.random.default_rng(5)
    m, A, S, d = 1, 2, 5, 4
    q, k, v = (rng.standard_normal((m, A, S, d)) for _ in range(3))
    dO = rng.standard_normal((m, A, S, d))
    for causal in (True, False):
        O, P = L.attention_fwd(q, k, v, causal)
        dQ, dK, dV = L.attention_bwd(dO, q, k, v, P)
        # rowsum(dP*P) equals rowsum(dO*O)
        dP = dO @ v.transpose(0, 1, 3, 2)
        assert np.allclose((dP * P).sum(-1), (dO * O).sum(-1), atol=1e-13)
        h = 1e-6
        for name, t, dt in (("q", q, dQ), ("k", k, dK), ("v", v, dV)):
            for idx in [(0, 0, 1, 2), (0, 1, 4, 0), (0, 1, 2, 3)]:
                old = t[idx]
                t[idx] = old + h
                lp = (dO * L.attention_fwd(q, k, v, causal)[0]).sum()
                t[idx] = old - h
                lm = (dO * L.attention_fwd(q, k, v, causal)[0]).sum()
                t[idx] = old
                assert abs((lp - lm) / (2 * h) - dt[idx]) < 1e-8, (name, idx, causal)


# ------------------------------------------------------------------ whole layer: finite differences
@pytest.mark.parametrize("causal", [True, False])
def test_layer_bwd_finite_differences(causal):
    rng = np.random.default_rng(6)
    m, S, H, F, A = 2, 4, 8, 16, 2
    p = tiny_params(rng, H, F)
    x = rng.standard_normal((m, S, H))
    dy = rng.standard_normal((m, S, H))
    y, cache = L.layer_fwd(p, x, A, causal)
    dx, g = L.layer_bwd(p, cache, dy, A)

    def loss():
        return (dy * L.layer_fwd(p, x, A, causal)[0]).sum()

    h = 1e-5
    worst = 0.0
    tensors = dict(p)
    tensors["x"] = x
    grads = dict(g)
    grads["x"] = dx
    for name, t in tensors.items():
        flat = t.reshape(-1)                # view: edits reach the layer
        gf = grads[name].reshape(-1)
        for i in rng.choice(flat.size, size=min(flat.size, 12), replace=False):
            old = flat[i]
            flat[i] = old + h
            lp = loss()
            flat[i] = old - h
            lm = loss()
            flat[i] = old
            fd = (lp - lm) / (2 * h)
            err = abs(fd - gf[i]) / max(1.0, abs(fd))
            worst = max(worst, err)
            assert err < 1e-6, (name, i, fd, gf[i])
    assert worst < 1e-6


# ------------------------------------------------------------------ whole layer: torch autograd
def torch_layer(p, x, A, causal, eps):
    """The same layer built from torch library routines (independent of oracle.layer)."""
    F_ = torch.nn.functional
    H = x.shape[-1]
    m, S, _ = x.shape
    u = F_.layer_norm(x, (H,), p["ln1_g"], p["ln1_b"], eps)
    qkv = F_.linear(u, p["w_qkv"], p["b_qkv"])
    q, k, v = qkv.split(H, dim=-1)
    hd = lambda t: t.view(m, S, A, H // A).transpose(1, 2)
    o = F_.scaled_dot_product_attention(hd(q), hd(k), hd(v), is_causal=causal)
    o = o.transpose(1, 2).reshape(m, S, H)
    x1 = x + F_.linear(o, p["w_o"], p["b_o"])
    u2 = F_.layer_norm(x1, (H,), p["ln2_g"], p["ln2_b"], eps)
    h = F_.gelu(F_.linear(u2, p["w_fc1"], p["b_fc1"]))
    return x1 + F_.linear(h, p["w_fc2"], p["b_fc2"])


@pytest.mark.parametrize("causal", [True, False])
def test_layer_matches_torch_autograd(causal):
    rng = np.random.default_rng(7)
    m, S, H, F, A = 2, 9, 24, 40, 3
    p = tiny_params(rng, H, F)
    x = rng.standard_normal((m, S, H))
    dy = rng.standard_normal((m, S, H))
    y, cache = L.layer_fwd(p, x, A, causal)
    dx, g = L.layer_bwd(p, cache, dy, A)
    tp = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()}
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    ty = torch_layer(tp, tx, A, causal, 1e-5)
    ty.backward(torch.tensor(dy))
    assert np.max(np.abs(ty.detach().numpy() - y)) < 1e-11
    assert np.max(np.abs(tx.grad.numpy() - dx)) < 1e-10
    for k in p:
        assert np.max(np.abs(tp[k].grad.numpy() - g[k])) < 1e-10, k


# ------------------------------------------------------------------ planted mistakes are caught
def test_pins_catch_a_planted_mistake(monkeypatch):
    """A dropped term in the LayerNorm backward must fail the finite-difference pin."""
    def broken(du, xhat, rstd, gamma):
        g = du * gamma
        dx = rstd * (g - g.mean(axis=-1, keepdims=True))          # xhat term dropped
        H = du.shape[-1]
        return dx, (du * xhat).reshape(-1, H).sum(0), du.reshape(-1, H).sum(0)
    monkeypatch.setattr(L, "layer_norm_bwd", broken)
    with pytest.raises(AssertionError):
        test_layer_bwd_finite_differences(True)
