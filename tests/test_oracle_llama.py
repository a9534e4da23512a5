"""Pins of the Llama-style layer oracle: closed forms, invariants, finite differences, torch autograd."""
import numpy as np
import pytest
import torch

from oracle import llama as ol


def draw(seed, m=2, S=6, H=16, F=24, A=2):
    rng = np.random.default_rng(seed)
    p = {k: rng.standard_normal(s) * (0.3 if len(s) == 2 else 0.2) + (1.0 if len(s) == 1 else 0.0) for k, s in ol.shapes(H, F).items()}
    x = rng.standard_normal((m, S, H))
    dy = rng.standard_normal((m, S, H))
    return p, x, dy, A


def test_rms_norm_closed_forms():
    x = np.full((1, 3, 8), -2.5)
    u, xhat, rstd = ol.rms_norm_fwd(x, np.arange(1.0, 9.0), 0.0)
    assert np.allclose(u, -np.arange(1.0, 9.0))                   # a constant row has unit RMS: xhat = sign
    x = np.random.default_rng(0).standard_normal((2, 5, 32))
    u, xhat, rstd = ol.rms_norm_fwd(x, np.ones(32), 1e-5)
    assert np.allclose((xhat ** 2).mean(-1), (x ** 2).mean(-1) / ((x ** 2).mean(-1) + 1e-5))
    du = np.random.default_rng(1).standard_normal(x.shape)
    dx, dg = ol.rms_norm_bwd(du, xhat, rstd, np.ones(32))
    _, xhat0, rstd0 = ol.rms_norm_fwd(x, np.ones(32), 0.0)        # eps = 0: the output is scale-invariant, so dx is orthogonal to x
    dx0, _ = ol.rms_norm_bwd(du, xhat0, rstd0, np.ones(32))
    assert np.allclose((dx0 * x).sum(-1), 0.0, atol=1e-10)


def test_rotary_properties():
    rng = np.random.default_rng(2)
    q, k = rng.standard_normal((1, 2, 9, 8)), rng.standard_normal((1, 2, 9, 8))
    rq, rk = ol.rotary(q), ol.rotary(k)
    assert np.allclose(rq[:, :, 0], q[:, :, 0])                   # position 0: identity
    assert np.allclose((rq ** 2).sum(-1), (q ** 2).sum(-1))       # an orthogonal map
    assert np.allclose(ol.rotary(rq, -1.0), q)                    # inverse = rotation by the negative angle
    # scores depend on the distance only: the same vectors placed at positions (2, 5) and (4, 7) score alike
    qq, kk = np.zeros_like(q), np.zeros_like(k)
    for pos in (2, 4):
        qq[:, :, pos + 3] = q[:, :, 0]
        kk[:, :, pos] = k[:, :, 0]
    s = ol.rotary(qq) @ ol.rotary(kk).transpose(0, 1, 3, 2)
    assert np.allclose(s[:, :, 5, 2], s[:, :, 7, 4])
    # first pair at position 1 is rotated by one radian (base^0), as a complex multiplication says
    z = (q[0, 0, 1, 0] + 1j * q[0, 0, 1, 1]) * np.exp(1j * 1.0)
    assert np.allclose([rq[0, 0, 1, 0], rq[0, 0, 1, 1]], [z.real, z.imag])
    ang = ol.rotary_angles(4, 8)
    assert np.allclose(ang[3, 2], 3 * 10000.0 ** (-4.0 / 8.0))


def test_silu_identities():
    z = np.linspace(-6, 6, 41)
    assert ol.silu(0.0) == 0.0 and ol.silu_grad(0.0) == 0.5
    assert np.allclose(ol.silu(z) - ol.silu(-z), z)               # silu(z) - silu(-z) = z
    num = (ol.silu(z + 1e-6) - ol.silu(z - 1e-6)) / 2e-6
    assert np.allclose(num, ol.silu_grad(z), atol=1e-8)


def loss_of(p, x, dy, A):
    y, _ = ol.layer_fwd(p, x, A)
    return float((y * dy).sum())


@pytest.mark.parametrize("seed", [0, 1])
def test_layer_gradients_by_finite_differences(seed):
    p, x, dy, A = draw(seed)
    y, cache = ol.layer_fwd(p, x, A)
    dx, g = ol.layer_bwd(p, cache, dy, A)
    rng = np.random.default_rng(10 + seed)
    eps = 1e-6
    for name in ol.NAMES:
        for _ in range(6):
            idx = tuple(int(rng.integers(0, n)) for n in p[name].shape)
            pp = {k: v.copy() for k, v in p.items()}; pm = {k: v.copy() for k, v in p.items()}
            pp[name][idx] += eps; pm[name][idx] -= eps
            num = (loss_of(pp, x, dy, A) - loss_of(pm, x, dy, A)) / (2 * eps)
            assert abs(num - g[name][idx]) <= 1e-6 * max(1.0, abs(num)), (name, idx)
    for _ in range(8):
        idx = tuple(int(rng.integers(0, n)) for n in x.shape)
        xp, xm = x.copy(), x.copy()
        xp[idx] += eps; xm[idx] -= eps
        num = (loss_of(p, xp, dy, A) - loss_of(p, xm, dy, A)) / (2 * eps)
        assert abs(num - dx[idx]) <= 1e-6 * max(1.0, abs(num))


def torch_layer(p, x, A, eps=1e-5):
    """An independent implementation with torch ops (complex multiplication for the rotation, library softmax / silu)."""
    H = x.shape[-1]; m, S, _ = x.shape; d = H // A; F = p["w_down"].shape[1]
    rms = lambda t, g: g * t * torch.rsqrt((t * t).mean(-1, keepdim=True) + eps)
    u = rms(x, p["rms1_g"])
    qkv = u @ p["w_qkv"].T
    heads = lambda t: t.reshape(m, S, A, d).permute(0, 2, 1, 3)
    q, k, v = heads(qkv[..., :H]), heads(qkv[..., H:2 * H]), heads(qkv[..., 2 * H:])
    inv = 10000.0 ** (-2.0 * torch.arange(d // 2, dtype=torch.float64) / d)
    rot = torch.polar(torch.ones(S, d // 2, dtype=torch.float64), torch.arange(S, dtype=torch.float64)[:, None] * inv[None, :])
    rope = lambda t: torch.view_as_real(torch.view_as_complex(t.reshape(m, A, S, d // 2, 2).contiguous()) * rot).reshape(m, A, S, d)
    q, k = rope(q), rope(k)
    sc = q @ k.transpose(-1, -2) / d ** 0.5
    sc = sc.masked_fill(torch.triu(torch.ones(S, S, dtype=torch.bool), 1), float("-inf"))
    O = (torch.softmax(sc, -1) @ v).permute(0, 2, 1, 3).reshape(m, S, H)
    x1 = x + O @ p["w_o"].T
    gu = rms(x1, p["rms2_g"]) @ p["w_gu"].T
    return x1 + (torch.nn.functional.silu(gu[..., :F]) * gu[..., F:]) @ p["w_down"].T


def test_layer_against_torch_autograd():
    p, x, dy, A = draw(3, m=2, S=7, H=24, F=20, A=3)
    y, cache = ol.layer_fwd(p, x, A)
    dx, g = ol.layer_bwd(p, cache, dy, A)
    tp = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()}
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    ty = torch_layer(tp, tx, A)
    (ty * torch.tensor(dy)).sum().backward()
    assert np.allclose(ty.detach().numpy(), y, rtol=1e-10, atol=1e-10)
    assert np.allclose(tx.grad.numpy(), dx, rtol=1e-9, atol=1e-10)
    for k in ol.NAMES:
        assert np.allclose(tp[k].grad.numpy(), g[k], rtol=1e-9, atol=1e-10), k


def test_share_step_sums_micro_batches():
    p, x, dy, A = draw(4, m=4)
    y1, dx1, g1 = ol.share_step(p, x, dy, A, micro_batch=4)
    y2, dx2, g2 = ol.share_step(p, x, dy, A, micro_batch=1, scale=1.0)
    assert np.allclose(y1, y2) and np.allclose(dx1, dx2)
    for k in ol.NAMES:
        assert np.allclose(g1[k], g2[k], rtol=1e-10, atol=1e-12)


def test_planted_mistake_is_caught():
    # rotating the gradient with the forward angle instead of its inverse must fail the finite-difference pin
    p, x, dy, A = draw(5)
    y, cache = ol.layer_fwd(p, x, A)
    orig = ol.rotary
    try:
        ol.rotary = lambda t, sign=1.0, base=10000.0: orig(t, 1.0, base)
        dx, g = ol.layer_bwd(p, cache, dy, A)
    finally:
        ol.rotary = orig
    eps = 1e-6
    idx = (1, 2)
    pp = {k: v.copy() for k, v in p.items()}; pm = {k: v.copy() for k, v in p.items()}
    pp["w_qkv"][idx] += eps; pm["w_qkv"][idx] -= eps
    num = (loss_of(pp, x, dy, A) - loss_of(pm, x, dy, A)) / (2 * eps)
    assert abs(num - g["w_qkv"][idx]) > 1e-4 * max(1.0, abs(num))


# ---- the stack

def tiny_stack(rng, V, H, F, L):
    shp = ol.shapes(H, F)
    layers = [{k: (1 + 0.2 * rng.standard_normal(s)) if k.endswith("_g") else 0.4 * rng.standard_normal(s) for k, s in shp.items()}
              for _ in range(L)]
    return {"wte": 0.5 * rng.standard_normal((V, H)), "layers": layers, "normf_g": 1 + 0.2 * rng.standard_normal(H),
            "w_head": 0.5 * rng.standard_normal((V, H))}


def test_stack_against_torch_autograd_and_microbatch_invariance():
    rng = np.random.default_rng(31)
    V, S, H, F, L, A, b = 11, 5, 8, 12, 2, 2, 4
    p = tiny_stack(rng, V, H, F, L)
    ids = rng.integers(0, V, (b, S))
    ids[0, :3] = 4                       # repeated tokens: their embedding gradients must add up
    tgt = rng.integers(0, V, (b, S))
    loss, g = ol.stack_step(p, ids, tgt, A, True, m=2)
    tp = {k: torch.tensor(v, requires_grad=True) for k, v in p.items() if k != "layers"}
    tl = [{k: torch.tensor(v, requires_grad=True) for k, v in lp.items()} for lp in p["layers"]]
    x = tp["wte"][torch.tensor(ids)]
    for lp in tl:
        x = torch_layer(lp, x, A)
    u = tp["normf_g"] * x * torch.rsqrt((x * x).mean(-1, keepdim=True) + 1e-5)
    tloss = torch.nn.functional.cross_entropy((u @ tp["w_head"].T).reshape(-1, V), torch.tensor(tgt).reshape(-1))
    tloss.backward()
    assert abs(tloss.item() - loss) < 1e-12
    for k in tp:
        assert np.max(np.abs(tp[k].grad.numpy() - g[k])) < 1e-11, k
    for li in range(L):
        for k in tl[li]:
            assert np.max(np.abs(tl[li][k].grad.numpy() - g["layers"][li][k])) < 1e-11, (li, k)
    for m in (1, 4):                     # any split of the share into micro-batches: the same loss and gradient
        loss2, g2 = ol.stack_step(p, ids, tgt, A, True, m=m)
        assert abs(loss2 - loss) < 1e-13
        assert np.max(np.abs(g2["wte"] - g["wte"])) < 1e-13 and np.max(np.abs(g2["w_head"] - g["w_head"])) < 1e-13
        assert np.max(np.abs(g2["layers"][0]["w_gu"] - g["layers"][0]["w_gu"])) < 1e-13


def test_stack_finite_differences_scale_and_closed_forms():
    rng = np.random.default_rng(32)
    V, S, H, F, L, A, b = 7, 4, 8, 8, 1, 2, 2
    p = tiny_stack(rng, V, H, F, L)
    ids, tgt = rng.integers(0, V, (b, S)), rng.integers(0, V, (b, S))
    loss, g = ol.stack_step(p, ids, tgt, A, True, m=1)
    _, g3 = ol.stack_step(p, ids, tgt, A, True, m=1, scale=3.0)
    assert np.allclose(g3["w_head"], 3.0 * g["w_head"], rtol=1e-13, atol=0)
    h = 1e-6
    for t, gt in ((p["wte"], g["wte"]), (p["w_head"], g["w_head"]), (p["normf_g"], g["normf_g"]),
                  (p["layers"][0]["w_qkv"], g["layers"][0]["w_qkv"]), (p["layers"][0]["w_gu"], g["layers"][0]["w_gu"])):
        flat, gf = t.reshape(-1), gt.reshape(-1)          # views: the perturbation reaches the stack's own arrays
        for i in rng.choice(flat.size, 6, replace=False):
            keep = flat[i]
            flat[i] = keep + h; lp = ol.stack_step(p, ids, tgt, A, True, m=2)[0]
            flat[i] = keep - h; lm = ol.stack_step(p, ids, tgt, A, True, m=2)[0]
            flat[i] = keep
            assert abs((lp - lm) / (2 * h) - gf[i]) <= 1e-7 * max(1.0, abs(gf[i]))
    unused = np.setdiff1d(np.arange(V), ids.reshape(-1))
    assert np.all(g["wte"][unused] == 0.0)                # a token that does not occur gets no embedding gradient
    z = dict(p, w_head=np.zeros_like(p["w_head"]))        # zero logits: the loss is ln V and nothing flows below the head
    lz, gz = ol.stack_step(z, ids, tgt, A, True, m=2)
    assert abs(lz - np.log(V)) < 1e-14 and np.all(gz["wte"] == 0.0) and np.all(gz["layers"][0]["w_o"] == 0.0)
    assert np.allclose(gz["w_head"].sum(axis=0), 0.0, atol=1e-15)      # softmax - onehot sums to zero over the vocabulary
