"""Pins for oracle.stack: torch autograd on an independent build of the same stack, finite differences,
micro-batch invariance, and the closed form of the loss at zero logits."""
import numpy as np
import torch

from oracle import layout, stack
from tests.test_oracle_layer import tiny_params, torch_layer


def tiny_stack(rng, V, S, H, F, L):
    return {"wte": rng.standard_normal((V, H)) * 0.3, "wpe": rng.standard_normal((S, H)) * 0.3,
            "layers": [tiny_params(rng, H, F) for _ in range(L)],
            "lnf_g": 1 + 0.2 * rng.standard_normal(H), "lnf_b": 0.2 * rng.standard_normal(H)}


def test_stack_matches_torch_autograd_and_is_microbatch_invariant():
    rng = np.random.default_rng(21)
    V, S, H, F, L, A, b = 13, 6, 8, 16, 2, 2, 4
    p = tiny_stack(rng, V, S, H, F, L)
    ids = rng.integers(0, V, (b, S))
    ids[0, :3] = 5                       # repeated tokens: their embedding gradients must add up
    tgt = rng.integers(0, V, (b, S))
    loss, g = stack.stack_step(p, ids, tgt, A, True, m=2)
    # independent torch build
    tp = {k: torch.tensor(v, requires_grad=True) for k, v in p.items() if k != "layers"}
    tl = [{k: torch.tensor(v, requires_grad=True) for k, v in lp.items()} for lp in p["layers"]]
    x = tp["wte"][torch.tensor(ids)] + tp["wpe"][None]
    for lp in tl:
        x = torch_layer(lp, x, A, True, 1e-5)
    u = torch.nn.functional.layer_norm(x, (H,), tp["lnf_g"], tp["lnf_b"], 1e-5)
    logits = u @ tp["wte"].T
    tloss = torch.nn.functional.cross_entropy(logits.reshape(-1, V), torch.tensor(tgt).reshape(-1))
    tloss.backward()
    assert abs(tloss.item() - loss) < 1e-12
    for k in tp:
        assert np.max(np.abs(tp[k].grad.numpy() - g[k])) < 1e-11, k
    for li in range(L):
        for k in tl[li]:
            assert np.max(np.abs(tl[li][k].grad.numpy() - g["layers"][li][k])) < 1e-11, (li, k)
    # any split of the share into micro-batches gives the same loss and gradient
    for m in (1, 4):
        loss2, g2 = stack.stack_step(p, ids, tgt, A, True, m=m)
        assert abs(loss2 - loss) < 1e-13
        assert np.max(np.abs(g2["wte"] - g["wte"])) < 1e-13
        assert np.max(np.abs(g2["layers"][0]["w_qkv"] - g["layers"][0]["w_qkv"])) < 1e-13


def test_stack_finite_differences_and_scale():
    rng = np.random.default_rng(22)
    V, S, H, F, L, A, b = 7, 4, 8, 8, 1, 2, 2
    p = tiny_stack(rng, V, S, H, F, L)
    ids, tgt = rng.integers(0, V, (b, S)), rng.integers(0, V, (b, S))
    loss, g = stack.stack_step(p, ids, tgt, A, False, m=1)
    _, g3 = stack.stack_step(p, ids, tgt, A, False, m=1, scale=3.0)
    assert np.allclose(g3["wpe"], 3.0 * g["wpe"], rtol=1e-13, atol=0)
    h = 1e-6
    for name, t, gt in (("wte", p["wte"], g["wte"]), ("wpe", p["wpe"], g["wpe"]), ("lnf_g", p["lnf_g"], g["lnf_g"]),
                        ("w_o", p["layers"][0]["w_o"], g["layers"][0]["w_o"])):
        flat, gf = t.reshape(-1), gt.reshape(-1)
        for i in rng.choice(flat.size, 6, replace=False):
            old = flat[i]
            flat[i] = old + h
            lp = stack.stack_step(p, ids, tgt, A, False, m=2)[0]
            flat[i] = old - h
            lm = stack.stack_step(p, ids, tgt, A, False, m=2)[0]
            flat[i] = old
            assert abs((lp - lm) / (2 * h) - gf[i]) < 1e-7, (name, i)


def test_loss_closed_form_at_zero_logits():
    rng = np.random.default_rng(23)
    V, S, H, F = 11, 3, 8, 8
    p = tiny_stack(rng, V, S, H, F, 1)
    p["wte"][:] = 0.0                    # logits = 0 -> uniform distribution -> loss = ln V exactly
    loss, _ = stack.stack_step(p, rng.integers(0, V, (2, S)), rng.integers(0, V, (2, S)), 2, True, m=1)
    assert abs(loss - np.log(V)) < 1e-14
    # stack layout count at the paper-scale sizes
    assert layout.stack_param_count(2048, 8192, 2048, 50257, 24) == 1315723264
