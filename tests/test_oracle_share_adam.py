"""Pins for oracle.share, oracle.adam, oracle.layout and oracle.precision."""
import numpy as np
import pytest
import torch

from oracle import adam as A
from oracle import layer as L
from oracle import layout
from oracle import share
from oracle.precision import round_to_bf16


def rand_layer(rng, H, F):
    p = {k: rng.standard_normal(s) * 0.3 for k, s in layout.layer_shapes(H, F).items()}
    p["ln1_g"] += 1.0
    p["ln2_g"] += 1.0
    return p


# ------------------------------------------------------------------ layout bookkeeping
def test_layout_enumerates_every_index_once():
    H, F = 4, 6
    offs = layout.layer_offsets(H, F)
    P = layout.layer_param_count(H, F)
    assert P == 4 * H * H + 2 * H * F + 9 * H + F
    owner = [None] * P
    for name, (start, shape) in offs.items():
        for i in range(int(np.prod(shape))):
            assert owner[start + i] is None
            owner[start + i] = name
    assert all(o is not None for o in owner)
    assert [n for n in layout.LAYER_ORDER] == sorted(offs, key=lambda n: offs[n][0])
    # round trip, and row-major [out, in]
    rng = np.random.default_rng(0)
    p = rand_layer(rng, H, F)
    flat = layout.flatten_layer(p, H, F)
    s = offs["w_fc1"][0]
    assert flat[s + 2 * H + 3] == p["w_fc1"][2, 3]
    q = layout.unflatten_layer(flat, H, F)
    assert all(np.array_equal(p[k], q[k]) for k in p)
    assert layout.state_bytes(P) == 16 * P


def test_stack_layout_counts():
    H, F, S, V, Lr = 8, 32, 5, 11, 3
    offs = layout.stack_offsets(H, F, S, V, Lr)
    pos = 0
    for name, start, shape in offs:
        assert start == pos
        pos += int(np.prod(shape))
    assert pos == layout.stack_param_count(H, F, S, V, Lr)
    # the paper-scale stack: 24 layers of width 2048, vocabulary 50257, 2048 positions
    assert layout.stack_param_count(2048, 8192, 2048, 50257, 24) == 1315723264
    assert layout.layer_param_count(4096, 16384) == 201379840


# ------------------------------------------------------------------ micro-batch split
def test_split_share_validation():
    assert share.split_share(6, 2) == [(0, 2), (2, 4), (4, 6)]
    for b, m in ((5, 2), (0, 1), (4, 0), (4, -2)):
        with pytest.raises(ValueError):
            share.split_share(b, m)


def test_microbatch_sum_equals_full_batch():
    rng = np.random.default_rng(11)
    b, S, H, F, heads = 6, 5, 8, 16, 2
    flat = layout.flatten_layer(rand_layer(rng, H, F), H, F)
    x = rng.standard_normal((b, S, H))
    dy = rng.standard_normal((b, S, H))
    ref = share.share_layer_step(flat, x, dy, H, F, heads, True, m=b)      # one batch
    for m in (1, 2, 3):
        got = share.share_layer_step(flat, x, dy, H, F, heads, True, m=m)
        for r, g in zip(ref, got):
            assert np.max(np.abs(r - g)) <= 1e-12 * max(1.0, np.max(np.abs(r)))


def test_eq1_uneven_shares_reproduce_global_mean():
    """N = 3 GPUs with shares (5, 2, 1) of B = 8: scaling each local mean gradient by
    N*b_i/B and averaging over GPUs gives the plain mean over all 8 samples (Eq. 1)."""
    rng = np.random.default_rng(12)
    S, H, F, heads = 4, 8, 16, 2
    shares = (5, 2, 1)
    B, N = sum(shares), len(shares)
    flat = layout.flatten_layer(rand_layer(rng, H, F), H, F)
    x = rng.standard_normal((B, S, H))
    dy = rng.standard_normal((B, S, H))
    _, _, G_all = share.share_layer_step(flat, x, dy, H, F, heads, True, m=1)
    global_mean = G_all / B
    acc = np.zeros_like(flat)
    lo = 0
    for b_i in shares:
        # local mean (1/b_i) times Eq. 1's factor, folded into the accumulation scale
        s = share.eq1_scale(N, b_i, B) / b_i
        _, _, G_i = share.share_layer_step(flat, x[lo:lo + b_i], dy[lo:lo + b_i], H, F, heads, True, m=1, scale=s)
        acc += G_i
        lo += b_i
    assert np.max(np.abs(acc / N - global_mean)) < 1e-12
    assert abs(sum(share.eq1_scale(N, b, B) for b in shares) / N - 1.0) < 1e-15


# ------------------------------------------------------------------ Adam
HYP = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8)


def test_adam_first_step_closed_form():
    rng = np.random.default_rng(13)
    P = 64
    p = rng.standard_normal(P)
    g = rng.standard_normal(P)
    g[5] = 0.0
    z = np.zeros(P)
    p1, m1, v1 = A.shard_adam(p, g, z, z, 0, P, t=1, **HYP)
    expect = p - HYP["lr"] * g / (np.abs(g) + HYP["eps"])
    assert np.allclose(p1, expect, rtol=0, atol=1e-15)
    assert p1[5] == p[5]
    big = np.abs(g) > 1e-3
    assert np.allclose(np.abs(p1 - p)[big], HYP["lr"], rtol=1e-4)
    assert np.allclose(m1, 0.1 * g) and np.allclose(v1, 0.001 * g * g)


def test_adam_unsharded_matches_torch_optimizer():
    rng = np.random.default_rng(14)
    P = 257
    p0 = rng.standard_normal(P)
    tp = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([tp], lr=HYP["lr"], betas=(HYP["beta1"], HYP["beta2"]), eps=HYP["eps"])
    p, m, v = p0.copy(), np.zeros(P), np.zeros(P)
    for t in range(1, 8):
        g = rng.standard_normal(P) * 0.1
        tp.grad = torch.tensor(g)
        opt.step()
        p, m, v = A.shard_adam(p, g, m, v, 0, P, t=t, **HYP)
        assert np.max(np.abs(tp.detach().numpy() - p)) < 1e-13, t


def test_adam_weight_decay_is_the_l2_term_of_torch_adam():
    """weight_decay * p joins the gradient (torch.optim.Adam's weight_decay), not the decoupled AdamW form."""
    rng = np.random.default_rng(17)
    P, wd = 129, 0.05
    p0 = rng.standard_normal(P)
    tp = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([tp], lr=HYP["lr"], betas=(HYP["beta1"], HYP["beta2"]), eps=HYP["eps"], weight_decay=wd)
    tw = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
    optw = torch.optim.AdamW([tw], lr=HYP["lr"], betas=(HYP["beta1"], HYP["beta2"]), eps=HYP["eps"], weight_decay=wd)
    p, m, v = p0.copy(), np.zeros(P), np.zeros(P)
    for t in range(1, 6):
        g = rng.standard_normal(P) * 0.1
        tp.grad = torch.tensor(g)
        tw.grad = torch.tensor(g)
        opt.step()
        optw.step()
        p, m, v = A.shard_adam(p, g, m, v, 0, P, t=t, weight_decay=wd, **HYP)
        assert np.max(np.abs(tp.detach().numpy() - p)) < 1e-13, t
    assert np.max(np.abs(tw.detach().numpy() - p)) > 1e-6          # the decoupled form is a different update
    # closed form at t = 1 from zero moments: the step is -lr * g' / (|g'| + eps) with g' = g + wd * p
    z = np.zeros(P)
    g = rng.standard_normal(P)
    p1, m1, v1 = A.shard_adam(p0, g, z, z, 0, P, t=1, weight_decay=wd, **HYP)
    gp = g + wd * p0
    assert np.allclose(p1, p0 - HYP["lr"] * gp / (np.abs(gp) + HYP["eps"]), rtol=0, atol=1e-15)
    assert np.allclose(m1, 0.1 * gp) and np.allclose(v1, 0.001 * gp * gp)
    # zero gradient: only the decay moves p, towards zero; weight_decay = 0 is the plain update, bit for bit
    pz, _, _ = A.shard_adam(p0, z, z, z, 0, P, t=1, weight_decay=wd, **HYP)
    assert np.all(np.abs(pz) < np.abs(p0))
    a = A.shard_adam(p0, g, m, v, 3, 100, t=4, weight_decay=0.0, **HYP)
    b = A.shard_adam(p0, g, m, v, 3, 100, t=4, **HYP)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    # partition invariance holds with decay as well (each element's update reads only its own p, g, m, v)
    full = A.shard_adam(p0, g, m, v, 0, P, t=4, weight_decay=wd, **HYP)
    left = A.shard_adam(p0, g, m, v, 0, 50, t=4, weight_decay=wd, **HYP)
    right = A.shard_adam(p0, g, m, v, 50, P - 50, t=4, weight_decay=wd, **HYP)
    for f, l, r in zip(full, left, right):
        assert np.array_equal(f[:50], l[:50]) and np.array_equal(f[50:], r[50:])


def test_adam_partition_invariant_and_outside_untouched():
    rng = np.random.default_rng(15)
    P = 1000
    p, g, m = (rng.standard_normal(P) for _ in range(3))
    v = rng.standard_normal(P) ** 2
    full = A.shard_adam(p, g, m, v, 0, P, t=7, **HYP)
    cuts = [0, 0, 137, 138, 611, 999, 1000]            # includes an empty shard and a 1-element shard
    got = [np.empty(P) for _ in range(3)]
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        out = A.shard_adam(p, g, m, v, lo, hi - lo, t=7, **HYP)
        for k, (o, src) in enumerate(zip(out, (p, m, v))):
            assert np.array_equal(o[:lo], src[:lo]) and np.array_equal(o[hi:], src[hi:])
            got[k][lo:hi] = o[lo:hi]
    for a, b in zip(full, got):
        assert np.array_equal(a, b)
    same = A.shard_adam(p, g, m, v, 400, 0, t=7, **HYP)    # len = 0: no-op
    assert all(np.array_equal(a, b) for a, b in zip(same, (p, m, v)))
    for bad in ((-1, 3), (0, P + 1), (P, 1), (3, -1)):
        with pytest.raises(ValueError):
            A.shard_adam(p, g, m, v, bad[0], bad[1], t=7, **HYP)


# ------------------------------------------------------------------ bf16 rounding
def test_round_to_bf16_matches_torch_and_ties_to_even():
    rng = np.random.default_rng(16)
    a = np.concatenate([rng.standard_normal(4096).astype(np.float32) * 3,
                        np.array([1.00390625, 1.01171875, 0.0, -0.0, 65280.0, 3.0e38, 1e-40], dtype=np.float32)])
    ref = torch.tensor(a).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(round_to_bf16(a), ref)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: even mantissa wins -> 1.0; 1 + 3*2^-8 -> 1 + 2^-6
    assert round_to_bf16(np.float32([1.00390625]))[0] == 1.0
    assert round_to_bf16(np.float32([1.01171875]))[0] == 1.015625
