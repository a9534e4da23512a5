"""GPU parity of the flat training-state kernels: slice Adam, gradient accumulation, bf16 copy."""
import numpy as np
import pytest
import torch

import paper_2411_01075_amd as C
from oracle import adam as oadam
from oracle import share as oshare
from oracle.precision import round_to_bf16
from workloads import CONFIGS, shard_of, draw_adam_state
from workloads.configs import split4_boundaries

pytestmark = pytest.mark.gpu
# The ABI carries the hyper-parameters as fp32; the oracle gets the same fp32 values (as doubles), so
# both sides start from identical inputs.
HYP = {k: float(np.float32(x)) for k, x in dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8).items()}


def shifted(a, shift):
    """A device copy of `a` whose first element sits `shift` floats after a 512-byte boundary (torch's allocations
    start on one), so that the kernel's head, the part before its 256-byte aligned body, takes every length."""
    buf = torch.empty(a.size + shift, dtype=torch.float32, device="cuda")
    buf[shift:].copy_(torch.from_numpy(a))
    return buf[shift:]


def run_adam(p, g, m, v, off, ln, t, lowp=False, wd=0.0, shift=0):
    """shift: a multiple of 4 floats (the base pointers must stay 16-byte aligned)."""
    P = p.size
    dp, dg, dm, dv = (shifted(a, shift) for a in (p, g, m, v))
    dl = torch.full((P,), -7.0, dtype=torch.bfloat16, device="cuda") if lowp else None
    C.cephalo_shard_adam(dp, dg, dm, dv, dl, P, off, ln, HYP["lr"], HYP["beta1"], HYP["beta2"], HYP["eps"], wd, t)
    torch.cuda.synchronize()
    out = [a.cpu().numpy() for a in (dp, dm, dv)]
    if lowp:
        out.append(dl.float().cpu().numpy())
    return out


def check_against_oracle(p, g, m, v, off, ln, t, got, wd=0.0):
    ref = oadam.shard_adam(*(a.astype(np.float64) for a in (p, g, m, v)), off, ln, t=t, weight_decay=float(np.float32(wd)), **HYP)
    for name, gq, rq, src in zip("pmv", got, ref, (p, m, v)):
        # outside the slice: bit-identical to the input
        assert np.array_equal(gq[:off], src[:off]) and np.array_equal(gq[off + ln:], src[off + ln:]), name
        d = np.abs(gq[off:off + ln].astype(np.float64) - rq[off:off + ln])
        assert np.all(d <= 1e-4 * np.abs(rq[off:off + ln]) + 1e-7), (name, d.max())
        if ln:
            assert d.max() / max(np.abs(rq[off:off + ln]).max(), 1e-300) <= 1e-4


@pytest.mark.parametrize("P,off,ln", [(1000, 0, 1000), (1000, 1, 998), (1000, 3, 2), (1000, 997, 3), (4099, 1027, 2051),
                                      (1 << 20, 12345, 777777), (64, 5, 0), (7, 0, 7), (5, 2, 1),
                                      (200, 1, 30), (200, 1, 31), (200, 1, 34), (200, 1, 35), (200, 33, 100), (4099, 31, 4068)])
@pytest.mark.parametrize("t", [1, 7])
def test_shard_adam_matches_oracle(P, off, ln, t):
    print("adam P", P, "off", off, "len", ln, "t", t, flush=True)
    rng = np.random.default_rng(P + off + t)
    p = rng.standard_normal(P).astype(np.float32) * 0.02
    g = rng.standard_normal(P).astype(np.float32) * 1e-2
    if t == 1:
        m = np.zeros(P, np.float32); v = np.zeros(P, np.float32)
    else:
        m = rng.standard_normal(P).astype(np.float32) * 1e-2
        v = (rng.standard_normal(P).astype(np.float32) * 1e-2) ** 2
    got = run_adam(p, g, m, v, off, ln, t)
    check_against_oracle(p, g, m, v, off, ln, t, got)


@pytest.mark.parametrize("shift", [4, 8, 28, 36, 60])
@pytest.mark.parametrize("off,ln", [(0, 5000), (3, 4000), (29, 131), (125, 4875), (1, 62), (1, 63), (1, 66), (1, 67), (65, 70)])
def test_shard_adam_wherever_the_buffers_sit(shift, off, ln):
    """The kernel's scalar head runs until p's address is a multiple of 256 bytes: every head length, and buffers
    whose bases are not themselves on such a boundary, give the bits of the aligned run."""
    P = 5000
    rng = np.random.default_rng(shift + off)
    p = rng.standard_normal(P).astype(np.float32) * 0.02
    g, m, v = draw_adam_state(CONFIGS["c1"], P)
    ref = run_adam(p, g, m, v, off, ln, 7, lowp=True)
    got = run_adam(p, g, m, v, off, ln, 7, lowp=True, shift=shift)
    for a, b in zip(ref, got):
        assert np.array_equal(a, b)
    check_against_oracle(p, g, m, v, off, ln, 7, got[:3])


@pytest.mark.parametrize("P,off,ln", [(1000, 0, 1000), (4099, 1027, 2051), (1 << 18, 12345, 77777)])
def test_shard_adam_with_weight_decay_matches_oracle(P, off, ln):
    """The decay term joins the gradient (plain Adam's L2 term); partitions still concatenate bit for bit."""
    rng = np.random.default_rng(P + off)
    p = rng.standard_normal(P).astype(np.float32)
    g, m, v = draw_adam_state(CONFIGS["c2"], P)
    wd = 0.05
    got = run_adam(p, g, m, v, off, ln, 7, wd=wd, lowp=True)
    check_against_oracle(p, g, m, v, off, ln, 7, got[:3], wd=wd)
    plain = run_adam(p, g, m, v, off, ln, 7)
    assert not np.array_equal(plain[0], got[0])                      # the decay does act
    cut = off + ln // 3 + 1
    left = run_adam(p, g, m, v, off, cut - off, 7, wd=wd, lowp=True)
    right = run_adam(p, g, m, v, cut, off + ln - cut, 7, wd=wd, lowp=True)
    for f, l, r in zip(got, left, right):
        assert np.array_equal(f[off:cut], l[off:cut]) and np.array_equal(f[cut:off + ln], r[cut:off + ln])


def test_partition_concatenation_is_bitwise_the_unsharded_update():
    """Updates over any partition of [0,P) concatenate to the unsharded update bit for bit,
    wherever the cuts fall relative to the 16-byte vector body."""
    P = 300001
    rng = np.random.default_rng(5)
    p = rng.standard_normal(P).astype(np.float32) * 0.02
    g, m, v = draw_adam_state(CONFIGS["c3"], P)
    full = run_adam(p, g, m, v, 0, P, 7, lowp=True)
    for cuts in ([0, 1, 2, 3, 7, 100003, 200001, P], split4_boundaries(P, 1003), [0, 0, 150000, 150000, P]):
        cat = [np.empty_like(a) for a in full]
        for lo, hi in zip(cuts[:-1], cuts[1:]):
            part = run_adam(p, g, m, v, lo, hi - lo, 7, lowp=True)
            for c, q in zip(cat, part):
                c[lo:hi] = q[lo:hi]
        for a, b in zip(full, cat):
            assert np.array_equal(a, b)


def test_lowp_copy_is_rounding_of_new_param_and_untouched_outside():
    P, off, ln = 70001, 1237, 50001
    rng = np.random.default_rng(6)
    p = rng.standard_normal(P).astype(np.float32) * 0.02
    g, m, v = draw_adam_state(CONFIGS["c2"], P)
    newp, _, _, lowp = run_adam(p, g, m, v, off, ln, 7, lowp=True)
    assert np.array_equal(lowp[off:off + ln].astype(np.float64), round_to_bf16(newp[off:off + ln]))
    assert np.all(lowp[:off] == -7.0) and np.all(lowp[off + ln:] == -7.0)


def test_shifted_base_pointers_give_shard_length_state():
    """Shard-length m and v (only the slice is stored) work by passing bases shifted by -offset,
    provided the shift keeps 16-byte alignment."""
    P, off, ln = 5000, 1024, 2000
    rng = np.random.default_rng(8)
    p = rng.standard_normal(P).astype(np.float32)
    g, m, v = draw_adam_state(CONFIGS["c1"], P)
    ref = run_adam(p, g, m, v, off, ln, 7)
    dp, dg = torch.from_numpy(p).cuda(), torch.from_numpy(g).cuda()
    ms, vs = torch.from_numpy(m[off:off + ln].copy()).cuda(), torch.from_numpy(v[off:off + ln].copy()).cuda()
    lib = C.binding.lib()
    rc = lib.cephalo_shard_adam(dp.data_ptr(), dg.data_ptr(), ms.data_ptr() - 4 * off, vs.data_ptr() - 4 * off, None,
                                P, off, ln, HYP["lr"], HYP["beta1"], HYP["beta2"], HYP["eps"], 0.0, 7,
                                torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    torch.cuda.synchronize()
    assert np.array_equal(dp.cpu().numpy(), ref[0])
    assert np.array_equal(ms.cpu().numpy(), ref[1][off:off + ln])
    assert np.array_equal(vs.cpu().numpy(), ref[2][off:off + ln])


@pytest.mark.parametrize("n", [0, 1, 3, 4, 1023, 1 << 20, (1 << 20) + 5])
def test_grad_accum(n):
    rng = np.random.default_rng(n)
    acc = rng.standard_normal(n + 8).astype(np.float32)
    g = rng.standard_normal(n + 8).astype(np.float32)
    da, dg = torch.from_numpy(acc.copy()).cuda(), torch.from_numpy(g).cuda()
    C.cephalo_grad_accum(da, dg, 0.375, n)
    torch.cuda.synchronize()
    out = da.cpu().numpy()
    ref = oshare.grad_accum(acc[:n].astype(np.float64), g[:n].astype(np.float64), 0.375)
    assert np.array_equal(out[n:], acc[n:])
    if n:
        assert np.max(np.abs(out[:n] - ref)) <= 1e-6 * max(1.0, np.abs(ref).max())


@pytest.mark.parametrize("n", [1, 5, 4096, 100003])
def test_cast_bf16_is_round_to_nearest_even(n):
    rng = np.random.default_rng(n)
    a = (rng.standard_normal(n) * 3).astype(np.float32)
    a[0] = 1.00390625       # a tie: rounds to even
    src = torch.from_numpy(a).cuda()
    dst = torch.zeros(n + 3, dtype=torch.bfloat16, device="cuda")
    C.cephalo_cast_bf16(dst, src, n)
    torch.cuda.synchronize()
    out = dst.float().cpu().numpy()
    assert np.array_equal(out[:n].astype(np.float64), round_to_bf16(a))
    assert np.all(out[n:] == 0)


def test_full_size_shards_of_every_workload_sampled():
    """Each workload's real shard (offset, length) at full P: the slice edges and a sample of interior
    elements against the oracle, everything outside the slice bit-identical."""
    from oracle import layout
    for name in ("c1", "c2", "c3", "c4", "c5"):
        cfg = CONFIGS[name]
        if cfg.layers > 1:      # the stack's flat buffer: embeddings, layers, final LayerNorm
            P = C.cephalo_stack_param_count(C.stack_desc_from_config(cfg))
            assert P == (cfg.vocab + cfg.seq) * cfg.hidden + cfg.layers * layout.layer_param_count(cfg.hidden, cfg.mlp) + 2 * cfg.hidden
        else:
            P = layout.layer_param_count(cfg.hidden, cfg.mlp)
        off, ln = shard_of(cfg, P)
        print(name, "P", P, "offset", off, "len", ln, flush=True)
        gen = torch.Generator(device="cuda").manual_seed(cfg.seed)
        p = torch.randn(P, device="cuda", generator=gen) * 0.02
        g = torch.randn(P, device="cuda", generator=gen) * 1e-2
        m = torch.randn(P, device="cuda", generator=gen) * 1e-2
        v = (torch.randn(P, device="cuda", generator=gen) * 1e-2) ** 2
        p0, m0, v0 = p.clone(), m.clone(), v.clone()
        lowp = torch.full((P,), -7.0, dtype=torch.bfloat16, device="cuda")
        C.cephalo_shard_adam(p, g, m, v, lowp, P, off, ln, cfg.lr, 0.9, 0.999, 1e-8, 0.0, 7)
        torch.cuda.synchronize()
        assert bool((lowp[:off] == -7.0).all()) and bool((lowp[off + ln:] == -7.0).all())
        assert torch.equal(lowp[off:off + ln], p[off:off + ln].to(torch.bfloat16))      # nearest-even, as torch rounds
        for a, a0 in ((p, p0), (m, m0), (v, v0)):
            assert torch.equal(a[:off], a0[:off]) and torch.equal(a[off + ln:], a0[off + ln:])
        rng = np.random.default_rng(cfg.seed)
        idx = np.unique(np.concatenate([np.arange(off, off + 9), np.arange(off + ln - 9, off + ln),
                                        rng.integers(off, off + ln, 20000)]))
        ti = torch.from_numpy(idx).cuda()
        sub = [a[ti].cpu().numpy().astype(np.float64) for a in (p0, g, m0, v0)]
        ref = oadam.shard_adam(*sub, 0, idx.size, lr=float(np.float32(cfg.lr)), beta1=HYP['beta1'], beta2=HYP['beta2'], eps=HYP['eps'], t=7)
        for a, r in zip((p, m, v), ref):
            d = np.abs(a[ti].cpu().numpy().astype(np.float64) - r)
            assert np.all(d <= 1e-4 * np.abs(r) + 1e-7)
