"""The C-ABI library loads, exports every symbol the header declares, and rejects bad
arguments on the host (no kernel is launched by anything in this file)."""
import ctypes
import os
import re

import pytest

import paper_2411_01075_amd as C
from paper_2411_01075_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    text = open(os.path.join(ROOT, "include", "cephalo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cephalo_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.lib()
    names = header_symbols()
    assert len(names) >= 10
    for n in names:
        assert hasattr(lib, n), n
        assert n in binding.SIGNATURES, "binding lacks %s" % n
    assert sorted(binding.SIGNATURES) == names


def test_param_count_and_offsets_match_formula():
    d = C.layer_desc(256, 4, 1024, 128, True, C.F32)
    P = C.cephalo_layer_param_count(d)
    H, F = 256, 1024
    assert P == 4 * H * H + 2 * H * F + 9 * H + F == 789760
    offs = C.cephalo_layer_param_offsets(d)
    sizes = [H, H, 3 * H * H, 3 * H, H * H, H, H, H, F * H, F, H * F, H]
    pos = 0
    for o, s in zip(offs, sizes):
        assert o == pos
        pos += s
    assert pos == P
    assert C.cephalo_layer_param_count(C.layer_desc(4096, 32, 16384, 2048, True, C.BF16)) == 201379840


def test_workspace_is_independent_of_number_of_microbatches():
    # compute memory depends on the micro-batch size m only (Sec. 3.3): the query has no l argument; the saved
    # activations are proportional to m, the scratch area is a constant part (transposed weights, partial weight
    # gradients) plus a part proportional to m
    d = C.layer_desc(1024, 16, 4096, 512, False, C.BF16)
    sizes = {m: C.cephalo_layer_workspace_bytes(d, m) for m in (1, 2, 3, 4, 8)}
    s1, w1 = sizes[1]
    assert s1 > 0 and w1 > 0
    for m, (s, w) in sizes.items():
        assert abs(s / (m * s1) - 1.0) < 0.01
        assert w <= m * w1
    assert sizes[1][1] < sizes[2][1] < sizes[3][1] < sizes[4][1] < sizes[8][1]


@pytest.mark.parametrize("kw", [dict(hidden=0), dict(heads=3), dict(mlp=-4), dict(seq=0), dict(dtype=7), dict(ln_eps=-1.0)])
def test_bad_desc_is_rejected(kw):
    base = dict(hidden=256, heads=4, mlp=1024, seq=128, causal=True, dtype=C.F32, ln_eps=1e-5)
    base.update(kw)
    with pytest.raises(C.CephaloError) as e:
        C.cephalo_layer_param_count(C.layer_desc(**base))
    assert "cephalo error -1" in str(e.value)


def test_widths_the_norm_kernels_cannot_hold_are_refused_up_front():
    """A row of the norm kernels lives in one wavefront's registers: up to 8192 columns of bf16-mode activations, 4096
    in fp32 mode.  The desc check refuses wider layers, so no launch sequence starts that could not finish."""
    assert C.cephalo_layer_param_count(C.layer_desc(8192, 64, 8192, 16, True, C.BF16)) > 0
    assert C.cephalo_layer_param_count(C.layer_desc(4096, 32, 4096, 16, True, C.F32)) > 0
    for H, dt in ((8200, C.BF16), (4104, C.F32), (8192, C.F32)):
        with pytest.raises(C.CephaloError) as e:
            C.cephalo_layer_param_count(C.layer_desc(H, H // 8, 64, 16, True, dt))
        assert "cephalo error -2" in str(e.value)


def test_unsupported_head_dim():
    with pytest.raises(C.CephaloError) as e:
        C.cephalo_layer_param_count(C.layer_desc(200, 2, 384, 16, True, C.BF16))   # head dim 100: not a multiple of 8
    assert "cephalo error -2" in str(e.value)


def test_host_validation_of_slices_and_shares():
    lib = binding.lib()
    fake = ctypes.c_void_p(0x1000)       # never dereferenced: validation fails first
    # slice outside [0, P)
    for P, off, ln in ((100, -1, 5), (100, 0, 101), (100, 100, 1), (100, 50, -1), (-1, 0, 0)):
        assert lib.cephalo_shard_adam(fake, fake, fake, fake, None, P, off, ln, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1, None) == -1
    assert b"slice" in lib.cephalo_last_error()
    assert lib.cephalo_shard_adam(fake, fake, fake, fake, None, 100, 0, 10, 1e-3, 0.9, 0.999, 1e-8, 0.0, 0, None) == -1   # step 0
    assert lib.cephalo_shard_adam(fake, fake, fake, fake, None, 100, 0, 10, 1e-3, 0.9, 0.999, 1e-8, -0.1, 1, None) == -1  # negative decay
    assert lib.cephalo_shard_adam(fake, fake, fake, fake, None, 100, 0, 10, 1e-3, 1.0, 0.999, 1e-8, 0.0, 1, None) == -1   # beta1 = 1
    assert lib.cephalo_shard_adam(ctypes.c_void_p(0x1004), fake, fake, fake, None, 100, 0, 10, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1, None) == -1
    assert lib.cephalo_shard_adam(None, None, None, None, None, 100, 40, 0, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1, None) == 0   # len 0: no-op
    assert lib.cephalo_grad_accum(fake, fake, 1.0, -3, None) == -1
    assert lib.cephalo_grad_accum(None, None, 1.0, 0, None) == 0
    # b must be a positive multiple of m
    d = C.layer_desc(256, 4, 1024, 128, True, C.F32)
    args = lambda b, m: (ctypes.byref(d), fake, fake, ctypes.c_void_p(0x2000), fake, ctypes.c_void_p(0x3000), b, m,
                         fake, 1 << 40, fake, 1.0, fake, 1 << 40, None)
    assert lib.cephalo_share_layer_step(*args(5, 2)) == -1
    assert b"multiple" in lib.cephalo_last_error()
    assert lib.cephalo_share_layer_step(*args(0, 2)) == -1
    assert lib.cephalo_share_layer_step(*args(4, 0)) == -1
    # workspace too small
    a = list(args(4, 2)); a[9] = 16
    assert lib.cephalo_share_layer_step(*a) == -3
    with pytest.raises(C.CephaloError):
        C.cephalo_share_workspace_bytes(d, 5, 2)
    s_share, w_share = C.cephalo_share_workspace_bytes(d, 4, 2)
    s_mb, w_mb = C.cephalo_layer_workspace_bytes(d, 2)
    assert s_share <= 2 * s_mb and w_share >= w_mb
