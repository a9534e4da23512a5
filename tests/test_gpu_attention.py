"""GPU parity of attention forward/backward (plain fp32 kernel and matrix-core bf16 kernel)
against the oracle's definition, on the packed [tokens, 3H] projection layout."""
import numpy as np
import pytest
import torch

import paper_2411_01075_amd as C
from oracle import layer as olayer
from oracle.precision import round_to_bf16
from tests.harness import rel_errors

pytestmark = pytest.mark.gpu

CASES = [  # bf16?, m, S, heads, head dim, causal
    (True, 2, 256, 2, 64, True),
    (True, 1, 200, 3, 64, False),      # ragged: S not a multiple of the 64/128 tiles
    (True, 2, 333, 2, 128, True),
    (True, 1, 128, 1, 128, False),
    (True, 1, 40, 2, 64, True),        # shorter than one tile
    (True, 1, 1024, 2, 64, True),
    # head widths between the 64- and 128-wide tiles (the paper's model table has 32, 104 and 112 among others)
    (True, 2, 200, 3, 32, True),
    (True, 1, 333, 2, 104, True),
    (True, 2, 197, 2, 112, False),
    (True, 1, 150, 5, 8, True),
    (True, 1, 260, 2, 96, False),
    (True, 1, 130, 3, 40, False),
    # the 128-wide causal forward (two wavefront groups in turns): a single tile, an even tile count, a narrow head on the wide tile
    (True, 1, 100, 2, 128, True),
    (True, 2, 256, 2, 128, True),
    (True, 1, 300, 2, 72, True),
    (True, 1, 640, 1, 128, True),
    (False, 2, 70, 3, 24, True),
    (False, 1, 128, 2, 64, False),
]


def oracle_attention(qkv, dO, m, S, A, d, causal):
    H = A * d
    t = qkv.reshape(m, S, 3 * H)
    q, k, v = (olayer.split_heads(t[..., i * H:(i + 1) * H], A) for i in range(3))
    Oh, P = olayer.attention_fwd(q, k, v, causal)
    # log-sum-exp of the scaled, masked scores
    Z = (q @ k.transpose(0, 1, 3, 2)) / np.sqrt(d)
    if causal:
        Z = np.where(np.triu(np.ones((S, S), dtype=bool), 1), -np.inf, Z)
    zmax = Z.max(-1, keepdims=True)
    lse = (zmax + np.log(np.exp(Z - zmax).sum(-1, keepdims=True)))[..., 0]
    dQ, dK, dV = olayer.attention_bwd(olayer.split_heads(dO.reshape(m, S, H), A), q, k, v, P)
    dqkv = np.concatenate([olayer.merge_heads(g) for g in (dQ, dK, dV)], axis=-1).reshape(m * S, 3 * H)
    return olayer.merge_heads(Oh).reshape(m * S, H), lse, dqkv


@pytest.mark.parametrize("bf16,m,S,A,d,causal", CASES)
def test_attention_fwd_bwd(bf16, m, S, A, d, causal):
    print("attention", bf16, m, S, A, d, causal, flush=True)
    H = A * d
    rng = np.random.default_rng(S + d)
    qkv = rng.standard_normal((m * S, 3 * H)).astype(np.float32)
    dO = rng.standard_normal((m * S, H)).astype(np.float32)
    rnd = round_to_bf16 if bf16 else (lambda a: a.astype(np.float64))
    O_ref, lse_ref, dqkv_ref = oracle_attention(rnd(qkv), rnd(dO), m, S, A, d, causal)
    dt = torch.bfloat16 if bf16 else torch.float32
    desc = C.layer_desc(H, A, 4 * H, S, causal, C.BF16 if bf16 else C.F32)
    dqkv_in = torch.from_numpy(qkv).cuda().to(dt)
    ddO = torch.from_numpy(dO).cuda().to(dt)
    O = torch.full((m * S, H), float("nan"), dtype=dt, device="cuda")
    lse = torch.full((m, A, S), float("nan"), dtype=torch.float32, device="cuda")
    C.cephalo_op_attention_fwd(desc, dqkv_in, O, lse, m)
    torch.cuda.synchronize()
    tol_max, tol_mean = (2e-2, 5e-3) if bf16 else (1e-4, 1e-4)
    e = rel_errors(O.double().cpu().numpy(), O_ref)
    print("O", e, flush=True)
    assert e[0] < tol_max and e[1] < tol_mean
    assert np.max(np.abs(lse.double().cpu().numpy() - lse_ref)) < (2e-3 if bf16 else 1e-4)
    dvec = torch.empty((m, A, S), dtype=torch.float32, device="cuda")
    dqkv = torch.full((m * S, 3 * H), float("nan"), dtype=dt, device="cuda")
    C.cephalo_op_attention_bwd(desc, dqkv_in, O, ddO, lse, dvec, dqkv, m)
    torch.cuda.synchronize()
    got = dqkv.double().cpu().numpy()
    for name, sl in (("dQ", slice(0, H)), ("dK", slice(H, 2 * H)), ("dV", slice(2 * H, 3 * H))):
        e = rel_errors(got[:, sl], dqkv_ref[:, sl])
        print(name, e, flush=True)
        assert e[0] < tol_max and e[1] < tol_mean, name
