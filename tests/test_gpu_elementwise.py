"""GPU parity of the bandwidth-bound building blocks on their own, through the C ABI: LayerNorm / RMSNorm forward and
backward, the bias column sum and the cross-entropy of the stack's head, each against the oracle's definition."""
import numpy as np
import pytest
import torch

import paper_2411_01075_amd as C
from oracle import layer as olayer
from oracle import llama as ollama
from oracle import stack as ostack
from oracle.precision import round_to_bf16
from tests.harness import rel_errors, TOL

pytestmark = pytest.mark.gpu

# rows x H: ragged against the 4 rows per block of the forward and the 8 of the backward, one vector per lane up to
# sixteen, the widest row each mode takes
SHAPES = [(5, 72), (37, 256), (130, 1600), (64, 2048), (9, 4096)]


def act(a, bf16):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


@pytest.mark.parametrize("rms", [False, True])
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("rows,H", SHAPES + [(3, 8192)])
def test_norm_forward_and_backward(rows, H, bf16, rms):
    if H > 4096 and not bf16:
        pytest.skip("fp32 rows stop at 4096 columns (refused by the library; covered by the ABI test)")
    print("norm", rows, H, "bf16" if bf16 else "f32", "rms" if rms else "ln", flush=True)
    rng = np.random.default_rng(rows * 7 + H)
    x = (rng.standard_normal((rows, H)) * 1.7 + 0.3).astype(np.float32)
    gamma = (1.0 + 0.1 * rng.standard_normal(H)).astype(np.float32)
    beta = (0.1 * rng.standard_normal(H)).astype(np.float32)
    du = rng.standard_normal((rows, H)).astype(np.float32)
    resid = rng.standard_normal((rows, H)).astype(np.float32)
    rnd = round_to_bf16 if bf16 else (lambda a: a.astype(np.float64))
    g64, b64, x64 = rnd(gamma), rnd(beta), x.astype(np.float64)
    eps = 1e-5
    if rms:
        u_ref, xhat, rstd_ref = ollama.rms_norm_fwd(x64, g64, eps)
        dx_ref, dg_ref = ollama.rms_norm_bwd(du.astype(np.float64), xhat, rstd_ref, g64)
        mean_ref, db_ref = np.zeros((rows, 1)), None
    else:
        u_ref, xhat, rstd_ref = olayer.layer_norm_fwd(x64, g64, b64, eps)
        dx_ref, dg_ref, db_ref = olayer.layer_norm_bwd(du.astype(np.float64), xhat, rstd_ref, g64)
        mean_ref = x64.mean(axis=-1, keepdims=True)
    dt = C.BF16 if bf16 else C.F32
    dx_, dgam, dbet = torch.from_numpy(x).cuda(), act(gamma, bf16), act(beta, bf16)
    u = torch.full((rows, H), float("nan"), device="cuda", dtype=torch.bfloat16 if bf16 else torch.float32)
    mean = torch.full((rows,), float("nan"), device="cuda")
    rstd = torch.full((rows,), float("nan"), device="cuda")
    C.cephalo_op_norm_fwd(dt, rms, dx_, dgam, None if rms else dbet, u, mean, rstd, rows, H, eps)
    torch.cuda.synchronize()
    tol = TOL["bf16" if bf16 else "f32"]
    e = rel_errors(u.double().cpu().numpy(), u_ref)
    assert e[0] <= tol[0] and e[1] <= tol[1], ("u", e)
    assert np.max(np.abs(rstd.double().cpu().numpy() - rstd_ref[:, 0])) <= 1e-5 * np.max(np.abs(rstd_ref))
    assert np.max(np.abs(mean.double().cpu().numpy() - mean_ref[:, 0])) <= 1e-5
    # backward: every operand but gamma is fp32 in both modes
    ws = torch.empty(C.cephalo_op_norm_bwd_workspace(rows, H), dtype=torch.uint8, device="cuda")
    dx = torch.full((rows, H), float("nan"), device="cuda")
    dxl = torch.full((rows, H), float("nan"), device="cuda", dtype=torch.bfloat16) if bf16 else None
    dg = torch.full((H,), float("nan"), device="cuda")
    db = torch.full((H,), float("nan"), device="cuda")
    C.cephalo_op_norm_bwd(dt, rms, torch.from_numpy(du).cuda(), dx_, mean, rstd, dgam, torch.from_numpy(resid).cuda(), dx, dxl,
                          dg, None if rms else db, rows, H, ws)
    torch.cuda.synchronize()
    assert rel_errors(dx.double().cpu().numpy(), dx_ref + resid)[0] <= 1e-4
    assert rel_errors(dg.double().cpu().numpy(), dg_ref)[0] <= 1e-4
    if not rms:
        assert rel_errors(db.double().cpu().numpy(), db_ref)[0] <= 1e-4
    if bf16:
        assert torch.equal(dxl, dx.to(torch.bfloat16))            # the operand copy is the rounding of the fp32 result
    if not rms:
        # the same with the column sums of dx (the bias gradient of the projection whose output joined the stream there)
        ws3 = torch.empty(C.cephalo_op_norm_bwd_sums_workspace(rows, H), dtype=torch.uint8, device="cuda")
        ws3.fill_(0xFF)
        dx2, dg2, db2 = torch.full_like(dx, float("nan")), torch.full_like(dg, float("nan")), torch.full_like(db, float("nan"))
        dxl2 = torch.full_like(dxl, float("nan")) if bf16 else None
        dsum = torch.full((H,), float("nan"), device="cuda")
        C.cephalo_op_norm_bwd_sums(dt, torch.from_numpy(du).cuda(), dx_, mean, rstd, dgam, torch.from_numpy(resid).cuda(), dx2, dxl2,
                                   dg2, db2, dsum, rows, H, ws3)
        torch.cuda.synchronize()
        assert torch.equal(dx2, dx) and torch.equal(dg2, dg) and torch.equal(db2, db)
        if bf16:
            assert torch.equal(dxl2, dxl)
        assert rel_errors(dsum.double().cpu().numpy(), dx.double().cpu().numpy().sum(axis=0))[0] <= 1e-5   # sums of the very values written
        assert rel_errors(dsum.double().cpu().numpy(), (dx_ref + resid).sum(axis=0))[0] <= 1e-4
    # without a residual
    C.cephalo_op_norm_bwd(dt, rms, torch.from_numpy(du).cuda(), dx_, mean, rstd, dgam, None, dx, dxl, dg, None if rms else db, rows, H, ws)
    torch.cuda.synchronize()
    assert rel_errors(dx.double().cpu().numpy(), dx_ref)[0] <= 1e-4


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("rows,N", [(1, 8), (63, 72), (64, 256), (65, 1600), (5000, 384), (24576, 2048)])
def test_bias_column_sum(rows, N, bf16):
    rng = np.random.default_rng(rows + N)
    X = rng.standard_normal((rows, N)).astype(np.float32)
    g0 = rng.standard_normal(N).astype(np.float32)
    Xr = round_to_bf16(X) if bf16 else X.astype(np.float64)
    ws = torch.empty(C.cephalo_op_colsum_workspace(rows, N), dtype=torch.uint8, device="cuda")
    g = torch.from_numpy(g0.copy()).cuda()
    dt = C.BF16 if bf16 else C.F32
    C.cephalo_op_colsum(dt, act(X, bf16), rows, N, g, 0.5, 0, ws)
    torch.cuda.synchronize()
    ref = 0.5 * Xr.sum(axis=0)
    assert np.max(np.abs(g.double().cpu().numpy() - ref)) <= 1e-5 * max(1.0, np.abs(ref).max())
    C.cephalo_op_colsum(dt, act(X, bf16), rows, N, g, 0.25, 1, ws)
    torch.cuda.synchronize()
    assert np.max(np.abs(g.double().cpu().numpy() - 1.5 * ref)) <= 1e-5 * max(1.0, np.abs(ref).max())


@pytest.mark.parametrize("bf16", [False, True])
# (a row of up to 64 Ki columns stays in registers; 70001 and 140003 columns take the two-pass kernel)
@pytest.mark.parametrize("rows,V", [(7, 101), (130, 1031), (16, 50257), (5, 20011), (3, 70001), (2, 140003)])
def test_cross_entropy_rows(rows, V, bf16):
    rng = np.random.default_rng(rows + V)
    ld = (V + 63) // 64 * 64
    logits = np.full((rows, ld), 1e30, dtype=np.float32)              # the padding must not be read as logits
    logits[:, :V] = (rng.standard_normal((rows, V)) * 3).astype(np.float32)
    tgt = rng.integers(0, V, rows).astype(np.int32)
    tgt[0] = V - 1
    coef = 0.125
    loss_ref, p = ostack.cross_entropy(logits[:, :V].astype(np.float64), tgt)
    d_ref = p.copy()
    d_ref[np.arange(rows), tgt] -= 1.0
    d_ref *= coef
    dl = torch.full((rows, ld), float("nan"), device="cuda", dtype=torch.bfloat16 if bf16 else torch.float32)
    loss = torch.full((rows,), float("nan"), device="cuda")
    C.cephalo_op_cross_entropy(C.BF16 if bf16 else C.F32, torch.from_numpy(logits).cuda(), ld, torch.from_numpy(tgt).cuda(), dl, loss, rows, V, coef)
    torch.cuda.synchronize()
    assert np.max(np.abs(loss.double().cpu().numpy() - loss_ref)) <= 1e-5 * np.max(np.abs(loss_ref))
    got = dl.double().cpu().numpy()
    assert np.all(got[:, V:] == 0.0)
    e = rel_errors(got[:, :V], d_ref)
    tol = TOL["bf16" if bf16 else "f32"]
    assert e[0] <= tol[0] and e[1] <= tol[1], e
