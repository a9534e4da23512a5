"""GPU parity of the GEMM family (forward, input-gradient and weight-gradient contractions with
their fused epilogues) against plain fp64 definitions evaluated by the oracle's pieces."""
import numpy as np
import pytest
import torch

import paper_2411_01075_amd as C
from oracle import layer as olayer
from oracle.precision import round_to_bf16
from tests.harness import rel_errors

pytestmark = pytest.mark.gpu


def dev(a, bf16):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if bf16 else t


def host(t):
    return t.double().cpu().numpy()


SHAPES = [  # tokens T, out features N, in features K
    (256, 384, 128),      # exact tiles
    (200, 1600, 320),     # ragged rows, 12.5 tiles of 128 columns
    (520, 328, 72),       # ragged in all three, k not a multiple of the 64-slab
    (1024, 3072, 1024),   # the BERT-large-shaped QKV projection
    (64, 64, 64),
    (1, 8, 8),            # one row, one group of 8 columns
    (8, 72, 40),          # less than a wavefront's 64 rows, less than a k-slab
    (72, 2056, 264),      # a last tile column of 8 columns, a second wavefront row of 8 rows
]


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("T,N,K", SHAPES)
def test_linear_forward_epilogues(T, N, K, bf16):
    print("fwd", T, N, K, "bf16" if bf16 else "f32", flush=True)
    rng = np.random.default_rng(T + N + K)
    X = rng.standard_normal((T, K)).astype(np.float32)
    W = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    b = (rng.standard_normal(N) * 0.1).astype(np.float32)
    R = rng.standard_normal((T, N)).astype(np.float32)
    rnd = round_to_bf16 if bf16 else (lambda a: a.astype(np.float64))
    Xr, Wr, br, Rr = rnd(X), rnd(W), rnd(b), rnd(R)
    acc = Xr @ Wr.T
    dt = C.BF16 if bf16 else C.F32
    tol = 6e-3 if bf16 else 1e-5      # one bf16 rounding of the output: 2^-9 relative, tensor-normalised
    dX, dW, db, dR = dev(X, bf16), dev(W, bf16), dev(b, bf16), dev(R, bf16)
    out = torch.empty_like(dR)
    Z = torch.empty_like(dR)
    C.cephalo_op_gemm(dt, dX, K, 1, dW, K, 1, T, N, K, C.EPI_NONE, C=out)
    assert rel_errors(host(out), acc)[0] < tol
    C.cephalo_op_gemm(dt, dX, K, 1, dW, K, 1, T, N, K, C.EPI_BIAS, C=out, bias=db)
    assert rel_errors(host(out), acc + br)[0] < tol
    C.cephalo_op_gemm(dt, dX, K, 1, dW, K, 1, T, N, K, C.EPI_BIAS_RESID, C=out, bias=db, R=dR)
    assert rel_errors(host(out), acc + br + Rr)[0] < tol
    C.cephalo_op_gemm(dt, dX, K, 1, dW, K, 1, T, N, K, C.EPI_BIAS_GELU, C=out, bias=db, Z=Z)
    assert rel_errors(host(Z), acc + br)[0] < tol
    assert rel_errors(host(out), olayer.gelu(acc + br))[0] < tol
    # what the layer's forward uses: the same output, with gelu'(z) saved in place of z
    out.fill_(float("nan"))
    Z = torch.full_like(Z, float("nan"), dtype=torch.float16 if bf16 else torch.float32)      # a saved factor: half beside bf16 operands
    C.cephalo_op_gemm(dt, dX, K, 1, dW, K, 1, T, N, K, C.EPI_BIAS_GELU_DERIV, C=out, bias=db, Z=Z)
    assert rel_errors(host(Z), olayer.gelu_grad(acc + br))[0] < (1e-3 if bf16 else tol)
    assert rel_errors(host(out), olayer.gelu(acc + br))[0] < tol


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("T,N,K", SHAPES)
def test_linear_input_and_weight_gradients(T, N, K, bf16):
    print("bwd", T, N, K, "bf16" if bf16 else "f32", flush=True)
    rng = np.random.default_rng(T * 3 + N + K)
    X = rng.standard_normal((T, K)).astype(np.float32)
    W = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    dY = rng.standard_normal((T, N)).astype(np.float32)
    Zp = rng.standard_normal((T, K)).astype(np.float32)
    rnd = round_to_bf16 if bf16 else (lambda a: a.astype(np.float64))
    Xr, Wr, dYr, Zr = rnd(X), rnd(W), rnd(dY), rnd(Zp)
    dt = C.BF16 if bf16 else C.F32
    tol = 6e-3 if bf16 else 1e-5
    dX_, dW_, ddY, dZ = dev(X, bf16), dev(W, bf16), dev(dY, bf16), dev(Zp, bf16)
    # input gradient: dX[T,K] = dY[T,N] W[N,K]
    out = torch.empty_like(dX_)
    C.cephalo_op_gemm(dt, ddY, N, 1, dW_, 1, K, T, K, N, C.EPI_NONE, C=out)
    assert rel_errors(host(out), dYr @ Wr)[0] < tol
    C.cephalo_op_gemm(dt, ddY, N, 1, dW_, 1, K, T, K, N, C.EPI_DGELU, C=out, Z=dZ)
    assert rel_errors(host(out), (dYr @ Wr) * olayer.gelu_grad(Zr))[0] < tol
    dZf = torch.from_numpy(Zp).cuda().to(torch.float16 if bf16 else torch.float32)             # Z: a saved factor (half beside bf16 operands)
    C.cephalo_op_gemm(dt, ddY, N, 1, dW_, 1, K, T, K, N, C.EPI_MUL, C=out, Z=dZf)
    assert rel_errors(host(out), (dYr @ Wr) * dZf.double().cpu().numpy())[0] < tol
    # weight gradient with accumulation: G = (acc ? G : 0) + s * dY^T X
    G = torch.full((N, K), float("nan"), dtype=torch.float32, device="cuda")
    C.cephalo_op_gemm(dt, ddY, 1, N, dX_, 1, K, N, K, T, C.EPI_GRAD, G=G, scale=0.5, accumulate=0)
    ref = 0.5 * (dYr.T @ Xr)
    assert rel_errors(host(G), ref)[0] < 1e-5
    C.cephalo_op_gemm(dt, ddY, 1, N, dX_, 1, K, N, K, T, C.EPI_GRAD, G=G, scale=0.25, accumulate=1)
    assert rel_errors(host(G), 1.5 * ref)[0] < 1e-5


@pytest.mark.parametrize("T,N,K", [(256, 384, 128), (200, 1600, 320), (520, 328, 72), (1024, 1024, 4096)])
def test_input_gradient_through_transposed_weight_and_fp32_outputs(T, N, K):
    """The layer's bf16 backward reads W^T (made once per layer and step), so dX = dY W is a contraction with both
    operands contiguous along the contracted axis; results entering LayerNorm's backward and the residual stream
    leave the GEMM in fp32."""
    print("dgrad-wt", T, N, K, flush=True)
    rng = np.random.default_rng(T + 7 * N + K)
    W = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    dY = rng.standard_normal((T, N)).astype(np.float32)
    Zp = rng.standard_normal((T, K)).astype(np.float32)
    b = (rng.standard_normal(K) * 0.1).astype(np.float32)
    R = rng.standard_normal((T, K)).astype(np.float32)
    Wr, dYr, Zr, br = round_to_bf16(W), round_to_bf16(dY), round_to_bf16(Zp), round_to_bf16(b)
    ref = dYr @ Wr
    dWT, ddY, dZ, db = dev(np.ascontiguousarray(W.T), True), dev(dY, True), dev(Zp, True), dev(b, True)
    dR = torch.from_numpy(R).cuda()
    out32 = torch.full((T, K), float("nan"), dtype=torch.float32, device="cuda")
    C.cephalo_op_gemm(C.BF16, ddY, N, 1, dWT, N, 1, T, K, N, C.EPI_NONE_F32, C=out32)
    assert rel_errors(host(out32), ref)[0] < 1e-5            # fp32 out: only the order of the fp32 additions differs
    out = torch.empty((T, K), dtype=torch.bfloat16, device="cuda")
    C.cephalo_op_gemm(C.BF16, ddY, N, 1, dWT, N, 1, T, K, N, C.EPI_DGELU, C=out, Z=dZ)
    assert rel_errors(host(out), ref * olayer.gelu_grad(Zr))[0] < 6e-3
    dZf = torch.from_numpy(Zp).cuda().to(torch.float16)
    C.cephalo_op_gemm(C.BF16, ddY, N, 1, dWT, N, 1, T, K, N, C.EPI_MUL, C=out, Z=dZf)
    assert rel_errors(host(out), ref * dZf.double().cpu().numpy())[0] < 6e-3
    C.cephalo_op_gemm(C.BF16, ddY, N, 1, dWT, N, 1, T, K, N, C.EPI_BIAS_RESID_F32, C=out32, bias=db, R=dR)
    assert rel_errors(host(out32), ref + br + R.astype(np.float64))[0] < 1e-5


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("T,N,K", [(4096, 256, 256),      # one output tile: the token axis is cut into pieces
                                   (4104, 320, 200),      # ragged everything, pieces of unequal length
                                   (2048, 1024, 512), (300, 72, 136), (8192, 512, 256)])
def test_linear_weight_gradient_op(T, N, K, bf16):
    print("wgrad op", T, N, K, bf16, flush=True)
    rng = np.random.default_rng(T + N * 3 + K)
    X = rng.standard_normal((T, K)).astype(np.float32)
    dY = rng.standard_normal((T, N)).astype(np.float32)
    rnd = round_to_bf16 if bf16 else (lambda a: a.astype(np.float64))
    ref = rnd(dY).T @ rnd(X)
    dt = C.BF16 if bf16 else C.F32
    ws = torch.empty(max(16, C.cephalo_op_linear_wgrad_workspace(dt, T, N, K)), dtype=torch.uint8, device="cuda")
    G = torch.full((N, K), float("nan"), dtype=torch.float32, device="cuda")
    C.cephalo_op_linear_wgrad(dt, dev(dY, bf16), dev(X, bf16), T, N, K, G, 0.5, 0, ws)
    assert rel_errors(host(G), 0.5 * ref)[0] < 1e-5
    first = G.clone()
    C.cephalo_op_linear_wgrad(dt, dev(dY, bf16), dev(X, bf16), T, N, K, G, 0.25, 1, ws)
    assert rel_errors(host(G), 0.75 * ref)[0] < 1e-5
    G2 = torch.full((N, K), float("nan"), dtype=torch.float32, device="cuda")
    C.cephalo_op_linear_wgrad(dt, dev(dY, bf16), dev(X, bf16), T, N, K, G2, 0.5, 0, ws)
    assert torch.equal(first, G2)                              # fixed summation order: bit-reproducible
    if bf16:
        small = torch.empty(16, dtype=torch.uint8, device="cuda")
        with pytest.raises(C.CephaloError, match="error -3"):
            C.cephalo_op_linear_wgrad(dt, dev(dY, bf16), dev(X, bf16), T, N, K, G, 1.0, 0, small)


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("T,N,K", [(4096, 256, 256),      # one tile, the token axis in pieces: one owner per piece and wavefront column
                                   (4104, 320, 200),      # ragged rows, columns and tokens
                                   (2048, 1024, 512),     # 256 x 256 tiles
                                   (1000, 2048, 1024),    # several tile rows and columns: the k-slabs go round 8 owners
                                   (192, 512, 4096),      # more owners than k-slabs: most pieces stay zero
                                   (300, 72, 136),        # smaller than a tile in every direction
                                   (8192, 512, 256)])
def test_weight_gradient_with_bias_gradient_beside_it(T, N, K, bf16):
    """Sec. 3.2's accumulated gradient holds, for every projection, dW = dY^T X and db = the column sums of dY.  The
    bf16 GEMM forms db from the dY tiles that pass through its registers; the weight gradient must not change by a
    bit, and db is the sum of the very bf16 values, in fp32."""
    print("wgrad+bias op", T, N, K, bf16, flush=True)
    rng = np.random.default_rng(T + N * 5 + K)
    X = rng.standard_normal((T, K)).astype(np.float32)
    dY = (rng.standard_normal((T, N)) + 0.25).astype(np.float32)      # (a mean: the sums do not cancel to noise)
    rnd = round_to_bf16 if bf16 else (lambda a: a.astype(np.float64))
    ref_b = rnd(dY).sum(axis=0)
    dt = C.BF16 if bf16 else C.F32
    ws = torch.empty(C.cephalo_op_linear_wgrad_bias_workspace(dt, T, N, K), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)                                                     # NaN patterns: nothing may be read before it is written
    ws0 = torch.empty(max(16, C.cephalo_op_linear_wgrad_workspace(dt, T, N, K)), dtype=torch.uint8, device="cuda")
    G = torch.full((N, K), float("nan"), dtype=torch.float32, device="cuda")
    G0 = torch.full((N, K), float("nan"), dtype=torch.float32, device="cuda")
    gb = torch.full((N,), float("nan"), dtype=torch.float32, device="cuda")
    C.cephalo_op_linear_wgrad_bias(dt, dev(dY, bf16), dev(X, bf16), T, N, K, G, gb, 0.5, 0, ws)
    C.cephalo_op_linear_wgrad(dt, dev(dY, bf16), dev(X, bf16), T, N, K, G0, 0.5, 0, ws0)
    assert torch.equal(G, G0)
    assert rel_errors(host(gb), 0.5 * ref_b)[0] < 1e-5
    first = gb.clone()
    C.cephalo_op_linear_wgrad_bias(dt, dev(dY, bf16), dev(X, bf16), T, N, K, G, gb, 0.25, 1, ws)
    assert rel_errors(host(gb), 0.75 * ref_b)[0] < 1e-5
    gb2 = torch.full((N,), float("nan"), dtype=torch.float32, device="cuda")
    C.cephalo_op_linear_wgrad_bias(dt, dev(dY, bf16), dev(X, bf16), T, N, K, G0, gb2, 0.5, 0, ws)
    assert torch.equal(first, gb2)                             # fixed summation order: bit-reproducible
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(C.CephaloError, match="error -3"):
        C.cephalo_op_linear_wgrad_bias(dt, dev(dY, bf16), dev(X, bf16), T, N, K, G, gb, 1.0, 0, small)
