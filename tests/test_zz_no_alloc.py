"""The allocation-free weight-gradient entry point (partial sums in the library's fixed device array) against the
entry point that takes a work area: the same kernels, so bit-identical results; both against the oracle's definition."""
import ctypes
import numpy as np
import pytest
import torch

import paper_2411_01075_amd as C
from oracle.precision import round_to_bf16

pytestmark = pytest.mark.gpu


def one_case(T, N, K, seed, accumulate):
    rng = np.random.default_rng(seed)
    dY = rng.standard_normal((T, N)).astype(np.float32)
    X = rng.standard_normal((T, K)).astype(np.float32)
    G0 = rng.standard_normal((N, K)).astype(np.float32)
    d_dY, d_X = torch.from_numpy(dY).cuda().to(torch.bfloat16), torch.from_numpy(X).cuda().to(torch.bfloat16)
    ws = torch.empty(C.cephalo_op_linear_wgrad_workspace(C.BF16, T, N, K), dtype=torch.uint8, device="cuda")
    Ga, Gb = torch.from_numpy(G0.copy()).cuda(), torch.from_numpy(G0.copy()).cuda()
    C.cephalo_op_linear_wgrad(C.BF16, d_dY, d_X, T, N, K, Ga, 0.5, accumulate, ws)
    lib = C.binding.lib()        # straight through the C ABI
    rc = lib.cephalo_op_linear_wgrad_static(C.BF16, d_dY.data_ptr(), d_X.data_ptr(), T, N, K, Gb.data_ptr(), 0.5, accumulate,
                                            torch.cuda.current_stream().cuda_stream)
    assert rc == 0, C.cephalo_last_error()
    torch.cuda.synchronize()
    a, b = Ga.cpu().numpy(), Gb.cpu().numpy()
    assert np.array_equal(a, b)                                              # same kernels, same order of additions
    ref = 0.5 * (round_to_bf16(dY).T @ round_to_bf16(X)) + (G0.astype(np.float64) if accumulate else 0.0)
    assert np.max(np.abs(b - ref)) <= 1e-4 * np.max(np.abs(ref))             # fp32 path of the bf16 mode: products exact, fp32 sums


def test_static_area_gives_the_bits_of_the_work_area_form_twice_in_a_row():
    # few output tiles and a long token axis: the contraction is cut into 8 and then 4 pieces whose partial sums go
    # through the fixed array; the second call is smaller and finds the first call's values there
    assert C.cephalo_op_linear_wgrad_workspace(C.BF16, 8192, 512, 384) > 8 * 512 * 384 * 4 - 1
    one_case(8192, 512, 384, 1, accumulate=0)
    one_case(4100, 256, 264, 2, accumulate=1)
    one_case(300, 200, 72, 3, accumulate=0)           # no split at all: the array is not touched


def test_static_area_limit_and_fp32():
    lib = C.binding.lib()
    fake = ctypes.c_void_p(0x1000)       # never dereferenced: refused on the host
    # c5's qkv weight gradient over the whole share: 4 pieces x 6144 x 2048 x 4 B = 192 MiB > the 64 MiB array
    assert lib.cephalo_op_linear_wgrad_static(C.BF16, fake, fake, 24576, 6144, 2048, fake, 1.0, 0, None) == -3
    assert b"fixed area" in lib.cephalo_last_error()
    assert lib.cephalo_op_linear_wgrad_static(C.BF16, fake, fake, 0, 6, 2, fake, 1.0, 0, None) == -1
    assert lib.cephalo_op_linear_wgrad_static(C.BF16, None, fake, 8, 6, 2, fake, 1.0, 0, None) == -1
    # fp32 operands: no split, no scratch
    rng = np.random.default_rng(5)
    dY, X = rng.standard_normal((70, 24)).astype(np.float32), rng.standard_normal((70, 40)).astype(np.float32)
    G = torch.full((24, 40), float("nan"), device="cuda")
    C.cephalo_op_linear_wgrad_static(C.F32, torch.from_numpy(dY).cuda(), torch.from_numpy(X).cuda(), 70, 24, 40, G, 2.0, 0)
    torch.cuda.synchronize()
    ref = 2.0 * dY.astype(np.float64).T @ X.astype(np.float64)
    assert np.max(np.abs(G.cpu().numpy() - ref)) <= 1e-5 * np.max(np.abs(ref))
