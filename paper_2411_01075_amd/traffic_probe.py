"""Launches, three times each, the kernels whose HBM traffic the benchmark reports: the input-gradient GEMM of the
largest workload's three N = H projections (through the transposed weight and on the tile the interleaved step runs
them on, two side by side, as the layer's backward issues them), a
1 GiB device copy (the calibration of the counters) and the shard Adam on a 64 Mi-element slice.  Meant to run under

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dir> -o t -- python3 paper_2411_01075_amd/traffic_probe.py
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <dir> -o t -- python3 paper_2411_01075_amd/traffic_probe.py

(one counter per run); the per-dispatch values are in <dir>/t_counter_collection.csv, in KiB.
"""
import os
import sys

import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import paper_2411_01075_amd as C  # noqa: E402

T, H, F = 4096, 2048, 8192
bt = torch.bfloat16
C.cephalo_gemm_side_by_side(2)      # the tile choice of the step with two micro-batches in flight
def dgrad(n_out, k_in, f32):
    # input gradient dX[T,k_in] = dY[T,n_out] W through W^T [k_in, n_out]
    dY = torch.randn(T, n_out, device='cuda').to(bt); WT = (torch.randn(k_in, n_out, device='cuda') * 0.02).to(bt)
    dX = torch.empty(T, k_in, device='cuda', dtype=torch.float32 if f32 else bt)
    for _ in range(3):
        C.cephalo_op_gemm(C.BF16, dY, n_out, 1, WT, n_out, 1, T, k_in, n_out, C.EPI_NONE_F32 if f32 else C.EPI_NONE, C=dX)
    torch.cuda.synchronize()
dgrad(3 * H, H, True)     # qkv
dgrad(H, H, False)        # out-proj
dgrad(F, H, True)         # fc1
# plain copy of 1 GiB (calibration: 2^30 bytes read, 2^30 bytes written)
a = torch.empty(1 << 28, device='cuda'); b = torch.empty(1 << 28, device='cuda')
a.fill_(1.0)
for _ in range(3):
    b.copy_(a)
# shard Adam on a 64 Mi-element slice with the bf16 copy
n = 1 << 26
p = torch.zeros(n, device='cuda'); g = torch.ones(n, device='cuda') * 1e-2; m = torch.zeros(n, device='cuda'); v = torch.zeros(n, device='cuda')
lp = torch.empty(n, device='cuda', dtype=bt)
for i in range(3):
    C.cephalo_shard_adam(p, g, m, v, lp, n, 0, n, 1e-3, 0.9, 0.999, 1e-8, i + 1)
torch.cuda.synchronize()
