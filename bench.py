#!/usr/bin/env python3
"""Benchmark of one GPU's share of a sharded data-parallel training step on one MI355X.

A "step" is one pass of the whole hot path over one batch share: forward of every micro-batch,
backward of every micro-batch with fp32 gradient accumulation, then Adam on this GPU's uneven
slice of the flat training state (with the bf16 parameter copy refreshed for the slice).
Inputs are seeded synthetic tensors already resident in HBM when the timed region starts.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4]

Prints ONE JSON line (metric, value, roofline of the dominant kernel, CPU-oracle baseline).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E, published


def model_flops_per_microbatch(cfg):
    """fwd+bwd model FLOPs of one layer on one micro-batch: GEMMs 6 * T * (4H^2 + 2HF)
    (2 per multiply-add, x3 for fwd + dgrad + wgrad) and attention 12 m S^2 H non-causal,
    half of it under a causal mask.  Recompute and masked-out work are not counted."""
    T, H, F, S, m = cfg.tokens_per_micro, cfg.hidden, cfg.mlp, cfg.seq, cfg.micro_batch
    gemm = 6.0 * T * (4 * H * H + 2 * H * F)
    attn = 12.0 * m * S * S * H * (0.5 if cfg.causal else 1.0)
    return gemm, attn


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c4", choices=["c1", "c2", "c3", "c4"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build covers one GPU's share of the step; it has no collectives and runs on exactly "
              "one GPU (--gpus %d was asked for)." % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2411_01075_amd as C
    from workloads import CONFIGS, shard_of, draw_layer_params, draw_activations, draw_adam_state

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    C.binding.lib()     # fail loudly if the HIP library is missing
    cfg = CONFIGS[args.workload]
    desc = C.desc_from_config(cfg)
    bf16 = cfg.dtype == "bf16"
    dt = torch.bfloat16 if bf16 else torch.float32
    P = C.cephalo_layer_param_count(desc)
    off, ln = shard_of(cfg, P)
    b, m, l = cfg.batch_share, cfg.micro_batch, cfg.n_micro

    # ---- seeded inputs, generated on the host, then made resident in HBM
    tensors = draw_layer_params(cfg)
    x_h, dy_h = draw_activations(cfg)
    flat32_h = C.flatten_layer_params(desc, tensors)
    _, m_h, v_h = draw_adam_state(cfg, ln)            # moments of the slice only (a mid-training state)
    p32 = torch.from_numpy(flat32_h).cuda()
    p32_init = p32.clone()
    if bf16:
        plow = torch.empty(P, dtype=torch.bfloat16, device="cuda")
        C.cephalo_cast_bf16(plow, p32)
        pcomp = plow
    else:
        plow, pcomp = None, p32
    x = torch.from_numpy(x_h).cuda().to(dt).contiguous()
    dy = torch.from_numpy(dy_h).cuda().to(dt).contiguous()
    y, dx = torch.empty_like(x), torch.empty_like(x)
    G = torch.zeros(P, dtype=torch.float32, device="cuda")
    mom = torch.zeros(P, dtype=torch.float32, device="cuda")
    var = torch.zeros(P, dtype=torch.float32, device="cuda")
    mom[off:off + ln] = torch.from_numpy(m_h).cuda()
    var[off:off + ln] = torch.from_numpy(v_h).cuda()
    save_b, scr_b = C.cephalo_share_workspace_bytes(desc, b, m)
    save = torch.empty(save_b, dtype=torch.uint8, device="cuda")
    scratch = torch.empty(scr_b, dtype=torch.uint8, device="cuda")
    lr = float(np.float32(cfg.lr))

    def step(t):
        C.cephalo_share_layer_step(desc, pcomp, x, y, dy, dx, b, m, save, G, 1.0, scratch)
        C.cephalo_shard_adam(p32, G, mom, var, plow, P, off, ln, lr, 0.9, 0.999, 1e-8, t)

    for i in range(args.warmup):
        step(7 + i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(7 + args.warmup + i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    tokens_per_s = cfg.tokens_per_step * args.steps / elapsed
    gemm_fl, attn_fl = model_flops_per_microbatch(cfg)
    step_flops = l * (gemm_fl + attn_fl)

    # ---- per-kernel legs, HIP events on the launch stream (torch's current stream is the one passed to the library)
    def timed(fn, iters):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / iters

    extras = {}
    T, H, F = cfg.tokens_per_micro, cfg.hidden, cfg.mlp
    if bf16:
        # dominant kernel: the weight-gradient GEMM (one kernel instantiation, four launches per micro-batch
        # of the shapes dW_qkv, dW_o, dW_fc1, dW_fc2), exactly as the layer's backward issues it
        shapes = [(3 * H, H), (H, H), (F, H), (H, F)]          # (N_out, K_in) of each linear
        acts = {}
        for n_out, k_in in shapes:
            acts[(n_out, k_in)] = (torch.randn(T, n_out, device="cuda").to(dt), torch.randn(T, k_in, device="cuda").to(dt),
                                   torch.zeros(n_out, k_in, device="cuda"))

        def wgrads():
            for (n_out, k_in), (dY_, X_, G_) in acts.items():
                C.cephalo_op_gemm(C.BF16, dY_, 1, n_out, X_, 1, k_in, n_out, k_in, T, C.EPI_GRAD, G=G_, scale=1.0, accumulate=1)

        sec = timed(wgrads, max(3, args.steps))
        flops_per_launch = sum(2.0 * T * n * k for n, k in shapes) / len(shapes)
        avg_launch = sec / len(shapes)
        achieved = flops_per_launch / avg_launch / 1e12
        roofline = {"kernel": "gemm_mfma_kernel<..., EPI_GRAD> (weight gradient, 4 launches per micro-batch)",
                    "bound": "mfma", "achieved": round(achieved, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": None,
                    "avg_launch_us": round(avg_launch * 1e6, 1), "flops_per_launch": flops_per_launch}
        extras["whole_step_model_tflops"] = round(step_flops / (elapsed / args.steps) / 1e12, 1)
        extras["whole_step_frac_of_bf16_peak"] = round(step_flops / (elapsed / args.steps) / 1e12 / PEAK_BF16_TFLOPS, 4)
    else:
        roofline = {"kernel": "none (launch-latency bound workload)", "bound": "alu", "achieved": None, "peak": 157.3,
                    "unit": "TFLOP/s", "frac": None, "traffic": None}
    # shard Adam alone: 28 algorithmic bytes per element (+2 for the bf16 copy)
    adam_sec = timed(lambda: C.cephalo_shard_adam(p32, G, mom, var, plow, P, off, ln, lr, 0.9, 0.999, 1e-8, 9), 20)
    adam_bytes = ln * (28 + (2 if bf16 else 0))
    extras["shard_adam"] = {"elements": ln, "us": round(adam_sec * 1e6, 1), "GB/s": round(adam_bytes / adam_sec / 1e9, 1),
                            "frac_of_hbm_peak": round(adam_bytes / adam_sec / 1e9 / PEAK_HBM_GBS, 4)}

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import adam as oadam
        from tests.harness import oracle_share_step
        import dataclasses
        sample_cfg = dataclasses.replace(cfg, n_micro=1)
        xs, dys = x_h[:m], dy_h[:m]
        n_ad = min(ln, max(1, ln // l))
        threads = len(os.sched_getaffinity(0))
        t0 = time.perf_counter()
        _, _, G_ref = oracle_share_step(sample_cfg, tensors, xs, dys)
        sl = slice(off, off + n_ad)
        oadam.shard_adam(flat32_h[sl].astype(np.float64), G_ref[sl], m_h[:n_ad].astype(np.float64),
                         v_h[:n_ad].astype(np.float64), 0, n_ad, lr, 0.9, 0.999, 1e-8, 7)
        cpu_sec = time.perf_counter() - t0
        cpu = {"value": round(cfg.tokens_per_micro / cpu_sec, 2), "unit": "tokens/s", "cores": threads, "kind": "oracle",
               "sample": "1 of %d micro-batches (%d tokens) fwd+bwd in fp64 numpy + Adam on %d of %d slice elements, %.1f s"
                         % (l, cfg.tokens_per_micro, n_ad, ln, cpu_sec)}

    out = {
        "metric": "tokens/s per fwd+bwd+shard-Adam step on 1 MI355X",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": "%s: 1 layer H=%d A=%d F=%d S=%d %s, batch share %d = %d micro-batches x %d, shard [%d, %d) of P=%d"
                               % (cfg.name, cfg.hidden, cfg.heads, cfg.mlp, cfg.seq, "causal" if cfg.causal else "non-causal",
                                  b, l, m, off, off + ln, P)},
        "roofline": roofline, "cpu_baseline": cpu, "extras": extras,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
