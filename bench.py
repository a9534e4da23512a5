#!/usr/bin/env python3
"""Benchmark of one GPU's share of a sharded data-parallel training step on one MI355X.

A "step" is one pass of the whole hot path over one batch share: forward of every micro-batch,
backward of every micro-batch with fp32 gradient accumulation (layered order: all micro-batches
through a layer before the next layer), then Adam on this GPU's uneven slice of the flat training
state (with the bf16 parameter copy refreshed for the slice).  Inputs are seeded synthetic tensors
already resident in HBM when the timed region starts.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5]

The default workload is c5, the largest one: the full 24-layer stack with embeddings, tied LM head
and mean cross-entropy.  c2..c4 are single-layer workloads (upstream gradient supplied).
Prints ONE JSON line (metric, value, roofline of the dominant kernel, CPU-oracle baseline).
"""
import argparse
import dataclasses
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E, published
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "gemm_input_gradient_and_adam_hbm_traffic.txt")


def traffic_from_profiles(key):
    """HBM bytes per launch of a kernel, as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by the
    copy-kernel calibration) and recorded in profiles/: the line 'BENCH <key> = <bytes>'.  None if it is not there."""
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 4 and parts[0] == "BENCH" and parts[1] == key and parts[2] == "=":
                    return float(parts[3])
    except OSError:
        pass
    return None


def layer_flops_per_microbatch(cfg):
    """fwd+bwd model FLOPs of one layer on one micro-batch: GEMMs 6 * T * (4H^2 + 2HF)
    (2 per multiply-add, x3 for fwd + dgrad + wgrad) and attention 12 m S^2 H non-causal,
    half of it under a causal mask.  Recompute and masked-out work are not counted."""
    T, H, F, S, m = cfg.tokens_per_micro, cfg.hidden, cfg.mlp, cfg.seq, cfg.micro_batch
    gemm = 6.0 * T * (4 * H * H + (3 if cfg.kind == "llama" else 2) * H * F)      # gated feed-forward: three F x H matrices
    attn = 12.0 * m * S * S * H * (0.5 if cfg.causal else 1.0)
    return gemm, attn


def step_model_flops(cfg):
    gemm, attn = layer_flops_per_microbatch(cfg)
    per_micro = cfg.layers * (gemm + attn)
    if cfg.vocab:
        per_micro += 6.0 * cfg.tokens_per_micro * cfg.hidden * cfg.vocab      # LM head (tied or not): logits, dgrad, wgrad
    return cfg.n_micro * per_micro


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c5", choices=["c1", "c2", "c3", "c4", "c5", "l7b", "ltiny", "vitl", "vitg", "g27"],
                    help="c5 (default) is the metric's workload; l7b: a Llama-style 7B-class layer; ltiny: a TinyLlama-shaped 22-layer "
                         "stack; vitl / vitg: ViT-Large- / ViT-G-shaped layers; g27: a GPT 2.7B-shaped layer (80 heads of 32)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-legs", action="store_true", help="skip the per-kernel legs (whole step only)")
    ap.add_argument("--checkpoint", action="store_true",
                    help="stacks only: layer-boundary activation checkpointing with recomputation in the backward (one extra forward)")
    ap.add_argument("--single-stream", action="store_true",
                    help="one micro-batch at a time on one stream (the default runs two micro-batches side by side on two streams)")
    ap.add_argument("--legs-only", action="store_true",
                    help="skip the timed steps and run only the per-kernel legs (for a profile in which each GEMM kernel's line holds "
                         "the legs' launches and nothing else); `value` is then null")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="instead of the benchmark: launch, three times each, the kernels whose HBM traffic the roofline quotes (the "
                         "dominant GEMM's shapes, a 1 GiB copy as calibration, the shard Adam), for a run under rocprofv3 --pmc")
    ap.add_argument("--offload", action="store_true",
                    help="stacks only, implies --checkpoint: the boundary activations live in pinned host memory and move on a second stream")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build covers one GPU's share of the step; it has no collectives and runs on exactly "
              "one GPU (--gpus %d was asked for)." % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2411_01075_amd as C
    from workloads import CONFIGS, shard_of, draw_layer_params, draw_stack_params, draw_activations, draw_token_ids, draw_adam_state

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    C.binding.lib()     # fail loudly if the HIP library is missing
    if args.traffic_probe:
        traffic_probe(C, torch, CONFIGS[args.workload])
        return
    cfg = CONFIGS[args.workload]
    stack = cfg.layers > 1
    bf16 = cfg.dtype == "bf16"
    b, m, l = cfg.batch_share, cfg.micro_batch, cfg.n_micro
    lr = float(np.float32(cfg.lr))

    # ---- seeded inputs, generated on the host, then made resident in HBM
    if stack:
        interleave = not (args.single_stream or args.offload)
        sd = C.stack_desc_from_config(cfg, checkpoint=args.checkpoint or args.offload, offload=args.offload, interleave=interleave)
        desc = sd.layer
        P = C.cephalo_stack_param_count(sd)
        params = draw_stack_params(cfg)
        flat32_h = C.flatten_stack_params(sd, params)
        ids_h, tgt_h = draw_token_ids(cfg)
    else:
        desc = C.desc_from_config(cfg)
        P = C.cephalo_layer_param_count(desc)
        params = draw_layer_params(cfg)
        flat32_h = C.flatten_layer_params(desc, params)
        x_h, dy_h = draw_activations(cfg)
    off, ln = shard_of(cfg, P)
    _, m_h, v_h = draw_adam_state(cfg, ln)            # moments of the slice only (a mid-training state)
    p32 = torch.from_numpy(flat32_h).cuda()
    if bf16:
        plow = torch.empty(P, dtype=torch.bfloat16, device="cuda")
        C.cephalo_cast_bf16(plow, p32)
        pcomp = plow
    else:
        plow, pcomp = None, p32
    G = torch.zeros(P, dtype=torch.float32, device="cuda")
    mom = torch.zeros(P, dtype=torch.float32, device="cuda")
    var = torch.zeros(P, dtype=torch.float32, device="cuda")
    mom[off:off + ln] = torch.from_numpy(m_h).cuda()
    var[off:off + ln] = torch.from_numpy(v_h).cuda()
    if stack:
        ids = torch.from_numpy(ids_h).cuda()
        tgt = torch.from_numpy(tgt_h).cuda()
        loss = torch.zeros(1, dtype=torch.float32, device="cuda")
        ws = torch.empty(C.cephalo_stack_workspace_bytes(sd, b, m), dtype=torch.uint8, device="cuda")

        if args.offload:
            host_area = torch.empty(C.cephalo_stack_host_bytes(sd, b, m) // 4, dtype=torch.float32).pin_memory()
            copy_in, copy_out = torch.cuda.Stream(), torch.cuda.Stream()

        if interleave:
            side = torch.cuda.Stream()

        def step(t):
            if args.offload:
                C.cephalo_stack_step_offload(sd, pcomp, ids, tgt, b, m, G, 1.0, loss, ws, host_area, copy_in, copy_out)
            elif interleave:
                C.cephalo_stack_step_interleaved(sd, pcomp, ids, tgt, b, m, G, 1.0, loss, ws, side)
            else:
                C.cephalo_stack_step(sd, pcomp, ids, tgt, b, m, G, 1.0, loss, ws)
            C.cephalo_shard_adam(p32, G, mom, var, plow, P, off, ln, lr, 0.9, 0.999, 1e-8, 0.0, t)
    else:
        x = torch.from_numpy(x_h).cuda().float().contiguous()       # the residual stream is fp32
        dy = torch.from_numpy(dy_h).cuda().float().contiguous()
        y, dx = torch.empty_like(x), torch.empty_like(x)
        save_b, scr_b = C.cephalo_share_workspace_bytes(desc, b, m)
        save = torch.empty(save_b, dtype=torch.uint8, device="cuda")
        scratch = torch.empty(scr_b, dtype=torch.uint8, device="cuda")

        interleave = not args.single_stream and l > 1
        if interleave:
            side = torch.cuda.Stream()

        def step(t):
            if interleave:
                C.cephalo_share_layer_step_interleaved(desc, pcomp, x, y, dy, dx, b, m, save, G, 1.0, scratch, side)
            else:
                C.cephalo_share_layer_step(desc, pcomp, x, y, dy, dx, b, m, save, G, 1.0, scratch)
            C.cephalo_shard_adam(p32, G, mom, var, plow, P, off, ln, lr, 0.9, 0.999, 1e-8, 0.0, t)

    if args.legs_only:
        args.steps, args.warmup = 0, 0
    for i in range(args.warmup):
        step(7 + i)
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]      # on the stream every step starts and ends on
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        step(7 + args.warmup + i)
        marks[i + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0 if args.steps else float("nan")
    ms_per_step = 1e3 * elapsed / max(args.steps, 1)
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)) or [float("nan")]
    tokens_per_s = cfg.tokens_per_step * args.steps / elapsed
    step_flops = step_model_flops(cfg)
    extras = {"step_ms_median": round(per_step[len(per_step) // 2], 4), "step_ms_min": round(per_step[0], 4)} if args.steps else {}
    if stack:
        extras["loss"] = round(float(loss.item()), 4)
        extras["activation_checkpointing"] = bool(args.checkpoint or args.offload)
        extras["activation_offload"] = bool(args.offload)

        if args.offload:
            extras["host_area_GB"] = round(host_area.numel() * 4 / 1e9, 2)
        extras["workspace_GB"] = round(ws.numel() / 1e9, 2)
    extras["micro_batches_in_flight"] = 2 if interleave else 1
    if bf16 and args.steps:
        extras["whole_step_model_tflops"] = round(step_flops / (elapsed / args.steps) / 1e12, 1)
        extras["whole_step_frac_of_bf16_peak"] = round(step_flops / (elapsed / args.steps) / 1e12 / PEAK_BF16_TFLOPS, 4)

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

    def timed_pairs(fn, iters):
        """fn(i) launches on stream i of two; pairs run side by side as in the interleaved step.  Returns the time of a pair."""
        s0 = torch.cuda.current_stream()
        fn(0, s0); fn(1, side)
        torch.cuda.synchronize()
        e0, e1, ej = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True), torch.cuda.Event()
        e0.record(s0)
        side.wait_event(e0)
        for _ in range(iters):
            fn(0, s0)
            fn(1, side)
        ej.record(side)
        s0.wait_event(ej)
        e1.record(s0)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / iters

    roofline = {"kernel": "not broken out (the GEMM legs are timed for the bf16 GPT-style workloads; see whole_step_model_tflops)",
                "bound": "mfma" if bf16 else "alu", "achieved": None, "peak": PEAK_BF16_TFLOPS if bf16 else 157.3,
                "unit": "TFLOP/s", "frac": None, "traffic": None}
    T, H, F, V = cfg.tokens_per_micro, cfg.hidden, cfg.mlp, cfg.vocab
    n_tok = cfg.tokens_per_step
    if bf16 and not args.no_legs and cfg.kind == "gpt":      # (the legs carry the GPT-style layer's epilogues)
        if stack:
            del ws                      # the legs allocate their own operands
            torch.cuda.empty_cache()
        bt = torch.bfloat16
        # The GEMM kernels of the step, each launched through the C ABI with the shapes, operand layouts and epilogues
        # the step uses.  Forward and input-gradient GEMMs run per micro-batch on T tokens (the input gradients read
        # the per-layer transposed weights, so they are the same contraction as the forward); the weight gradient
        # runs once per linear layer over all b*S tokens (token-minor copy of one operand + GEMM + split reduction).
        L = cfg.layers
        lin = [("qkv", 3 * H, H), ("o", H, H), ("fc1", F, H), ("fc2", H, F)]
        legs = {}

        pairs = interleave      # per-micro-batch GEMMs run two side by side, one per stream, as in the step

        def add_leg(key, fn, flops, count, alone=False):
            # enough back-to-back launches (about 30 ms) that the clocks settle where they sit during the step.
            # fn(i, stream): launch number i of a pair (its own output buffers) on that stream.
            # Every leg is timed alone on one stream; a per-micro-batch leg of a two-stream step is also timed the way
            # that step launches it, in pairs, one kernel per stream, on the tile chosen for half the device.
            # (--legs-only: the same number of launches for every shape, so that a profile's per-kernel average weighs the
            #  shapes that share a kernel as the step does, equally)
            reps = (lambda first: 40) if args.legs_only else (lambda first: max(3, min(400, int(0.03 / max(first, 1e-6)))))
            one = lambda: fn(0, None)
            first = timed(one, 2)
            dur1 = timed(one, reps(first))
            if pairs and not alone:
                C.cephalo_gemm_side_by_side(2)
                first = timed_pairs(fn, 2)
                dur = timed_pairs(fn, reps(first))      # a kernel's duration = the pair's
                sec = dur / 2                                                                  # device time per launch
                C.cephalo_gemm_side_by_side(1)
            else:
                dur = sec = dur1
            g = legs.setdefault(key, {"sec": 0.0, "dur": 0.0, "dur1": 0.0, "flops": 0.0, "launches": 0, "side_by_side": 2 if (pairs and not alone) else 1})
            g["sec"] += sec * count
            g["dur"] += dur * count
            g["dur1"] += dur1 * count
            g["flops"] += flops * count
            g["launches"] += count

        def rnd(*shape, scale=1.0, dtype=bt):
            return (torch.randn(*shape, device="cuda") * scale).to(dtype)

        def two(*shape, dtype=bt):
            return [torch.empty(*shape, device="cuda", dtype=dtype) for _ in range(2)]

        for name, n_out, k_in in lin:
            X, W, WT, dY = rnd(T, k_in), rnd(n_out, k_in, scale=0.02), rnd(k_in, n_out, scale=0.02), rnd(T, n_out)
            bias = torch.zeros(n_out, device="cuda", dtype=bt)
            fl = 2.0 * T * n_out * k_in
            fwd_args = (C.BF16, X, k_in, 1, W, k_in, 1, T, n_out, k_in)
            if name == "qkv":
                Y = two(T, n_out)
                add_leg("forward, bias epilogue (qkv)", lambda i, st: C.cephalo_op_gemm(*fwd_args, C.EPI_BIAS, C=Y[i], bias=bias, stream=st), fl, L * l)
            elif name == "fc1":
                Y, Z = two(T, n_out), two(T, n_out, dtype=torch.float16)      # the saved derivative is a half-precision factor
                add_leg("forward, bias+GELU epilogue, derivative saved (fc1)",
                        lambda i, st: C.cephalo_op_gemm(*fwd_args, C.EPI_BIAS_GELU_DERIV, C=Y[i], bias=bias, Z=Z[i], stream=st), fl, L * l)
            else:
                R, Y = rnd(T, n_out, dtype=torch.float32), two(T, n_out, dtype=torch.float32)
                add_leg("forward, bias+residual epilogue, fp32 stream (out-proj, fc2)",
                        lambda i, st: C.cephalo_op_gemm(*fwd_args, C.EPI_BIAS_RESID_F32, C=Y[i], bias=bias, R=R, stream=st), fl, L * l)
            # input gradient dX[T, k_in] = dY[T, n_out] W, through W^T [k_in, n_out]
            dg_args = (C.BF16, dY, n_out, 1, WT, n_out, 1, T, k_in, n_out)
            if name == "fc2":
                Zs, dZ = rnd(T, k_in, dtype=torch.float16), two(T, k_in)
                add_leg("input gradient, times the saved GELU' (fc2)", lambda i, st: C.cephalo_op_gemm(*dg_args, C.EPI_MUL, C=dZ[i], Z=Zs, stream=st), fl, L * l)
            elif name == "o":
                dX = two(T, k_in)
                add_leg("input gradient, plain epilogue (qkv, out-proj, fc1)", lambda i, st: C.cephalo_op_gemm(*dg_args, C.EPI_NONE, C=dX[i], stream=st), fl, L * l)
            else:
                dX = two(T, k_in, dtype=torch.float32)
                add_leg("input gradient, plain epilogue (qkv, out-proj, fc1)", lambda i, st: C.cephalo_op_gemm(*dg_args, C.EPI_NONE_F32, C=dX[i], stream=st), fl, L * l)
            del X, W, WT, dY
            # weight gradient over the whole share: alone on the main stream
            Xs, dYs = rnd(n_tok, k_in), rnd(n_tok, n_out)
            Gw = torch.zeros(n_out, k_in, device="cuda")
            wsb = torch.empty(C.cephalo_op_linear_wgrad_workspace(C.BF16, n_tok, n_out, k_in), dtype=torch.uint8, device="cuda")
            add_leg("weight gradient over the share (GEMM + split reduction)",
                    lambda i, st: C.cephalo_op_linear_wgrad(C.BF16, dYs, Xs, n_tok, n_out, k_in, Gw, 1.0, 0, wsb), 2.0 * n_tok * n_out * k_in, L, alone=True)
            del Xs, dYs, Gw, wsb
        for g in legs.values():
            g["TFLOP/s"] = round(g["flops"] / g["sec"] / 1e12, 1)
            g["frac_of_bf16_peak"] = round(g["flops"] / g["sec"] / 1e12 / PEAK_BF16_TFLOPS, 4)
            g["avg_launch_us"] = round(1e6 * g.pop("dur") / g["launches"], 1)      # a kernel's own duration (side by side: while sharing the device)
            g["ms_per_step"] = round(1e3 * g.pop("sec"), 3)
            one = g.pop("dur1")
            g["one_stream"] = {"TFLOP/s": round(g["flops"] / one / 1e12, 1), "frac_of_bf16_peak": round(g["flops"] / one / 1e12 / PEAK_BF16_TFLOPS, 4),
                               "avg_launch_us": round(1e6 * one / g["launches"], 1), "ms_per_step": round(1e3 * one, 3)}
            g["flops_per_launch"] = g.pop("flops") / g["launches"]
        single = [k for k in legs if not k.startswith("weight gradient")]      # one kernel launch per call
        key = max(single, key=lambda k: legs[k]["ms_per_step"])
        d = legs[key]
        # HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, read from the committed summary of
        # `bench.py --traffic-probe` (measured for the c5 shapes of this leg only)
        traffic = traffic_from_profiles("c5_input_gradient_bytes_per_launch") if (cfg.name == "c5" and key.startswith("input gradient, plain")) else None
        roofline = {"kernel": "gemm_mfma_kernel (v_mfma_f32_16x16x32_bf16), " + key, "bound": "mfma", "achieved": d["TFLOP/s"], "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(d["TFLOP/s"] / PEAK_BF16_TFLOPS, 4), "traffic": traffic,
                    "avg_launch_us": d["avg_launch_us"], "flops_per_launch": d["flops_per_launch"], "launches_per_step": d["launches"],
                    # side_by_side = 2: two such kernels share the device, one per stream, as the step runs them; `achieved`
                    # is their joint rate, 2 * flops_per_launch / avg_launch_us, against the whole device's peak.  one_stream:
                    # the same launches one at a time (each kernel has the device to itself, on the tile chosen for that).
                    "side_by_side": d["side_by_side"], "one_stream": d["one_stream"]}
        tot_pair = sum(g["ms_per_step"] for g in legs.values())
        tot_one = sum(g["one_stream"]["ms_per_step"] for g in legs.values())
        gemm_flops = sum(g["flops_per_launch"] * g["launches"] for g in legs.values())
        extras["gemm_all_legs"] = {"flops_per_step": gemm_flops, "ms_per_step": round(tot_pair, 3),
                                   "frac_of_bf16_peak": round(gemm_flops / (tot_pair * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                                   "one_stream_ms_per_step": round(tot_one, 3),
                                   "one_stream_frac_of_bf16_peak": round(gemm_flops / (tot_one * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
        extras["gemm_legs"] = legs

        # ---- attention alone (forward; backward = rowsum(dO*O) + dQ kernel + dK/dV kernel), at the workload's shape.
        # Model flops: 4 m S^2 H forward (half under a causal mask), twice that backward; the backward kernels recompute
        # the scores and dP (7 products instead of 4), which is not counted.
        A, S, m_ = cfg.heads, cfg.seq, cfg.micro_batch
        qkv = rnd(T, 3 * H)
        dO = rnd(T, H)
        O = torch.empty(T, H, device="cuda", dtype=bt)
        lse = torch.empty(m_ * A * S, device="cuda")
        dvec = torch.empty(m_ * A * S, device="cuda")
        dqkv = torch.empty(T, 3 * H, device="cuda", dtype=bt)
        af = 4.0 * m_ * S * S * H * (0.5 if cfg.causal else 1.0)
        t_f = timed(lambda: C.cephalo_op_attention_fwd(desc, qkv, O, lse, m_), 50)
        t_b = timed(lambda: C.cephalo_op_attention_bwd(desc, qkv, O, dO, lse, dvec, dqkv, m_), 30)
        extras["attention"] = {
            "forward": {"us": round(t_f * 1e6, 1), "model_TFLOP/s": round(af / t_f / 1e12, 1), "frac_of_bf16_peak": round(af / t_f / 1e12 / PEAK_BF16_TFLOPS, 4)},
            "backward": {"us": round(t_b * 1e6, 1), "model_TFLOP/s": round(2 * af / t_b / 1e12, 1), "frac_of_bf16_peak": round(2 * af / t_b / 1e12 / PEAK_BF16_TFLOPS, 4)},
            "ms_per_step": round(1e3 * (t_f + t_b) * cfg.layers * l, 3)}
        del qkv, dO, O, dqkv

        # ---- the bandwidth-bound kernels alone: algorithmic bytes / time against the HBM peak
        def gbs(nbytes, sec):
            return {"us": round(sec * 1e6, 1), "GB/s": round(nbytes / sec / 1e9, 1), "frac_of_hbm_peak": round(nbytes / sec / 1e9 / PEAK_HBM_GBS, 4)}
        xr = torch.randn(T, H, device="cuda")
        gam, bet = torch.ones(H, device="cuda", dtype=bt), torch.zeros(H, device="cuda", dtype=bt)
        u_ = torch.empty(T, H, device="cuda", dtype=bt)
        mean_, rstd_ = torch.empty(T, device="cuda"), torch.empty(T, device="cuda")
        t_lnf = timed(lambda: C.cephalo_op_norm_fwd(C.BF16, False, xr, gam, bet, u_, mean_, rstd_, T, H, 1e-5), 100)
        du_, res_, dx_ = torch.randn(T, H, device="cuda"), torch.randn(T, H, device="cuda"), torch.empty(T, H, device="cuda")
        dxl_ = torch.empty(T, H, device="cuda", dtype=bt)
        dg_, db_ = torch.empty(H, device="cuda"), torch.empty(H, device="cuda")
        wsn = torch.empty(C.cephalo_op_norm_bwd_workspace(T, H), dtype=torch.uint8, device="cuda")
        t_lnb = timed(lambda: C.cephalo_op_norm_bwd(C.BF16, False, du_, xr, mean_, rstd_, gam, res_, dx_, dxl_, dg_, db_, T, H, wsn), 100)
        dzs = rnd(n_tok, F)
        wsc = torch.empty(C.cephalo_op_colsum_workspace(n_tok, F), dtype=torch.uint8, device="cuda")
        gF = torch.empty(F, device="cuda")
        t_cs = timed(lambda: C.cephalo_op_colsum(C.BF16, dzs, n_tok, F, gF, 1.0, 0, wsc), 30)
        extras["elementwise"] = {
            # LayerNorm forward: reads the fp32 row, writes it in bf16 (+ 8 B of statistics per row)
            "layer_norm_forward": gbs(T * (H * 6 + 8), t_lnf),
            # backward with the partial sums of d gamma / d beta and their fixed-order reduction: reads du, x and the
            # residual in fp32 (+ statistics), writes dx in fp32 and in bf16
            "layer_norm_backward": gbs(T * (H * 18 + 8), t_lnb),
            # bias gradient of the first feed-forward projection over the whole share: reads d z [b*S, F] in bf16
            "bias_column_sum": gbs(n_tok * F * 2, t_cs),
        }
        del xr, u_, du_, res_, dx_, dxl_, dzs
        if stack:
            ldv = (V + 63) // 64 * 64
            lg = torch.randn(T, ldv, device="cuda")
            tg = torch.randint(0, V, (T,), device="cuda", dtype=torch.int32)
            dl_ = torch.empty(T, ldv, device="cuda", dtype=bt)
            lr_ = torch.empty(T, device="cuda")
            t_ce = timed(lambda: C.cephalo_op_cross_entropy(C.BF16, lg, ldv, tg, dl_, lr_, T, V, 1.0 / n_tok), 30)
            # two passes over the fp32 logits of a micro-batch, one write of their bf16 gradient
            extras["elementwise"]["cross_entropy"] = gbs(T * ldv * (4 + 2), t_ce)      # fp32 logits read once (the row stays in registers), bf16 gradient written
            del lg, dl_

    # ---- what this device sustains (probes of the library): a register-only stream of the GEMM's matrix instruction on
    # random operands, and streaming reads / writes / copies of 1 GiB
    if bf16:
        seed = (torch.randn(32768, device="cuda")).to(torch.bfloat16)
        sink = torch.zeros(4, device="cuda")
        fl = C.cephalo_probe_mfma(seed, 1024, 2000, sink)
        t_m = timed(lambda: C.cephalo_probe_mfma(seed, 1024, 2000, sink), 10)      # about 50 ms of back-to-back launches: a sustained rate
        nb = 1 << 30
        a_ = torch.empty(nb // 4, device="cuda"); b_ = torch.empty(nb // 4, device="cuda")
        a_.fill_(1.0); b_.fill_(2.0)
        t_r = timed(lambda: C.cephalo_probe_stream(0, None, a_, nb, sink), 20)
        t_w = timed(lambda: C.cephalo_probe_stream(1, b_, None, nb, sink), 20)
        t_c = timed(lambda: C.cephalo_probe_stream(2, b_, a_, nb, sink), 20)
        mp = {"mfma_16x16x32_bf16_registers_only_TFLOP/s": round(fl / t_m / 1e12, 1), "read_GB/s": round(nb / t_r / 1e9, 1),
              "write_GB/s": round(nb / t_w / 1e9, 1), "copy_GB/s": round(2 * nb / t_c / 1e9, 1)}
        extras["measured_on_this_device"] = mp
        if roofline.get("achieved"):
            roofline["frac_of_measured_mfma_stream"] = round(roofline["achieved"] / mp["mfma_16x16x32_bf16_registers_only_TFLOP/s"], 4)
        del a_, b_
    # shard Adam alone: 28 algorithmic bytes per element (+2 for the bf16 copy)
    adam_sec = timed(lambda: C.cephalo_shard_adam(p32, G, mom, var, plow, P, off, ln, lr, 0.9, 0.999, 1e-8, 0.0, 9), 10)
    adam_bytes = ln * (28 + (2 if bf16 else 0))
    extras["shard_adam"] = {"elements": ln, "us": round(adam_sec * 1e6, 1), "GB/s": round(adam_bytes / adam_sec / 1e9, 1),
                            "frac_of_hbm_peak": round(adam_bytes / adam_sec / 1e9 / PEAK_HBM_GBS, 4),
                            "traffic_bytes_per_element": traffic_from_profiles("shard_adam_bytes_per_element")}
    if "measured_on_this_device" in extras:
        extras["shard_adam"]["frac_of_measured_copy"] = round(adam_bytes / adam_sec / 1e9 / extras["measured_on_this_device"]["copy_GB/s"], 4)

    # bf16 GEMMs that fell off the matrix-core kernel onto the general one (0 for every workload here)
    extras["gemm_calls_on_general_kernel"] = C.cephalo_gemm_general_count()

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, params, flat32_h, m_h, v_h, off, ln, lr,
                           None if stack else (x_h, dy_h), (ids_h, tgt_h) if stack else None)

    what = ("%d %s layers + embeddings + %s LM head (V=%d)" % (cfg.layers, "Llama-style" if cfg.kind == "llama" else "GPT-style",
                                                               "untied" if cfg.kind == "llama" else "tied", V)) if stack else "1 layer"
    out = {
        "metric": "tokens/s per fwd+bwd+shard-Adam step on 1 MI355X",
        "value": round(tokens_per_s, 1) if args.steps else None, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4) if args.steps else None, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": "%s: %s H=%d A=%d F=%d S=%d %s, batch share %d = %d micro-batches x %d, shard [%d, %d) of P=%d"
                               % (cfg.name, what, cfg.hidden, cfg.heads, cfg.mlp, cfg.seq, "causal" if cfg.causal else "non-causal",
                                  b, l, m, off, off + ln, P)},
        "roofline": roofline, "cpu_baseline": cpu, "extras": extras,
    }
    print(json.dumps(out))


def traffic_probe(C, torch, cfg):
    """Launches, three times each, the kernels whose HBM traffic the benchmark quotes: the input-gradient GEMM of the
    workload's three projections with N = H outputs (through the transposed weight, on the tile the two-stream step runs
    them on), a 1 GiB device copy (the calibration of the counters: 2^30 bytes read, 2^30 written) and the shard Adam
    on a 64 Mi-element slice with the bf16 copy.  Meant to run under
        rocprofv3 --pmc FETCH_SIZE --output-format csv -d <dir> -o t -- python3 bench.py --traffic-probe
        rocprofv3 --pmc WRITE_SIZE --output-format csv -d <dir> -o t -- python3 bench.py --traffic-probe
    (one counter per run); the per-dispatch values are in <dir>/t_counter_collection.csv, in KiB."""
    T, H, F = cfg.tokens_per_micro, cfg.hidden, cfg.mlp
    bt = torch.bfloat16
    C.cephalo_gemm_side_by_side(2)

    def dgrad(n_out, k_in, f32):      # dX[T, k_in] = dY[T, n_out] W through W^T [k_in, n_out]
        dY = torch.randn(T, n_out, device="cuda").to(bt)
        WT = (torch.randn(k_in, n_out, device="cuda") * 0.02).to(bt)
        dX = torch.empty(T, k_in, device="cuda", dtype=torch.float32 if f32 else bt)
        for _ in range(3):
            C.cephalo_op_gemm(C.BF16, dY, n_out, 1, WT, n_out, 1, T, k_in, n_out, C.EPI_NONE_F32 if f32 else C.EPI_NONE, C=dX)
        torch.cuda.synchronize()
    dgrad(3 * H, H, True)     # qkv
    dgrad(H, H, False)        # out-proj
    dgrad(F, H, True)         # fc1
    a = torch.empty(1 << 28, device="cuda"); b = torch.empty(1 << 28, device="cuda")
    a.fill_(1.0)
    for _ in range(3):
        b.copy_(a)
    n = 1 << 26
    p = torch.zeros(n, device="cuda"); g = torch.ones(n, device="cuda") * 1e-2; m = torch.zeros(n, device="cuda"); v = torch.zeros(n, device="cuda")
    lp = torch.empty(n, device="cuda", dtype=bt)
    for i in range(3):
        C.cephalo_shard_adam(p, g, m, v, lp, n, 0, n, 1e-3, 0.9, 0.999, 1e-8, 0.0, i + 1)
    torch.cuda.synchronize()
    print("traffic probe done", flush=True)


def cpu_baseline(cfg, params, flat32_h, m_h, v_h, off, ln, lr, acts, tokens):
    """The numpy fp64 oracle, untouched, on a bounded sample; tokens/s scaled to the whole step."""
    from oracle import adam as oadam
    from oracle import layer as olayer
    from oracle import stack as ostack
    from oracle.precision import round_to_bf16
    from tests.harness import oracle_share_step
    threads = len(os.sched_getaffinity(0))
    l, m = cfg.n_micro, cfg.micro_batch
    if cfg.layers == 1:
        x_h, dy_h = acts
        sample_cfg = dataclasses.replace(cfg, n_micro=1)
        n_ad = min(ln, max(1, ln // l))
        t0 = time.perf_counter()
        if cfg.kind == "llama":
            from oracle import llama as ollama
            p64 = {k: round_to_bf16(v) if cfg.dtype == "bf16" else v.astype(np.float64) for k, v in params.items()}
            _, _, g = ollama.share_step(p64, x_h[:m].astype(np.float64), dy_h[:m].astype(np.float64), cfg.heads, m, cfg.causal)
            G_ref = np.concatenate([g[k].reshape(-1) for k in ollama.NAMES])
        else:
            _, _, G_ref = oracle_share_step(sample_cfg, params, x_h[:m], dy_h[:m])
        sl = slice(off, off + n_ad)
        oadam.shard_adam(flat32_h[sl].astype(np.float64), G_ref[sl], m_h[:n_ad].astype(np.float64),
                         v_h[:n_ad].astype(np.float64), 0, n_ad, lr, 0.9, 0.999, 1e-8, 7)
        sec = time.perf_counter() - t0
        return {"value": round(cfg.tokens_per_micro / sec, 2), "unit": "tokens/s", "cores": threads, "kind": "oracle",
                "sample": "1 of %d micro-batches (%d tokens) fwd+bwd in fp64 numpy + Adam on %d of %d slice elements, %.1f s"
                          % (l, cfg.tokens_per_micro, n_ad, ln, sec)}
    # full stack: (a) one layer, forward + backward, on one micro-batch; (b) the oracle's whole step on a 1-layer,
    # 1-micro-batch relative with the full vocabulary (embeddings, that layer, final LN, LM head, cross-entropy and
    # back); (c) Adam on 1/64 of the slice.  Whole step ~ l * (L * a + (b - a)) + 64 * c.
    ids_h, tgt_h = tokens
    rb = (lambda a: round_to_bf16(a)) if cfg.dtype == "bf16" else (lambda a: a.astype(np.float64))
    lp = {k: rb(v) for k, v in params["layers"][0].items()}
    x = np.random.default_rng(0).standard_normal((m, cfg.seq, cfg.hidden))
    if cfg.kind == "llama":
        from oracle import llama as olayer          # the Llama-style layer and stack
        stack_step = olayer.stack_step
        p1 = {"wte": rb(params["wte"]), "normf_g": rb(params["normf_g"]), "w_head": rb(params["w_head"]), "layers": [lp]}
    else:
        stack_step = ostack.stack_step
        p1 = {"wte": rb(params["wte"]), "wpe": rb(params["wpe"]), "lnf_g": rb(params["lnf_g"]), "lnf_b": rb(params["lnf_b"]), "layers": [lp]}
    t0 = time.perf_counter()
    y, cache = olayer.layer_fwd(lp, x, cfg.heads, cfg.causal)
    olayer.layer_bwd(lp, cache, x, cfg.heads)
    t_layer = time.perf_counter() - t0
    del y, cache
    t0 = time.perf_counter()
    stack_step(p1, ids_h[:m], tgt_h[:m], cfg.heads, cfg.causal, m)
    t_stack1 = time.perf_counter() - t0
    n_ad = max(1, ln // 64)
    sl = slice(off, off + n_ad)
    t0 = time.perf_counter()
    oadam.shard_adam(flat32_h[sl].astype(np.float64), flat32_h[sl].astype(np.float64), m_h[:n_ad].astype(np.float64),
                     v_h[:n_ad].astype(np.float64), 0, n_ad, lr, 0.9, 0.999, 1e-8, 7)
    t_adam = time.perf_counter() - t0
    est = l * (cfg.layers * t_layer + max(0.0, t_stack1 - t_layer)) + 64 * t_adam
    return {"value": round(cfg.tokens_per_step / est, 3), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "extrapolated: one layer fwd+bwd on one micro-batch of %d tokens (%.1f s), the oracle's whole step on a "
                      "1-layer 1-micro-batch relative with the full vocabulary (%.1f s), Adam on 1/64 of the slice (%.2f s); "
                      "whole step estimated as l*(L*layer + head) + Adam = %.0f s" % (cfg.tokens_per_micro, t_layer, t_stack1, t_adam, est)}


if __name__ == "__main__":
    main()
