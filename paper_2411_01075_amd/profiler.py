"""Profiler of Sec. 3.3 / 4.1 on one MI355X: times one transformer layer's forward and backward through the C ABI
for micro-batch sizes 1..B, reads the compute memory from the library's workspace query, and fits the paper's
models: latency = profiled values inside the profiled range, a line beyond it (T(m, l) = l T(m)); compute memory =
a line in m; training state = 16 bytes per parameter.  The tables it produces feed cephalo_plan_compute.

    python -m paper_2411_01075_amd.profiler --workload c5 --max-m 8 --check 12 16
"""
import argparse
import json
import sys


def fit_line(xs, ys):
    """Closed-form least squares: returns (intercept, slope)."""
    n = float(len(xs))
    sx, sy = float(sum(xs)), float(sum(ys))
    sxx = float(sum(x * x for x in xs))
    sxy = float(sum(x * y for x, y in zip(xs, ys)))
    den = n * sxx - sx * sx
    if den == 0.0:
        return sy / n, 0.0
    b = (n * sxy - sx * sy) / den
    return (sy - b * sx) / n, b


class LatencyModel:
    """Profiled latencies of one micro-batch for m = 1..B; beyond B the line through the upper half of the profile."""

    def __init__(self, ms, ts):
        self.table = dict(zip(ms, ts))
        top = max(ms)
        hi = [(m, t) for m, t in zip(ms, ts) if 2 * m >= top]
        self.a, self.b = fit_line([m for m, _ in hi], [t for _, t in hi])

    def __call__(self, m, l=1):
        one = self.table[m] if m in self.table else self.a + self.b * m
        return l * one

    def as_table(self, max_m):
        """[0, T(1), ..., T(max_m)] for cephalo_plan_compute."""
        return [0.0] + [self(m) for m in range(1, max_m + 1)]


class MemoryModel:
    def __init__(self, ms, mem):
        self.a, self.b = fit_line(ms, mem)

    def __call__(self, m):
        return self.a + self.b * m


def measure_layer(desc, ms, iters=5, warmup=2):
    """Forward and backward time (ms) of one micro-batch of each size in `ms`, HIP events on the launch stream, and the
    compute memory (save + scratch bytes) the library needs for it."""
    import torch
    from . import binding as C
    P = C.cephalo_layer_param_count(desc)
    bf16 = desc.dtype == C.BF16
    flat = torch.randn(P, device="cuda") * 0.02
    if bf16:
        low = torch.empty(P, dtype=torch.bfloat16, device="cuda")
        C.cephalo_cast_bf16(low, flat)
        flat = low
    G = torch.zeros(P, device="cuda")
    out = []
    for m in ms:
        x = torch.randn(m, desc.seq, desc.hidden, device="cuda")
        dy = torch.randn(m, desc.seq, desc.hidden, device="cuda")
        y, dx = torch.empty_like(x), torch.empty_like(x)
        save_b, scr_b = C.cephalo_layer_workspace_bytes(desc, m)
        save = torch.empty(save_b, dtype=torch.uint8, device="cuda")
        scratch = torch.empty(scr_b, dtype=torch.uint8, device="cuda")

        def fwd():
            C.cephalo_layer_fwd(desc, flat, x, y, m, save, scratch)

        def bwd():
            C.cephalo_layer_bwd(desc, flat, x, dy, dx, m, save, G, 1.0, 1, scratch)

        times = []
        for fn in (fwd, bwd):
            for _ in range(warmup):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(iters):
                fn()
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1) / iters)
        out.append({"m": m, "t_fwd_ms": times[0], "t_bwd_ms": times[1], "compute_bytes": save_b + scr_b})
        del x, dy, y, dx, save, scratch
    return out


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="c5")
    ap.add_argument("--max-m", type=int, default=8)
    ap.add_argument("--check", type=int, nargs="*", default=[12, 16], help="held-out micro-batch sizes to test the models on")
    args = ap.parse_args(argv)
    import os
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    from workloads import CONFIGS
    from . import binding as C
    cfg = CONFIGS[args.workload]
    desc = C.desc_from_config(cfg)
    ms = list(range(1, args.max_m + 1))
    prof = measure_layer(desc, ms)
    tf = LatencyModel(ms, [p["t_fwd_ms"] for p in prof])
    tb = LatencyModel(ms, [p["t_bwd_ms"] for p in prof])
    mem = MemoryModel(ms, [p["compute_bytes"] for p in prof])
    held = measure_layer(desc, args.check) if args.check else []
    errs = []
    for p in held:
        errs.append({"m": p["m"],
                     "t_fwd_rel_err": abs(tf(p["m"]) - p["t_fwd_ms"]) / p["t_fwd_ms"],
                     "t_bwd_rel_err": abs(tb(p["m"]) - p["t_bwd_ms"]) / p["t_bwd_ms"],
                     "mem_rel_err": abs(mem(p["m"]) - p["compute_bytes"]) / p["compute_bytes"]})
    print(json.dumps({"workload": cfg.name, "profile": prof, "fwd_line_ms": [tf.a, tf.b], "bwd_line_ms": [tb.a, tb.b],
                      "memory_line_bytes": [mem.a, mem.b], "state_bytes_per_layer": 16 * C.cephalo_layer_param_count(desc),
                      "held_out": held, "held_out_errors": errs}))


if __name__ == "__main__":
    main()
