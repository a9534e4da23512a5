"""The profiler on the device: latency of a layer against micro-batch size, the models fitted to it, and a plan
computed from them (Sec. 3.3, 3.4, 4.1)."""
import dataclasses
import pytest

import paper_2411_01075_amd as C
from paper_2411_01075_amd import profiler as prof
from workloads import CONFIGS

pytestmark = pytest.mark.gpu


def test_profile_fit_and_plan():
    cfg = dataclasses.replace(CONFIGS["c2"], hidden=512, heads=8, mlp=2048, seq=256)
    desc = C.desc_from_config(cfg)
    ms = [1, 2, 3, 4, 5, 6]
    p = prof.measure_layer(desc, ms, iters=5, warmup=2)
    tf = prof.LatencyModel(ms, [q["t_fwd_ms"] for q in p])
    tb = prof.LatencyModel(ms, [q["t_bwd_ms"] for q in p])
    mem = prof.MemoryModel(ms, [q["compute_bytes"] for q in p])
    assert all(q["t_fwd_ms"] > 0 and q["t_bwd_ms"] > q["t_fwd_ms"] for q in p)        # backward is the larger part
    assert p[-1]["t_fwd_ms"] > p[0]["t_fwd_ms"] and tf.b > 0 and tb.b > 0
    # compute memory: linear in m and independent of the number of micro-batches (the query has no l)
    held = prof.measure_layer(desc, [8], iters=3, warmup=1)[0]
    assert abs(mem(8) - held["compute_bytes"]) / held["compute_bytes"] < 0.25
    # the latency model within 35 % on a held-out size (a small, launch-bound layer: the timings are noisy)
    assert abs(tf(8) - held["t_fwd_ms"]) / held["t_fwd_ms"] < 0.35
    # two such GPUs, one with half the memory: the plan covers the batch and respects the capacities
    P = C.cephalo_layer_param_count(desc)
    cl = C.cluster_model(0.05, 0.05, mem.a, mem.b, 16.0 * P)
    big = (tf.as_table(16), tb.as_table(16), mem(16) + 16.0 * P)
    small = (tf.as_table(16), tb.as_table(16), mem(4) + 1.0)
    m, l, lat = C.cephalo_plan_compute([big, small], 16, cl)
    assert sum(a * b for a, b in zip(m, l)) == 16 and m[1] <= 4 and lat > 0
    r = C.cephalo_plan_state([big, small], m, cl)
    assert abs(sum(r) - 1) < 1e-12 and r[0] > r[1]
