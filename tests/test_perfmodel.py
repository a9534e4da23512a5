"""The performance models of Sec. 3.3 (oracle and the profiler's own fit) against closed forms and against the
latencies and memory the paper plots for BERT-Large on four GPUs (tests/golden/paper_fig_latency_memory.txt)."""
import os
import numpy as np
import pytest

from oracle import perfmodel as om
from paper_2411_01075_amd import profiler as prof

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_fig_latency_memory.txt")


def load_gold():
    lat, mem, block = [], [], 0
    for line in open(GOLD):
        if line.startswith("# memory"):
            block = 1
        if line.startswith("#") or not line.strip():
            continue
        v = [float(t) for t in line.split()]
        (lat if block == 0 else mem).append(v)
    return np.array(lat), np.array(mem)


def test_line_fit_closed_forms():
    xs = [1, 2, 3, 5, 8]
    a, b = om.least_squares_line(xs, [3.0 + 0.25 * x for x in xs])           # points on a line: that line
    assert abs(a - 3.0) < 1e-12 and abs(b - 0.25) < 1e-12
    a, b = om.least_squares_line([2, 6], [1.0, 9.0])                         # two points: the line through them
    assert abs(a + 3.0) < 1e-12 and abs(b - 2.0) < 1e-12
    ys = [2.0, 2.9, 4.2, 6.1, 8.7]
    a0, b0 = om.least_squares_line(xs, ys)
    a1, b1 = om.least_squares_line(xs, [y + 10 for y in ys])                 # shifting y shifts the intercept only
    assert abs(a1 - a0 - 10) < 1e-9 and abs(b1 - b0) < 1e-12
    r = np.array(ys) - (a0 + b0 * np.array(xs))                              # normal equations: residuals orthogonal to 1 and x
    assert abs(r.sum()) < 1e-9 and abs((r * np.array(xs)).sum()) < 1e-9
    assert om.state_bytes(10) == 160


def test_models_predict_the_papers_held_out_points():
    """Profile m = 1..8 as the paper's profiler does (Sec. 4.1) and predict m = 9..16.  The paper reports a mean model
    error of 2.9 % and a maximum below 10 % (supplementary, model accuracy) for whole configurations; its own plotted
    points give the same picture: A6000 and P100 stay within 5 % (mean 2.8 %), L4 is at 5.2 % on average with its worst
    point (m = 16, where its curve bends upwards) at 10.6 %.  P40 has outliers inside the profiled range of the plot
    (m = 7) and beyond (m = 11) and is left out."""
    lat, mem = load_gold()
    ms = lat[:8, 0].astype(int).tolist()
    for col, name, bound_max, bound_mean in ((1, "A6000", 0.05, 0.03), (2, "L4", 0.12, 0.06), (3, "P100", 0.05, 0.03)):
        model = om.latency_model(ms, lat[:8, col].tolist())
        errs = [abs(model(int(m)) - t) / t for m, t in zip(lat[8:, 0], lat[8:, col])]
        assert max(errs) < bound_max and np.mean(errs) < bound_mean, (name, errs)
        assert model(3) == lat[2, col] and model(3, 4) == 4 * lat[2, col]     # inside the profile: the measured value; l micro-batches: l times
    mm = om.memory_model(mem[:8, 0].tolist(), mem[:8, 1].tolist())
    assert max(abs(mm(m) - v) / v for m, v in mem[8:]) < 0.005


def test_profiler_fit_equals_oracle_fit():
    lat, mem = load_gold()
    ms = lat[:8, 0].astype(int).tolist()
    rng = np.random.default_rng(0)
    for col in (1, 2, 3, 4):
        a = om.latency_model(ms, lat[:8, col].tolist())
        b = prof.LatencyModel(ms, lat[:8, col].tolist())
        for m in range(1, 33):
            assert abs(a(m) - b(m)) <= 1e-9 * abs(a(m))
        assert b.as_table(12)[5] == lat[4, col] and len(b.as_table(12)) == 13
    xs = list(range(1, 9)); ys = (rng.uniform(1, 2) * np.array(xs) + rng.normal(0, 0.1, 8)).tolist()
    assert np.allclose(om.least_squares_line(xs, ys), prof.fit_line(xs, ys), rtol=1e-10)
    assert abs(om.memory_model(xs, ys)(20) - prof.MemoryModel(xs, ys)(20)) < 1e-9
