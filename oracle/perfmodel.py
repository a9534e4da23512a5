"""Performance models of Sec. 3.3: compute latency and compute memory as functions of the micro-batch size.

Latency (Sec. 3.3 "Compute Latency Model"): the profiled values are used as they are for the profiled micro-batch
sizes (they capture the sub-linear start), and larger sizes are extrapolated linearly; l micro-batches cost l times
one micro-batch.  The paper does not say which points fix the line: here, the least-squares line through the upper
half of the profiled sizes (m >= B/2, where the device is saturated).  Memory (Sec. 3.3 "Memory Utilization Model"):
one least-squares line through all profiled sizes; M_state = 16 bytes per parameter.  Test infrastructure.
"""
import numpy as np


def least_squares_line(xs, ys):
    """Intercept and slope minimising sum (a + b x - y)^2."""
    A = np.stack([np.ones(len(xs)), np.asarray(xs, dtype=np.float64)], axis=1)
    (a, b), *_ = np.linalg.lstsq(A, np.asarray(ys, dtype=np.float64), rcond=None)
    return a, b


def latency_model(ms, ts):
    """Returns predict(m, l): profiled table inside the profiled range, line through the upper half beyond it."""
    ms = list(ms); ts = list(ts)
    table = dict(zip(ms, ts))
    top = max(ms)
    hi = [(m, t) for m, t in zip(ms, ts) if 2 * m >= top]
    a, b = least_squares_line([m for m, _ in hi], [t for _, t in hi])

    def predict(m, l=1):
        one = table[m] if m in table else a + b * m
        return l * one
    return predict


def memory_model(ms, mem):
    a, b = least_squares_line(ms, mem)
    return lambda m: a + b * m


def state_bytes(n_params):
    """4 (parameter) + 4 (gradient) + 8 (two Adam moments) bytes per parameter."""
    return 16 * n_params
