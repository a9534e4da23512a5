"""The optimizer's problem by exhaustive search (Sec. 3.4 "Optimization Formulation", Eqs. 2-3, constraints I-III) and
the training-state partition as a linear programme -- only for tiny clusters; test infrastructure.

For every assignment of (m_i, l_i) to the N GPUs with sum_i m_i l_i = B:
  layer latency = max_i [ max(l_i T_f^i(m_i), AG') + max(l_i T_b^i(m_i), AG' + RS') ]
  (AG', RS' uneven if GPU i cannot hold its compute memory plus an even share of the training state),
  feasible iff M(m_i) <= cap_i for every i (II) and M_state + sum_i M(m_i) <= sum_i cap_i (III);
the optimum is the least latency over the feasible assignments.  M(m) = mem_base + mem_per_sample * m (Sec. 3.3).
Readings of the garbled notation: N is the number of GPUs, B the global batch size.
"""
import itertools
import numpy as np


def table_latency(table, m):
    """Profiled latencies for m = 1..len(table)-1, extended linearly through the last two points (Sec. 3.3)."""
    top = len(table) - 1
    if m <= top:
        return table[m]
    slope = table[top] - table[top - 1] if top >= 2 else table[1]
    return table[top] + slope * (m - top)


def gpu_latency(tf, tb, cap, m, l, mem_base, mem_per_sample, state_even, ag, rs, ag_u, rs_u):
    uneven = mem_base + mem_per_sample * m + state_even > cap
    a, r = (ag_u, rs_u) if uneven else (ag, rs)
    return max(l * table_latency(tf, m), a) + max(l * table_latency(tb, m), a + r)


def brute_force_plan(gpus, B, ag, rs, ag_u, rs_u, mem_base, mem_per_sample, state_bytes):
    """gpus: list of (t_fwd table, t_bwd table, mem_cap).  Returns (best latency, list of optimal assignments)."""
    n = len(gpus)
    cap_sum = sum(g[2] for g in gpus)
    options = [(m, l) for m in range(1, B + 1) for l in range(1, B // m + 1)]
    best, arg = np.inf, []
    for combo in itertools.product(options, repeat=n):
        if sum(m * l for m, l in combo) != B:
            continue
        if any(mem_base + mem_per_sample * m > gpus[i][2] for i, (m, l) in enumerate(combo)):
            continue
        if state_bytes + sum(mem_base + mem_per_sample * m for m, l in combo) > cap_sum:
            continue
        t = max(gpu_latency(gpus[i][0], gpus[i][1], gpus[i][2], m, l, mem_base, mem_per_sample, state_bytes / n, ag, rs, ag_u, rs_u)
                for i, (m, l) in enumerate(combo))
        if t < best - 1e-12:
            best, arg = t, [combo]
        elif abs(t - best) <= 1e-12:
            arg.append(combo)
    return best, arg


def min_max_utilisation(used, cap, state_bytes):
    """Least possible value of max_i (used_i + s_i) / cap_i over s >= 0 with sum s = state_bytes, by linear programming
    (variables s_1..s_n, u; minimise u)."""
    from scipy.optimize import linprog
    n = len(used)
    c = np.zeros(n + 1); c[-1] = 1.0
    A_ub = np.zeros((n, n + 1)); b_ub = np.zeros(n)
    for i in range(n):
        A_ub[i, i] = 1.0 / cap[i]; A_ub[i, -1] = -1.0; b_ub[i] = -used[i] / cap[i]
    A_eq = np.ones((1, n + 1)); A_eq[0, -1] = 0.0
    res = linprog(c, A_ub=A_ub, b_ub=b_ub, A_eq=A_eq, b_eq=[state_bytes], bounds=[(0, None)] * n + [(None, None)])
    assert res.success
    return res.x[-1]


def max_even_units_bruteforce(targets, n_units, unit_len):
    """Sec. 4 "Uneven Parameter Sharding": the largest number of units that can be sharded evenly (every GPU the same
    whole share unit_len / N; unit_len must be a multiple of N here) when GPU i is to hold targets[i] elements in all
    (sum = n_units * unit_len).  Exhaustive: every way of cutting every unit into N non-negative whole parts whose
    column sums meet the targets is enumerated, and the even rows counted.  Tiny inputs only."""
    n = len(targets)
    assert unit_len % n == 0 and sum(targets) == n_units * unit_len
    even = tuple([unit_len // n] * n)

    def rows(left, parts):      # all ways to write `left` as `parts` ordered non-negative integers
        if parts == 1:
            yield (left,)
            return
        for first in range(left + 1):
            for rest in rows(left - first, parts - 1):
                yield (first,) + rest

    all_rows = list(rows(unit_len, n))
    best = -1
    for combo in itertools.product(all_rows, repeat=n_units):
        if all(sum(r[i] for r in combo) == targets[i] for i in range(n)):
            best = max(best, sum(1 for r in combo if r == even))
    return best
