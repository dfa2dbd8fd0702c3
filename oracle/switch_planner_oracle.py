"""Plain Python statement of the host-side planners.  TEST INFRASTRUCTURE ONLY.

* greedy_switch_plan: the steps of the appendix "Greedy Algorithm for Ad Hoc Model
  Switching" (paper section 5.2) in its notation: counters C[s -> t] per device pair, shards in
  order, for each target that does not hold the shard the intra-machine holders if any, else the
  others, the one with the smallest C[s -> t] (first listed among equals), then C grows by V.
* capacity_normalise: section 4.2's least common multiple M_k and per-request units M_k / n_kj.
* assign_workload: section 4.2's constraints C1-C3 written out as a linear program and handed to
  scipy's linprog (the library primitive); the optimum value is what is compared.

Pins (tests/test_switch_planner.py): the paper's own numbers 80 and 50 -> 400, 5 and 8; closed
forms of one- and two-type single-replica assignments; an integer grid search on tiny instances;
hand-worked switch plans.
"""
from __future__ import annotations

import math

import numpy as np


def greedy_switch_plan(device_machine, sources, targets, volumes):
    """sources[m], targets[m]: lists of devices; volumes[m][i]: volume of (m, targets[m][i]).
    Returns (plan: list of lists of chosen sources or -1, C: dict (s, t) -> volume)."""
    C = {}
    plan = []
    for m, (S_m, T_m) in enumerate(zip(sources, targets)):
        row = []
        for i, t in enumerate(T_m):
            if t in S_m:
                row.append(-1)
                continue
            intra = [s for s in S_m if device_machine[s] == device_machine[t]]
            inter = [s for s in S_m if device_machine[s] != device_machine[t]]
            cand = intra if intra else inter
            if not cand:
                raise ValueError("a needed shard has no holder")
            s_star = min(cand, key=lambda s: C.get((s, t), 0))      # min() keeps the first of equals
            C[(s_star, t)] = C.get((s_star, t), 0) + volumes[m][i]
            row.append(s_star)
        plan.append(row)
    return plan, C


def capacity_normalise(n_row):
    M = 1
    for n in n_row:
        if n > 0:
            M = M * n // math.gcd(M, n)
    return M, [M // n if n > 0 else 0 for n in n_row]


def assign_workload(arrivals, node_capacity, edge_capacity=None):
    """Maximum of sum x subject to C1-C3; returns (total, x [K, J])."""
    from scipy.optimize import linprog
    n = np.asarray(node_capacity, dtype=np.int64)
    K, J = n.shape
    A, b = [], []
    for j in range(J):                         # C1
        row = np.zeros(K * J); row[[k * J + j for k in range(K)]] = 1.0
        A.append(row); b.append(float(arrivals[j]))
    for k in range(K):                         # C3, in units of M_k
        M, units = capacity_normalise([int(v) for v in n[k]])
        row = np.zeros(K * J)
        for j in range(J):
            row[k * J + j] = float(units[j])
        A.append(row); b.append(float(M))
    bounds = []
    for k in range(K):
        for j in range(J):
            if n[k, j] == 0:
                bounds.append((0.0, 0.0))
            elif edge_capacity is not None and np.isfinite(edge_capacity[k][j]):
                bounds.append((0.0, float(edge_capacity[k][j])))      # C2
            else:
                bounds.append((0.0, None))
    res = linprog(-np.ones(K * J), A_ub=np.asarray(A), b_ub=np.asarray(b), bounds=bounds, method="highs")
    if res.status != 0:
        raise RuntimeError(res.message)
    return -res.fun, res.x.reshape(K, J)
