"""Host-side planners (no GPU): oracle pins, and the library against the oracle."""
import itertools

import numpy as np
import pytest

from oracle import switch_planner_oracle as po
from paper_2602_12151_amd import binding, workloads as wl


# ------------------------------------------------------------------ capacity normalisation (section 4.2)
def test_the_papers_80_and_50_give_400_5_and_8():
    """Section 4.2's example: 80 type-1 and 50 type-2 requests per unit time -> common capacity 400,
    a type-1 request consumes 5 units, a type-2 request 8."""
    assert po.capacity_normalise([80, 50]) == (400, [5, 8])
    assert binding.capacity_normalise([80, 50]) == (400, [5, 8])


def test_normalise_skips_types_the_replica_cannot_serve_and_rejects_overflow():
    assert binding.capacity_normalise([6, 0, 4]) == (12, [2, 0, 3]) == po.capacity_normalise([6, 0, 4])
    with pytest.raises(binding.OserveError):
        binding.capacity_normalise([2**40 + 1, 2**40 - 1, 2**39 + 7])
    with pytest.raises(binding.OserveError):
        binding.capacity_normalise([3, -1])


# ------------------------------------------------------------------ workload assignment (section 4.2)
def test_assignment_closed_forms():
    # one replica, one type: min(arrivals, capacity, edge)
    for lam, n, e, want in [(30, 80, None, 30), (100, 80, None, 80), (100, 80, [[25.0]], 25)]:
        for fn in (po.assign_workload, binding.assign_workload):
            total, _ = fn([lam], [[n]], e)
            assert abs(total - want) < 1e-9
    # the 80 / 50 replica with 40 type-1 and 100 type-2 arrivals: 5 x1 + 8 x2 <= 400 -> x1 = 40, x2 = 25
    for fn in (po.assign_workload, binding.assign_workload):
        total, x = fn([40, 100], [[80, 50]])
        assert abs(total - 65.0) < 1e-9 and np.allclose(x, [[40.0, 25.0]])
    # two replicas that each serve one type twice as fast: the optimum specialises them
    for fn in (po.assign_workload, binding.assign_workload):
        total, x = fn([1000, 1000], [[100, 50], [50, 100]])
        assert abs(total - 200.0) < 1e-9 and np.allclose(x, [[100.0, 0.0], [0.0, 100.0]])


def feasible(x, lam, n, e, tol=1e-7):
    x = np.asarray(x)
    if (x < -tol).any() or (x.sum(axis=0) > np.asarray(lam) + tol).any():
        return False
    for k in range(n.shape[0]):
        share = sum(x[k, j] / n[k, j] for j in range(n.shape[1]) if n[k, j] > 0)
        if share > 1 + tol or any(x[k, j] > tol for j in range(n.shape[1]) if n[k, j] == 0):
            return False
    return e is None or (x <= np.asarray(e) + tol).all()


def test_oracle_assignment_against_integer_grid_search():
    """Tiny instances: the LP optimum is at least the best integer point and less than one request per
    variable above it."""
    rng = wl.CounterRng(5)
    for trial in range(6):
        n = rng.integers(1, 6, 4).reshape(2, 2).astype(np.int64)
        lam = rng.integers(1, 7, 2).astype(float)
        best = 0
        for pt in itertools.product(range(7), repeat=4):
            x = np.array(pt, dtype=float).reshape(2, 2)
            if feasible(x, lam, n, None, tol=1e-12):
                best = max(best, int(x.sum()))
        total, x = po.assign_workload(lam, n)
        assert feasible(x, lam, n, None)
        assert best - 1e-9 <= total < best + 4


@pytest.mark.parametrize("seed", range(8))
def test_library_assignment_matches_the_oracle(seed):
    rng = wl.CounterRng(100 + seed)
    K, J = int(rng.integers(1, 6, 1)[0]), int(rng.integers(1, 4, 1)[0])
    n = rng.integers(0, 120, K * J).reshape(K, J).astype(np.int64)
    lam = rng.integers(0, 300, J).astype(float)
    e = rng.integers(0, 150, K * J).reshape(K, J).astype(float) if seed % 2 else None
    want, _ = po.assign_workload(lam, n, e)
    total, x = binding.assign_workload(lam, n, e)
    assert abs(total - want) <= 1e-7 * max(1.0, want)
    assert feasible(x, lam, n, e) and abs(x.sum() - total) < 1e-9


# ------------------------------------------------------------------ greedy switch plan (section 5.2, appendix)
def test_hand_worked_switch_plans():
    machines = [0, 0, 1, 1]                       # devices 0,1 on machine 0; 2,3 on machine 1
    # shard 0 held by {0, 2}, needed by {1, 3}: each target has a holder on its own machine
    for fn in (po.greedy_switch_plan, binding.switch_plan):
        plan, _ = fn(machines, [[0, 2]], [[1, 3]], [[10, 10]])
        assert plan == [[0, 2]]
    # a target that already holds the shard needs nothing
    for fn in (po.greedy_switch_plan, binding.switch_plan):
        plan, _ = fn(machines, [[0, 1]], [[1, 2]], [[5, 5]])
        assert plan == [[-1, 0]]
    # two shards held by {0, 1}, both needed by device 2 (other machine): the second goes to the
    # holder whose counter towards device 2 is still zero
    for fn in (po.greedy_switch_plan, binding.switch_plan):
        plan, load = fn(machines, [[0, 1], [0, 1]], [[2], [2]], [[7], [3]])
        assert plan == [[0], [1]]
        got = load if isinstance(load, dict) else {(s, t): int(load[s, t]) for s in range(4) for t in range(4) if load[s, t]}
        assert got == {(0, 2): 7, (1, 2): 3}


@pytest.mark.parametrize("seed", range(6))
def test_library_switch_plan_equals_the_oracle_and_obeys_the_rules(seed):
    rng = wl.CounterRng(300 + seed)
    D, S = 16, 40
    machines = [d // 8 for d in range(D)]
    sources, targets, volumes = [], [], []
    for m in range(S):
        ns, nt = int(rng.integers(1, 4, 1)[0]), int(rng.integers(1, 5, 1)[0])
        sources.append(sorted(set(int(v) for v in rng.integers(0, D - 1, ns))))
        targets.append(sorted(set(int(v) for v in rng.integers(0, D - 1, nt))))
        volumes.append([int(v) for v in rng.integers(1, 100, len(targets[-1]))])
    plan, load = binding.switch_plan(machines, sources, targets, volumes)
    want, C = po.greedy_switch_plan(machines, sources, targets, volumes)
    assert plan == want
    assert {(s, t): int(load[s, t]) for s in range(D) for t in range(D) if load[s, t]} == C
    for m in range(S):
        for i, t in enumerate(targets[m]):
            s = plan[m][i]
            if t in sources[m]:
                assert s == -1
            else:
                assert s in sources[m]
                if any(machines[h] == machines[t] for h in sources[m]):
                    assert machines[s] == machines[t]          # intra-machine sources first


def test_switch_plan_errors():
    with pytest.raises(binding.OserveError):
        binding.switch_plan([0, 0], [[]], [[1]], [[4]])          # needed, nobody holds it
    with pytest.raises(binding.OserveError):
        binding.switch_plan([0, 0], [[0]], [[5]], [[4]])         # device out of range
