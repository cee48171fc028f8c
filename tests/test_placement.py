"""Table placement (Section 3.1, "Embedding PS"): the oracle's packing against brute force,
and the library's host-side planner against the oracle (no GPU: host logic only)."""
import itertools

import numpy as np
import pytest

from oracle import placement as oplace
from paper_2003_03477_amd import binding


def _brute_force_makespan(costs, m):
    best = float("inf")
    for assign in itertools.product(range(m), repeat=len(costs)):
        load = [0.0] * m
        for c, p in zip(costs, assign):
            load[p] += c
        best = min(best, max(load))
    return best


@pytest.mark.parametrize("seed", range(6))
def test_oracle_packing_within_the_lpt_bound_of_the_optimum(seed):
    rng = np.random.default_rng(seed)
    n, m = int(rng.integers(4, 9)), int(rng.integers(2, 4))
    rows = [int(v) for v in rng.integers(10, 1000, n)]
    cost = [float(v) for v in rng.uniform(0.1, 10.0, n)]
    shards, load = oplace.plan_placement(rows, cost, m)
    assert sorted(s[0] for s in shards) == list(range(n))          # every table placed once
    assert abs(sum(load) - sum(cost)) < 1e-9
    opt = _brute_force_makespan(cost, m)
    assert max(load) <= (4.0 / 3.0 - 1.0 / (3.0 * m)) * opt + 1e-12
    assert max(load) >= opt - 1e-12


def test_oracle_partitions_large_tables_by_rows():
    shards, load = oplace.plan_placement([1000, 10, 2501], [4.0, 1.0, 10.0], 3, max_rows_per_shard=1000)
    by_table = {}
    for t, first, n, c, ps in shards:
        by_table.setdefault(t, []).append((first, n, c))
    assert by_table[0] == [(0, 1000, 4.0)] and by_table[1] == [(0, 10, 1.0)]
    parts = by_table[2]
    assert [p[0] for p in parts] == [0, 834, 1668] and sum(p[1] for p in parts) == 2501
    assert abs(sum(p[2] for p in parts) - 10.0) < 1e-12
    assert all(0 <= s[4] < 3 for s in shards)


@pytest.mark.parametrize("seed", range(5))
def test_library_planner_equals_the_oracle(seed):
    rng = np.random.default_rng(100 + seed)
    n, m = int(rng.integers(3, 30)), int(rng.integers(1, 9))
    rows = [int(v) for v in np.exp(rng.uniform(np.log(1e3), np.log(4e7), n))]
    cost = [float(v) for v in rng.uniform(0.5, 20.0, n)]
    limit = int(rng.choice([0, 1_000_000, 5_000_000]))
    got, got_load = binding.ss_plan_placement(rows, cost, m, limit)
    want, want_load = oplace.plan_placement(rows, cost, m, limit)
    assert [(g[0], g[1], g[2], g[4]) for g in got] == [(w[0], w[1], w[2], w[4]) for w in want]
    np.testing.assert_allclose([g[3] for g in got], [w[3] for w in want], rtol=1e-14)
    np.testing.assert_allclose(got_load, want_load, rtol=1e-12)


def test_library_planner_rejects_bad_arguments():
    lib = binding.load()
    assert lib.ss_plan_placement(0, None, None, 1, 0, None, 0, None, None) == -1
