"""respec_solver_pick (host code of the library, no GPU needed) against the oracle's Solver
choice: the hand-worked table, random profile tables, and the error paths."""
import json
import os

import numpy as np
import pytest

from paper_2510_26475_amd import binding, build

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module", autouse=True)
def _lib():
    if not os.path.exists(build.LIB_PATH):
        build.build()
    return binding.load()


def test_hand_worked_case():
    case = json.load(open(os.path.join(GOLDEN, "solver_hand_case.json")))
    for c in case["cases"]:
        best, speedup, cost = binding.respec_solver_pick(case["points"], c["active_batch"], c["draft_us_fixed"],
                                                         c["draft_us_per_seq"])
        assert best == c["best_k"]
        assert speedup == pytest.approx(c["speedup"], rel=1e-6) and cost == pytest.approx(c["cost"], rel=1e-6)


def test_random_tables_equal_the_oracle(oracle):
    rng = np.random.default_rng(42)
    for trial in range(200):
        Bs = sorted(rng.choice(np.arange(1, 2000), size=rng.integers(1, 6), replace=False).tolist())
        ks = [0] + sorted(rng.choice(np.arange(1, 12), size=rng.integers(0, 5), replace=False).tolist())
        pts = []
        for B in Bs:
            for k in ks:
                if k and rng.random() < 0.15 and len(Bs) > 1:
                    continue                       # a hole in the table
                t = (40 + rng.uniform(0.5, 3) * B) * (1 + 0.1 * k * rng.uniform(0, 1))
                e = 1.0 if k == 0 else rng.uniform(1.0, 1.0 + k)
                pts.append((B, k, t, e))
        pts = [pts[i] for i in rng.permutation(len(pts))]
        b = int(rng.integers(1, 3000))
        fixed, per_seq = float(rng.uniform(0, 50)), float(rng.uniform(0, 0.5))
        want = oracle.solver_pick(pts, b, fixed, per_seq)
        got = binding.respec_solver_pick(pts, b, fixed, per_seq)
        costs = sorted(want[3].values())
        if len(costs) > 1 and costs[1] - costs[0] < 1e-9 * costs[0]:
            continue                               # a tie up to rounding: either k is right
        assert got[0] == want[0], (trial, got, want[:3])
        assert got[1] == pytest.approx(want[1], rel=1e-12) and got[2] == pytest.approx(want[2], rel=1e-12)


def test_errors():
    with pytest.raises(binding.RespecError) as e:
        binding.respec_solver_pick([(64, 2, 100.0, 1.5)], 64, 0.0, 0.0)          # no k = 0 point
    assert e.value.status == 1
    for bad in ([], [(64, 0, -1.0, 1.0)], [(64, 0, 100.0, 0.0)], [(0, 0, 100.0, 1.0)], [(64, 0, float("nan"), 1.0)]):
        with pytest.raises(binding.RespecError):
            binding.respec_solver_pick(bad, 64, 0.0, 0.0)
    with pytest.raises(binding.RespecError):
        binding.respec_solver_pick([(64, 0, 100.0, 1.0)], 0, 0.0, 0.0)
    with pytest.raises(binding.RespecError):
        binding.respec_solver_pick([(64, 0, 100.0, 1.0)], 64, -1.0, 0.0)
