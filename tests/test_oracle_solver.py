"""Pins for the oracle's Solver choice (CPU only): a hand-worked table, numpy's interp as the
interpolation routine, and properties that follow from Eq. 4's cost per produced token."""
import json
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_worked_case(oracle):
    case = json.load(open(os.path.join(GOLDEN, "solver_hand_case.json")))
    for c in case["cases"]:
        best, speedup, cost, _ = oracle.solver_pick(case["points"], c["active_batch"], c["draft_us_fixed"],
                                                    c["draft_us_per_seq"])
        assert best == c["best_k"], c
        assert speedup == pytest.approx(c["speedup"], rel=1e-6) and cost == pytest.approx(c["cost"], rel=1e-6)


def _random_table(rng, Bs, ks):
    pts = []
    for B in Bs:
        for k in ks:
            t = (50 + 2.0 * B) * (1 + 0.05 * k) * rng.uniform(0.9, 1.1)
            e = 1.0 if k == 0 else 1 + (1 - 0.6 ** k) / 0.4 * 0.6 * rng.uniform(0.9, 1.1)
            pts.append((B, k, t, e))
    rng.shuffle(pts)
    return pts


def test_against_numpy_interp_and_argmin(oracle):
    rng = np.random.default_rng(0)
    Bs, ks = [16, 64, 256, 1024], [0, 1, 2, 4, 8]
    for trial in range(50):
        pts = _random_table(rng, Bs, ks)
        b = float(rng.choice([8, 16, 40, 64, 100, 256, 700, 1024, 5000]))
        fixed, per_seq = rng.uniform(0, 30), rng.uniform(0, 0.3)
        cost = {}
        for k in ks:
            rows = sorted((B, t, e) for (B, kk, t, e) in pts if kk == k)
            xs = [r[0] for r in rows]
            t = np.interp(b, xs, [r[1] for r in rows])
            e = np.interp(b, xs, [r[2] for r in rows])
            cost[k] = (k * (fixed + per_seq * b) + t) / e
        want = min(ks, key=lambda k: (cost[k], k))
        best, speedup, c, all_cost = oracle.solver_pick(pts, b, fixed, per_seq)
        assert best == want and c == pytest.approx(cost[want], rel=1e-12)
        assert speedup == pytest.approx(cost[0] / cost[want], rel=1e-12)
        assert all(all_cost[k] == pytest.approx(cost[k], rel=1e-12) for k in ks)


def test_properties_of_the_cost_model(oracle):
    rng = np.random.default_rng(1)
    pts = _random_table(rng, [32, 128, 512], [0, 2, 4, 8])
    base = oracle.solver_pick(pts, 200, 4.0, 0.02)
    # the unit of time does not matter
    scaled = oracle.solver_pick([(B, k, 7 * t, e) for (B, k, t, e) in pts], 200, 28.0, 0.14)
    assert scaled[0] == base[0] and scaled[1] == pytest.approx(base[1], rel=1e-12)
    # drafts that are never accepted (one token per step whatever k): speculation cannot pay
    assert oracle.solver_pick([(B, k, t, 1.0) for (B, k, t, e) in pts], 200, 4.0, 0.02)[0] == 0
    # a free drafter and a verify step as cheap as a decode step: the k that emits the most wins
    flat = [(B, k, 100.0, e) for (B, k, t, e) in pts]
    emits = {k: max(e for (B, kk, t, e) in pts if kk == k) for k in (0, 2, 4, 8)}
    same_e = [(B, k, t, emits[k]) for (B, k, t, e) in flat]
    assert oracle.solver_pick(same_e, 200, 0.0, 0.0)[0] == max(emits, key=emits.get)
    # a dearer drafter never raises the chosen draft length
    ks = [oracle.solver_pick(pts, 200, f, 0.02)[0] for f in (0, 5, 20, 80, 320, 5000)]
    assert ks == sorted(ks, reverse=True) and ks[-1] == 0
    # the speedup of the choice is never below 1 (k = 0 is always a candidate)
    for b in (1, 32, 77, 512, 9999):
        assert oracle.solver_pick(pts, b, 4.0, 0.02)[1] >= 1.0


def test_needs_the_plain_decoding_baseline(oracle):
    with pytest.raises(ValueError):
        oracle.solver_pick([(64, 2, 100.0, 1.5)], 64, 0.0, 0.0)
