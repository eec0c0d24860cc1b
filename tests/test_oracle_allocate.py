"""Pins for oracle/allocate.py: Eq. (1)-(4), brute force on tiny inputs,
hand-worked cases, limiting behaviour.  CPU only."""
import itertools
import json
import os

import numpy as np
import pytest

from oracle import allocate as al

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def const_curve(speed, mbs, pts=(1, 2, 4, 8)):
    bs = [b for b in pts if b <= mbs] + ([mbs] if mbs not in pts else [])
    return (bs, [b / speed for b in bs], mbs)


def test_hand_cases_from_fixture():
    with open(os.path.join(GOLDEN, "alloc_hand_cases.json")) as f:
        gold = json.load(f)
    for case in gold["cases"]:
        curves = [const_curve(s, 64, (1, 2, 4, 8, 16, 32, 64)) for s in case["speeds"]]
        out = al.allocate(1, case["gbs"], curves)
        assert out["gmbs"] == case["gmbs"]
        assert abs(out["T"] - case["T"]) < 1e-12
        t = [g / s for g, s in zip(out["gmbs"], case["speeds"])]
        if case["equal_time"]:
            assert max(t) - min(t) < 1e-12
            assert abs(al.under_utilization(t, case["speeds"])) < 1e-9


def test_dipping_and_negative_splines_from_fixture():
    # pins the running maximum of the step-time curve, the speed floor and `find`
    with open(os.path.join(GOLDEN, "alloc_dip_cases.json")) as f:
        gold = json.load(f)
    for case in gold["cases"]:
        curve = (case["batches"], case["times"], case["mbs"])
        sp = al.speed_curve(*curve)
        np.testing.assert_allclose(sp[1:], case["speed"], rtol=1e-12)
        tm = al.time_curve(sp)
        assert tm[0] == 0.0
        np.testing.assert_allclose(tm[1:], case["time"], rtol=1e-12)
        assert np.all(np.diff(tm) >= 0)
        for t, b in case["find"]:
            assert al.find(tm, t) == b, (case["name"], t)
        a = case["alloc"]
        out = al.allocate(a["stage"], a["gbs"], [curve], a["time_communication"])
        assert out["b"] == a["b"] and out["gas"] == a["gas"] and out["lbs"] == a["lbs"] and out["gmbs"] == a["gmbs"]
        assert abs(out["t"] - a["t"]) < 1e-12 and abs(out["wall"] - a["wall"]) < 1e-12


def test_find_is_the_largest_batch_within_t():
    tm = np.array([0.0, 1.0, 1.0, 2.5, 2.5, 7.0])
    assert [al.find(tm, t) for t in (0.5, 1.0, 2.4, 2.5, 6.9, 7.0, 1e9)] == [0, 2, 2, 4, 4, 5, 5]
    assert al.find(np.zeros(1), 3.0) == 0       # a device that cannot run one sample


def compositions(total, n):
    for c in itertools.combinations(range(total + n - 1), n - 1):
        yield [b - a - 1 for a, b in zip((-1,) + c, c + (total + n - 1,))]


def test_stage01_matches_brute_force_optimum():
    rng = np.random.default_rng(0)
    for _ in range(60):
        n = int(rng.integers(2, 5))
        gbs = int(rng.integers(1, 21))
        speeds = [float(rng.integers(1, 9)) / 2 for _ in range(n)]
        out = al.allocate(0, gbs, [const_curve(s, 32, (1, 2, 4, 8, 16, 32)) for s in speeds])
        assert sum(out["gmbs"]) == gbs and min(out["gmbs"]) >= 0
        best_T, best_U = np.inf, np.inf
        for B in compositions(gbs, n):
            t = [b / s for b, s in zip(B, speeds)]
            best_T = min(best_T, al.iteration_time(t))
            best_U = min(best_U, al.under_utilization(t, speeds))
        t = [g / s for g, s in zip(out["gmbs"], speeds)]
        assert abs(al.iteration_time(t) - best_T) < 1e-12      # Eq. 1 minimal
        assert abs(al.under_utilization(t, speeds) - best_U) < 1e-9  # Eq. 4 minimal
        # Eq. 4 == T * sum(p) - gbs under constant speeds
        assert abs(al.under_utilization(t, speeds) - (max(t) * sum(speeds) - gbs)) < 1e-9
        assert abs(out["T"] - max(t)) < 1e-12


def test_stage01_micro_batches_and_accumulation():
    # speed saturates: 1,2,3,3.9,4,4,... -> peak range (>=95% of 4) starts at b=4
    bs = list(range(1, 9))
    sp = [1.0, 2.0, 3.0, 3.9, 4.0, 4.0, 4.0, 4.0]
    fast = (bs, [b / s for b, s in zip(bs, sp)], 8)
    slow = (bs, [b / (s / 2) for b, s in zip(bs, sp)], 6)   # half speed, less memory
    out = al.allocate(1, 30, [fast, slow])
    assert out["gmbs"] == [20, 10]
    assert out["b"] == [8, 6]                 # largest batch of the peak range, capped by mbs
    assert out["gas"] == [3, 2] and out["lbs"] == [4, 4]
    for i in range(2):
        assert (out["gas"][i] - 1) * out["b"][i] + out["lbs"][i] == out["gmbs"][i]
        assert 1 <= out["lbs"][i] <= out["b"][i]
    # Eq. 1 on the peak speeds (what the split was made for) against Eq. 1 on the steps that will really run:
    # fast: two steps of 8 at speed 4 and one of 4 at speed 3.9; slow: one of 6 at speed 2 and one of 4 at 1.95
    assert abs(out["T"] - 5.0) < 1e-12
    assert abs(out["T_steps"] - max(2 * 8 / 4.0 + 4 / 3.9, 6 / 2.0 + 4 / 1.95)) < 1e-12
    # a device that gets nothing
    out = al.allocate(1, 1, [fast, slow])
    assert out["gmbs"] == [1, 0] and out["b"] == [1, 0] and out["gas"] == [1, 0] and out["lbs"] == [1, 0]


def test_speed_curve_interpolates_and_clamps():
    s = al.speed_curve([1, 2, 4, 8], [1.0, 1.25, 2.0, 3.2], 10)
    np.testing.assert_allclose(s[[1, 2, 4, 8]], [1.0, 1.6, 2.0, 2.5], rtol=1e-12)
    assert s[9] == s[8] == s[10]             # clamped outside the sampled range
    assert np.all(s[1:] > 0)
    # duplicates are averaged as speeds
    s2 = al.speed_curve([2, 2], [1.0, 2.0], 3)
    np.testing.assert_allclose(s2[1:], 1.5)
    # scipy opinion on the interior
    from scipy.interpolate import CubicSpline
    ref = CubicSpline([1, 2, 4, 8], [1.0, 1.6, 2.0, 2.5], bc_type="natural")(np.arange(1, 9))
    np.testing.assert_allclose(s[1:9], ref, rtol=1e-10)


def _tm(curve):
    return al.time_curve(al.speed_curve(*curve))


def brute_stage23(gbs, curves, tc):
    tms = [_tm(c) for c in curves]
    best = np.inf
    for B in itertools.product(*[range(0, c[2] + 1) for c in curves]):
        if sum(B) == 0:
            continue
        t = max(tms[i][b] for i, b in enumerate(B))
        best = min(best, (t + tc) * -(-gbs // sum(B)))
    return best


def test_stage23_matches_brute_force_wall_time():
    rng = np.random.default_rng(1)
    for _ in range(40):
        n = int(rng.integers(2, 4))
        curves = []
        for _i in range(n):
            mbs = int(rng.integers(1, 7))
            bs = sorted(set([1, mbs] + [int(b) for b in rng.integers(1, mbs + 1, 2)]))
            sat = float(rng.uniform(1, 6))
            half = float(rng.uniform(0.5, 4))
            curves.append((bs, [b / (sat * b / (b + half)) for b in bs], mbs))
        gbs = int(rng.integers(1, 40))
        tc = float(rng.choice([0.0, 0.3, 5.0]))
        out = al.allocate(2, gbs, curves, tc)
        assert abs(out["wall"] - brute_stage23(gbs, curves, tc)) < 1e-9
        assert sum(out["gmbs"]) == gbs
        for i, c in enumerate(curves):
            assert 0 <= out["lbs"][i] <= out["b"][i] <= c[2]
            assert _tm(c)[out["b"][i]] <= out["t"] + 1e-15
        assert out["gas"] == -(-gbs // sum(out["b"]))


def test_stage23_limits():
    curves = [const_curve(2.0, 8), const_curve(1.0, 4)]
    # communication dominates -> as few accumulation steps as possible -> max batches
    out = al.allocate(3, 48, curves, time_communication=1e6)
    assert out["b"] == [8, 4] and out["gas"] == 4
    # no communication, constant speeds: any t with balanced load has the same
    # per-sample rate; wall must equal gbs / sum(speed) when it divides
    out = al.allocate(3, 48, curves, time_communication=0.0)
    assert abs(out["wall"] - 48 / 3.0) < 1e-12
    # fewest steps first, then the smallest t that still reaches that count
    out = al.allocate(2, 50, curves, time_communication=1e6)
    assert out["gas"] == 5 and out["b"] == [7, 3] and out["lbs"] == [7, 3]
    # last step carries the remainder: 26 = 2 * 9 + 8, eight samples handed out
    # one by one to the device that finishes earliest (ties to the lower index)
    out = al.allocate(2, 26, curves, time_communication=1e6)
    assert out["gas"] == 3 and out["b"] == [6, 3] and out["lbs"] == [6, 2]
    assert out["gmbs"] == [18, 8]


def test_invalid_stage():
    with pytest.raises(ValueError):
        al.allocate(5, 4, [const_curve(1.0, 4)])
