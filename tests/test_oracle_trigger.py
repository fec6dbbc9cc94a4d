"""Pins for the oracle's Optimization Trigger (Section 3.3 "Optimization trigger": 5 % gain threshold,
10 % prediction-error threshold): hand-worked cases, brute force, edge cases."""
import math
import os

import numpy as np

from oracle import oracle as orc

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "trigger_cases.txt")


def test_hand_worked_cases():
    n = 0
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        sc, cur, obs, best, gain, rec, ad = [x.strip() for x in line.split("|")]
        scores = np.array([[float(x) for x in sc.split(",")]], dtype=np.float32)
        b, g, r, a = orc.trigger(scores, [int(cur)], [float(obs)])
        assert b[0] == int(best), line
        assert abs(float(g[0]) - float(gain)) <= 1e-6, line
        assert bool(r[0]) == bool(int(rec)) and bool(a[0]) == bool(int(ad)), line
        n += 1
    assert n == 7


def test_brute_force_random_rows():
    rng = np.random.default_rng(0)
    sc = (1.0 + 0.2 * rng.standard_normal((300, 17))).astype(np.float32)
    cur = rng.integers(0, 17, 300)
    obs = (1.0 + 0.2 * rng.standard_normal(300)).astype(np.float32)
    b, g, r, a = orc.trigger(sc, cur, obs, 0.05, 0.10)
    for s in range(300):
        best = max(range(17), key=lambda c: (sc[s, c], -c))
        vc = np.float32(sc[s, cur[s]])
        gain = np.float32(np.float32(sc[s, best] - vc) / np.float32(abs(vc)))
        err = np.float32(np.float32(abs(np.float32(vc - obs[s]))) / np.float32(abs(obs[s])))
        assert b[s] == best and g[s] == gain
        assert bool(r[s]) == bool(gain >= np.float32(0.05)) and bool(a[s]) == bool(err > np.float32(0.10))
    assert 0.1 < r.mean() < 0.95 and 0.1 < a.mean() < 0.95      # both outcomes occur


def test_edge_cases():
    sc = np.array([[np.nan, np.nan, np.nan],        # no valid best
                   [1.0, 2.0, np.nan],               # current candidate is NaN
                   [1.0, 2.0, 3.0],                  # current index out of range
                   [-2.0, -1.0, -4.0],               # negative speeds: |V_cur| in the denominator
                   [0.0, 1.0, 0.5]], dtype=np.float32)
    b, g, r, a = orc.trigger(sc, [0, 2, 7, 0, 0], [1.0, 1.0, 1.0, -2.1, 0.0])
    assert list(b) == [-1, 1, 2, 1, 1]
    assert math.isnan(g[0]) and math.isnan(g[1]) and math.isnan(g[2])
    assert not r[0] and not r[1] and not r[2] and not a[0] and not a[1] and not a[2]
    assert g[3] == np.float32(0.5) and r[3] and not a[3]
    assert g[4] == np.inf and r[4] and not a[4]       # 0/0 error ratio is NaN -> no adaptation
    # without observations nothing asks for adaptation; padding columns are ignored with a row stride
    b2, g2, r2, a2 = orc.trigger(sc, [0, 0, 0, 0, 0], None)
    assert not a2.any() and list(b2) == list(b)
