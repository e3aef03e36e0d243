"""Pins for the training-side scale state oracle (ALS window scheduler, PTS scale update).
CPU only."""
import math

import numpy as np
import pytest

from conftest import golden_lines
from oracle import pts_oracle as po
from oracle import hif8_oracle as orc

OVERFLOWS = {
    "clean": set(),
    "storm": set(range(1, 10000)),
    "mixed": {1, 2, 23, 24, 45, 46, 47},
}


def test_als_constants_are_the_papers():
    assert po.ALS_WINDOWS == (1, 20, 50, 100, 200, 500, 1000)
    a = po.ALS()
    assert a.scale == 2.0 ** 32 and a.window == 20


@pytest.mark.parametrize("name", ["clean", "storm", "mixed"])
def test_als_hand_worked_traces(name):
    want = {int(it): (int(lg), int(w)) for n, it, lg, w in golden_lines("als_traces.txt") if n == name}
    assert len(want) >= 5
    a = po.ALS()
    for it in range(1, max(want) + 1):
        scale, window = a.update(it in OVERFLOWS[name])
        if it in want:
            assert (math.log2(scale), window) == want[it], (name, it)


def test_als_window_saturates_and_scale_is_clamped():
    a = po.ALS()
    for _ in range(20000):
        a.update(False)
    assert a.window == 1000 and a.scale <= po.ALS_MAX_SCALE
    for _ in range(200):
        a.update(True)
    assert a.window == 1 and a.scale == 1.0
    # a decrease does not clear the count of increases, an increase clears the decrease streak
    a = po.ALS()
    a.window_index = 0
    a.update(False); a.update(False)            # two increases
    a.update(True)                              # one decrease
    a.update(False)                             # third increase since the last window change
    assert a.window == 20
    a = po.ALS()
    a.update(True); a.update(True)
    for _ in range(20):
        a.update(False)                         # doubling breaks the streak
    a.update(True); a.update(True)
    assert a.window == 20
    a.update(True)
    assert a.window == 1


def test_pts_scale_is_the_largest_power_of_two_that_fits():
    rng = np.random.default_rng(5)
    amax = np.concatenate([np.exp2(rng.uniform(-40, 40, 5000)), np.exp2(np.arange(-30.0, 31.0)),
                           np.nextafter(np.exp2(np.arange(-30.0, 31.0)), np.inf)]).astype(np.float32)
    for target in (32768.0, 8192.0, 1.0):
        for a in amax.tolist():
            s = po.pts_scale(a, 1.0, target)
            m, e = math.frexp(s)
            assert m == 0.5                                  # a power of two
            assert a * s <= target < a * s * 2.0
            # same answer as the conversion oracle's pow2 scale rule (typed separately in C)
            assert s == float(orc.scale_from_amax(np.float32(a), np.float32(target), True))
    for bad in (0.0, -0.0, float("inf"), float("nan")):
        assert po.pts_scale(bad, 0.25) == 0.25


def test_pts_schedule():
    p = po.PTS(2, interval=10, target=32768.0)
    seen = []
    for it in range(25):
        collects = p.collects()
        assert collects == (it % 10 == 0)
        seen.append(p.end_iteration([3.0 * (it + 1), 0.0] if collects else None))
    assert seen[0] == [8192.0, 1.0]                          # amax 3 -> 2^13; amax 0 keeps 1
    assert seen[9] == [8192.0, 1.0]
    assert seen[10] == [512.0, 1.0]                          # amax 33 -> 2^9 (33 * 1024 > 32768)
    assert seen[20] == [512.0, 1.0]                          # amax 63 -> 2^9
