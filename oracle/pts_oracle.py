"""CPU oracle for the training-side scale state of the HiF8 method -- TEST INFRASTRUCTURE,
NOT PRODUCT CODE.  Plain Python, written from the paper (Sec. 5.1, training methods).

Adaptive loss scaling (ALS)
    A dynamic loss scaler as in FP16 mixed-precision training (scale halves on an overflow,
    doubles after `window` overflow-free iterations), whose window itself moves along the
    list {1, 20, 50, 100, 200, 500, 1000}: initial scale 2^32, initial window 20; when the
    scale has increased three times the window moves one place up the list, when the scale
    has decreased three times in a row it moves one place down.
    Readings where the text is silent:
      - "increases three times" is counted since the last window change and is not reset by
        a decrease; "decreases three times in a row" is reset by any increase;
      - both counters restart after a window change; the window stays put at the list ends;
      - halving stops at scale 1 and doubling stops at 2^126 (the counters still advance).

Per-tensor scaling (PTS)
    One scale per GEMM input tensor, initially 1; every `interval` (10) iterations the
    tensor's amax is taken and the scale becomes the largest power of two s with
    amax * s <= target ("a certain algorithm" in the paper; power-of-two restriction stated).
    A tensor whose amax is zero, Inf or NaN keeps its previous scale.
"""
import math

ALS_WINDOWS = (1, 20, 50, 100, 200, 500, 1000)
ALS_INIT_SCALE = 2.0 ** 32
ALS_INIT_WINDOW_INDEX = 1          # window 20
ALS_MIN_SCALE = 1.0
ALS_MAX_SCALE = 2.0 ** 126


class ALS:
    def __init__(self):
        self.scale = ALS_INIT_SCALE
        self.window_index = ALS_INIT_WINDOW_INDEX
        self.good_steps = 0            # overflow-free iterations since the last scale change
        self.increases = 0             # scale increases since the last window change
        self.decrease_streak = 0       # consecutive scale decreases

    @property
    def window(self):
        return ALS_WINDOWS[self.window_index]

    def update(self, found_overflow: bool):
        """One training iteration.  Returns (scale, window) in effect for the next one."""
        if found_overflow:
            self.scale = max(self.scale / 2.0, ALS_MIN_SCALE)
            self.good_steps = 0
            self.decrease_streak += 1
            if self.decrease_streak == 3:
                self.window_index = max(self.window_index - 1, 0)
                self.decrease_streak = 0
                self.increases = 0
        else:
            self.good_steps += 1
            if self.good_steps >= self.window:
                self.scale = min(self.scale * 2.0, ALS_MAX_SCALE)
                self.good_steps = 0
                self.decrease_streak = 0
                self.increases += 1
                if self.increases == 3:
                    self.window_index = min(self.window_index + 1, len(ALS_WINDOWS) - 1)
                    self.increases = 0
                    self.decrease_streak = 0
        return self.scale, self.window


def pts_scale(amax: float, old_scale: float, target: float = 32768.0) -> float:
    """Scale of one tensor after an amax update: the largest power of two s with
    amax * s <= target; degenerate amax keeps the old scale."""
    if not (amax > 0.0) or math.isinf(amax) or math.isnan(amax):
        return old_scale
    s = 2.0 ** math.floor(math.log2(target / amax))
    # log2 of a quotient near a power of two can be off by one ulp: fix up exactly
    while amax * s > target:
        s /= 2.0
    while amax * (2.0 * s) <= target:
        s *= 2.0
    # binary32 normal range (the device holds the scale and its reciprocal as floats)
    return min(max(s, 2.0 ** -126), 2.0 ** 126)


class PTS:
    """Scale state of `count` tensors over training iterations (interval in iterations)."""

    def __init__(self, count, interval=10, target=32768.0):
        self.scale = [1.0] * count
        self.interval = interval
        self.target = target
        self.iteration = 0

    def collects(self):
        return self.iteration % self.interval == 0

    def end_iteration(self, amax_list=None):
        """amax_list: the amax of each tensor gathered during this iteration (needed on
        collecting iterations only)."""
        if self.collects():
            self.scale = [pts_scale(a, s, self.target) for a, s in zip(amax_list, self.scale)]
        self.iteration += 1
        return list(self.scale)
