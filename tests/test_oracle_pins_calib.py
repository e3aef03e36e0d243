"""Pins for the oracle's scale sweep (cast-and-score step of Algorithm 1 on one tensor) and
per-channel scaling functions.  CPU only."""
import numpy as np
import pytest

from oracle import hif8_oracle as orc

TA, HR, TE, SR = orc.RM_TA, orc.RM_HR, orc.RM_TE, orc.RM_SR
SAT = orc.FLAG_SAT


def brute_sweep_ta(x, e_lo, count):
    """Independent fp64 derivation: nearest HiF8 magnitude by argmin over the value set (a tie
    goes to the larger magnitude), values at or above the midpoint to 1.5 * 2^15 overflow."""
    vals, _ = orc.value_table()
    grid = np.concatenate([vals, [1.5 * 2.0 ** 15]])
    out = []
    x = x.astype(np.float64)
    for k in range(count):
        s = 2.0 ** (e_lo + k)
        a = np.abs(x) * s
        d = np.abs(a[:, None] - grid[None, :])
        # argmin returns the first minimum; flip so that ties resolve to the larger magnitude
        j = grid.size - 1 - np.argmin(d[:, ::-1], axis=1)
        q = np.where(j == grid.size - 1, np.inf, grid[np.minimum(j, grid.size - 1)])
        q = np.where(a >= grid[-1], np.inf, q)
        with np.errstate(invalid="ignore", over="ignore"):
            err = (np.abs(x) - q / s) ** 2
        out.append(err.sum())
    return np.array(out)


def test_sweep_matches_brute_force_nearest():
    rng = np.random.default_rng(7)
    x = (rng.standard_normal(3000) * np.exp2(rng.uniform(-20, 9, 3000))).astype(np.float32)
    want = brute_sweep_ta(x, -4, 10)
    got = orc.scale_sweep(x, orc.SRC_F32, -4, 10, TA)
    assert np.all(np.isfinite(want))
    np.testing.assert_allclose(got, want, rtol=1e-13)
    xb = (x.view(np.uint32) >> 16).astype(np.uint16)
    xbf = (xb.astype(np.uint32) << 16).view(np.float32)
    np.testing.assert_allclose(orc.scale_sweep(xb, orc.SRC_BF16, -6, 12, TA), brute_sweep_ta(xbf, -6, 12), rtol=1e-13)
    xh = x.astype(np.float16)
    np.testing.assert_allclose(orc.scale_sweep(xh.view(np.uint16), orc.SRC_F16, -3, 5, TA),
                               brute_sweep_ta(xh.astype(np.float32), -3, 5), rtol=1e-13)


def test_sweep_power_of_two_shift_invariance():
    """Q(2^j x * 2^e) * 2^-e = 2^j * Q(x * 2^(e+j)) * 2^-(e+j): every term scales by exactly 4^j
    (the fp64 sums agree up to the order in which the threads' partial sums are combined)."""
    rng = np.random.default_rng(8)
    x = (rng.standard_normal(20000) * np.exp2(rng.uniform(-8, 4, 20000))).astype(np.float32)
    for mode in (TA, HR, TE):
        base = orc.scale_sweep(x, orc.SRC_F32, -6, 14, mode)
        for j in (-2, 1, 3):
            shifted = orc.scale_sweep((x * np.float32(2.0 ** j)).astype(np.float32), orc.SRC_F32, -6 - j + 2, 8, mode)
            np.testing.assert_allclose(shifted, base[2:10] * 4.0 ** j, rtol=1e-13, err_msg=str((mode, j)))


@pytest.mark.parametrize("E,k", [(0, 3), (2, 3), (5, 2), (-6, 2), (9, 1), (-12, 1)])
def test_sweep_uniform_binade_gives_step_squared_over_12(E, k):
    """Textbook: rounding to nearest on a uniform grid of step h has MSE h^2 / 12 for inputs
    uniform over many steps.  In the binade of 2^E HiF8 keeps k mantissa bits: h = 2^(E-k)."""
    rng = np.random.default_rng(100 + E)
    n = 400000
    x = (np.ldexp(1.0 + rng.random(n), E)).astype(np.float32)
    h = 2.0 ** (E - k)
    mse = orc.scale_sweep(x, orc.SRC_F32, 0, 1, TA)[0] / x.size
    assert abs(mse / (h * h / 12.0) - 1.0) < 0.01, (mse, h * h / 12)


def test_sweep_exact_and_non_finite_cases():
    p2 = np.ldexp(1.0, np.arange(-16, 9)).astype(np.float32)          # 2^j * 2^e stays in [2^-22, 2^15]
    assert np.all(orc.scale_sweep(np.concatenate([p2, -p2]), orc.SRC_F32, -4, 10, TA) == 0.0)
    x = np.array([3.0e4, 1.0], np.float32)
    e = orc.scale_sweep(x, orc.SRC_F32, 0, 2, TA)
    assert np.isfinite(e[0]) and np.isinf(e[1]) and e[1] > 0              # 6e4 is beyond 1.25 * 2^15
    es = orc.scale_sweep(x, orc.SRC_F32, 0, 2, TA | SAT)
    assert es[1] == (3.0e4 - 32768.0 / 2) ** 2 + 0.0
    assert np.isnan(orc.scale_sweep(np.array([1.0, np.nan], np.float32), orc.SRC_F32, 0, 1, TA)[0])
    assert orc.scale_sweep(np.zeros(0, np.float32), orc.SRC_F32, -4, 10, TA).tolist() == [0.0] * 10
    # one element, by hand: 1.3 -> nearest multiple of 1/8 is 1.25; at 2^3: 10.4 -> 10 (step 1) -> 1.25
    x = np.array([1.3], np.float32)
    d = float(x[0]) - 1.25
    assert orc.scale_sweep(x, orc.SRC_F32, 0, 1, TA)[0] == d * d
    assert orc.scale_sweep(x, orc.SRC_F32, 3, 1, TA)[0] == d * d
    # at 2^4: 20.8 -> step 4 in [16, 32) -> 20 -> 1.25 as well; at 2^5: 41.6 -> step 8 -> 40 -> 1.25
    assert orc.scale_sweep(x, orc.SRC_F32, 4, 2, TA).tolist() == [d * d, d * d]
    # at 2^8: 332.8 -> binade [256, 512), one mantissa bit: step 128 -> 384 -> 1.5
    assert orc.scale_sweep(x, orc.SRC_F32, 8, 1, TA)[0] == (float(x[0]) - 1.5) ** 2


def test_sweep_standard_sr_uses_the_element_index():
    rng = np.random.default_rng(9)
    x = rng.standard_normal(5000).astype(np.float32)
    orc.set_sr_seed(123)
    try:
        got = orc.scale_sweep(x, orc.SRC_F32, 1, 1, SR)[0]
        out, _ = orc.fake_quant_f32(x, 2.0, SR)
    finally:
        orc.set_sr_seed(0)
    want = ((x.astype(np.float64) - out.astype(np.float64)) ** 2).sum()
    assert abs(got / want - 1) < 1e-13


# ---------------------------------------------------------------- per-channel
@pytest.mark.parametrize("axis", [0, 1])
def test_per_channel_functions_reduce_to_the_per_tensor_ones(axis):
    rng = np.random.default_rng(11)
    rows, cols = 37, 53
    x = (rng.standard_normal((rows, cols)) * np.exp2(rng.uniform(-6, 6, (rows, 1 if axis == 0 else cols)))).astype(np.float32)
    am = orc.amax_axis(x, orc.SRC_F32, axis)
    assert np.array_equal(am, np.abs(x).max(axis=1 - axis))             # library routine
    scale = np.array([orc.scale_from_amax(a, 32768.0, True) for a in am], np.float32)
    codes = orc.encode_axis(x, scale, orc.SRC_F32, axis, TA)
    xt = x if axis == 0 else np.ascontiguousarray(x.T)
    ct = codes if axis == 0 else np.ascontiguousarray(codes.T)
    for c in range(xt.shape[0]):
        assert np.array_equal(ct[c], orc.encode_f32(xt[c], scale[c], TA))
        assert (ct[c] & 0x7F).max() in (0x6C, 0x6D, 0x6E)                 # each channel reaches the top binade
    back = orc.decode_axis(codes, scale, orc.SRC_F32, axis)
    bt = back if axis == 0 else np.ascontiguousarray(back.T)
    for c in range(xt.shape[0]):
        assert np.array_equal(bt[c].view(np.uint32), orc.decode_f32(ct[c], scale[c]).view(np.uint32))
    # 16-bit containers
    xb = (x.view(np.uint32) >> 16).astype(np.uint16)
    assert np.array_equal(orc.amax_axis(xb, orc.SRC_BF16, axis),
                          np.abs((xb.astype(np.uint32) << 16).view(np.float32)).max(axis=1 - axis))
    xh = x.astype(np.float16)
    assert np.array_equal(orc.amax_axis(xh.view(np.uint16), orc.SRC_F16, axis), np.abs(xh.astype(np.float32)).max(axis=1 - axis))
    cb = orc.encode_axis(xb, scale, orc.SRC_BF16, axis, HR)
    xbt = xb if axis == 0 else np.ascontiguousarray(xb.T)
    cbt = cb if axis == 0 else np.ascontiguousarray(cb.T)
    for c in range(xbt.shape[0]):
        assert np.array_equal(cbt[c], orc.encode_bf16(xbt[c], scale[c], HR))


def test_per_channel_sr_thresholds_follow_the_flat_index():
    rng = np.random.default_rng(12)
    x = rng.standard_normal((8, 100)).astype(np.float32)
    one = np.ones(8, np.float32)
    orc.set_sr_seed(77)
    try:
        a = orc.encode_axis(x, one, orc.SRC_F32, 0, SR)
        b = orc.encode_f32(x.reshape(-1), 1.0, SR).reshape(8, 100)
    finally:
        orc.set_sr_seed(0)
    assert np.array_equal(a, b)
