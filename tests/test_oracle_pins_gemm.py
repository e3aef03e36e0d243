"""Pins for the GEMM / layer-calibration oracle.  CPU only."""
from fractions import Fraction

import numpy as np

from oracle import gemm_oracle as go
from oracle import hif8_oracle as orc


def test_gemm_against_exact_rational_arithmetic():
    """Brute force: triple loop over exact rationals on a small problem."""
    rng = np.random.default_rng(3)
    finite = [c for c in range(256) if np.isfinite(orc.decode_value(c))]
    M, N, K = 5, 4, 23
    ca = rng.choice(finite, size=(M, K)).astype(np.uint8)
    cb = rng.choice(finite, size=(N, K)).astype(np.uint8)
    val = {c: Fraction(orc.decode_value(c)) for c in finite}
    sa, sb = 0.25, 8.0
    got = go.gemm_hif8(ca, cb, sa, sb)
    for i in range(M):
        for j in range(N):
            exact = sum(val[int(ca[i, k])] * val[int(cb[j, k])] for k in range(K)) * Fraction(1 / sa) * Fraction(1 / sb)
            assert abs(Fraction(got[i, j]) - exact) <= abs(exact) * Fraction(1, 2 ** 48) + Fraction(1, 2 ** 80)
    bound = go.gemm_abs_bound(ca, cb, sa, sb)
    assert np.all(np.abs(got) <= bound * (1 + 1e-12))


def test_gemm_hand_example_and_specials():
    # codes: 1.0 = 0x08, 2.0 = 0x10, 0.5 = 0x18, -1.0 = 0x88, 1.5 = 0x0C, zero = 0x00 (Tables 1-3)
    a = np.array([[0x08, 0x10, 0x18, 0x00]], np.uint8)          # 1, 2, 0.5, 0
    b = np.array([[0x0C, 0x88, 0x10, 0x6E],                      # 1.5, -1, 2, 2^15
                  [0x08, 0x08, 0x08, 0x08]], np.uint8)
    assert go.gemm_hif8(a, b).tolist() == [[1.5 - 2.0 + 1.0 + 0.0, 3.5]]
    assert go.gemm_hif8(a, b, 2.0, 4.0).tolist() == [[0.5 / 8, 3.5 / 8]]
    inf = np.array([[0x6F, 0x08, 0x08, 0x08]], np.uint8)
    r = go.gemm_hif8(inf, b)
    assert np.isposinf(r[0, 0]) and np.isposinf(r[0, 1])
    nan = np.array([[0x80, 0x08, 0x08, 0x08]], np.uint8)
    assert np.all(np.isnan(go.gemm_hif8(nan, b)))
    assert np.isnan(go.gemm_hif8(np.array([[0x6F, 0, 0, 0]], np.uint8), np.array([[0, 8, 8, 8]], np.uint8))[0, 0])  # Inf * 0


def test_calibration_properties():
    rng = np.random.default_rng(4)
    vals, codes = orc.value_table()
    mid = vals[(vals >= 2.0 ** -6) & (vals <= 2.0 ** 5)]
    # inputs already on the HiF8 grid with room to spare: scale 2^0 reproduces the exact product
    a = (rng.choice(mid, size=(6, 32)) * rng.choice([-1.0, 1.0], size=(6, 32))).astype(np.float32)
    w = (rng.choice(mid, size=(7, 32)) * rng.choice([-1.0, 1.0], size=(7, 32))).astype(np.float32)
    o = a.astype(np.float64) @ w.astype(np.float64).T
    err, best = go.calibrate_layer(a, w, o, orc.SRC_F32, -2, 5, -2, 5)
    assert err[2, 2] == 0.0 and err.min() == 0.0
    assert err[best[0] + 2, best[1] + 2] == 0.0
    # generic inputs: the search square is symmetric under swapping the roles of the two inputs
    a = rng.standard_normal((9, 40)).astype(np.float32)
    w = (rng.standard_normal((11, 40)) * 0.05).astype(np.float32)
    o = a.astype(np.float64) @ w.astype(np.float64).T
    e1, b1 = go.calibrate_layer(a, w, o, orc.SRC_F32, -4, 10, -4, 10)
    e2, b2 = go.calibrate_layer(w, a, o.T, orc.SRC_F32, -4, 10, -4, 10)
    np.testing.assert_allclose(e1, e2.T, rtol=1e-12)
    assert b1 == (b2[1], b2[0])
    # the small-magnitude weight tensor wants a larger scale than 2^0 (that is the point of PTS)
    assert b1[1] > 0
    # error of one cell, recomputed from fake-quantised inputs (the paper's simulation route)
    qa, _ = orc.fake_quant_f32(a.reshape(-1), 2.0 ** 1, orc.RM_TA)
    qw, _ = orc.fake_quant_f32(w.reshape(-1), 2.0 ** 3, orc.RM_TA)
    oq = qa.reshape(a.shape).astype(np.float64) @ qw.reshape(w.shape).astype(np.float64).T
    np.testing.assert_allclose(e1[5, 7], np.sum((oq - o) ** 2), rtol=1e-12)
