"""Pins for the oracle's comparison modes (TE, simplified SR everywhere, standard SR) and for
FP16 sources.  CPU only; same approach as test_oracle_pins.py: printed examples, a second
bit-level derivation typed here, invariants and library routines."""
import numpy as np
import pytest

from conftest import golden_lines
from oracle import hif8_oracle as orc
from test_oracle_pins import (all_values, bits_f32, closed_form_round, f32_bits,
                              kept_bits_of_exponent, oracle_values_f32)

TA, HR, TE, SSR, SR = orc.RM_TA, orc.RM_HR, orc.RM_TE, orc.RM_SSR, orc.RM_SR
SAT, N2Z = orc.FLAG_SAT, orc.FLAG_NAN2ZERO


# ---------------------------------------------------------------- FP16 container
def test_f16_conversions_match_numpy():
    pats = np.arange(65536, dtype=np.uint16)
    w = orc.widen_f16(pats)
    ref = pats.view(np.float16).astype(np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(w), nan)
    assert np.array_equal(w[~nan].view(np.uint32), ref[~nan].view(np.uint32))
    rng = np.random.default_rng(51)
    x = (rng.standard_normal(300000) * np.exp2(rng.uniform(-28, 18, 300000))).astype(np.float32)
    # exact ties between neighbouring binary16 values, even and odd
    h = rng.integers(0, 0x7BFF, size=20000).astype(np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    ties = ((lo + hi) / 2).astype(np.float32)
    special = np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e9, -1e9, np.inf, -np.inf, 2.0 ** -24, 2.0 ** -25,
                        1.5 * 2.0 ** -25, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -25], np.float32)
    x = np.concatenate([x, ties, -ties, special])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(orc.narrow_f16(x), want)
    assert orc.narrow_f16(np.array([np.nan], np.float32))[0] == 0x7E00
    # round trip on every non-NaN pattern
    assert np.array_equal(orc.narrow_f16(w[~nan]), pats[~nan])
    fin = ~nan
    assert orc.amax_f16(pats[fin & (pats != 0x7C00) & (pats != 0xFC00)]) == 65504.0


@pytest.mark.parametrize("mode", [TA, HR, TE, SSR, TA | SAT, HR | N2Z])
def test_f16_source_encode_matches_bit_level_rule(mode):
    pats = np.arange(65536, dtype=np.uint16)
    x = pats.view(np.float16).astype(np.float32)
    ok = ~np.isnan(x)
    v = all_values()
    rm = mode & 0xF
    for scale in (np.float32(1.0), np.float32(0.37), np.float32(2.0 ** -7)):
        prod = (x[ok] * scale).astype(np.float32)
        codes = orc.encode_f16(pats[ok], scale, mode)
        want = closed_form_round(f32_bits(prod), rm, 2)
        got = v[codes]
        if mode & SAT:
            want = np.where(np.isinf(want), np.sign(want) * 2.0 ** 15, want)
        assert np.array_equal(got, want)
    assert orc.encode_f16(pats[~ok], 1.0, mode).tolist() == [0x00 if mode & N2Z else 0x80] * int((~ok).sum())
    # fake-quant back to binary16: every HiF8 value is a binary16 value, so scale 1 is idempotent
    out, codes = orc.fake_quant_f16(pats[ok], 1.0, TA)
    out2, codes2 = orc.fake_quant_f16(out, 1.0, TA)
    assert np.array_equal(out, out2) and np.array_equal(codes, codes2)
    assert np.array_equal(orc.decode_f16(np.arange(256, dtype=np.uint8), 1.0)[[0x6E, 0x01, 0x80, 0x6F]],
                          np.array([0x7800, 0x0004, 0x7E00, 0x7C00], np.uint16))


# ---------------------------------------------------------------- TE
def test_te_worked_example_from_paper():
    rows = [r for r in golden_lines("rounding_examples.txt") if "." in r[0] and len(r) == 3]
    for src, ta, te in rows:
        x = int(src.replace(".", ""), 2) / 2.0
        for sgn in (1.0, -1.0):
            c = orc.encode_one(sgn * (8.0 + x), TE)
            assert orc.decode_value(c) == sgn * (8.0 + int(te, 2))
    # the three inputs give two distinct TE results and three distinct TA results
    assert len({orc.encode_one(8.0 + d, TE) for d in (0.5, 1.5, 2.5)}) == 2
    assert len({orc.encode_one(8.0 + d, TA) for d in (0.5, 1.5, 2.5)}) == 3


def test_te_differs_from_ta_only_on_ties_and_tie_probability():
    want_log2 = int([r for r in golden_lines("rounding_examples.txt") if r[0] == "te_special_case_probability_log2"][0][1])
    # all 2^20 discarded patterns below a 3-bit mantissa, even and odd kept values
    low = np.arange(1 << 20, dtype=np.uint32)
    for keep, expect in ((0b010, 1), (0b011, 0)):
        yb = (np.uint32(127) << 23) | (np.uint32(keep) << 20) | low
        ta = orc.encode_f32(bits_f32(yb), 1.0, TA)
        te = orc.encode_f32(bits_f32(yb), 1.0, TE)
        assert int((ta != te).sum()) == expect
    assert np.log2(1.0 / (1 << 20)) == want_log2         # one tie among 2^20 equally likely patterns
    rng = np.random.default_rng(52)
    yb = rng.integers(0, 2 ** 32, size=1 << 20, dtype=np.uint64).astype(np.uint32)
    yb[::3] &= np.uint32(0xFFF80000)                    # plenty of exact ties and representables
    yb[1::3] &= np.uint32(0xFFFC0000)
    yb = yb[~np.isnan(bits_f32(yb))]
    got, _ = oracle_values_f32(yb, TE)
    assert np.array_equal(got, closed_form_round(yb, TE, False))
    ta, _ = oracle_values_f32(yb, TA)
    diff = got != ta
    assert diff.any()
    # wherever they differ the input is exactly halfway between the two results
    x = bits_f32(yb).astype(np.float64)
    fin = diff & np.isfinite(ta) & np.isfinite(got)
    assert np.array_equal((got[fin] + ta[fin]) / 2, x[fin])
    # |error| <= half a step, like TA
    v = all_values()
    sel = (np.abs(x) >= 2.0 ** -22) & (np.abs(x) < 2.0 ** 15)
    E = np.floor(np.log2(np.abs(x[sel]))).astype(np.int64)
    ulp = np.ldexp(1.0, E - kept_bits_of_exponent(E))
    assert np.all(np.abs(got[sel] - x[sel]) <= 0.5 * ulp)


def test_te_edges():
    e = orc.encode_one
    assert e(2.0 ** -23, TE) == 0x00 and e(np.nextafter(np.float32(2.0 ** -23), np.float32(1)), TE) == 0x01
    assert e(40960.0, TE) == 0x6E and e(np.nextafter(np.float32(40960.0), np.float32(1e9)), TE) == 0x6F
    assert e(1.5 * 2.0 ** -20, TE) == 0x04                # denormal range: lo is 1 * step, odd
    assert e(1.0625, TE) == 0x08 and e(1.1875, TE) == 0x0A  # 1 + 1/16 -> 1.0 (even); 1 + 3/16 -> 1.25 (even)
    for c in range(256):
        v = orc.decode_value(c)
        assert e(v, TE) == c


# ---------------------------------------------------------------- simplified SR in every binade
def test_ssr_matches_bit_level_rule_and_hr_outside_the_switch():
    rng = np.random.default_rng(53)
    yb = rng.integers(0, 2 ** 32, size=1 << 20, dtype=np.uint64).astype(np.uint32)
    ex = rng.integers(127 - 30, 127 + 18, size=yb.size).astype(np.uint32)
    yb[::2] = (yb[::2] & np.uint32(0x807FFFFF)) | (ex[::2] << 23)
    yb[::8] &= np.uint32(0xFFFFC000)
    yb = yb[~np.isnan(bits_f32(yb))]
    got, codes = oracle_values_f32(yb, SSR)
    assert np.array_equal(got, closed_form_round(yb, SSR, False))
    hr = orc.encode_f32(bits_f32(yb), 1.0, HR)
    E = ((yb >> 23) & 0xFF).astype(np.int64) - 127
    out = np.abs(E) >= 4
    assert np.array_equal(codes[out], hr[out])
    assert np.any(codes[~out] != hr[~out])
    b = np.arange(65536, dtype=np.uint16)
    bb = b.astype(np.uint32) << 16
    ok = ~np.isnan(bits_f32(bb))
    c16 = orc.encode_bf16(b[ok], 1.0, SSR)
    assert np.array_equal(all_values()[c16], closed_form_round(bb[ok], SSR, True))


# ---------------------------------------------------------------- standard SR
def np_fmix32(x):
    x = x.astype(np.uint64)
    x ^= x >> np.uint64(16); x = (x * np.uint64(0x85EBCA6B)) & np.uint64(0xFFFFFFFF)
    x ^= x >> np.uint64(13); x = (x * np.uint64(0xC2B2AE35)) & np.uint64(0xFFFFFFFF)
    x ^= x >> np.uint64(16)
    return x


def np_threshold(seed, idx):
    """The generator as the oracle's header states it, typed again in numpy (so that whole arrays of
    thresholds can be formed quickly; test_sr_threshold_generator compares it with the C function)."""
    idx = np.asarray(idx, np.uint64)
    m32 = np.uint64(0xFFFFFFFF)
    with np.errstate(over="ignore"):
        z = np.uint64(seed) + np.uint64(0x9E3779B97F4A7C15) * ((idx >> np.uint64(32)) + np.uint64(1))
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    k1, k2 = z & m32, z >> np.uint64(32)
    x = (idx & m32) ^ k1
    x ^= x >> np.uint64(16); x = (x * np.uint64(0x85EBCA6B)) & m32
    x = (x + k2) & m32
    x ^= x >> np.uint64(13); x = (x * np.uint64(0xC2B2AE35)) & m32
    x ^= x >> np.uint64(16)
    return x.astype(np.uint32)


def test_sr_threshold_generator():
    idx = np.concatenate([np.arange(100000, dtype=np.uint64), np.uint64(1 << 32) + np.arange(1000, dtype=np.uint64),
                          np.array([2 ** 40 + 17, 2 ** 63], np.uint64)])
    for seed in (0, 1, 0x123456789ABCDEF):
        got = np.array([orc.sr_threshold(seed, int(i)) for i in idx[:3000]], np.uint32)
        assert np.array_equal(got, np_threshold(seed, idx[:3000]))
    t = np_threshold(7, np.arange(1 << 20, dtype=np.uint64)).astype(np.float64) / 2.0 ** 32
    assert abs(t.mean() - 0.5) < 2e-3
    hist, _ = np.histogram(t, bins=64, range=(0, 1))
    assert hist.min() > 0.9 * t.size / 64 and hist.max() < 1.1 * t.size / 64
    assert np.unique(np_threshold(7, np.arange(1 << 16, dtype=np.uint64))).size > 0.99 * (1 << 16)
    assert not np.array_equal(np_threshold(7, np.arange(64, dtype=np.uint64)), np_threshold(8, np.arange(64, dtype=np.uint64)))


def test_sr_threshold_generator_statistics():
    """What standard SR needs of its thresholds (Sec. 3.2: a uniform random number per element): every bit
    balanced, neighbours uncorrelated, streams of different seeds and of different 2^32-element blocks
    uncorrelated.  Measured on the oracle's own generator (the C function), 2^18 draws per stream."""
    n = 1 << 18
    def stream(seed, base):
        return np.array([orc.sr_threshold(seed, base + i) for i in range(n)], np.uint32)
    def corr(a, b):
        a = a.astype(np.float64) - a.mean(); b = b.astype(np.float64) - b.mean()
        return float((a * b).sum() / np.sqrt((a * a).sum() * (b * b).sum()))
    bound = 5.0 / np.sqrt(n)                                 # 5 sigma of a sample correlation / of a bit mean * 2
    s7 = stream(7, 0)
    for b in range(32):
        assert abs(((s7 >> np.uint32(b)) & np.uint32(1)).mean() - 0.5) < bound / 2, b
    for lag in (1, 2, 3, 4, 8, 64, 1024):
        assert abs(corr(s7[:-lag], s7[lag:])) < bound, lag
    assert abs(corr(s7, stream(8, 0))) < bound               # neighbouring seeds
    assert abs(corr(s7, stream(7 + (1 << 32), 0))) < bound   # seeds that differ in the high word only
    assert abs(corr(s7, stream(7, 1 << 32))) < bound         # the next 2^32-element block
    assert abs(corr(s7, stream(7, 1 << 33))) < bound
    # top bits (the ones that decide a carry) of neighbours: all 16 pairs of 2-bit values about equally often
    top = (s7 >> np.uint32(30)).astype(np.int64)
    pairs = np.bincount(top[:-1] * 4 + top[1:], minlength=16)
    assert pairs.min() > 0.95 * (n - 1) / 16 and pairs.max() < 1.05 * (n - 1) / 16



def _oracle_thresholds(seed, n, base=0):
    return np.array([orc.sr_threshold(seed, base + i) for i in range(n)], np.uint32)


def test_sr_seeds_are_different_draws_not_permutations():
    """Sec. 3.2: standard SR draws one uniform random number per element.  Two seeds must therefore give
    two draws, not one draw in another order: (a) the thresholds that fall into one aligned 16-element block
    must differ as a multiset between seeds, (b) the number of carries over a constant tensor (a binomial
    count) must vary from seed to seed with about the binomial spread, (c) no small index displacement d maps
    the stream of seed s onto the stream of seed s ^ d."""
    n = 1 << 12
    base_seeds = (0, 7, 1234, 1 << 40)
    for s in base_seeds:
        a = np.sort(_oracle_thresholds(s, n).reshape(-1, 16), axis=1)
        for s2 in (s + 1, s ^ 5, s + (1 << 32), s + (1 << 33) + 1):
            b = np.sort(_oracle_thresholds(s2, n).reshape(-1, 16), axis=1)
            same = int((a == b).all(axis=1).sum())
            assert same == 0, (s, s2, same)
    # (c) t(s, i) == t(s ^ d, i ^ d) would make seeds permutations of each other
    for s in base_seeds:
        t0 = _oracle_thresholds(s, 256)
        for d in range(1, 64):
            t1 = _oracle_thresholds(s ^ d, 256)
            idx = np.arange(256) ^ d
            assert int((t0 == t1[idx]).sum()) <= 1, (s, d)
    # (b) 2^16 copies of 20.5 (between 20 and 24: discarded fraction 1/8): carries ~ Binomial(2^16, 1/8)
    m = 1 << 16
    x = np.full(m, 20.5, np.float32)
    v = all_values()
    sums = []
    try:
        for seed in range(16):
            orc.set_sr_seed(seed)
            sums.append(float(v[orc.encode_f32(x, 1.0, SR)].sum()))
    finally:
        orc.set_sr_seed(0)
    carries = (np.array(sums) - 20.0 * m) / 4.0
    sd = np.sqrt(m * 0.125 * 0.875)                      # 84.7
    assert len(set(sums)) >= 14                           # not one value for every seed
    assert np.all(np.abs(carries - m / 8) < 5 * sd)
    assert 0.4 * sd < carries.std(ddof=1) < 2.0 * sd      # chi-square bounds for 15 degrees of freedom, wide


def test_sr_index_base_continues_the_stream():
    """A slice of a tensor cast with index base b uses the thresholds its elements have inside the tensor."""
    rng = np.random.default_rng(7)
    x = (rng.standard_normal(5000) * 3).astype(np.float32)
    try:
        orc.set_sr_seed(11)
        whole = orc.encode_f32(x, 1.0, SR)
        orc.set_sr_index_base(1234)
        part = orc.encode_f32(x[1234:], 1.0, SR)
        orc.set_sr_index_base((1 << 32) - 100)
        hi = orc.encode_f32(x[:200], 1.0, SR)
        t = np.array([orc.sr_threshold(11, (1 << 32) - 100 + i) for i in range(200)], np.uint32)
        want = [orc.encode_one(float(x[i]), SR, 0, int(t[i])) for i in range(200)]
    finally:
        orc.set_sr_seed(0)
        orc.set_sr_index_base(0)
    assert np.array_equal(part, whole[1234:])
    assert hi.tolist() == want

def test_sr_matches_bit_level_rule_and_is_unbiased():
    rng = np.random.default_rng(54)
    n = 1 << 20
    yb = rng.integers(0, 2 ** 32, size=n, dtype=np.uint64).astype(np.uint32)
    ex = rng.integers(127 - 60, 127 + 18, size=n).astype(np.uint32)
    yb[::2] = (yb[::2] & np.uint32(0x807FFFFF)) | (ex[::2] << 23)
    yb[::16] &= np.uint32(0xFFF00000)
    x = bits_f32(yb)
    ok = ~np.isnan(x)
    for seed in (0, 99):
        orc.set_sr_seed(seed)
        try:
            codes = orc.encode_f32(x, 1.0, SR)
        finally:
            orc.set_sr_seed(0)
        t32 = np_threshold(seed, np.arange(n, dtype=np.uint64))
        want = closed_form_round(yb[ok], SR, False, t32[ok])
        assert np.array_equal(all_values()[codes[ok]], want)
    # extreme thresholds: 0 carries whenever anything is discarded, 2^32 - 1 never does (<= 23-bit fractions)
    v = all_values()
    for val in (1.03, 100.3, 3e-6, 2.0 ** -24, 1.2e-8):
        lo_c, hi_c = orc.encode_one(val, SR, 0, 0xFFFFFFFF), orc.encode_one(val, SR, 0, 0)
        assert v[lo_c] < val < v[hi_c]
    for c in range(256):                                  # representable inputs never move
        for t in (0, 1, 0x80000000, 0xFFFFFFFF):
            assert orc.encode_one(v[c], SR, 0, t) == c
    # carry probability equals the discarded fraction; the mean is preserved
    idx = np.arange(1 << 16, dtype=np.uint64)
    t = np_threshold(5, idx)
    for val, lo, hi in ((1.03125, 1.0, 1.125), (20.5, 20.0, 24.0), (2.0 ** -20 * 1.7, 2.0 ** -20, 2.0 ** -19), (3e-8, 0.0, 2.0 ** -22)):
        frac = (np.float64(np.float32(val)) - lo) / (hi - lo)
        ups = np.array([orc.encode_one(val, SR, 0, int(tt)) for tt in t[:20000]])
        p = np.mean(v[ups] == hi)
        assert set(np.unique(v[ups])) <= {lo, hi}
        assert abs(p - frac) < 4 * np.sqrt(frac * (1 - frac) / 20000) + 1e-4
