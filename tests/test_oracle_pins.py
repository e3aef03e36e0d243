"""Pins the CPU oracle to what the paper and the mathematics fix (CPU only).

Nothing here touches the HIP library.  The checks are chosen so that a plausible
mistake anywhere in the oracle (a dropped term, a wrong sign or index, a swapped
field) fails at least one of them:
  * printed patterns / values and counts (golden fixtures, each with its citation);
  * a second, bit-level derivation of each rounding rule written here in numpy
    ("add half at the band's width, truncate"; "compare discarded bits with threshold
    bits"), which must agree with the oracle's value-level brute-force search;
  * invariants: error bounds, nearest-neighbour property, identity on representable
    values, odd symmetry, dependence on the top 13 bits only;
  * library routines for the textbook parts (BF16 round-to-nearest-even, max-abs).
"""
import math

import numpy as np
import pytest
import torch

from conftest import golden_lines
from oracle import hif8_oracle as orc

TA, HR = orc.RM_TA, orc.RM_HR
TE, SSR, SR = orc.RM_TE, orc.RM_SSR, orc.RM_SR
SAT, N2Z = orc.FLAG_SAT, orc.FLAG_NAN2ZERO


# ---------------------------------------------------------------- helpers
def bits_to_code(pattern: str) -> int:
    return int(pattern.replace("_", ""), 2)


def f32_bits(x):
    return np.asarray(x, np.float32).view(np.uint32)


def bits_f32(u):
    return np.asarray(u, np.uint32).view(np.float32)


def all_values():
    return np.array([orc.decode_value(c) for c in range(256)], np.float64)


def kept_bits_of_exponent(E):
    """Mantissa width per binary exponent, typed from Table 3 (E ranges per dot value)
    and Eq. (2) (denormals are pure powers of two)."""
    aE = np.abs(E)
    k = np.full(E.shape, -1, np.int64)
    k[aE <= 3] = 3
    k[(aE >= 4) & (aE <= 7)] = 2
    k[(aE >= 8) & (aE <= 15)] = 1
    k[(E >= -22) & (E <= -16)] = 0
    return k


def closed_form_round(ybits, rm, src_bf16, t32=None):
    """Bit-level rounding of binary32 patterns (non-NaN) to HiF8 *values* (float64;
    +-inf on overflow, 0 on underflow), written from the prose of Sec. 3: keep k(E)
    mantissa bits, look only at the discarded bits.  TA: carry iff the top discarded bit
    is 1.  SR: carry iff F >= T (F top 14 / 2 discarded bits; T the 14 LSBs of the pattern
    / {LSB of the 16-bit source pattern, 1}), no carry when F = T = 0.  Below 2^-22 the discarded
    fraction is the fixed-point fraction of one 2^-22 step.
    src_bf16: False/0 = FP32 source, True/1 = BF16 (LSB at bit 16), 2 = FP16 (LSB at bit 13).
    Comparison modes: TE carries iff the discarded part is above half, or exactly half with an
    odd kept significand; SSR is the SR rule in every binade; SR carries iff the threshold
    t32 / 2^32 is below the discarded fraction."""
    src_kind = int(src_bf16)
    ybits = np.asarray(ybits, np.uint32)
    sign = np.where(ybits >> 31, -1.0, 1.0)
    a = (ybits & 0x7FFFFFFF).astype(np.int64)
    val = bits_f32(a.astype(np.uint32)).astype(np.float64)
    out = np.zeros(a.shape, np.float64)

    is_inf = a == 0x7F800000
    e = a >> 23
    E = e - 127
    m = a & 0x7FFFFF

    # --- underflow region: |y| < 2^-22, one step of 2^-22, fraction f = |y| / 2^-22
    under = (val < 2.0 ** -22)
    # f * 2^24 as an exact integer when possible: floor() of a float64 is exact here
    f = np.where(under, val, 0.0) * 2.0 ** 22
    if src_kind:
        F_u = np.floor(f * 4).astype(np.int64)
    else:
        F_u = np.floor(f * 16384).astype(np.int64)
    ta_up_u = f >= 0.5
    te_up_u = f > 0.5                      # the tie f = 1/2 sits next to lo = 0, an even multiple

    # --- regular region
    k = kept_bits_of_exponent(E)
    k = np.where(E >= 16, 0, k)  # overflow anyway
    k = np.where(k < 0, 0, k)
    d = 23 - k  # number of discarded bits
    disc = m & ((1 << d) - 1)
    keep = m >> d
    top = (disc >> (d - 1)) & 1
    if src_kind:
        F_r = disc >> (d - 2)
    else:
        F_r = disc >> (d - 14)

    if src_kind:
        T = 2 * ((a >> (16 if src_kind == 1 else 13)) & 1) + 1
    else:
        T = a & 0x3FFF
    F = np.where(under, F_u, F_r)
    sr_up = (F >= T) & ~((F == 0) & (T == 0))
    ta_up = np.where(under, ta_up_u, top == 1)
    if rm == TA:
        up = ta_up
    elif rm == TE:
        half = np.int64(1) << (d - 1)
        n_odd = np.where(k > 0, keep & 1, 1)
        te_up = (disc > half) | ((disc == half) & (n_odd == 1))
        up = np.where(under, te_up_u, te_up)
    elif rm == SSR:
        up = sr_up
    elif rm == SR:
        t = np.asarray(t32, np.uint32).astype(np.int64)
        up_r = (t >> (32 - d)) < disc
        up_u = (t.astype(np.float64) / 2.0 ** 32) < f
        up = np.where(under, up_u, up_r)
    else:
        use_sr = (np.abs(E) >= 4)
        up = np.where(use_sr, sr_up, ta_up)

    # assemble the rounded value
    step = np.ldexp(1.0, (E - k).astype(np.int64))
    lo = np.ldexp(1.0, E.astype(np.int64)) + keep * step
    res = np.where(up, lo + step, lo)
    res_u = np.where(up, 2.0 ** -22, 0.0)
    res = np.where(under, res_u, res)
    res = np.where(res >= 1.5 * 2.0 ** 15, np.inf, res)
    res = np.where(is_inf, np.inf, res)
    out = sign * res
    out = np.where(res == 0, 0.0, out)
    return out


def oracle_values_f32(ybits, mode):
    x = bits_f32(ybits)
    codes = orc.encode_f32(x, 1.0, mode)
    return all_values()[codes], codes


# ---------------------------------------------------------------- decode pins
def test_table4_patterns_and_values():
    rows = golden_lines("table4_typical_values.txt")
    seen = 0
    for r in rows:
        if r[0].startswith("exponent_range"):
            continue
        name, pattern, kind, lg = r
        code = bits_to_code(pattern)
        v = orc.decode_value(code)
        if kind == "inf":
            assert math.isinf(v) and (v < 0) == (pattern[0] == "1")
        elif kind == "nan":
            assert math.isnan(v)
        elif kind == "zero":
            assert v == 0.0 and not math.copysign(1, v) < 0
        else:
            assert v == 2.0 ** int(lg), name
        seen += 1
    assert seen == 8
    # well known byte values of those patterns
    assert bits_to_code("0_11_0111_1") == 0x6F and bits_to_code("1_0000_000") == 0x80


def test_table4_exponent_ranges():
    rng = {r[0]: (int(r[1]), int(r[2])) for r in golden_lines("table4_typical_values.txt")
           if r[0].startswith("exponent_range")}
    E_nml, E_all = set(), set()
    for c in range(256):
        f = orc.decode_fields(c)
        if f["kind"] == "nml":
            E_nml.add(f["E"])
            E_all.add(f["E"])
        elif f["kind"] == "dml":
            E_all.add(f["E"])
    assert (min(E_nml), max(E_nml)) == rng["exponent_range_nml"]
    assert (min(E_all), max(E_all)) == rng["exponent_range_all"]


def test_field_counts_match_paper():
    g = golden_lines("format_counts.txt")
    want = {r[0]: int(r[1]) for r in g if r[0] != "dot"}
    dots = {int(r[1]): (int(r[2]), int(r[3]), int(r[4])) for r in g if r[0] == "dot"}
    width_of_E = {}
    dml_E = set()
    per_dot = {}
    for c in range(128):
        f = orc.decode_fields(c)
        if f["kind"] in ("nml", "inf"):
            width_of_E.setdefault(f["E"], set()).add(f["mant_width"])
            per_dot.setdefault(f["D"], []).append(f)
        elif f["kind"] == "dml":
            dml_E.add(f["E"])
    assert all(len(w) == 1 for w in width_of_E.values())
    by_w = {}
    for E, w in width_of_E.items():
        by_w.setdefault(next(iter(w)), []).append(E)
    assert len(by_w[3]) == want["exponents_with_3bit_mantissa"]
    assert len(by_w[2]) == want["exponents_with_2bit_mantissa"]
    assert len(by_w[1]) == want["exponents_with_1bit_mantissa"]
    assert sorted(by_w[3]) == list(range(-3, 4))
    assert len(dml_E) == want["denormal_binades"] and sorted(dml_E) == list(range(-22, -15))
    assert len(width_of_E) == want["binades_normal"]
    assert len(width_of_E) + len(dml_E) == want["binades_total"]
    # Table 1 / Table 3 rows, per dot value
    for D, (emin, emax, w) in dots.items():
        fs = per_dot[D]
        assert {abs(f["E"]) for f in fs} == set(range(emin, emax + 1))
        assert {f["mant_width"] for f in fs} == {w}
        # each exponent value has all 2^w mantissas (sign of exponent doubles it for D > 0)
        n_exp = (emax - emin + 1) * (2 if D > 0 else 1)
        assert len(fs) == n_exp * (1 << w)


def test_specials_and_code_space():
    kinds = [orc.decode_fields(c)["kind"] for c in range(256)]
    assert kinds.count("zero") == 1 and kinds[0x00] == "zero"   # single zero pattern
    assert kinds.count("nan") == 1 and kinds[0x80] == "nan"
    assert kinds.count("inf") == 2 and kinds[0x6F] == "inf" and kinds[0xEF] == "inf"
    assert kinds.count("dml") == 14 and kinds.count("nml") == 256 - 4 - 14
    v = all_values()
    fin = v[np.isfinite(v)]
    assert fin.size == 253
    assert np.unique(fin).size == 253                      # non-redundant encoding
    # negative half mirrors the positive half
    for c in range(1, 128):
        if c == 0x6F:
            continue
        assert v[c | 0x80] == -v[c]
    # largest finite magnitude below the Inf slot value 1.5 * 2^15
    assert fin.max() == 2.0 ** 15 and fin.min() == -2.0 ** 15
    assert np.min(fin[fin > 0]) == 2.0 ** -22


def test_value_order_and_precision_taper():
    vals, codes = orc.value_table()
    assert vals.size == 127 and vals[0] == 0.0 and codes[0] == 0
    assert np.all(np.diff(vals) > 0)
    # within one (dot, exponent) prefix the value grows with the mantissa
    for c in range(128):
        f = orc.decode_fields(c)
        if f["kind"] == "nml" and f["M"] > 0:
            assert orc.decode_value(c) > orc.decode_value(c - 1)
    # Sec. 2.2: the mantissa width never drops by more than one bit between adjacent exponents
    E = np.arange(-22, 16)
    k = kept_bits_of_exponent(E)
    assert np.all(np.abs(np.diff(k)) <= 1)
    # and the oracle's parse agrees with that table
    for c in range(1, 128):
        f = orc.decode_fields(c)
        if f["kind"] == "nml":
            assert f["mant_width"] == kept_bits_of_exponent(np.array([f["E"]]))[0]
    # every finite value is an integer multiple of its binade's step (<= 4 significant bits)
    for v in vals[1:]:
        m, e = math.frexp(v)
        assert (m * 16) == int(m * 16)


def test_decode_arrays_and_descale():
    codes = np.arange(256, dtype=np.uint8)
    v = all_values()
    out = orc.decode_f32(codes, 1.0)
    assert out.view(np.uint32)[0x80] == 0x7FC00000
    assert out.view(np.uint32)[0x6F] == 0x7F800000 and out.view(np.uint32)[0xEF] == 0xFF800000
    assert out.view(np.uint32)[0x00] == 0
    fin = np.isfinite(v)
    assert np.array_equal(out[fin].astype(np.float64), v[fin])
    # power-of-two scale: exact division
    out4 = orc.decode_f32(codes, 4.0)
    assert np.array_equal(out4[fin].astype(np.float64), v[fin] / 4.0)
    # general scale: value * fl32(1/scale) in binary32
    s = np.float32(3.7)
    inv = np.float32(1.0) / s
    want = (v[fin].astype(np.float32) * inv).astype(np.float32)
    assert np.array_equal(orc.decode_f32(codes, s)[fin], want)
    # bf16 output: every HiF8 value is exact in bf16
    ob = orc.decode_bf16(codes, 1.0)
    back = (ob.astype(np.uint32) << 16).view(np.float32)
    assert np.array_equal(back[fin].astype(np.float64), v[fin])
    assert ob[0x80] == 0x7FC0 and ob[0x6F] == 0x7F80 and ob[0xEF] == 0xFF80


def test_bf16_rne_matches_torch():
    rng = np.random.default_rng(7)
    u = rng.integers(0, 2 ** 32, size=200000, dtype=np.uint64).astype(np.uint32)
    special = np.array([0, 0x80000000, 0x7F800000, 0xFF800000, 0x7F7FFFFF, 0x7F7F8000, 0x7F7F7FFF,
                        0x00000001, 0x00008000, 0x00018000, 0x3F808000, 0x3F818000, 0x3F80FFFF,
                        0x3F807FFF, 0x3F808001], np.uint32)
    u = np.concatenate([u, special])
    x = u.view(np.float32)
    keep = ~np.isnan(x)
    x = x[keep]
    want = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    # exact ties (low half = 0x8000) on even and odd kept patterns
    t = (rng.integers(0, 2 ** 16, size=5000, dtype=np.uint64).astype(np.uint32) << 16) | np.uint32(0x8000)
    t = t[~np.isnan(t.view(np.float32))]
    x = np.concatenate([x, t.view(np.float32)])
    want = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(orc.narrow_bf16(x), want)
    assert orc.narrow_bf16(np.array([np.nan], np.float32))[0] == 0x7FC0
    codes = np.arange(256, dtype=np.uint8)
    for s in [np.float32(3.7), np.float32(0.013), np.float32(1234.567)]:
        f = orc.decode_f32(codes, s)
        fin = ~np.isnan(f)
        w = torch.from_numpy(f[fin].copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        got = orc.decode_bf16(codes, s)[fin]
        assert np.array_equal(got, w)
    assert want.size > 0


# ---------------------------------------------------------------- TA pins
def test_ta_worked_example_from_paper():
    rows = [r for r in golden_lines("rounding_examples.txt") if "." in r[0] and len(r) == 3]
    assert len(rows) == 3
    # the example is about integers with ulp 1; HiF8 has ulp 1 in the binade [8, 16)
    for src, ta, te in rows:
        x = int(src.replace(".", ""), 2) / 2.0
        want = int(ta, 2)
        for sgn in (1.0, -1.0):
            c = orc.encode_one(sgn * (8.0 + x))
            assert orc.decode_value(c) == sgn * (8.0 + want)
        # and at ulp 2^-3 around 1.0
        c = orc.encode_one(1.0 + x / 8.0)
        assert orc.decode_value(c) == 1.0 + want / 8.0


def test_ta_matches_bit_level_rule_on_all_top13_patterns():
    top = np.arange(1 << 13, dtype=np.uint32) << 19
    rng = np.random.default_rng(1)
    fillers = [0, 1, 0x7FFFF, 0x40000, 0x3FFFF, 0x2000, 0x1FFF] + list(rng.integers(0, 1 << 19, 24))
    for fill in fillers:
        yb = top | np.uint32(fill)
        keep = ~np.isnan(bits_f32(yb))
        yb = yb[keep]
        got, codes = oracle_values_f32(yb, TA)
        want = closed_form_round(yb, TA, False)
        assert np.array_equal(got, want)
        # the TA code of a non-NaN binary32 value depends only on bits [31:19]
        base, base_codes = oracle_values_f32(yb & np.uint32(0xFFF80000), TA)
        assert np.array_equal(codes, base_codes)


def test_ta_matches_bit_level_rule_random_and_16bit_sources():
    rng = np.random.default_rng(2)
    yb = rng.integers(0, 2 ** 32, size=1 << 21, dtype=np.uint64).astype(np.uint32)
    yb = yb[~np.isnan(bits_f32(yb))]
    got, _ = oracle_values_f32(yb, TA)
    assert np.array_equal(got, closed_form_round(yb, TA, False))
    # all FP16 patterns widened, all BF16 patterns
    h = np.arange(65536, dtype=np.uint16).view(np.float16).astype(np.float32)
    hb = f32_bits(h)
    hb = hb[~np.isnan(h)]
    got, _ = oracle_values_f32(hb, TA)
    assert np.array_equal(got, closed_form_round(hb, TA, False))
    b = np.arange(65536, dtype=np.uint16)
    bb = b.astype(np.uint32) << 16
    ok = ~np.isnan(bits_f32(bb))
    codes = orc.encode_bf16(b[ok], 1.0, TA)
    assert np.array_equal(all_values()[codes], closed_form_round(bb[ok], TA, True))


def test_ta_is_nearest_with_ties_away_bruteforce():
    """Independent of any bit trick: for each x the result minimises |v - x| over the value
    set {finite values} + {+-1.5*2^15 standing for Inf}, and on an exact tie has the larger
    magnitude."""
    v = all_values()
    fin = np.sort(v[np.isfinite(v)])
    ext = np.concatenate([[-1.5 * 2 ** 15], fin, [1.5 * 2 ** 15]])
    rng = np.random.default_rng(3)
    x = np.concatenate([
        (rng.standard_normal(4000) * np.exp2(rng.uniform(-26, 17, 4000))).astype(np.float32),
        # exact midpoints and representable values
        ((ext[1:] + ext[:-1]) / 2).astype(np.float32),
        fin.astype(np.float32),
    ])
    x = x[np.abs(x) < 1.5 * 2 ** 15]
    codes = orc.encode_f32(x, 1.0, TA)
    q = v[codes]
    q = np.where(np.isinf(q), np.sign(q) * 1.5 * 2 ** 15, q)
    dist = np.abs(ext[None, :] - x[:, None].astype(np.float64))
    best = dist.min(axis=1)
    assert np.array_equal(np.abs(q - x.astype(np.float64)), best)
    # ties: two candidates at the same distance -> the one farther from zero
    tie = (dist == best[:, None]).sum(axis=1) == 2
    assert tie.sum() > 200
    cand = np.where(dist == best[:, None], np.abs(ext)[None, :], -1.0).max(axis=1)
    assert np.array_equal(np.abs(q[tie]), cand[tie])


def test_ta_error_at_most_half_ulp():
    rng = np.random.default_rng(4)
    x = (rng.standard_normal(1 << 18) * np.exp2(rng.uniform(-21, 14, 1 << 18))).astype(np.float32)
    x = x[(np.abs(x) >= 2.0 ** -22) & (np.abs(x) < 2.0 ** 15)]
    q = all_values()[orc.encode_f32(x, 1.0, TA)]
    E = np.floor(np.log2(np.abs(x.astype(np.float64)))).astype(np.int64)
    ulp = np.ldexp(1.0, E - kept_bits_of_exponent(E))
    assert np.all(np.abs(q - x) <= 0.5 * ulp)
    assert np.max(np.abs(q - x) / ulp) > 0.49


@pytest.mark.parametrize("mode", [TA, HR, TA | SAT, HR | SAT, TA | N2Z, HR | N2Z])
@pytest.mark.parametrize("src_bf16", [False, True])
def test_decode_encode_identity_all_codes(mode, src_bf16):
    v = all_values()
    for c in range(256):
        x = v[c]
        if src_bf16:
            got = orc.encode_bf16(np.array([np.float32(x)], np.float32).view(np.uint32)[:1].astype(np.uint32).__rshift__(16).astype(np.uint16), 1.0, mode)[0]
        else:
            got = orc.encode_f32(np.array([x], np.float32), 1.0, mode)[0]
        want = c
        if c == 0x80 and (mode & N2Z):
            want = 0x00
        if (c & 0x7F) == 0x6F and (mode & SAT):
            want = (c & 0x80) | 0x6E
        assert got == want, (hex(c), hex(got))


def test_specials_edges_and_options():
    e = orc.encode_one
    inf = float("inf")
    assert e(float("nan")) == 0x80 and e(float("nan"), TA | N2Z) == 0x00
    assert e(-float("nan")) == 0x80
    assert e(inf) == 0x6F and e(-inf) == 0xEF
    assert e(inf, TA | SAT) == 0x6E and e(-inf, TA | SAT) == 0xEE
    assert e(float("nan"), TA | SAT) == 0x80            # saturation leaves NaN alone
    assert e(inf, TA | N2Z) == 0x6F
    # overflow threshold: halfway between 2^15 and the Inf slot 1.5*2^15, tie away
    assert e(40960.0) == 0x6F and e(np.nextafter(np.float32(40960.0), np.float32(0))) == 0x6E
    assert e(40960.0, TA | SAT) == 0x6E and e(-1e30, TA | SAT) == 0xEE and e(-1e30) == 0xEF
    # underflow threshold: halfway between 0 and 2^-22, tie away
    assert e(2.0 ** -23) == 0x01 and e(np.nextafter(np.float32(2.0 ** -23), np.float32(0))) == 0x00
    # negative results of magnitude zero and -0.0 give the single zero pattern, never NaN's 0x80
    assert e(-0.0) == 0x00 and e(-1e-30) == 0x00 and e(-2.0 ** -24) == 0x00
    assert e(-2.0 ** -23) == 0x81
    # denormal range: pure powers of two, tie at 1.5 * 2^k goes up
    assert e(1.5 * 2.0 ** -20) == 0x04 and e(1.4999 * 2.0 ** -20) == 0x03
    assert e(1.5 * 2.0 ** -16) == 0x7E                   # crosses from denormal to normal
    # FP32 subnormal inputs
    assert e(1e-45) == 0x00 and e(-1e-40) == 0x00


def test_encode_is_odd_symmetric_except_zero():
    rng = np.random.default_rng(5)
    x = (rng.standard_normal(1 << 16) * np.exp2(rng.uniform(-30, 20, 1 << 16))).astype(np.float32)
    for mode in (TA, HR, TA | SAT):
        cp = orc.encode_f32(x, 1.0, mode)
        cn = orc.encode_f32(-x, 1.0, mode)
        nz = (cp & 0x7F) != 0
        assert np.array_equal(cp[nz] ^ 0x80, cn[nz])
        assert np.all(cn[~nz] == 0) and np.all(cp[~nz] == 0)


def test_deterministic_rounding_is_monotone():
    """Round-to-nearest cannot reorder values: for x <= y the TA (and saturating TA) results satisfy Q(x) <= Q(y),
    on random inputs over every binade and on a fine sweep across every boundary between two bands of the format
    (powers of two where the mantissa width changes, the denormal range, underflow and overflow).  A misplaced band
    boundary, a wrong mantissa width for one exponent or a carry that lands in the wrong exponent breaks it."""
    rng = np.random.default_rng(61)
    x = (rng.standard_normal(1 << 17) * np.exp2(rng.uniform(-30, 20, 1 << 17))).astype(np.float32)
    edges = np.array([2.0 ** e for e in range(-26, 18)], np.float32)
    fine = (edges[:, None] * np.linspace(0.75, 1.5, 193, dtype=np.float32)[None, :]).reshape(-1)
    allx = np.sort(np.concatenate([x, fine, -fine, np.array([0.0], np.float32)]))
    for mode in (TA, TA | SAT):
        v = orc.decode_f32(orc.encode_f32(allx, 1.0, mode), 1.0).astype(np.float64)
        assert not np.any(np.isnan(v))
        assert np.all(v[1:] >= v[:-1]), mode


def test_fake_quant_is_composition_and_idempotent():
    rng = np.random.default_rng(6)
    x = (rng.standard_normal(1 << 16) * np.exp2(rng.uniform(-25, 16, 1 << 16))).astype(np.float32)
    for s in (np.float32(1.0), np.float32(8.0), np.float32(0.37)):
        fq, codes = orc.fake_quant_f32(x, s, TA)
        assert np.array_equal(codes, orc.encode_f32(x, s, TA))
        assert np.array_equal(fq.view(np.uint32), orc.decode_f32(codes, s).view(np.uint32))
    fq, _ = orc.fake_quant_f32(x, 1.0, TA)
    fq2, _ = orc.fake_quant_f32(fq, 1.0, TA)
    assert np.array_equal(fq.view(np.uint32), fq2.view(np.uint32))
    # scaled encode = plain encode of the binary32 product
    s = np.float32(0.37)
    assert np.array_equal(orc.encode_f32(x, s, TA), orc.encode_f32((x * s).astype(np.float32), 1.0, TA))
    xb = (f32_bits(x) >> 16).astype(np.uint16)
    xw = (xb.astype(np.uint32) << 16).view(np.float32)
    assert np.array_equal(orc.encode_bf16(xb, s, TA), orc.encode_f32((xw * s).astype(np.float32), 1.0, TA))


# ---------------------------------------------------------------- SR / HR pins
def test_hr_equals_ta_inside_and_sr_outside_switch():
    """Eq. (3): |E| < 4 -> TA.  Outside, results are lo/hi of the same bracket."""
    rng = np.random.default_rng(8)
    yb = rng.integers(0, 2 ** 32, size=1 << 20, dtype=np.uint64).astype(np.uint32)
    yb = yb[~np.isnan(bits_f32(yb))]
    E = ((yb >> 23) & 0xFF).astype(np.int64) - 127
    inside = np.abs(E) < 4
    ta = orc.encode_f32(bits_f32(yb), 1.0, TA)
    hr = orc.encode_f32(bits_f32(yb), 1.0, HR)
    assert np.array_equal(ta[inside], hr[inside])
    assert np.any(ta[~inside] != hr[~inside])
    # boundaries of the switch: 2^-3 and just below 2^4 are TA; 2^4 and just below 2^-3 are SR
    x = np.array([15.9999], np.float32)
    assert orc.encode_f32(x, 1.0, HR)[0] == orc.encode_f32(x, 1.0, TA)[0]


def test_sr14_matches_bit_level_rule():
    rng = np.random.default_rng(9)
    yb = rng.integers(0, 2 ** 32, size=1 << 21, dtype=np.uint64).astype(np.uint32)
    # concentrate half of them where the format lives
    ex = rng.integers(127 - 40, 127 + 18, size=yb.size).astype(np.uint32)
    yb[::2] = (yb[::2] & np.uint32(0x807FFFFF)) | (ex[::2] << 23)
    # and force small thresholds / fractions often
    yb[::8] &= np.uint32(0xFFFFC000)
    yb[1::8] &= np.uint32(0xFFFF0000)
    yb = yb[~np.isnan(bits_f32(yb))]
    got, _ = oracle_values_f32(yb, HR)
    want = closed_form_round(yb, HR, False)
    assert np.array_equal(got, want)


def test_sr2_matches_bit_level_rule_all_bf16_patterns_and_scaled():
    b = np.arange(65536, dtype=np.uint16)
    bb = b.astype(np.uint32) << 16
    ok = ~np.isnan(bits_f32(bb))
    codes = orc.encode_bf16(b[ok], 1.0, HR)
    assert np.array_equal(all_values()[codes], closed_form_round(bb[ok], HR, True))
    # non-power-of-two scale: SR2 is applied to the binary32 product's bits
    s = np.float32(0.37)
    prod = (bits_f32(bb[ok]) * s).astype(np.float32)
    codes = orc.encode_bf16(b[ok], s, HR)
    assert np.array_equal(all_values()[codes], closed_form_round(f32_bits(prod), HR, True))


def test_sr2_thresholds_and_max_error():
    g = {r[0]: r[1:] for r in golden_lines("rounding_examples.txt") if r[0].startswith("sr")}
    want_thr = sorted(float(t) for t in g["sr2_thresholds"])
    want_err = float(g["sr2_max_error_ulp"][0])
    v = all_values()
    thr_seen = set()
    max_err = 0.0
    # every BF16 pattern in the SR range of HR with |E| in [4, 15] (normal bands, k = 2 or 1)
    b = np.arange(65536, dtype=np.uint16)
    x = (b.astype(np.uint32) << 16).view(np.float32)
    E = ((b >> 7) & 0xFF).astype(np.int64) - 127
    sel = (np.abs(E) >= 4) & (np.abs(E) <= 15) & (np.abs(x) < 2.0 ** 15)
    b, x, E = b[sel], x[sel].astype(np.float64), E[sel]
    q = v[orc.encode_bf16(b, 1.0, HR)]
    k = kept_bits_of_exponent(E)
    ulp = np.ldexp(1.0, E - k)
    lo = np.floor(np.abs(x) / ulp) * ulp
    frac = (np.abs(x) - lo) / ulp
    up = np.abs(q) > lo
    err = np.abs(np.abs(q) - np.abs(x)) / ulp
    assert np.all(np.isfinite(q))
    max_err = err.max()
    assert max_err == want_err                       # attained exactly, never exceeded
    for lsb in (0, 1):
        s = (b & 1) == lsb
        # a clean threshold: exactly one of the two printed values explains every decision
        fits = [t for t in want_thr if np.array_equal(up[s], frac[s] >= t)]
        assert len(fits) == 1
        thr_seen.add(fits[0])
    assert sorted(thr_seen) == want_thr
    assert not np.any(up & (frac == 0))              # representable values stay


def test_sr14_mean_preservation_and_error_bound():
    """E[Q(x)] = x when the threshold bits are uniform (Sec. 3.2), and |Q(x) - x| < 1 ulp."""
    v = all_values()
    rng = np.random.default_rng(10)
    for E, k in [(5, 2), (-6, 2), (10, 1), (-12, 1), (-18, 0)]:
        d = 23 - k
        # all 2^14 threshold patterns, each with random upper discarded bits
        low = np.arange(1 << 14, dtype=np.uint32)
        for trial in range(4):
            upper = np.uint32(rng.integers(0, 1 << (d - 14)))
            keep = np.uint32(rng.integers(0, 1 << k)) if k else np.uint32(0)
            m = (keep << d) | (upper << 14) | low
            yb = (np.uint32(E + 127) << 23) | m
            x = bits_f32(yb).astype(np.float64)
            q = v[orc.encode_f32(bits_f32(yb), 1.0, HR)]
            ulp = 2.0 ** (E - k)
            assert np.all(np.abs(q - x) < ulp)
            assert abs(np.mean(q - x)) / ulp < 2.0 ** -6
    # over fully random discarded bits the mean error is tiny compared to TA's worst case
    yb = (np.uint32(127 + 9) << 23) | rng.integers(0, 1 << 23, size=1 << 20).astype(np.uint32)
    x = bits_f32(yb).astype(np.float64)
    q = v[orc.encode_f32(bits_f32(yb), 1.0, HR)]
    assert abs(np.mean(q - x)) / 2.0 ** 8 < 2e-3


def test_sr_literal_zero_switch_is_the_only_difference():
    """The no-carry-at-F=T=0 reading changes results only where the literal rule would move
    an exactly representable input, or lift a value below 2^-36 (fraction F = 0) to 2^-22."""
    rng = np.random.default_rng(11)
    yb = rng.integers(0, 2 ** 32, size=1 << 18, dtype=np.uint64).astype(np.uint32)
    yb[::4] &= np.uint32(0xFFE00000)
    yb = yb[~np.isnan(bits_f32(yb))]
    x = bits_f32(yb)
    a = orc.encode_f32(x, 1.0, HR)
    orc.set_literal_sr_zero(True)
    try:
        lit = orc.encode_f32(x, 1.0, HR)
    finally:
        orc.set_literal_sr_zero(False)
    diff = a != lit
    assert diff.any()
    v = all_values()
    xd = x[diff].astype(np.float64)
    tiny = np.abs(xd) < 2.0 ** -36
    assert np.all(v[a[diff]][tiny] == 0.0)
    assert np.array_equal(v[a[diff]][~tiny], xd[~tiny])             # input was representable
    assert (~tiny).sum() > 100 and tiny.sum() > 100


# ---------------------------------------------------------------- amax / scale pins
def test_amax_and_scale():
    rng = np.random.default_rng(12)
    x = (rng.standard_normal(100001) * 3).astype(np.float32)
    assert orc.amax_f32(x) == np.max(np.abs(x))
    xb = (f32_bits(x) >> 16).astype(np.uint16)
    xw = (xb.astype(np.uint32) << 16).view(np.float32)
    assert orc.amax_bf16(xb) == np.max(np.abs(xw))
    assert orc.amax_f32(np.zeros(0, np.float32)) == 0.0
    x[17] = -np.inf
    assert np.isinf(orc.amax_f32(x))
    x[99] = np.nan
    assert np.isnan(orc.amax_f32(x))
    for am in [np.float32(0.1234), np.float32(5.5), np.float32(3e-5), np.float32(7e4)]:
        s = orc.scale_from_amax(am, 32768.0, False)
        assert s == np.float32(32768.0) / am
        p = orc.scale_from_amax(am, 32768.0, True)
        assert p <= s < 2 * p and math.frexp(float(p))[0] == 0.5
    for am in [np.float32(0), np.float32(np.inf), np.float32(np.nan)]:
        assert orc.scale_from_amax(am, 32768.0, False) == 1.0
