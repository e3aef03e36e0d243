"""CPU build of the HIP library's device bit logic, checked against the oracle (no GPU).

The header with the device functions is compiled for the host with g++ through a small
shim (tests/devfn_host).  This is not the parity test proper (that one runs the kernels
on the GPU through the C ABI); it checks the integer encode / decode logic the kernels
are built from on every binary32 top-13-bit pattern, every 16-bit source pattern and
random patterns, under every rounding method and option.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest

from oracle import hif8_oracle as orc

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "devfn_host", "devfn_host.cpp")
HDR = os.path.join(HERE, "..", "paper_2409_16626_amd", "csrc", "hif8_device.hpp")
HDR2 = os.path.join(HERE, "..", "paper_2409_16626_amd", "csrc", "hif8_gemm_split.hpp")
LIB = os.path.join(HERE, "devfn_host", "libdevfn_host.so")


@pytest.fixture(scope="module")
def dev():
    newest = max(os.path.getmtime(SRC), os.path.getmtime(HDR), os.path.getmtime(HDR2))
    if not os.path.exists(LIB) or os.path.getmtime(LIB) < newest:
        subprocess.run(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-o", LIB, SRC], check=True)
    lib = ctypes.CDLL(LIB)
    return lib


def _enc(lib, ybits, mode, srck, seed=0):
    ybits = np.ascontiguousarray(ybits, np.uint32)
    out = np.empty(ybits.shape, np.uint8)
    lib.devfn_encode_bits(ybits.ctypes.data_as(ctypes.c_void_p), out.ctypes.data_as(ctypes.c_void_p),
                          ctypes.c_size_t(ybits.size), ctypes.c_uint32(mode), ctypes.c_int(srck),
                          ctypes.c_uint64(seed))
    if (mode & 0xF) in (orc.RM_HR, orc.RM_SSR):
        # the streaming kernels' table-driven forms must agree with the generic form
        out2 = np.empty(ybits.shape, np.uint8)
        if srck == 0:
            lib.devfn_encode_bits_hr_table(ybits.ctypes.data_as(ctypes.c_void_p), out2.ctypes.data_as(ctypes.c_void_p),
                                           ctypes.c_size_t(ybits.size), ctypes.c_uint32(mode))
        else:
            # 16-bit sources: the clamped sum looked up in the truncating table
            lib.devfn_encode_bits_hr16_stream(ybits.ctypes.data_as(ctypes.c_void_p), out2.ctypes.data_as(ctypes.c_void_p),
                                              ctypes.c_size_t(ybits.size), ctypes.c_uint32(mode), ctypes.c_int(srck))
        bad = np.nonzero(out != out2)[0]
        assert bad.size == 0, [(hex(ybits[i]), hex(out[i]), hex(out2[i])) for i in bad[:8]]
    if (mode & 0xF) == orc.RM_SR:
        # the streaming kernels' add-and-truncate form of standard SR must agree as well
        out2 = np.empty(ybits.shape, np.uint8)
        lib.devfn_encode_bits_sr_table(ybits.ctypes.data_as(ctypes.c_void_p), out2.ctypes.data_as(ctypes.c_void_p),
                                       ctypes.c_size_t(ybits.size), ctypes.c_uint32(mode), ctypes.c_uint64(seed))
        bad = np.nonzero(out != out2)[0]
        assert bad.size == 0, [(hex(ybits[i]), hex(out[i]), hex(out2[i])) for i in bad[:8]]
    return out


MODES = [orc.RM_TA, orc.RM_HR, orc.RM_TA | orc.FLAG_SAT, orc.RM_HR | orc.FLAG_SAT,
         orc.RM_TA | orc.FLAG_NAN2ZERO, orc.RM_HR | orc.FLAG_SAT | orc.FLAG_NAN2ZERO,
         orc.RM_TE, orc.RM_SSR, orc.RM_SR, orc.RM_TE | orc.FLAG_SAT, orc.RM_SR | orc.FLAG_SAT | orc.FLAG_NAN2ZERO]


@pytest.mark.parametrize("mode", MODES)
def test_device_encode_logic_f32(dev, mode):
    rng = np.random.default_rng(21)
    top = np.arange(1 << 13, dtype=np.uint32) << 19
    parts = [top, top | np.uint32(0x7FFFF), top | np.uint32(1), top | np.uint32(0x2000),
             top | rng.integers(0, 1 << 19, size=top.size).astype(np.uint32)]
    yb = rng.integers(0, 2 ** 32, size=1 << 20, dtype=np.uint64).astype(np.uint32)
    ex = rng.integers(127 - 40, 127 + 18, size=yb.size).astype(np.uint32)
    yb[::2] = (yb[::2] & np.uint32(0x807FFFFF)) | (ex[::2] << 23)
    yb[::8] &= np.uint32(0xFFFFC000)
    h = np.arange(65536, dtype=np.uint16).view(np.float16).astype(np.float32).view(np.uint32)
    allb = np.concatenate(parts + [yb, h])
    allb[5::16] &= np.uint32(0xFFF80000)      # exact ties and representable values for TE
    orc.set_sr_seed(0xABCDEF0123)
    try:
        want = orc.encode_f32(allb.view(np.float32), 1.0, mode)
    finally:
        orc.set_sr_seed(0)
    got = _enc(dev, allb, mode, 0, 0xABCDEF0123)
    bad = np.nonzero(want != got)[0]
    assert bad.size == 0, [(hex(allb[i]), hex(want[i]), hex(got[i])) for i in bad[:8]]


@pytest.mark.parametrize("mode", MODES)
def test_device_encode_logic_bf16(dev, mode):
    b = np.arange(65536, dtype=np.uint16)
    for scale in (np.float32(1.0), np.float32(0.37), np.float32(1311.7), np.float32(2.0 ** -20)):
        prod = ((b.astype(np.uint32) << 16).view(np.float32) * scale).astype(np.float32)
        want = orc.encode_bf16(b, scale, mode)
        got = _enc(dev, prod.view(np.uint32), mode, 1)
        bad = np.nonzero(want != got)[0]
        assert bad.size == 0, [(hex(b[i]), hex(want[i]), hex(got[i])) for i in bad[:8]]


@pytest.mark.parametrize("mode", MODES)
def test_device_encode_logic_f16(dev, mode):
    h = np.arange(65536, dtype=np.uint16)
    for scale in (np.float32(1.0), np.float32(0.37), np.float32(2.0 ** -9)):
        prod = (h.view(np.float16).astype(np.float32) * scale).astype(np.float32)
        want = orc.encode_f16(h, scale, mode)
        got = _enc(dev, prod.view(np.uint32), mode, 2)
        bad = np.nonzero(want != got)[0]
        assert bad.size == 0, [(hex(h[i]), hex(want[i]), hex(got[i])) for i in bad[:8]]


def test_device_decode_logic(dev):
    codes = np.arange(256, dtype=np.uint8)
    out = np.empty(256, np.uint32)
    dev.devfn_decode_bits(codes.ctypes.data_as(ctypes.c_void_p), out.ctypes.data_as(ctypes.c_void_p),
                          ctypes.c_size_t(256))
    assert np.array_equal(out, orc.decode_f32(codes, 1.0).view(np.uint32))


def test_device_narrow_logic(dev):
    rng = np.random.default_rng(22)
    u = rng.integers(0, 2 ** 32, size=1 << 18, dtype=np.uint64).astype(np.uint32)
    u[::7] = (u[::7] & np.uint32(0xFFFF0000)) | np.uint32(0x8000)
    out = np.empty(u.shape, np.uint16)
    dev.devfn_narrow_bf16(u.ctypes.data_as(ctypes.c_void_p), out.ctypes.data_as(ctypes.c_void_p),
                          ctypes.c_size_t(u.size))
    assert np.array_equal(out, orc.narrow_bf16(u.view(np.float32)))


def test_device_scale_from_amax_logic(dev):
    """The scale arithmetic of the scale kernels (fl32(target / amax), optional floor to a power of two,
    degenerate amax -> 1) against the oracle, bit for bit, on special values and random patterns."""
    rng = np.random.default_rng(23)
    special = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1e-45, 1.1754944e-38, 3.4028235e38, 1.0, 32768.0, 32767.99,
                        5e-39, 2.5e-41, 3.0e33, 6.1e-5], np.float32)
    rnd = rng.integers(0, 2 ** 31, size=200000, dtype=np.int64).astype(np.uint32).view(np.float32)   # non-negative patterns
    amax = np.concatenate([special, rnd, np.exp2(rng.uniform(-40, 40, 50000)).astype(np.float32)])
    out = np.empty(amax.shape, np.float32)
    for target in (32768.0, 1.0, 448.0, 3.0e38, 1e-30):
        for pow2 in (0, 1):
            dev.devfn_scale_from_amax(amax.ctypes.data_as(ctypes.c_void_p), out.ctypes.data_as(ctypes.c_void_p),
                                      ctypes.c_size_t(amax.size), ctypes.c_float(target), ctypes.c_int(pow2))
            want = np.array([orc.scale_from_amax(a, target, bool(pow2)) for a in amax[:2000]], np.float32)
            assert np.array_equal(out[:2000].view(np.uint32), want.view(np.uint32)), (target, pow2)
            assert np.all(out > 0) and np.all(np.isfinite(out))
            if pow2:      # a power of two: empty mantissa field, or (subnormal) a single mantissa bit
                b = out.view(np.uint32)
                normal = (b >> 23) != 0
                assert np.all((b[normal] & 0x7FFFFF) == 0)
                sub = b[~normal]
                assert np.all((sub & (sub - 1)) == 0)


def test_gemm_ragged_round_split_plan(dev):
    """Host-side planning of the GEMM launches: a second launch of small tiles only where the last round of
    256 x 256 tiles would be at most half full and whole tile columns fill the complete rounds; the split
    column is a multiple of 256 inside the matrix and the large tiles left of it fill whole rounds or less."""
    dev.devfn_ragged_round_split.restype = ctypes.c_uint32
    dev.devfn_ragged_round_split.argtypes = [ctypes.c_size_t, ctypes.c_size_t, ctypes.c_size_t]
    f = dev.devfn_ragged_round_split
    assert f(8192, 11008, 256) == 40 * 256            # 32 x 43 tiles = 5.375 rounds: 40 tile columns = 5 rounds exactly
    assert f(8192, 8192, 256) == 0                    # 1024 tiles = 4 whole rounds
    assert f(4096, 4096, 256) == 0                    # one round exactly
    assert f(2048, 2048, 256) == 0                    # fewer tiles than compute units
    assert f(8192, 11008, 0) == 0
    assert f(8192, 12288, 256) == 0                   # 6 rounds exactly
    assert f(8192, 12800, 256) == 48 * 256            # 32 x 50 = 6.25 rounds
    assert f(8192, 14336, 256) == 0                   # 7 rounds exactly
    assert f(8192, 15000, 256) == 56 * 256            # 32 x 59 = 7.4 rounds: 3 tile columns left = 96 tiles
    assert f(8192, 16000, 256) == 0                   # 32 x 63 = 7.9 rounds: the last round is nearly full
    rng = np.random.default_rng(3)
    for _ in range(2000):
        M, N, cus = int(rng.integers(1, 40000)), int(rng.integers(1, 40000)), int(rng.choice([64, 120, 256, 304]))
        s = f(M, N, cus)
        tm, tn = (M + 255) // 256, (N + 255) // 256
        if s:
            assert s % 256 == 0 and 0 < s < N
            big = tm * (s // 256)
            assert big <= (tm * tn // cus) * cus                  # the large tiles fit the complete rounds
            assert (tn - s // 256) * tm * 2 <= cus                # what is left is at most half a round of large tiles
            assert tm * tn > cus and (tm * tn) % cus != 0


def test_gemm_tile_order_is_a_bijection_and_compact_per_die(dev):
    """Workgroup -> tile of the expanded-operand GEMM: every tile is taken exactly once, only workgroups at the
    end of the grid go without one, and the 32 workgroups that run together on one die (b = die + 8 s for 32
    consecutive s) touch few operand panels: at most 8 tile rows and, for full groups, 4 to 5 tile columns."""
    dev.devfn_tile_order.restype = ctypes.c_uint32
    dev.devfn_tile_order.argtypes = [ctypes.c_uint32] * 3
    dev.devfn_tile_order_grid.restype = ctypes.c_uint32
    dev.devfn_tile_order_grid.argtypes = [ctypes.c_uint32]
    for tm, tn in [(1, 1), (1, 7), (3, 5), (8, 4), (32, 32), (32, 43), (16, 16), (9, 100), (100, 9), (13, 1), (64, 3)]:
        n = tm * tn
        grid = dev.devfn_tile_order_grid(n)
        assert grid % 8 == 0 and n <= grid < n + 8
        got = np.array([dev.devfn_tile_order(b, tm, tn) for b in range(grid)], np.int64)
        have = got[got != 0xFFFFFFFF]
        assert np.array_equal(np.sort(have), np.arange(n))
        assert len(have) == n
    # one round of 256 workgroups on the 32 x 43 tiles of the 8192 x 11008 product: panels per die
    tm, tn = 32, 43
    for die in range(8):
        tiles = [dev.devfn_tile_order(die + 8 * s, tm, tn) for s in range(32)]
        rows = {t // tn for t in tiles}
        cols = {t % tn for t in tiles}
        assert len(rows) <= 8 and len(cols) <= 5, (die, sorted(rows), sorted(cols))
