"""Every binary32 pattern: hif8_encode_f32 at scale 1 against the oracle on all 2^32 inputs, for TA
(Sec. 3.1), hybrid rounding with SR14 (Sec. 3.2, Eq. (3): the threshold is the low 14 bits of the
input, so all of them occur with every kept pattern), the options, and the comparison modes TE,
simplified SR in every binade and standard SR (threshold drawn per element index).  Bit-exact.

The patterns are produced in 16 chunks of 2^28 (consecutive integers reinterpreted as floats) on
both sides; the oracle takes well under a second per chunk on the host cores of a GPU machine.
"""
import numpy as np
import pytest
import torch

from oracle import hif8_oracle as orc
from gpu_util import dev

pytestmark = pytest.mark.gpu

CHUNK = 1 << 28


@pytest.fixture(scope="module")
def h():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2409_16626_amd import hif8
    hif8.hif8_init()
    return hif8


@pytest.mark.parametrize("mode", [orc.RM_TA, orc.RM_HR, orc.RM_TA | orc.FLAG_SAT | orc.FLAG_NAN2ZERO,
                                  orc.RM_HR | orc.FLAG_SAT, orc.RM_TE, orc.RM_SSR, orc.RM_SR],
                         ids=["TA", "HR", "TA+SAT+NAN2ZERO", "HR+SAT", "TE", "SSR", "SR"])
def test_every_binary32_pattern(h, mode):
    seed = 0x5EED0123456789
    h.hif8_set_sr_seed(seed)
    orc.set_sr_seed(seed)
    try:
        _run_all_patterns(h, mode)
    finally:
        h.hif8_set_sr_seed(0)
        orc.set_sr_seed(0)
        orc.set_sr_index_base(0)


def _run_all_patterns(h, mode):
    codes = torch.empty(CHUNK, dtype=torch.uint8, device=dev())
    for start in range(0, 1 << 32, CHUNK):
        x = torch.arange(start, start + CHUNK, dtype=torch.int64, device=dev()).to(torch.int32).view(torch.float32)
        h.hif8_encode_f32(x, codes, CHUNK, 1.0, mode)
        got = codes.cpu().numpy()                                      # synchronises
        del x
        bits = np.arange(start, start + CHUNK, dtype=np.uint32)
        orc.set_sr_index_base(0)                                       # each chunk is a call of its own on both sides
        want = orc.encode_f32(bits.view(np.float32), 1.0, mode)
        if not np.array_equal(got, want):
            bad = np.nonzero(got != want)[0]
            raise AssertionError("%d mismatches in chunk %#x; first: pattern %#010x got %#04x want %#04x" % (
                bad.size, start, int(bits[bad[0]]), int(got[bad[0]]), int(want[bad[0]])))


@pytest.mark.parametrize("scale,mode", [(0.37, orc.RM_TA), (2.0 ** -7, orc.RM_HR)], ids=["TA scale 0.37", "HR scale 2^-7"])
def test_fake_quant_every_binary32_pattern_scaled(h, scale, mode):
    """The fused round trip with a scale on all 2^32 inputs: the scale multiply, the cast, the decode
    and the descale multiply; outputs compared as raw bit patterns (0 ulp), codes bit for bit."""
    codes = torch.empty(CHUNK, dtype=torch.uint8, device=dev())
    out = torch.empty(CHUNK, dtype=torch.float32, device=dev())
    for start in range(0, 1 << 32, CHUNK):
        x = torch.arange(start, start + CHUNK, dtype=torch.int64, device=dev()).to(torch.int32).view(torch.float32)
        h.hif8_fake_quant_f32(x, out, codes, CHUNK, scale, mode)
        got_c = codes.cpu().numpy()
        got_o = out.view(torch.int32).cpu().numpy().view(np.uint32)
        del x
        bits = np.arange(start, start + CHUNK, dtype=np.uint32)
        want_o, want_c = orc.fake_quant_f32(bits.view(np.float32), scale, mode)
        assert np.array_equal(got_c, want_c), "codes differ in chunk %#x" % start
        if not np.array_equal(got_o, want_o.view(np.uint32)):
            bad = np.nonzero(got_o != want_o.view(np.uint32))[0]
            raise AssertionError("%d output mismatches in chunk %#x; first: pattern %#010x got %#010x want %#010x" % (
                bad.size, start, int(bits[bad[0]]), int(got_o[bad[0]]), int(want_o.view(np.uint32)[bad[0]])))
