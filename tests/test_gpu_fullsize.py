"""GPU parity at the baseline's full sizes, in the launch configuration bench.py times.

Every element of every configuration is checked:
  * FP32      : the oracle encodes the whole tensor, in slices of 2^26 elements for the 2^30-element
                gradient tensor (under standard SR each slice with the index base its elements have
                inside the tensor), under every rounding method;
  * BF16      : the oracle evaluates all 65,536 source patterns at the tensor's scale and every
                element is compared through that table (exhaustive, the op is element-wise); amax
                comes from the oracle's own reduction over the tensor.
"""
import numpy as np
import pytest
import torch

from oracle import hif8_oracle as orc
from gpu_util import assert_same_bytes, bf16_bits, dev, f32_bits

pytestmark = pytest.mark.gpu
TA, HR, SAT = orc.RM_TA, orc.RM_HR, orc.FLAG_SAT


@pytest.fixture(scope="module")
def h():
    assert torch.cuda.is_available()
    from paper_2409_16626_amd import hif8
    hif8.hif8_init()
    return hif8


def bf16_tables(scale, mode):
    """Oracle results for every BF16 source pattern at one scale: codes and fake-quant output."""
    pats = np.arange(65536, dtype=np.uint16)
    out, codes = orc.fake_quant_bf16(pats, scale, mode)
    return (torch.from_numpy(codes.copy()).to(dev()),
            torch.from_numpy(out.view(np.int16).copy()).to(dev()))


def gather_bf16(table, x_bits_i16, chunk=1 << 27):
    """table[pattern] for every element, in chunks (torch indexing needs int64 indices)."""
    outs = []
    for lo in range(0, x_bits_i16.numel(), chunk):
        idx = x_bits_i16[lo:lo + chunk].to(torch.int64) & 0xFFFF
        outs.append(table[idx])
    return torch.cat(outs)


def test_c2_full(h):
    from paper_2409_16626_amd import workloads
    n = 1 << 26
    x = workloads.dynamic_range_sweep(n, dev())
    codes = torch.empty(n, dtype=torch.uint8, device=dev())
    xn = x.cpu().numpy()
    for mode in (TA, TA | SAT):
        h.hif8_encode_f32(x, codes, n, 1.0, mode)
        torch.cuda.synchronize()
        assert_same_bytes(codes.cpu().numpy(), orc.encode_f32(xn, 1.0, mode), "C2 full mode %#x" % mode)
    # the tie positions really are ties: about 1 % of the inputs have no bit below the rounding position
    assert np.mean((xn.view(np.uint32) & 0x7FFFF) == 0) > 0.009


def test_c3_full(h):
    from paper_2409_16626_amd import workloads
    x = workloads.activation_bf16(8192, 8192, dev()).view(-1)
    n = x.numel()
    am = torch.zeros(1, dtype=torch.float32, device=dev())
    sc = torch.zeros(2, dtype=torch.float32, device=dev())
    out = torch.empty_like(x)
    codes = torch.empty(n, dtype=torch.uint8, device=dev())
    h.hif8_amax_bf16(x, n, am)
    h.hif8_scale_from_amax(am, sc, 32768.0, 0)
    h.hif8_fake_quant_bf16_ds(x, out, codes, n, sc, TA)
    torch.cuda.synchronize()
    w_am = orc.amax_bf16(bf16_bits(x))
    assert am.item() == float(w_am)
    w_s = orc.scale_from_amax(w_am, 32768.0, False)
    assert sc[0].item() == float(w_s)
    t_codes, t_out = bf16_tables(w_s, TA)
    xi = x.view(torch.int16)
    assert torch.equal(codes, gather_bf16(t_codes, xi))
    assert torch.equal(out.view(torch.int16), gather_bf16(t_out, xi))
    assert w_am > 100.0          # the x100 outliers set the scale
    # the same recipe as one call (two launches): identical outputs
    ws = torch.empty(h.hif8_quantize_workspace_bytes(), dtype=torch.uint8, device=dev())
    am2 = torch.zeros_like(am); sc2 = torch.zeros_like(sc)
    out2 = torch.empty_like(x); codes2 = torch.empty_like(codes)
    h.hif8_quantize_tensor_bf16(x, out2, codes2, n, am2, sc2, ws, 32768.0, 0, TA)
    torch.cuda.synchronize()
    assert torch.equal(am, am2) and torch.equal(sc, sc2) and torch.equal(codes, codes2)
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16))


SLICE = 1 << 26


def check_c4_against_oracle(x, codes, mode, what):
    """Every element of the 2^30-element tensor: the oracle encodes slice after slice on the host."""
    n = x.numel()
    try:
        for lo in range(0, n, SLICE):
            orc.set_sr_index_base(lo)
            want = orc.encode_f32(x[lo:lo + SLICE].cpu().numpy(), 1.0, mode)
            assert_same_bytes(codes[lo:lo + SLICE].cpu().numpy(), want, "%s, slice at %d" % (what, lo))
    finally:
        orc.set_sr_index_base(0)


@pytest.mark.parametrize("mode", [TA, HR])
def test_c4_full(h, mode):
    from paper_2409_16626_amd import workloads
    n = 1 << 30
    x = workloads.gradient_f32(n, dev())
    codes = torch.empty(n, dtype=torch.uint8, device=dev())
    h.hif8_encode_f32(x, codes, n, 1.0, mode)
    torch.cuda.synchronize()
    check_c4_against_oracle(x, codes, mode, "C4 mode %d" % mode)
    assert not torch.isnan(x).any()
    # the bulk of the data sits in the denormal binades 2^-22 .. 2^-16 and a visible share underflows
    mag = codes[:SLICE] & 0x7F
    assert float(((mag >= 1) & (mag <= 7)).float().mean().item()) > 0.3
    assert 0.08 < float((codes[:SLICE] == 0).float().mean().item()) < 0.25


@pytest.mark.parametrize("mode", [orc.RM_TE, orc.RM_SSR, orc.RM_SR])
def test_c4_full_comparison_modes(h, mode):
    """The gradient tensor under the rounding methods the paper compares TA / HR with, every element
    against the oracle (standard SR: with the thresholds the elements have at their place in the
    2^30-element tensor)."""
    from paper_2409_16626_amd import workloads
    n = 1 << 30
    x = workloads.gradient_f32(n, dev())
    codes = torch.empty(n, dtype=torch.uint8, device=dev())
    seed = 0x1234ABCD5678
    h.hif8_set_sr_seed(seed)
    orc.set_sr_seed(seed)
    try:
        h.hif8_encode_f32(x, codes, n, 1.0, mode)
        torch.cuda.synchronize()
        check_c4_against_oracle(x, codes, mode, "C4 mode %d" % mode)
    finally:
        orc.set_sr_seed(0)
        h.hif8_set_sr_seed(0)
    z = codes[:SLICE][x[:SLICE] == 0]
    assert int(z.max().item()) == 0


def test_c5_full(h):
    from paper_2409_16626_amd import workloads
    arena, index = workloads.llm_weights_bf16(dev())
    assert len(index) == 225 and arena.numel() == 6607077376
    codes = torch.empty(arena.numel(), dtype=torch.uint8, device=dev())
    items = [(arena.data_ptr() + 2 * off, codes.data_ptr() + off, m) for _, off, m in index]
    plan = h.hif8_multi_plan(items, src_is_16bit=True)
    d_items, count, tiles = plan
    am = torch.zeros(count, dtype=torch.float32, device=dev())
    sc = torch.zeros(count, 2, dtype=torch.float32, device=dev())
    h.hif8_multi_cast_bf16(d_items, count, tiles, am, sc, 32768.0, 0, TA, host_items=plan.host_items)   # group-wise schedule
    torch.cuda.synchronize()
    amn, scn = am.cpu().numpy(), sc.cpu().numpy()
    ai = arena.view(torch.int16)
    for i, (name, off, m) in enumerate(index):
        part = ai[off:off + m]
        w_am = orc.amax_bf16(part.cpu().numpy().view(np.uint16))
        assert amn[i] == w_am, name
        w_s = orc.scale_from_amax(w_am, 32768.0, False)
        assert scn[i, 0] == w_s, name
        t_codes, _ = bf16_tables(w_s, TA)
        assert torch.equal(codes[off:off + m], gather_bf16(t_codes, part)), name
    # the four-launch form (no host copy of the plan) gives the same bytes
    codes4 = torch.empty_like(codes)
    items4 = [(arena.data_ptr() + 2 * off, codes4.data_ptr() + off, m) for _, off, m in index]
    plan4 = h.hif8_multi_plan(items4, src_is_16bit=True)
    am4 = torch.zeros_like(am); sc4 = torch.zeros_like(sc)
    h.hif8_multi_cast_bf16(plan4.d_items, plan4.count, plan4.total_tiles, am4, sc4, 32768.0, 0, TA)
    torch.cuda.synchronize()
    assert torch.equal(codes, codes4) and torch.equal(am, am4) and torch.equal(sc, sc4)
    del codes4
    # the per-tensor call sequence gives the same bytes (checked on the first and last tensors)
    for i in (0, 4, 224):
        _, off, m = index[i]
        c2 = torch.empty(m, dtype=torch.uint8, device=dev())
        a1 = torch.zeros(1, dtype=torch.float32, device=dev())
        s2 = torch.zeros(2, dtype=torch.float32, device=dev())
        h.hif8_amax_bf16(arena.data_ptr() + 2 * off, m, a1)
        h.hif8_scale_from_amax(a1, s2, 32768.0, 0)
        h.hif8_encode_bf16_ds(arena.data_ptr() + 2 * off, c2, m, s2, TA)
        torch.cuda.synchronize()
        assert torch.equal(c2, codes[off:off + m])


@pytest.mark.parametrize("mode", [TA, HR])
def test_quantize_rows_weight_matrix_full(h, mode):
    """Per-row scaling of a [11008, 4096] BF16 weight matrix (the shape bench.py times) in one pass:
    every amax, scale pair and code against the oracle's amax -> scale -> cast composition."""
    rows, cols = 11008, 4096
    g = torch.Generator(device=dev()).manual_seed(4096)
    w = (torch.randn(rows, cols, generator=g, device=dev()) * 0.02
         * torch.exp2(torch.rand((rows, 1), generator=g, device=dev()) * 6 - 3)).to(torch.bfloat16)
    am = torch.zeros(rows, dtype=torch.float32, device=dev())
    sc = torch.zeros(rows, 2, dtype=torch.float32, device=dev())
    codes = torch.zeros(rows, cols, dtype=torch.uint8, device=dev())
    h.hif8_quantize_rows_bf16(w, codes, rows, cols, am, sc, 32768.0, 1, mode)
    torch.cuda.synchronize()
    wn = bf16_bits(w)
    w_am = orc.amax_axis(wn, orc.SRC_BF16, 0)
    assert_same_bytes(f32_bits(am), w_am.view(np.uint32), "amax")
    w_sc = np.array([orc.scale_from_amax(a, 32768.0, True) for a in w_am], np.float32)
    scn = sc.cpu().numpy()
    assert np.array_equal(scn[:, 0], w_sc) and np.array_equal(scn[:, 1], np.float32(1.0) / w_sc)
    want = orc.encode_axis(wn, w_sc, orc.SRC_BF16, 0, mode)
    assert_same_bytes(codes.cpu().numpy().reshape(-1), want.reshape(-1), "codes")
