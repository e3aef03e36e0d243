"""GPU parity for the comparison rounding modes (TE, simplified SR in every binade, standard
SR with the counter-based threshold) and for FP16 tensors, against the CPU oracle.

Bars as everywhere: u8 codes bit-exact, FP32 / BF16 / FP16 outputs as raw bit patterns.
"""
import numpy as np
import pytest
import torch

from oracle import hif8_oracle as orc
from gpu_util import assert_same_bytes, bf16_bits, dev, f32_bits, to_gpu

pytestmark = pytest.mark.gpu

TA, HR, TE, SSR, SR = orc.RM_TA, orc.RM_HR, orc.RM_TE, orc.RM_SSR, orc.RM_SR
SAT, N2Z = orc.FLAG_SAT, orc.FLAG_NAN2ZERO
NEW_MODES = [TE, SSR, SR, TE | SAT, SSR | N2Z, SR | SAT | N2Z]
ALL_RM = [TA, HR, TE, SSR, SR]
SEED = 0x5EED0123456789


@pytest.fixture(scope="module")
def h():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2409_16626_amd import hif8
    hif8.hif8_init()
    return hif8


@pytest.fixture(autouse=True)
def seeds(h):
    """Same standard-SR seed on both sides for the duration of a test."""
    h.hif8_set_sr_seed(SEED)
    orc.set_sr_seed(SEED)
    yield
    h.hif8_set_sr_seed(0)
    orc.set_sr_seed(0)


def f16_bits(t):
    if t.dtype == torch.float16:
        t = t.view(torch.int16)
    return t.cpu().numpy().view(np.uint16)


def enc(h, kind, x, scale, mode):
    dst = torch.empty(x.numel(), dtype=torch.uint8, device=dev())
    getattr(h, "hif8_encode_" + kind)(x, dst, x.numel(), scale, mode)
    torch.cuda.synchronize()
    return dst.cpu().numpy()


def test_threshold_generator_matches_the_oracle(h):
    rng = np.random.default_rng(3)
    for seed in (0, 1, SEED, 2 ** 64 - 1):
        for idx in [0, 1, 2 ** 32 - 1, 2 ** 32, 2 ** 40 + 17] + rng.integers(0, 2 ** 63, 50).tolist():
            assert h.hif8_sr_threshold(seed, idx) == orc.sr_threshold(seed, idx)
    assert h.hif8_get_sr_seed() == SEED


# ------------------------------------------------------------------ FP32 sources, new modes
@pytest.mark.parametrize("mode", NEW_MODES)
def test_f32_all_fp16_patterns_and_top13(h, mode):
    from paper_2409_16626_amd import workloads
    x = workloads.all_fp16_as_f32(dev())
    assert_same_bytes(enc(h, "f32", x, 1.0, mode), orc.encode_f32(x.cpu().numpy(), 1.0, mode), "fp16 pats")
    rng = np.random.default_rng(31)
    top = np.arange(1 << 13, dtype=np.uint32) << 19
    yb = np.concatenate([top, top | np.uint32(0x7FFFF), top | np.uint32(1), top | np.uint32(0x40000),
                         top | rng.integers(0, 1 << 19, size=top.size).astype(np.uint32)])
    xg = to_gpu(yb).view(torch.float32)
    assert_same_bytes(enc(h, "f32", xg, 1.0, mode), orc.encode_f32(yb.view(np.float32), 1.0, mode), "top13")


@pytest.mark.parametrize("mode", NEW_MODES)
def test_f32_dynamic_range_and_gradient(h, mode):
    from paper_2409_16626_amd import workloads
    x = workloads.dynamic_range_sweep((1 << 21) + 3, dev())
    assert_same_bytes(enc(h, "f32", x, 1.0, mode), orc.encode_f32(x.cpu().numpy(), 1.0, mode), "C2 small")
    g = workloads.gradient_f32((1 << 20) + 1, dev(), chunk=1 << 20)
    assert_same_bytes(enc(h, "f32", g, 1.0, mode), orc.encode_f32(g.cpu().numpy(), 1.0, mode), "C4 small")
    assert_same_bytes(enc(h, "f32", g, 3.7e3, mode), orc.encode_f32(g.cpu().numpy(), 3.7e3, mode), "C4 scaled")


def test_te_differs_from_ta_only_at_ties_and_sr_is_seeded(h):
    from paper_2409_16626_amd import workloads
    x = workloads.dynamic_range_sweep(1 << 20, dev())
    ta, te = enc(h, "f32", x, 1.0, TA), enc(h, "f32", x, 1.0, TE)
    diff = np.nonzero(ta != te)[0]
    assert 0 < diff.size < x.numel() // 50
    assert np.all((x.cpu().numpy().view(np.uint32)[diff] & 0x7FFFF) == 0)
    a = enc(h, "f32", x, 1.0, SR)
    h.hif8_set_sr_seed(SEED + 1)
    b = enc(h, "f32", x, 1.0, SR)
    h.hif8_set_sr_seed(SEED)
    c = enc(h, "f32", x, 1.0, SR)
    assert np.array_equal(a, c) and not np.array_equal(a, b)


@pytest.mark.parametrize("n", [0, 1, 5, 8, 9, 4097, (1 << 18) + 13])
def test_ragged_and_unaligned_new_modes(h, n):
    """The vector path, its ragged tail and the element-per-lane path give element i the same
    threshold (index within the tensor of the call)."""
    from paper_2409_16626_amd import workloads
    big = workloads.dynamic_range_sweep((1 << 18) + 64, dev())
    bigb = big.to(torch.bfloat16)
    bigh = (big * 2.0 ** -6).to(torch.float16)
    for off in (0, 1):
        x, xb, xh = big[off:off + n], bigb[off:off + n], bigh[off:off + n]
        xn = x.contiguous().cpu().numpy()
        xbn, xhn = bf16_bits(xb.contiguous()), f16_bits(xh.contiguous())
        codes = torch.zeros(n + 16, dtype=torch.uint8, device=dev())[off:off + n]
        for mode in (TE, SSR, SR | SAT):
            for scale in (1.0, 3.3):
                h.hif8_encode_f32(x.data_ptr(), codes.data_ptr(), n, scale, mode)
                torch.cuda.synchronize()
                assert_same_bytes(codes.cpu().numpy(), orc.encode_f32(xn, scale, mode), "f32 %d %d" % (n, off))
                h.hif8_encode_bf16(xb.data_ptr(), codes.data_ptr(), n, scale, mode)
                torch.cuda.synchronize()
                assert_same_bytes(codes.cpu().numpy(), orc.encode_bf16(xbn, scale, mode), "bf16 %d %d" % (n, off))
                h.hif8_encode_f16(xh.data_ptr(), codes.data_ptr(), n, scale, mode)
                torch.cuda.synchronize()
                assert_same_bytes(codes.cpu().numpy(), orc.encode_f16(xhn, scale, mode), "f16 %d %d" % (n, off))
            o = torch.zeros(n + 16, dtype=torch.float32, device=dev())[off:off + n]
            h.hif8_fake_quant_f32(x.data_ptr(), o.data_ptr(), codes.data_ptr(), n, 0.6, mode)
            torch.cuda.synchronize()
            wo, wc = orc.fake_quant_f32(xn, 0.6, mode)
            assert_same_bytes(codes.cpu().numpy(), wc, "fq codes")
            assert_same_bytes(f32_bits(o.contiguous()), wo.view(np.uint32), "fq out")


# ------------------------------------------------------------------ FP16 tensors
@pytest.mark.parametrize("mode", [TA, HR, TE, SSR, SR, TA | SAT, HR | N2Z, HR | SAT | N2Z])
@pytest.mark.parametrize("scale", [1.0, 0.37, 2.0 ** -9, 1311.7])
def test_f16_encode_all_patterns(h, mode, scale):
    pats = np.arange(65536, dtype=np.uint16)
    x = to_gpu(pats)
    assert_same_bytes(enc(h, "f16", x, scale, mode), orc.encode_f16(pats, scale, mode), "f16 patterns")


@pytest.mark.parametrize("scale", [1.0, 4.0, 0.37, 1311.7, 2.0 ** 20, 2.0 ** -12])
def test_f16_decode_all_codes(h, scale):
    """Includes scales whose descaled values are binary16 subnormals or overflow to Inf."""
    from paper_2409_16626_amd import workloads
    codes = workloads.all_codes(dev()).repeat(5)[:1275]
    n = codes.numel()
    out = torch.empty(n, dtype=torch.float16, device=dev())
    h.hif8_decode_f16(codes, out, n, scale)
    torch.cuda.synchronize()
    assert_same_bytes(f16_bits(out), orc.decode_f16(codes.cpu().numpy(), scale), "decode_f16")
    # unaligned destination: element path
    out2 = torch.zeros(n + 8, dtype=torch.float16, device=dev())[1:1 + n]
    h.hif8_decode_f16(codes.data_ptr(), out2.data_ptr(), n, scale)
    torch.cuda.synchronize()
    assert_same_bytes(f16_bits(out2.contiguous()), orc.decode_f16(codes.cpu().numpy(), scale), "decode_f16 elem")


@pytest.mark.parametrize("mode", [TA, HR, TE, SR])
def test_f16_fake_quant_amax_and_device_scale(h, mode):
    from paper_2409_16626_amd import workloads
    x = (workloads.activation_bf16(512, 1024 + 8, dev()).float()).to(torch.float16).view(-1)
    n = x.numel() - 3                      # ragged
    x = x[:n].contiguous()
    xn = f16_bits(x)
    am = torch.zeros(1, dtype=torch.float32, device=dev())
    sc = torch.zeros(2, dtype=torch.float32, device=dev())
    acc = torch.zeros(1, dtype=torch.float32, device=dev())
    out = torch.empty_like(x)
    codes = torch.empty(n, dtype=torch.uint8, device=dev())
    h.hif8_amax_f16(x, n, am)
    h.hif8_scale_from_amax(am, sc, 32768.0, 0)
    h.hif8_fake_quant_f16_ds(x, out, codes, n, sc, mode, d_amax_accum=acc)
    torch.cuda.synchronize()
    w_am = orc.amax_f16(xn)
    assert f32_bits(am)[0] == np.float32(w_am).view(np.uint32) and f32_bits(acc)[0] == f32_bits(am)[0]
    w_s = orc.scale_from_amax(w_am, 32768.0, False)
    assert sc[0].item() == w_s
    wo, wc = orc.fake_quant_f16(xn, w_s, mode)
    assert_same_bytes(codes.cpu().numpy(), wc, "f16 fq codes")
    assert_same_bytes(f16_bits(out), wo, "f16 fq out")
    c2 = torch.empty_like(codes)
    o2 = torch.empty_like(out)
    h.hif8_encode_f16_ds(x, c2, n, sc, mode)
    h.hif8_decode_f16_ds(c2, o2, n, sc)
    h.hif8_fake_quant_f16(x, out, None, n, float(w_s), mode)
    torch.cuda.synchronize()
    assert torch.equal(c2, codes) and torch.equal(o2.view(torch.int16), out.view(torch.int16))
    assert_same_bytes(f16_bits(out), wo, "f16 fq by-value scale")
    # amax of special values: Inf dominates finite, NaN dominates Inf (payload unspecified)
    y = x.clone()
    y[n // 2] = float("-inf")
    h.hif8_amax_f16(y, n, am)
    assert f32_bits(am)[0] == 0x7F800000
    y[7] = float("nan")
    h.hif8_amax_f16(y, n, am)
    assert np.isnan(am.cpu().numpy()[0])


@pytest.mark.parametrize("mode", [TA, TE, SR | SAT])
def test_multi_tensor_cast_f16_and_new_modes(h, mode):
    rng = np.random.default_rng(43)
    sizes = [8192 * 3, 0, 1, 7, 8, 8200, 12345, 100003, 16, 65536 + 24]
    for kind in ("f16", "bf16", "f32"):
        offs, total = [], 0
        for m in sizes:
            offs.append(total)
            total += (m + 15) // 16 * 16
        xf = torch.from_numpy((rng.standard_normal(total) * np.exp2(rng.uniform(-10, 3, total))).astype(np.float32)).to(dev())
        x = {"f16": xf.to(torch.float16), "bf16": xf.to(torch.bfloat16), "f32": xf}[kind]
        codes = torch.zeros(total, dtype=torch.uint8, device=dev())
        items = [(x[o:o + m].data_ptr() if m else 0, codes[o:o + m].data_ptr() if m else 0, m) for o, m in zip(offs, sizes)]
        d_items, count, tiles = h.hif8_multi_plan(items, src_is_16bit=(kind != "f32"))
        am = torch.full((count,), 3.0, dtype=torch.float32, device=dev())
        sc = torch.zeros(count, 2, dtype=torch.float32, device=dev())
        getattr(h, "hif8_multi_cast_" + kind)(d_items, count, tiles, am, sc, 32768.0, 1, mode)
        torch.cuda.synchronize()
        xn = {"f16": f16_bits, "bf16": bf16_bits, "f32": lambda t: t.cpu().numpy()}[kind](x)
        o_amax = {"f16": orc.amax_f16, "bf16": orc.amax_bf16, "f32": orc.amax_f32}[kind]
        o_enc = {"f16": orc.encode_f16, "bf16": orc.encode_bf16, "f32": orc.encode_f32}[kind]
        cg, amg, scg = codes.cpu().numpy(), am.cpu().numpy(), sc.cpu().numpy()
        for i, (o, m) in enumerate(zip(offs, sizes)):
            part = xn[o:o + m]
            w_am = o_amax(part)
            w_s = orc.scale_from_amax(w_am, 32768.0, True)
            assert amg[i] == w_am and scg[i, 0] == w_s, (kind, i, m)
            assert_same_bytes(cg[o:o + m], o_enc(part, w_s, mode), "multi %s item %d (n=%d)" % (kind, i, m))


def test_sr_threshold_index_beyond_32_bits(h):
    """2^32 + 2^20 BF16 elements under standard SR: the threshold of element i uses all 64 bits
    of i.  Checked on sampled elements with the oracle's one-element entry point."""
    n = (1 << 32) + (1 << 20)
    g = torch.Generator(device=dev()).manual_seed(77)
    x = torch.empty(n, dtype=torch.bfloat16, device=dev())
    chunk = 1 << 28
    for lo in range(0, n, chunk):
        m = min(chunk, n - lo)
        x[lo:lo + m] = (torch.randn(m, generator=g, device=dev()) * 40.0).to(torch.bfloat16)
    codes = torch.empty(n, dtype=torch.uint8, device=dev())
    h.hif8_encode_bf16(x, codes, n, 1.0, SR)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    idx = np.concatenate([np.arange(0, 64), np.arange((1 << 32) - 64, (1 << 32) + 64), np.arange(n - 64, n),
                          rng.integers(0, n, 2000)])
    it = torch.from_numpy(idx).to(dev())
    xs = bf16_bits(x[it])
    cs = codes[it].cpu().numpy()
    for i, xb, c in zip(idx.tolist(), xs.tolist(), cs.tolist()):
        y = np.array([xb << 16], np.uint32).view(np.float32)[0]
        want = orc.encode_one(y, SR, orc.SRC_BF16, orc.sr_threshold(SEED, i))
        assert c == want, (i, hex(xb), c, want)
    # the high word matters: the same values at index i - 2^32 get other thresholds
    lo_part = codes[:1 << 20]
    hi_src = x[1 << 32:]
    c_lo = torch.empty(1 << 20, dtype=torch.uint8, device=dev())
    h.hif8_encode_bf16(hi_src, c_lo, 1 << 20, 1.0, SR)
    torch.cuda.synchronize()
    assert not torch.equal(c_lo, codes[1 << 32:])
    del lo_part
