"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bars: u8 codes bit-exact; FP32 / BF16 outputs compared as raw bit patterns (0 ulp).
Sizes span several tiles, a ragged tail, and the element-per-lane path for unaligned
pointers.  Inputs come from the seeded generators in paper_2409_16626_amd.workloads.
"""
import numpy as np
import pytest
import torch

from oracle import hif8_oracle as orc

pytestmark = pytest.mark.gpu

TA, HR, SAT, N2Z = orc.RM_TA, orc.RM_HR, orc.FLAG_SAT, orc.FLAG_NAN2ZERO
ALL_MODES = [TA, HR, TA | SAT, HR | SAT, TA | N2Z, HR | N2Z, TA | SAT | N2Z, HR | SAT | N2Z]


@pytest.fixture(scope="module")
def h():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2409_16626_amd import hif8
    hif8.hif8_init()
    return hif8


from gpu_util import assert_same_bytes, bf16_bits, dev, f32_bits, to_gpu  # noqa: E402


def gpu_encode_f32(h, x, scale, mode):
    dst = torch.empty(x.numel(), dtype=torch.uint8, device=dev())
    h.hif8_encode_f32(x, dst, x.numel(), scale, mode)
    torch.cuda.synchronize()
    return dst.cpu().numpy()


def gpu_encode_bf16(h, x, scale, mode):
    dst = torch.empty(x.numel(), dtype=torch.uint8, device=dev())
    h.hif8_encode_bf16(x, dst, x.numel(), scale, mode)
    torch.cuda.synchronize()
    return dst.cpu().numpy()


# ------------------------------------------------------------------ config 1: exhaustive tiny
@pytest.mark.parametrize("scale", [1.0, 4.0, 0.37, 1311.7])
def test_c1_decode_all_codes(h, scale):
    from paper_2409_16626_amd import workloads
    codes = workloads.all_codes(dev())
    out32 = torch.empty(256, dtype=torch.float32, device=dev())
    out16 = torch.empty(256, dtype=torch.bfloat16, device=dev())
    h.hif8_decode_f32(codes, out32, 256, scale)
    h.hif8_decode_bf16(codes, out16, 256, scale)
    torch.cuda.synchronize()
    c = codes.cpu().numpy()
    assert_same_bytes(f32_bits(out32), orc.decode_f32(c, scale).view(np.uint32), "decode_f32")
    assert_same_bytes(bf16_bits(out16), orc.decode_bf16(c, scale), "decode_bf16")


@pytest.mark.parametrize("scale", [2.0 ** 110, 2.0 ** 120, 2.0 ** -100, 3.0e37, 1.7e-38])
def test_decode_and_fake_quant_extreme_scales(h, scale):
    """Descaled outputs that are binary32 / bfloat16 subnormals, or overflow to Inf."""
    from paper_2409_16626_amd import workloads
    codes = workloads.all_codes(dev()).repeat(5)[:1275]
    n = codes.numel()
    out32 = torch.empty(n, dtype=torch.float32, device=dev())
    out16 = torch.empty(n, dtype=torch.bfloat16, device=dev())
    h.hif8_decode_f32(codes, out32, n, scale)
    h.hif8_decode_bf16(codes, out16, n, scale)
    torch.cuda.synchronize()
    c = codes.cpu().numpy()
    assert_same_bytes(f32_bits(out32), orc.decode_f32(c, scale).view(np.uint32), "decode_f32 extreme")
    assert_same_bytes(bf16_bits(out16), orc.decode_bf16(c, scale), "decode_bf16 extreme")
    x = (workloads.normal_f32(1 << 12, dev()) / scale).to(torch.float32)
    xn = x.cpu().numpy()
    o = torch.empty_like(x)
    cc = torch.empty(x.numel(), dtype=torch.uint8, device=dev())
    h.hif8_fake_quant_f32(x, o, cc, x.numel(), scale, HR)
    torch.cuda.synchronize()
    wo, wc = orc.fake_quant_f32(xn, scale, HR)
    assert_same_bytes(cc.cpu().numpy(), wc, "fq extreme codes")
    assert_same_bytes(f32_bits(o), wo.view(np.uint32), "fq extreme out")


@pytest.mark.parametrize("mode", ALL_MODES)
def test_c1_encode_all_fp16_patterns(h, mode):
    from paper_2409_16626_amd import workloads
    x = workloads.all_fp16_as_f32(dev())
    got = gpu_encode_f32(h, x, 1.0, mode)
    assert_same_bytes(got, orc.encode_f32(x.cpu().numpy(), 1.0, mode), "fp16 patterns mode %#x" % mode)


@pytest.mark.parametrize("mode", ALL_MODES)
@pytest.mark.parametrize("scale", [1.0, 0.37, 2.0 ** -9, 1311.7])
def test_c1_encode_all_bf16_patterns(h, mode, scale):
    from paper_2409_16626_amd import workloads
    x = workloads.all_bf16(dev())
    got = gpu_encode_bf16(h, x, scale, mode)
    assert_same_bytes(got, orc.encode_bf16(bf16_bits(x), scale, mode), "bf16 patterns")


@pytest.mark.parametrize("mode", [TA, HR, TA | SAT, HR | N2Z])
def test_c1_encode_normal_1m(h, mode):
    from paper_2409_16626_amd import workloads
    x = workloads.normal_f32(1 << 20, dev())
    got = gpu_encode_f32(h, x, 1.0, mode)
    assert_same_bytes(got, orc.encode_f32(x.cpu().numpy(), 1.0, mode), "N(0,1)")


@pytest.mark.parametrize("mode", ALL_MODES)
def test_c1_decode_encode_round_trip(h, mode):
    from paper_2409_16626_amd import workloads
    codes = workloads.all_codes(dev())
    v = torch.empty(256, dtype=torch.float32, device=dev())
    h.hif8_decode_f32(codes, v, 256, 1.0)
    got = gpu_encode_f32(h, v, 1.0, mode)
    want = np.arange(256, dtype=np.uint8)
    if mode & N2Z:
        want[0x80] = 0
    if mode & SAT:
        want[0x6F], want[0xEF] = 0x6E, 0xEE
    assert_same_bytes(got, want, "round trip")
    vb = torch.empty(256, dtype=torch.bfloat16, device=dev())
    h.hif8_decode_bf16(codes, vb, 256, 1.0)
    assert_same_bytes(gpu_encode_bf16(h, vb, 1.0, mode), want, "round trip bf16")


def test_top13_bit_patterns_with_fillers(h):
    rng = np.random.default_rng(31)
    top = np.arange(1 << 13, dtype=np.uint32) << 19
    parts = [top, top | np.uint32(0x7FFFF), top | np.uint32(1),
             top | rng.integers(0, 1 << 19, size=top.size).astype(np.uint32)]
    yb = np.concatenate(parts)
    x = to_gpu(yb).view(torch.float32)
    for mode in (TA, HR, TA | SAT | N2Z):
        got = gpu_encode_f32(h, x, 1.0, mode)
        assert_same_bytes(got, orc.encode_f32(yb.view(np.float32), 1.0, mode), "top13 %#x" % mode)


# ------------------------------------------------------------------ ragged sizes / alignment
@pytest.mark.parametrize("n", [0, 1, 3, 4, 5, 7, 8, 9, 63, 64, 65, 1000, 4097, 8191, (1 << 18) + 13])
def test_ragged_sizes_all_entry_points(h, n):
    from paper_2409_16626_amd import workloads
    big = workloads.dynamic_range_sweep(1 << 19, dev())
    x = big[:n].contiguous()
    xb = big[:n].to(torch.bfloat16).contiguous()
    xn, xbn = x.cpu().numpy(), bf16_bits(xb)
    for mode in (TA, HR):
        for scale in (1.0, 3.3):
            assert_same_bytes(gpu_encode_f32(h, x, scale, mode), orc.encode_f32(xn, scale, mode), "enc f32")
            assert_same_bytes(gpu_encode_bf16(h, xb, scale, mode), orc.encode_bf16(xbn, scale, mode), "enc bf16")
            o = torch.empty_like(x)
            c = torch.empty(n, dtype=torch.uint8, device=dev())
            h.hif8_fake_quant_f32(x, o, c, n, scale, mode)
            ob = torch.empty_like(xb)
            cb = torch.empty(n, dtype=torch.uint8, device=dev())
            h.hif8_fake_quant_bf16(xb, ob, cb, n, scale, mode)
            torch.cuda.synchronize()
            wo, wc = orc.fake_quant_f32(xn, scale, mode)
            assert_same_bytes(f32_bits(o), wo.view(np.uint32), "fq f32")
            assert_same_bytes(c.cpu().numpy(), wc, "fq f32 codes")
            wob, wcb = orc.fake_quant_bf16(xbn, scale, mode)
            assert_same_bytes(bf16_bits(ob), wob, "fq bf16")
            assert_same_bytes(cb.cpu().numpy(), wcb, "fq bf16 codes")
    codes = torch.randint(0, 256, (n,), dtype=torch.int32, device=dev(),
                          generator=torch.Generator(device=dev()).manual_seed(5)).to(torch.uint8)
    o = torch.empty(n, dtype=torch.float32, device=dev())
    ob = torch.empty(n, dtype=torch.bfloat16, device=dev())
    h.hif8_decode_f32(codes, o, n, 2.5)
    h.hif8_decode_bf16(codes, ob, n, 2.5)
    torch.cuda.synchronize()
    assert_same_bytes(f32_bits(o), orc.decode_f32(codes.cpu().numpy(), 2.5).view(np.uint32), "dec f32")
    assert_same_bytes(bf16_bits(ob), orc.decode_bf16(codes.cpu().numpy(), 2.5), "dec bf16")
    am = torch.full((1,), 7.0, dtype=torch.float32, device=dev())
    h.hif8_amax_f32(x, n, am)
    assert f32_bits(am)[0] == np.float32(orc.amax_f32(xn)).view(np.uint32)
    h.hif8_amax_bf16(xb, n, am)
    assert f32_bits(am)[0] == np.float32(orc.amax_bf16(xbn)).view(np.uint32)


@pytest.mark.parametrize("off", [1, 2, 3])
def test_unaligned_pointers_use_element_path(h, off):
    from paper_2409_16626_amd import workloads
    n = 10007
    big = workloads.dynamic_range_sweep(1 << 15, dev())
    x = big[off:off + n]                       # 4*off bytes off a 16-byte boundary
    xb_all = big.to(torch.bfloat16)
    xb = xb_all[off:off + n]
    xn, xbn = x.cpu().numpy(), bf16_bits(xb.contiguous())
    dst_all = torch.zeros(n + 8, dtype=torch.uint8, device=dev())
    for mode in (TA, HR | SAT):
        dst = dst_all[off:off + n]
        h.hif8_encode_f32(x.data_ptr(), dst.data_ptr(), n, 1.7, mode)
        torch.cuda.synchronize()
        assert_same_bytes(dst.cpu().numpy(), orc.encode_f32(xn, 1.7, mode), "unaligned enc f32")
        h.hif8_encode_bf16(xb.data_ptr(), dst.data_ptr(), n, 1.7, mode)
        torch.cuda.synchronize()
        assert_same_bytes(dst.cpu().numpy(), orc.encode_bf16(xbn, 1.7, mode), "unaligned enc bf16")
        # destination only misaligned
        x0 = big[:n]
        h.hif8_encode_f32(x0.data_ptr(), dst.data_ptr(), n, 1.0, mode)
        torch.cuda.synchronize()
        assert_same_bytes(dst.cpu().numpy(), orc.encode_f32(x0.cpu().numpy(), 1.0, mode), "unaligned dst")
        o_all = torch.zeros(n + 8, dtype=torch.float32, device=dev())
        o = o_all[off:off + n]
        h.hif8_fake_quant_f32(x.data_ptr(), o.data_ptr(), dst.data_ptr(), n, 1.7, mode)
        torch.cuda.synchronize()
        wo, wc = orc.fake_quant_f32(xn, 1.7, mode)
        assert_same_bytes(f32_bits(o.contiguous()), wo.view(np.uint32), "unaligned fq")
        assert_same_bytes(dst.cpu().numpy(), wc, "unaligned fq codes")
        ob_all = torch.zeros(n + 8, dtype=torch.bfloat16, device=dev())
        ob = ob_all[off:off + n]
        h.hif8_fake_quant_bf16(xb.data_ptr(), ob.data_ptr(), None, n, 1.7, mode)
        torch.cuda.synchronize()
        wob, _ = orc.fake_quant_bf16(xbn, 1.7, mode)
        assert_same_bytes(bf16_bits(ob.contiguous()), wob, "unaligned fq bf16")
    codes = dst_all[off:off + n]
    o = torch.zeros(n + 8, dtype=torch.float32, device=dev())[off:off + n]
    h.hif8_decode_f32(codes.data_ptr(), o.data_ptr(), n, 0.7)
    torch.cuda.synchronize()
    assert_same_bytes(f32_bits(o.contiguous()), orc.decode_f32(codes.cpu().numpy(), 0.7).view(np.uint32), "unaligned dec")
    am = torch.zeros(1, dtype=torch.float32, device=dev())
    h.hif8_amax_f32(x.data_ptr(), n, am)
    assert f32_bits(am)[0] == np.float32(orc.amax_f32(xn)).view(np.uint32)
    h.hif8_amax_bf16(xb.data_ptr(), n, am)
    assert f32_bits(am)[0] == np.float32(orc.amax_bf16(xbn)).view(np.uint32)


def test_fake_quant_in_place(h):
    from paper_2409_16626_amd import workloads
    x = workloads.dynamic_range_sweep((1 << 20) + 5, dev())
    xn = x.cpu().numpy()
    h.hif8_fake_quant_f32(x, x, None, x.numel(), 2.0, TA)
    torch.cuda.synchronize()
    wo, _ = orc.fake_quant_f32(xn, 2.0, TA)
    assert_same_bytes(f32_bits(x), wo.view(np.uint32), "in place f32")
    xb = workloads.activation_bf16(512, 1024, dev()).view(-1)
    xbn = bf16_bits(xb)
    h.hif8_fake_quant_bf16(xb, xb, None, xb.numel(), 5.0, HR)
    torch.cuda.synchronize()
    wob, _ = orc.fake_quant_bf16(xbn, 5.0, HR)
    assert_same_bytes(bf16_bits(xb), wob, "in place bf16")


# ------------------------------------------------------------------ reduced-size configs 2-5
@pytest.mark.parametrize("mode", [TA, TA | SAT, HR])
def test_c2_dynamic_range_sweep_small(h, mode):
    from paper_2409_16626_amd import workloads
    x = workloads.dynamic_range_sweep((1 << 22) + 3, dev())
    got = gpu_encode_f32(h, x, 1.0, mode)
    assert_same_bytes(got, orc.encode_f32(x.cpu().numpy(), 1.0, mode), "C2 small")


def test_c3_activation_pipeline_small(h):
    """amax -> scale (2^15 / amax, device resident) -> fused fake-quant with codes."""
    from paper_2409_16626_amd import workloads
    x = workloads.activation_bf16(1024, 2048 + 8, dev()).view(-1)
    n = x.numel()
    xb = bf16_bits(x)
    am = torch.zeros(1, dtype=torch.float32, device=dev())
    sc = torch.zeros(2, dtype=torch.float32, device=dev())
    out = torch.empty_like(x)
    codes = torch.empty(n, dtype=torch.uint8, device=dev())
    for pow2 in (0, 1):
        h.hif8_amax_bf16(x, n, am)
        h.hif8_scale_from_amax(am, sc, 32768.0, pow2)
        h.hif8_fake_quant_bf16_ds(x, out, codes, n, sc, TA)
        torch.cuda.synchronize()
        w_am = orc.amax_bf16(xb)
        assert f32_bits(am)[0] == np.float32(w_am).view(np.uint32)
        w_s = orc.scale_from_amax(w_am, 32768.0, bool(pow2))
        s2 = sc.cpu().numpy()
        assert s2[0] == w_s and s2[1] == np.float32(1.0) / w_s
        wo, wc = orc.fake_quant_bf16(xb, w_s, TA)
        assert_same_bytes(codes.cpu().numpy(), wc, "C3 codes")
        assert_same_bytes(bf16_bits(out), wo, "C3 bf16 out")
        assert wc.max() >= 0x6C or (wc & 0x7F).max() >= 0x6C  # scaling uses the top of the range
        # separate encode_ds / decode_ds agree with the fused call
        c2 = torch.empty_like(codes)
        o2 = torch.empty_like(out)
        h.hif8_encode_bf16_ds(x, c2, n, sc, TA)
        h.hif8_decode_bf16_ds(c2, o2, n, sc)
        torch.cuda.synchronize()
        assert torch.equal(c2, codes) and torch.equal(o2.view(torch.int16), out.view(torch.int16))


@pytest.mark.parametrize("mode", [TA, HR])
def test_c4_gradient_small(h, mode):
    from paper_2409_16626_amd import workloads
    x = workloads.gradient_f32((1 << 22) + 1, dev(), chunk=1 << 20)
    got = gpu_encode_f32(h, x, 1.0, mode)
    want = orc.encode_f32(x.cpu().numpy(), 1.0, mode)
    assert_same_bytes(got, want, "C4 small")
    frac_dml = np.mean(((want & 0x7F) >= 1) & ((want & 0x7F) <= 7))
    assert frac_dml > 0.2      # the bulk of this workload lives in the denormal binades


def test_c5_weight_cast_small(h):
    from paper_2409_16626_amd import workloads
    arena, index = workloads.llm_weights_bf16(dev(), layers=2, hidden=256, ffn=688, vocab=2000)
    codes = torch.empty(arena.numel(), dtype=torch.uint8, device=dev())
    am = torch.zeros(len(index), dtype=torch.float32, device=dev())
    sc = torch.zeros(len(index), 2, dtype=torch.float32, device=dev())
    for i, (_, off, m) in enumerate(index):
        h.hif8_amax_bf16(arena[off:off + m].data_ptr(), m, am[i:i + 1].data_ptr())
        h.hif8_scale_from_amax(am[i:i + 1].data_ptr(), sc[i].data_ptr(), 32768.0, 0)
        h.hif8_encode_bf16_ds(arena[off:off + m].data_ptr(), codes[off:off + m].data_ptr(), m,
                              sc[i].data_ptr(), TA)
    torch.cuda.synchronize()
    ab = bf16_bits(arena)
    cg = codes.cpu().numpy()
    for i, (_, off, m) in enumerate(index):
        w_am = orc.amax_bf16(ab[off:off + m])
        w_s = orc.scale_from_amax(w_am, 32768.0, False)
        assert sc[i, 0].item() == w_s
        assert_same_bytes(cg[off:off + m], orc.encode_bf16(ab[off:off + m], w_s, TA), "C5 tensor %d" % i)


@pytest.mark.parametrize("mode", [TA, HR | SAT])
@pytest.mark.parametrize("pow2", [0, 1])
def test_multi_tensor_cast_matches_per_tensor_oracle(h, mode, pow2):
    """Tensor list with ragged, tiny and empty members: four launches for the whole list."""
    rng = np.random.default_rng(41)
    sizes = [8192 * 3, 0, 1, 7, 8, 8200, 12345, 8192, 100003, 16, 0, 65536 + 24]
    for bf16 in (True, False):
        offs, total = [], 0
        for m in sizes:
            offs.append(total)
            total += (m + 15) // 16 * 16          # keep every slice 16-byte aligned
        xf = torch.from_numpy((rng.standard_normal(total) * np.exp2(rng.uniform(-12, 3, total))).astype(np.float32)).to(dev())
        x = xf.to(torch.bfloat16) if bf16 else xf
        codes = torch.zeros(total, dtype=torch.uint8, device=dev())
        items = [(x[o:o + m].data_ptr() if m else 0, codes[o:o + m].data_ptr() if m else 0, m) for o, m in zip(offs, sizes)]
        d_items, count, tiles = h.hif8_multi_plan(items, src_is_16bit=bf16)
        am = torch.full((count,), 3.0, dtype=torch.float32, device=dev())
        sc = torch.zeros(count, 2, dtype=torch.float32, device=dev())
        fn = h.hif8_multi_cast_bf16 if bf16 else h.hif8_multi_cast_f32
        fn(d_items, count, tiles, am, sc, 32768.0, pow2, mode)
        torch.cuda.synchronize()
        xn = bf16_bits(x) if bf16 else x.cpu().numpy()
        cg, amg, scg = codes.cpu().numpy(), am.cpu().numpy(), sc.cpu().numpy()
        for i, (o, m) in enumerate(zip(offs, sizes)):
            part = xn[o:o + m]
            w_am = orc.amax_bf16(part) if bf16 else orc.amax_f32(part)
            w_s = orc.scale_from_amax(w_am, 32768.0, bool(pow2))
            assert amg[i] == w_am and scg[i, 0] == w_s and scg[i, 1] == np.float32(1.0) / w_s, (i, m)
            want = orc.encode_bf16(part, w_s, mode) if bf16 else orc.encode_f32(part, w_s, mode)
            assert_same_bytes(cg[o:o + m], want, "multi item %d (n=%d, bf16=%s)" % (i, m, bf16))
        # bytes between the slices were not touched
        for o, m in zip(offs, sizes):
            pad = (m + 15) // 16 * 16
            assert not cg[o + m:o + pad].any()


@pytest.mark.parametrize("mode", [TA, HR, orc.RM_SR | SAT])
def test_multi_tensor_encode_with_device_scales_and_amax_accumulation(h, mode):
    """Delayed scaling over a tensor list in one launch: codes under the given scales bit for bit the
    oracle's, accumulators = max(previous content, amax of the tensor), untouched without the pointer."""
    rng = np.random.default_rng(43)
    sizes = [8192 * 3, 0, 1, 7, 8, 8200, 12345, 8192, 100003, 16, 0, 65536 + 24, 3 * 8192 * 8 + 5]
    for kind in ("bf16", "f32", "f16"):
        offs, total = [], 0
        for m in sizes:
            offs.append(total)
            total += (m + 15) // 16 * 16
        xf = torch.from_numpy((rng.standard_normal(total) * np.exp2(rng.uniform(-12, 3, total))).astype(np.float32)).to(dev())
        x = {"bf16": xf.to(torch.bfloat16), "f16": xf.to(torch.float16), "f32": xf}[kind]
        codes = torch.zeros(total, dtype=torch.uint8, device=dev())
        items = [(x[o:o + m].data_ptr() if m else 0, codes[o:o + m].data_ptr() if m else 0, m) for o, m in zip(offs, sizes)]
        d_items, count, tiles = h.hif8_multi_plan(items, src_is_16bit=kind != "f32")
        scales = np.exp2(rng.integers(-3, 9, count)).astype(np.float32) * np.float32(1.25)
        sc = torch.from_numpy(np.stack([scales, np.float32(1.0) / scales], 1).copy()).to(dev())
        prev = np.where(np.arange(count) % 3 == 0, np.float32(1e9), np.float32(0.0)).astype(np.float32)   # some already above
        acc = torch.from_numpy(prev.copy()).to(dev())
        fn = getattr(h, "hif8_multi_encode_%s_ds" % kind)
        fn(d_items, count, tiles, sc, mode, d_amax_accum=acc)
        torch.cuda.synchronize()
        xn = x.cpu().numpy() if kind == "f32" else x.view(torch.int16).cpu().numpy().view(np.uint16)
        enc = {"bf16": orc.encode_bf16, "f16": orc.encode_f16, "f32": orc.encode_f32}[kind]
        amx = {"bf16": orc.amax_bf16, "f16": orc.amax_f16, "f32": orc.amax_f32}[kind]
        cg, ag = codes.cpu().numpy(), acc.cpu().numpy()
        for i, (o, m) in enumerate(zip(offs, sizes)):
            part = xn[o:o + m]
            assert_same_bytes(cg[o:o + m], enc(part, scales[i], mode), "multi ds item %d (n=%d, %s)" % (i, m, kind))
            assert ag[i] == max(prev[i], np.float32(amx(part))), (i, m, kind)
        codes2 = torch.zeros_like(codes)
        items2 = [(x[o:o + m].data_ptr() if m else 0, codes2[o:o + m].data_ptr() if m else 0, m) for o, m in zip(offs, sizes)]
        d_items2, count2, tiles2 = h.hif8_multi_plan(items2, src_is_16bit=kind != "f32")
        fn(d_items2, count2, tiles2, sc, mode)                      # no accumulator
        torch.cuda.synchronize()
        assert torch.equal(codes, codes2)


# ------------------------------------------------------------------ amax semantics, tuning, graphs
def test_amax_special_values(h):
    x = torch.randn(100003, device=dev())
    am = torch.zeros(1, dtype=torch.float32, device=dev())
    x[77777] = -float("inf")
    h.hif8_amax_f32(x, x.numel(), am)
    assert f32_bits(am)[0] == 0x7F800000
    x[5] = float("nan")
    h.hif8_amax_f32(x, x.numel(), am)
    assert np.isnan(am.cpu().numpy()[0])
    z = torch.zeros(4096, device=dev())
    h.hif8_amax_f32(z, z.numel(), am)
    assert f32_bits(am)[0] == 0
    z[4095] = -0.0
    h.hif8_amax_f32(z, z.numel(), am)
    assert f32_bits(am)[0] == 0
    # scale from a degenerate amax is 1
    sc = torch.zeros(2, dtype=torch.float32, device=dev())
    for v in (0.0, float("inf"), float("nan")):
        am.fill_(v)
        h.hif8_scale_from_amax(am, sc, 32768.0, 0)
        assert sc.cpu().tolist() == [1.0, 1.0]


@pytest.mark.parametrize("block,wg,unroll,impl,tpw,amax_nt",
                         [(64, 1, 1, 0, 0, 1), (256, 8, 2, 0, 0, 0), (1024, 2, 8, 0, 0, 1),
                          (512, 4, 4, 1, 0, 1), (128, 16, 8, 1, 1, 0), (320, 3, 2, 0, 3, 1),
                          (256, 4, 2, 0, 1, 1), (512, 4, 1, 0, 7, 0), (1024, 4, 4, 1, 16, 1),
                          (64, 4, 1, 0, 4096, 1)])
def test_launch_shapes_and_alu_variant(h, block, wg, unroll, impl, tpw, amax_nt):
    from paper_2409_16626_amd import workloads
    saved = [h.hif8_get_tuning(k) for k in range(h.N_TUNE_KEYS)]
    try:
        h.hif8_set_tuning(h.TUNE_BLOCK, block)
        h.hif8_set_tuning(h.TUNE_WG_PER_CU, wg)
        h.hif8_set_tuning(h.TUNE_UNROLL, unroll)
        h.hif8_set_tuning(h.TUNE_TA_IMPL, impl)
        h.hif8_set_tuning(h.TUNE_TILES_PER_WG, tpw)
        h.hif8_set_tuning(h.TUNE_AMAX_NT, amax_nt)
        x = workloads.dynamic_range_sweep((1 << 21) + 77, dev())
        xn = x.cpu().numpy()
        for mode in (TA, HR, TA | SAT | N2Z):
            assert_same_bytes(gpu_encode_f32(h, x, 1.0, mode), orc.encode_f32(xn, 1.0, mode), "tuned enc")
        xb = x.to(torch.bfloat16)
        xbn = bf16_bits(xb)
        o = torch.empty_like(xb)
        c = torch.empty(xb.numel(), dtype=torch.uint8, device=dev())
        h.hif8_fake_quant_bf16(xb, o, c, xb.numel(), 0.9, TA)
        torch.cuda.synchronize()
        wo, wc = orc.fake_quant_bf16(xbn, 0.9, TA)
        assert_same_bytes(c.cpu().numpy(), wc, "tuned fq codes")
        assert_same_bytes(bf16_bits(o), wo, "tuned fq out")
        am = torch.zeros(1, dtype=torch.float32, device=dev())
        h.hif8_amax_f32(x, x.numel(), am)
        assert f32_bits(am)[0] == np.float32(orc.amax_f32(xn)).view(np.uint32)
        h.hif8_amax_bf16(xb, xb.numel(), am)
        assert f32_bits(am)[0] == np.float32(orc.amax_bf16(xbn)).view(np.uint32)
        codes = c
        o32 = torch.empty(codes.numel(), dtype=torch.float32, device=dev())
        h.hif8_decode_f32(codes, o32, codes.numel(), 0.9)
        h.hif8_decode_bf16(codes, o, codes.numel(), 0.9)
        torch.cuda.synchronize()
        assert_same_bytes(f32_bits(o32), orc.decode_f32(wc, 0.9).view(np.uint32), "tuned dec f32")
        assert_same_bytes(bf16_bits(o), orc.decode_bf16(wc, 0.9), "tuned dec bf16")
    finally:
        for k, v in enumerate(saved):
            h.hif8_set_tuning(k, v)


@pytest.mark.parametrize("n,off", [(1 << 20, 0), ((1 << 18) + 5, 0), (10007, 1), (3, 0)])
def test_delayed_scaling_amax_accumulates_in_the_cast_pass(h, n, off):
    """_ds encode / fake-quant with an amax accumulator: codes as usual, plus the amax of the
    unscaled input; the accumulator keeps the maximum over consecutive calls."""
    from paper_2409_16626_amd import workloads
    big = workloads.dynamic_range_sweep((1 << 20) + 64, dev())
    x = big[off:off + n]
    y = (big[off + 8:off + 8 + n] * 0.01)
    xb_all = big.to(torch.bfloat16)
    xb = xb_all[off:off + n]
    sc = torch.tensor([0.75, 1.0 / 0.75], dtype=torch.float32, device=dev())
    acc = torch.zeros(1, dtype=torch.float32, device=dev())
    codes = torch.empty(n + 8, dtype=torch.uint8, device=dev())[off:off + n]
    xn, yn, xbn = x.cpu().numpy(), y.contiguous().cpu().numpy(), bf16_bits(xb.contiguous())
    s = np.float32(0.75)
    for mode in (TA, HR):
        h.hif8_amax_f32(0, 0, acc)                      # start a window: writes 0
        h.hif8_encode_f32_ds(x.data_ptr(), codes.data_ptr(), n, sc, mode, d_amax_accum=acc)
        torch.cuda.synchronize()
        assert_same_bytes(codes.cpu().numpy(), orc.encode_f32(xn, s, mode), "ds enc f32")
        assert f32_bits(acc)[0] == np.float32(orc.amax_f32(xn)).view(np.uint32)
        yc = y.contiguous()
        h.hif8_encode_f32_ds(yc, codes.data_ptr(), n, sc, mode, d_amax_accum=acc)   # smaller values: max stays
        torch.cuda.synchronize()
        assert f32_bits(acc)[0] == np.float32(max(orc.amax_f32(xn), orc.amax_f32(yn))).view(np.uint32)
        h.hif8_amax_f32(0, 0, acc)
        h.hif8_encode_bf16_ds(xb.data_ptr(), codes.data_ptr(), n, sc, mode, d_amax_accum=acc)
        torch.cuda.synchronize()
        assert_same_bytes(codes.cpu().numpy(), orc.encode_bf16(xbn, s, mode), "ds enc bf16")
        assert f32_bits(acc)[0] == np.float32(orc.amax_bf16(xbn)).view(np.uint32)
        o = torch.empty(n + 8, dtype=torch.float32, device=dev())[off:off + n]
        h.hif8_amax_f32(0, 0, acc)
        h.hif8_fake_quant_f32_ds(x.data_ptr(), o.data_ptr(), codes.data_ptr(), n, sc, mode, d_amax_accum=acc)
        torch.cuda.synchronize()
        wo, wc = orc.fake_quant_f32(xn, s, mode)
        assert_same_bytes(f32_bits(o.contiguous()), wo.view(np.uint32), "ds fq f32")
        assert f32_bits(acc)[0] == np.float32(orc.amax_f32(xn)).view(np.uint32)
        ob = torch.empty(n + 8, dtype=torch.bfloat16, device=dev())[off:off + n]
        h.hif8_amax_f32(0, 0, acc)
        h.hif8_fake_quant_bf16_ds(xb.data_ptr(), ob.data_ptr(), None, n, sc, mode, d_amax_accum=acc)
        torch.cuda.synchronize()
        wob, _ = orc.fake_quant_bf16(xbn, s, mode)
        assert_same_bytes(bf16_bits(ob.contiguous()), wob, "ds fq bf16")
        assert f32_bits(acc)[0] == np.float32(orc.amax_bf16(xbn)).view(np.uint32)


def test_hip_graph_replays_match_eager(h):
    """amax -> scale -> fused fake-quant captured in a HIP graph; every replay is checked against
    the eager result, with other eager work and synchronisations between replays."""
    from paper_2409_16626_amd import workloads
    x = workloads.activation_bf16(1024, 1024 + 8, dev()).view(-1)
    n = x.numel()
    am = torch.zeros(1, dtype=torch.float32, device=dev())
    sc = torch.zeros(2, dtype=torch.float32, device=dev())
    out = torch.empty_like(x)
    codes = torch.empty(n, dtype=torch.uint8, device=dev())

    def run():
        h.hif8_amax_bf16(x, n, am)
        h.hif8_scale_from_amax(am, sc, 32768.0, 0)
        h.hif8_fake_quant_bf16_ds(x, out, codes, n, sc, TA)

    run()
    torch.cuda.synchronize()
    ref_codes, ref_out, ref_sc = codes.clone(), out.clone(), sc.clone()
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            run()
    torch.cuda.synchronize()
    for rep in range(4):
        codes.zero_()
        out.zero_()
        sc.zero_()
        am.fill_(123.0)
        if rep == 2:                                   # new input between replays
            x.mul_(0.5)
            run()
            torch.cuda.synchronize()
            ref_codes, ref_out, ref_sc = codes.clone(), out.clone(), sc.clone()
            codes.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(codes, ref_codes) and torch.equal(out.view(torch.int16), ref_out.view(torch.int16))
        assert torch.equal(sc, ref_sc)
    wo, wc = orc.fake_quant_bf16(bf16_bits(x), np.float32(sc[0].item()), TA)
    assert_same_bytes(codes.cpu().numpy(), wc, "graph codes vs oracle")


def test_non_default_stream(h):
    from paper_2409_16626_amd import workloads
    x = workloads.normal_f32(1 << 18, dev())
    s = torch.cuda.Stream()
    dst = torch.empty(x.numel(), dtype=torch.uint8, device=dev())
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        h.hif8_encode_f32(x, dst, x.numel(), 1.0, TA)
    s.synchronize()
    assert_same_bytes(dst.cpu().numpy(), orc.encode_f32(x.cpu().numpy(), 1.0, TA), "stream")

