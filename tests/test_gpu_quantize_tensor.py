"""GPU parity of the per-tensor-scaling calls that do amax -> scale -> cast without leaving the device
(hif8_quantize_tensor_*, the group-wise hif8_multi_cast_*) and of the casts with an explicit standard-SR
threshold stream (hif8_*_sr), against the CPU oracle: amax, scale pair, codes and fake-quant outputs
bit for bit."""
import numpy as np
import pytest
import torch

from oracle import hif8_oracle as orc

pytestmark = pytest.mark.gpu

TA, HR, TE, SSR, SR = orc.RM_TA, orc.RM_HR, orc.RM_TE, orc.RM_SSR, orc.RM_SR
SAT, N2Z = orc.FLAG_SAT, orc.FLAG_NAN2ZERO

from gpu_util import assert_same_bytes, dev  # noqa: E402


@pytest.fixture(scope="module")
def h():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2409_16626_amd import hif8
    hif8.hif8_init()
    return hif8


KINDS = {
    "f32": (torch.float32, orc.amax_f32, orc.encode_f32, orc.fake_quant_f32),
    "bf16": (torch.bfloat16, orc.amax_bf16, orc.encode_bf16, orc.fake_quant_bf16),
    "f16": (torch.float16, orc.amax_f16, orc.encode_f16, orc.fake_quant_f16),
}


def host_view(x):
    """device tensor -> the numpy array the oracle takes (FP32 values, or uint16 patterns)."""
    if x.dtype == torch.float32:
        return x.cpu().numpy()
    return x.view(torch.int16).cpu().numpy().view(np.uint16)


def make_input(kind, n, seed, spread=(-12, 3)):
    rng = np.random.default_rng(seed)
    xf = (rng.standard_normal(n) * np.exp2(rng.uniform(spread[0], spread[1], n))).astype(np.float32)
    return torch.from_numpy(xf).to(dev()).to(KINDS[kind][0])


@pytest.mark.parametrize("kind", ["bf16", "f32", "f16"])
@pytest.mark.parametrize("n", [1, 7, 8, 4096, 8191, (1 << 16) + 3, (1 << 21) + 24, 5 * (1 << 20) + 1])
def test_quantize_tensor_matches_oracle(h, kind, n):
    """Sizes from one element to several hundred workgroups (more partial maxima than one wavefront reduces in
    one step), ragged tails included; codes only, fake-quant only, and both."""
    _, amx, enc, fq = KINDS[kind]
    fn = getattr(h, "hif8_quantize_tensor_" + kind)
    x = make_input(kind, n, 100 + n % 97)
    ws = torch.full((h.hif8_quantize_workspace_bytes() // 4,), -1, dtype=torch.int32, device=dev())   # garbage on purpose
    xh = host_view(x)
    w_am = amx(xh)
    for pow2, mode in ((0, TA), (1, HR | SAT)):
        w_s = orc.scale_from_amax(w_am, 32768.0, bool(pow2))
        want_out, want_codes = fq(xh, w_s, mode)
        for with_dst, with_codes in ((True, True), (False, True), (True, False)):
            am = torch.full((1,), 7.0, dtype=torch.float32, device=dev())
            sc = torch.zeros(2, dtype=torch.float32, device=dev())
            out = torch.zeros_like(x) if with_dst else None
            codes = torch.zeros(n, dtype=torch.uint8, device=dev()) if with_codes else None
            fn(x, out, codes, n, am, sc, ws, 32768.0, pow2, mode)
            torch.cuda.synchronize()
            assert am.item() == float(w_am), (kind, n, am.item(), w_am)
            assert sc[0].item() == float(w_s) and sc[1].item() == float(np.float32(1.0) / w_s)
            if with_codes:
                assert_same_bytes(codes.cpu().numpy(), want_codes, "codes %s n=%d" % (kind, n))
            if with_dst:
                got = out.view(torch.int32).cpu().numpy() if kind == "f32" else host_view(out)
                want = want_out.view(np.int32) if kind == "f32" else want_out
                assert_same_bytes(got, want, "fake-quant %s n=%d" % (kind, n))


def test_quantize_tensor_equals_the_three_separate_calls(h):
    """The C3 recipe (amax -> scale = 2^15 / amax -> fused fake-quant with codes) both ways, in place as well."""
    from paper_2409_16626_amd import workloads
    x = workloads.activation_bf16(1024, 1024 + 8, dev()).view(-1)
    n = x.numel()
    am1 = torch.zeros(1, dtype=torch.float32, device=dev()); sc1 = torch.zeros(2, dtype=torch.float32, device=dev())
    o1 = torch.empty_like(x); c1 = torch.empty(n, dtype=torch.uint8, device=dev())
    h.hif8_amax_bf16(x, n, am1)
    h.hif8_scale_from_amax(am1, sc1, 32768.0, 0)
    h.hif8_fake_quant_bf16_ds(x, o1, c1, n, sc1, TA)
    ws = torch.empty(1024, dtype=torch.int32, device=dev())
    am2 = torch.zeros(1, dtype=torch.float32, device=dev()); sc2 = torch.zeros(2, dtype=torch.float32, device=dev())
    o2 = x.clone(); c2 = torch.empty(n, dtype=torch.uint8, device=dev())
    h.hif8_quantize_tensor_bf16(o2, o2, c2, n, am2, sc2, ws, 32768.0, 0, TA)     # in place
    torch.cuda.synchronize()
    assert torch.equal(am1, am2) and torch.equal(sc1, sc2) and torch.equal(c1, c2)
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16))


def test_quantize_tensor_special_inputs(h):
    """Empty tensor, all zeros, Inf and NaN members (amax not finite -> scale 1), unaligned pointers."""
    ws = torch.empty(1024, dtype=torch.int32, device=dev())
    am = torch.full((1,), 5.0, dtype=torch.float32, device=dev()); sc = torch.full((2,), 9.0, dtype=torch.float32, device=dev())
    h.hif8_quantize_tensor_f32(None, None, None, 0, am, sc, ws)
    torch.cuda.synchronize()
    assert am.item() == 0.0 and sc.tolist() == [1.0, 1.0]
    for special in (0.0, float("inf"), float("nan")):
        x = make_input("f32", 20000, 3)
        x[::2] = 0.0 if special == 0.0 else x[::2]
        if special != 0.0:
            x[12345] = special
        else:
            x[:] = 0.0
        xh = host_view(x)
        codes = torch.zeros(x.numel(), dtype=torch.uint8, device=dev())
        h.hif8_quantize_tensor_f32(x, None, codes, x.numel(), am, sc, ws, 32768.0, 0, TA)
        torch.cuda.synchronize()
        w_am = orc.amax_f32(xh)
        w_s = orc.scale_from_amax(w_am, 32768.0, False)
        assert (np.isnan(w_am) and np.isnan(am.item())) or am.item() == float(w_am)
        assert sc[0].item() == float(w_s) == 1.0
        assert_same_bytes(codes.cpu().numpy(), orc.encode_f32(xh, w_s, TA), "special %r" % special)
    # element-per-lane path: source 2 bytes past a 16-byte boundary
    base = make_input("bf16", 40000 + 1, 4)
    x = base[1:]
    n = x.numel()
    out = torch.zeros_like(base)[1:]; codes = torch.zeros(n + 1, dtype=torch.uint8, device=dev())[1:]
    h.hif8_quantize_tensor_bf16(x, out, codes, n, am, sc, ws, 32768.0, 1, HR)
    torch.cuda.synchronize()
    xh = host_view(x.contiguous())
    w_s = orc.scale_from_amax(orc.amax_bf16(xh), 32768.0, True)
    wo, wc = orc.fake_quant_bf16(xh, w_s, HR)
    assert sc[0].item() == float(w_s)
    assert_same_bytes(codes.cpu().numpy(), wc, "unaligned codes")
    assert_same_bytes(host_view(out.contiguous()), wo, "unaligned fake-quant")


@pytest.mark.parametrize("group_mib", [1, 2, 192])
@pytest.mark.parametrize("mode,pow2", [(TA, 0), (HR | SAT, 1)])
def test_group_wise_multi_cast_matches_oracle_and_the_four_launch_form(h, group_mib, mode, pow2):
    """A tensor list with tiny, empty, ragged and large members, cut into groups of 1 MiB / 2 MiB / all in one:
    per-tensor amax, scale pair and codes equal the oracle's and those of the plain four-launch form."""
    rng = np.random.default_rng(77)
    sizes = [8192 * 3, 0, 1, 7, 8, 8200, 700001, 8192, 100003, 16, 0, 0, 65536 + 24, 1 << 20, 3, 0]
    h.hif8_set_tuning(h.TUNE_GROUP_MIB, group_mib)
    try:
        for kind in ("bf16", "f32"):
            _, amx, enc, _ = KINDS[kind]
            offs, total = [], 0
            for m in sizes:
                offs.append(total)
                total += (m + 15) // 16 * 16
            xf = torch.from_numpy((rng.standard_normal(total) * np.exp2(rng.uniform(-12, 3, total))).astype(np.float32)).to(dev())
            x = xf.to(KINDS[kind][0])
            codes = torch.zeros(total, dtype=torch.uint8, device=dev())
            items = [(x[o:o + m].data_ptr() if m else 0, codes[o:o + m].data_ptr() if m else 0, m) for o, m in zip(offs, sizes)]
            plan = h.hif8_multi_plan(items, src_is_16bit=kind != "f32")
            am = torch.full((plan.count,), 3.0, dtype=torch.float32, device=dev())
            sc = torch.full((plan.count, 2), 5.0, dtype=torch.float32, device=dev())
            fn = getattr(h, "hif8_multi_cast_" + kind)
            fn(plan.d_items, plan.count, plan.total_tiles, am, sc, 32768.0, pow2, mode, host_items=plan.host_items)
            torch.cuda.synchronize()
            xn = host_view(x)
            cg, amg, scg = codes.cpu().numpy(), am.cpu().numpy(), sc.cpu().numpy()
            for i, (o, m) in enumerate(zip(offs, sizes)):
                part = xn[o:o + m]
                w_am = amx(part)
                w_s = orc.scale_from_amax(w_am, 32768.0, bool(pow2))
                assert amg[i] == w_am and scg[i, 0] == w_s and scg[i, 1] == np.float32(1.0) / w_s, (kind, i, m, amg[i], scg[i])
                assert_same_bytes(cg[o:o + m], enc(part, w_s, mode), "grouped item %d (n=%d, %s)" % (i, m, kind))
            for o, m in zip(offs, sizes):          # bytes between the slices were not touched
                assert not cg[o + m:(o + m + 15) // 16 * 16].any()
            codes2 = torch.zeros_like(codes)
            items2 = [(x[o:o + m].data_ptr() if m else 0, codes2[o:o + m].data_ptr() if m else 0, m) for o, m in zip(offs, sizes)]
            plan2 = h.hif8_multi_plan(items2, src_is_16bit=kind != "f32")
            am2 = torch.zeros_like(am); sc2 = torch.zeros_like(sc)
            fn(plan2.d_items, plan2.count, plan2.total_tiles, am2, sc2, 32768.0, pow2, mode)   # no host copy: four launches
            torch.cuda.synchronize()
            assert torch.equal(codes, codes2) and torch.equal(am, am2) and torch.equal(sc, sc2)
    finally:
        h.hif8_set_tuning(h.TUNE_GROUP_MIB, 192)


@pytest.mark.parametrize("kind", ["f32", "bf16", "f16"])
def test_casts_with_an_explicit_threshold_stream(h, kind):
    """hif8_encode_*_sr / hif8_fake_quant_*_sr: element j draws t(seed, index_base + j) -- checked against the
    oracle with the same seed and base, across a multiple of 2^32 (where the key pair changes), with a base that
    is not a multiple of the vector width, and for slices of one tensor against the whole."""
    _, _, enc, fq = KINDS[kind]
    n = (1 << 16) + 13
    x = make_input(kind, n, 9, spread=(-26, 8))
    xh = host_view(x)
    e_sr, f_sr = getattr(h, "hif8_encode_%s_sr" % kind), getattr(h, "hif8_fake_quant_%s_sr" % kind)
    for seed, base in ((0, 0), (12345, 0), (12345, 1 << 20), (7, (1 << 32) - 1000), (7, (1 << 32) - 1001), (1 << 63, (5 << 32) - 30003)):
        codes = torch.zeros(n, dtype=torch.uint8, device=dev())
        e_sr(x, codes, n, 3.0, SR | SAT, seed, base)
        out = torch.zeros_like(x); codes2 = torch.zeros(n, dtype=torch.uint8, device=dev())
        f_sr(x, out, codes2, n, 3.0, SR | SAT, seed, base)
        torch.cuda.synchronize()
        try:
            orc.set_sr_seed(seed); orc.set_sr_index_base(base)
            want = enc(xh, 3.0, SR | SAT)
            want_out, _ = fq(xh, 3.0, SR | SAT)
        finally:
            orc.set_sr_seed(0); orc.set_sr_index_base(0)
        assert_same_bytes(codes.cpu().numpy(), want, "%s sr seed=%d base=%d" % (kind, seed, base))
        assert torch.equal(codes, codes2)
        got = out.view(torch.int32).cpu().numpy() if kind == "f32" else host_view(out)
        assert_same_bytes(got, want_out.view(np.int32) if kind == "f32" else want_out, "fq sr")
    # two tensors of one step share no thresholds when given consecutive index ranges; a slice continues the stream
    whole = torch.zeros(n, dtype=torch.uint8, device=dev())
    e_sr(x, whole, n, 1.0, SR, 99, 0)
    cut = 8 * 1000
    part = torch.zeros(n - cut, dtype=torch.uint8, device=dev())
    e_sr(x[cut:], part, n - cut, 1.0, SR, 99, cut)
    restart = torch.zeros(n - cut, dtype=torch.uint8, device=dev())
    e_sr(x[cut:], restart, n - cut, 1.0, SR, 99, 0)
    torch.cuda.synchronize()
    assert torch.equal(whole[cut:], part)
    assert not torch.equal(part, restart)
    # the process-wide seed is what a call without the arguments uses
    h.hif8_set_sr_seed(99)
    try:
        plain = torch.zeros(n, dtype=torch.uint8, device=dev())
        getattr(h, "hif8_encode_" + kind)(x, plain, n, 1.0, SR)
        torch.cuda.synchronize()
    finally:
        h.hif8_set_sr_seed(0)
    assert torch.equal(plain, whole)


def test_sr_seeds_give_different_carry_counts_on_the_gpu(h):
    """Sec. 3.2: a constant tensor under standard SR carries a binomial number of times; the count must move
    from seed to seed (it was one value for every seed while seeds only permuted one threshold sequence)."""
    n = 1 << 16
    x = torch.full((n,), 20.5, dtype=torch.float32, device=dev())
    counts = []
    for seed in range(16):
        c = torch.zeros(n, dtype=torch.uint8, device=dev())
        h.hif8_encode_f32_sr(x, c, n, 1.0, SR, seed, 0)
        torch.cuda.synchronize()
        try:
            orc.set_sr_seed(seed)
            want = orc.encode_f32(x.cpu().numpy(), 1.0, SR)
        finally:
            orc.set_sr_seed(0)
        assert_same_bytes(c.cpu().numpy(), want, "seed %d" % seed)
        counts.append(int((c != c.min()).sum().item()))
    assert len(set(counts)) >= 14
    assert all(abs(k - n / 8) < 5 * 84.7 for k in counts)
