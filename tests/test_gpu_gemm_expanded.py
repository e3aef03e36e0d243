"""GPU parity for the expanded-operand form of the simulated HiF8 GEMM: hif8_expand_bf16 (codes ->
bfloat16 patterns, rows padded with zeros to a multiple of 64) and hif8_gemm_expanded_* (tiles
loaded straight into LDS, bf16 MFMA, FP32 accumulation), against the fp64 oracle.

Bars: the expansion is bit-exact (every HiF8 value is exact in bfloat16); the GEMM carries the
same floating-point tolerance as the code-operand kernel, K * 2^-23 * sum_k |a b| * descale per
element (twice the worst case of an FP32 sum of exact products taken in any order), and is
bit-exact whenever every partial sum is exact in FP32.
"""
import numpy as np
import pytest
import torch

from oracle import gemm_oracle as go
from oracle import hif8_oracle as orc
from gpu_util import bf16_bits, dev

pytestmark = pytest.mark.gpu

FINITE = np.array([c for c in range(256) if np.isfinite(orc.decode_value(c))], np.uint8)


@pytest.fixture(scope="module")
def h():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2409_16626_amd import hif8
    hif8.hif8_init()
    yield hif8
    hif8.hif8_gemm_set_variant(0)


def random_codes(rng, shape, kind):
    if kind == "uniform_codes":
        return rng.choice(FINITE, size=shape).astype(np.uint8)
    x = rng.standard_normal(shape).astype(np.float32)
    return orc.encode_f32(x.reshape(-1), 8.0, orc.RM_TA).reshape(shape)


def expand(h, codes_np, poison=True):
    rows, K = codes_np.shape
    ld = h.hif8_expanded_ld(K)
    assert ld % 64 == 0 and K <= ld < K + 64
    dst = torch.full((rows, ld), 0x7FC1 if poison else 0, dtype=torch.int16, device=dev())   # NaN patterns: padding must be written
    h.hif8_expand_bf16(torch.from_numpy(codes_np).to(dev()), rows, K, dst, ld)
    return dst, ld


def want_expanded(codes_np, ld):
    rows, K = codes_np.shape
    f = orc.decode_f32(codes_np.reshape(-1), 1.0).view(np.uint32).reshape(rows, K)
    assert np.all((f & 0xFFFF) == 0)            # exact in bfloat16: the low half of the binary32 pattern is empty
    out = np.zeros((rows, ld), np.uint16)
    out[:, :K] = (f >> 16).astype(np.uint16)
    return out


@pytest.mark.parametrize("rows,K", [(1, 256), (3, 1), (7, 63), (5, 64), (9, 65), (33, 200), (300, 4104), (2, 8), (64, 1000)])
def test_expand_is_exact_and_pads_with_zeros(h, rows, K):
    rng = np.random.default_rng(rows * 1000 + K)
    codes = rng.integers(0, 256, size=(rows, K), dtype=np.uint8)          # NaN and Inf codes included
    if rows * K >= 256:
        codes.reshape(-1)[:256] = np.arange(256, dtype=np.uint8)          # every code at least once
    dst, ld = expand(h, codes)
    torch.cuda.synchronize()
    got = dst.cpu().numpy().view(np.uint16)
    assert np.array_equal(got, want_expanded(codes, ld))


def test_expand_unaligned_source(h):
    rng = np.random.default_rng(3)
    rows, K = 11, 72
    codes = rng.integers(0, 256, size=(rows, K), dtype=np.uint8)
    buf = torch.zeros(rows * K + 8, dtype=torch.uint8, device=dev())
    buf[3:3 + rows * K] = torch.from_numpy(codes.reshape(-1)).to(dev())
    ld = h.hif8_expanded_ld(K)
    dst = torch.full((rows, ld), -1, dtype=torch.int16, device=dev())
    h.hif8_expand_bf16(buf[3:].data_ptr(), rows, K, dst, ld)
    torch.cuda.synchronize()
    assert np.array_equal(dst.cpu().numpy().view(np.uint16), want_expanded(codes, ld))


def check(got, ca, cb, sa, sb, extra_rel=0.0):
    want = go.gemm_hif8(ca, cb, sa, sb)
    bound = go.gemm_abs_bound(ca, cb, sa, sb)
    K = ca.shape[1]
    tol = K * 2.0 ** -23 * bound + extra_rel * np.abs(want) + 1e-45
    diff = np.abs(got.astype(np.float64) - want)
    bad = np.argwhere(diff > tol)
    assert bad.size == 0, "%d outside the bound; first %s: got %r want %r tol %r" % (
        len(bad), bad[0], got[tuple(bad[0])], want[tuple(bad[0])], tol[tuple(bad[0])])
    return diff, bound


# several tiles of both tile shapes, ragged edges in M, N and K, K below one K step, single elements
SHAPES = [(32, 32, 16), (128, 128, 64), (100, 70, 48), (257, 129, 80), (1, 1, 1), (64, 300, 1040),
          (256, 256, 32), (300, 520, 4096), (33, 17, 19), (513, 259, 130), (1100, 1300, 72), (4200, 4100, 64),
          (300, 300, 256), (260, 140, 320), (270, 520, 448)]   # 4, 5 and 7 K steps: every length of the loop's tail


@pytest.mark.parametrize("variant", [0, 9, 10, 11])     # by problem size; 128 x 128; 256 x 256 as 2 x 2 and as 2 x 4 wavefronts
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_expanded_f32_matches_oracle(h, variant, M, N, K):
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    h.hif8_gemm_set_variant(variant)
    for kind in ("cast_normal", "uniform_codes"):
        ca, cb = random_codes(rng, (M, K), kind), random_codes(rng, (N, K), kind)
        a, ld = expand(h, ca)
        b, _ = expand(h, cb)
        out = torch.full((M, N), 7.0, dtype=torch.float32, device=dev())
        sa, sb = (8.0, 0.5) if kind == "cast_normal" else (1.0, 1.0)
        h.hif8_gemm_expanded_f32(a, b, out, M, N, K, ld, sa, sb)
        torch.cuda.synchronize()
        diff, bound = check(out.cpu().numpy(), ca, cb, sa, sb)
        assert np.mean(diff) <= 0.05 * K * 2.0 ** -23 * np.mean(bound) + 1e-45


@pytest.mark.parametrize("M,N,K", [(200, 136, 512), (4100, 4200, 192)])     # 128 x 128 tiles, then 256 x 256 tiles
def test_gemm_expanded_exact_when_sums_fit_24_bits(h, M, N, K):
    """Small integers as operands: every partial sum is an integer below 2^24, so FP32 accumulation
    is exact in any order and the result must equal the oracle bit for bit -- and the code-operand kernel."""
    rng = np.random.default_rng(5)
    ints = np.array([0x00, 0x08, 0x10, 0x14, 0x20, 0x88, 0x90, 0x94, 0xA0], np.uint8)   # 0, 1, 2, 3, 4, -1, -2, -3, -4
    assert [orc.decode_value(int(c)) for c in ints] == [0, 1, 2, 3, 4, -1, -2, -3, -4]
    ca, cb = rng.choice(ints, size=(M, K)), rng.choice(ints, size=(N, K))
    a, ld = expand(h, ca)
    b, _ = expand(h, cb)
    want64 = go.gemm_hif8(ca, cb)
    out = torch.zeros(M, N, dtype=torch.float32, device=dev())
    for variant in (9, 10, 11, 0):
        h.hif8_gemm_set_variant(variant)
        out.zero_()
        h.hif8_gemm_expanded_f32(a, b, out, M, N, K, ld, 1.0, 1.0)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().astype(np.float64), want64), variant
    other = torch.zeros(M, N, dtype=torch.float32, device=dev())
    h.hif8_gemm_f32(torch.from_numpy(ca).to(dev()), torch.from_numpy(cb).to(dev()), other, M, N, K, 1.0, 1.0)
    torch.cuda.synchronize()
    assert torch.equal(out, other)
    o16 = torch.zeros(M, N, dtype=torch.bfloat16, device=dev())
    oh = torch.zeros(M, N, dtype=torch.float16, device=dev())
    h.hif8_gemm_expanded_bf16(a, b, o16, M, N, K, ld, 4.0, 0.25)
    h.hif8_gemm_expanded_f16(a, b, oh, M, N, K, ld, 4.0, 0.25)
    torch.cuda.synchronize()
    want = torch.from_numpy(want64).to(torch.float32)
    assert torch.equal(o16.cpu(), want.to(torch.bfloat16)) and torch.equal(oh.cpu(), want.to(torch.float16))


def test_gemm_expanded_16bit_outputs_and_scales(h):
    rng = np.random.default_rng(6)
    M, N, K = 192, 160, 256
    ca, cb = random_codes(rng, (M, K), "cast_normal"), random_codes(rng, (N, K), "cast_normal")
    a, ld = expand(h, ca)
    b, _ = expand(h, cb)
    for sa, sb in ((8.0, 8.0), (0.37, 1311.7), (2.0 ** -20, 2.0 ** 10)):
        o16 = torch.zeros(M, N, dtype=torch.bfloat16, device=dev())
        oh = torch.zeros(M, N, dtype=torch.float16, device=dev())
        h.hif8_gemm_expanded_bf16(a, b, o16, M, N, K, ld, sa, sb)
        h.hif8_gemm_expanded_f16(a, b, oh, M, N, K, ld, sa, sb)
        torch.cuda.synchronize()
        check(o16.float().cpu().numpy(), ca, cb, sa, sb, extra_rel=2.0 ** -8)
        want = go.gemm_hif8(ca, cb, sa, sb)
        if np.abs(want).max() < 6.0e4 and np.abs(want)[want != 0].min() > 1e-4:
            check(oh.float().cpu().numpy(), ca, cb, sa, sb, extra_rel=2.0 ** -10)


def test_gemm_expanded_special_codes_follow_ieee(h):
    rng = np.random.default_rng(7)
    M, N, K = 64, 64, 64
    ca, cb = random_codes(rng, (M, K), "cast_normal"), random_codes(rng, (N, K), "cast_normal")
    ca[3, 5] = 0x6F       # +Inf
    ca[9, 0] = 0x80       # NaN
    ca[20, 7] = 0xEF      # -Inf, meeting a zero below: Inf * 0 = NaN
    cb[11, 7] = 0x00
    a, ld = expand(h, ca)
    b, _ = expand(h, cb)
    out = torch.zeros(M, N, dtype=torch.float32, device=dev())
    h.hif8_gemm_expanded_f32(a, b, out, M, N, K, ld, 1.0, 1.0)
    torch.cuda.synchronize()
    got, want = out.cpu().numpy(), go.gemm_hif8(ca, cb)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(np.isposinf(got), np.isposinf(want)) and np.array_equal(np.isneginf(got), np.isneginf(want))
    assert np.isnan(want[9]).all() and np.isnan(want[20, 11]) and np.isinf(want[3]).any()


def test_gemm_expanded_sqerr_epilogue(h):
    rng = np.random.default_rng(9)
    M, N, K = 300, 200, 520
    x = rng.standard_normal((M, K)).astype(np.float32)
    w = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    ref = (x.astype(np.float64) @ w.astype(np.float64).T).astype(np.float32)
    ca = orc.encode_f32(x.reshape(-1), 4.0, orc.RM_TA).reshape(M, K)
    cb = orc.encode_f32(w.reshape(-1), 64.0, orc.RM_TA).reshape(N, K)
    a, ld = expand(h, ca)
    b, _ = expand(h, cb)
    r = torch.from_numpy(ref).to(dev())
    want_o = go.gemm_hif8(ca, cb, 4.0, 64.0)
    S = np.sum((want_o - ref.astype(np.float64)) ** 2)
    e = K * 2.0 ** -23 * go.gemm_abs_bound(ca, cb, 4.0, 64.0)
    tol = 2 * np.sqrt(S * np.sum(e ** 2)) + np.sum(e ** 2)
    err = torch.zeros(2, dtype=torch.float64, device=dev())
    h.hif8_gemm_expanded_sqerr(a, b, r, M, N, K, ld, 4.0, 64.0, err)
    h.hif8_gemm_expanded_sqerr(a, b, r, M, N, K, ld, 4.0, 64.0, err)          # accumulates
    torch.cuda.synchronize()
    got = err.cpu().numpy()
    assert got[1] == 0.0 and abs(got[0] - 2 * S) <= 2 * tol, (got, S, tol)
    assert abs(got[0] / (2 * S) - 1) < 1e-4


def test_gemm_expanded_argument_checks(h):
    from paper_2409_16626_amd.hif8 import Hif8Error
    a = torch.zeros(64, 64, dtype=torch.int16, device=dev())
    out = torch.zeros(64, 64, dtype=torch.float32, device=dev())
    codes = torch.zeros(64, 64, dtype=torch.uint8, device=dev())
    for bad in (dict(ld=63), dict(ld=0), dict(K=0), dict(K=65), dict(sa=0.0), dict(sa=float("inf"))):
        kw = dict(K=64, ld=64, sa=1.0)
        kw.update(bad)
        with pytest.raises(Hif8Error):
            h.hif8_gemm_expanded_f32(a, a, out, 64, 64, kw["K"], kw["ld"], kw["sa"], 1.0)
    with pytest.raises(Hif8Error):
        h.hif8_gemm_expanded_f32(a.view(-1)[1:].data_ptr(), a, out, 32, 32, 64, 64, 1.0, 1.0)   # 2 bytes off alignment
    with pytest.raises(Hif8Error):
        h.hif8_expand_bf16(codes, 64, 64, a, 32)                                                  # pitch below K
    with pytest.raises(Hif8Error):
        h.hif8_expand_bf16(codes, 64, 64, a, 96)                                                  # not a multiple of 64
    h.hif8_gemm_expanded_f32(a, a, out, 0, 64, 64, 64, 1.0, 1.0)                                  # empty: nothing to do
    torch.cuda.synchronize()


def test_calibrate_layer_any_k(h):
    """Algorithm 1's inner loop on a layer whose K is not a multiple of the K step (the expanded
    operands are padded): error table and chosen (Ea, Ew) against the oracle."""
    rng = np.random.default_rng(13)
    M, N, K = 96, 130, 100
    x = rng.standard_normal((M, K)).astype(np.float32)
    w = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    tx, tw = torch.from_numpy(x).to(dev()).to(torch.bfloat16), torch.from_numpy(w).to(dev()).to(torch.bfloat16)
    xf, wf = tx.float().cpu().numpy(), tw.float().cpu().numpy()
    o_ref = (xf.astype(np.float64) @ wf.astype(np.float64).T).astype(np.float32)
    want, want_best = go.calibrate_layer(bf16_bits(tx), bf16_bits(tw), o_ref, orc.SRC_BF16, -3, 6, -2, 9)
    nbytes = h.hif8_calibrate_workspace_bytes(M, N, K, 6, 9)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev())
    err = torch.full((6, 9), -1.0, dtype=torch.float64, device=dev())
    best = torch.zeros(2, dtype=torch.int32, device=dev())
    h.hif8_calibrate_layer_bf16(tx, tw, torch.from_numpy(o_ref).to(dev()), M, N, K, -3, 6, -2, 9, orc.RM_TA, ws, nbytes, err, best)
    torch.cuda.synchronize()
    got = err.cpu().numpy()
    fin = np.isfinite(want)
    assert np.array_equal(np.isfinite(got), fin)
    np.testing.assert_allclose(got[fin], want[fin], rtol=2e-4)
    assert tuple(best.cpu().tolist()) == want_best


def expand_t(h, codes_np):
    rows, cols = codes_np.shape
    ld = h.hif8_expanded_ld(rows)
    dst = torch.full((cols, ld), 0x7FC1, dtype=torch.int16, device=dev())            # NaN patterns: padding must be written
    h.hif8_expand_bf16_t(torch.from_numpy(codes_np).to(dev()), rows, cols, dst, ld)
    return dst, ld


@pytest.mark.parametrize("rows,cols", [(1, 1), (3, 70), (64, 64), (65, 63), (100, 257), (1000, 48), (130, 4112), (7, 16)])
def test_transposing_expand_is_exact_and_pads_with_zeros(h, rows, cols):
    rng = np.random.default_rng(rows * 77 + cols)
    codes = rng.integers(0, 256, size=(rows, cols), dtype=np.uint8)
    dst, ld = expand_t(h, codes)
    torch.cuda.synchronize()
    assert np.array_equal(dst.cpu().numpy().view(np.uint16), want_expanded(np.ascontiguousarray(codes.T), ld))
    # a larger pitch than the minimum is filled with zeros as well; unaligned source
    ld2 = ld + 128
    buf = torch.zeros(rows * cols + 8, dtype=torch.uint8, device=dev())
    buf[5:5 + rows * cols] = torch.from_numpy(codes.reshape(-1)).to(dev())
    dst2 = torch.full((cols, ld2), -1, dtype=torch.int16, device=dev())
    h.hif8_expand_bf16_t(buf[5:].data_ptr(), rows, cols, dst2, ld2)
    torch.cuda.synchronize()
    assert np.array_equal(dst2.cpu().numpy().view(np.uint16), want_expanded(np.ascontiguousarray(codes.T), ld2))


def test_linear_layer_forward_and_backward_products(h):
    """The three GEMMs of a linear layer in simulated HiF8 (Sec. 5: activations, weights and activation
    gradients are cast): Y = X W^T, dX = dY W, dW = dY^T X, all on the K-contiguous kernel through plain and
    transposing expansions; each against the oracle on the correspondingly transposed code matrices."""
    rng = np.random.default_rng(31)
    M, N, K = 200, 136, 264
    cx = random_codes(rng, (M, K), "cast_normal")
    cw = random_codes(rng, (N, K), "cast_normal")
    cdy = random_codes(rng, (M, N), "cast_normal")
    xe, ldk = expand(h, cx)
    we, _ = expand(h, cw)
    dye, ldn = expand(h, cdy)
    wte, ldn2 = expand_t(h, cw)          # [K, ld(N)]
    dyte, ldm = expand_t(h, cdy)         # [N, ld(M)]
    xte, ldm2 = expand_t(h, cx)          # [K, ld(M)]
    assert ldn == ldn2 and ldm == ldm2
    y = torch.zeros(M, N, dtype=torch.float32, device=dev())
    dx = torch.zeros(M, K, dtype=torch.float32, device=dev())
    dw = torch.zeros(N, K, dtype=torch.float32, device=dev())
    h.hif8_gemm_expanded_f32(xe, we, y, M, N, K, ldk, 8.0, 8.0)
    h.hif8_gemm_expanded_f32(dye, wte, dx, M, K, N, ldn, 8.0, 8.0)
    h.hif8_gemm_expanded_f32(dyte, xte, dw, N, K, M, ldm, 8.0, 8.0)
    torch.cuda.synchronize()
    check(y.cpu().numpy(), cx, cw, 8.0, 8.0)
    check(dx.cpu().numpy(), cdy, np.ascontiguousarray(cw.T), 8.0, 8.0)
    check(dw.cpu().numpy(), np.ascontiguousarray(cdy.T), np.ascontiguousarray(cx.T), 8.0, 8.0)


@pytest.mark.parametrize("M,N,K", [(8192, 8192, 8192), (8192, 11008, 4096)])
def test_gemm_benchmark_shapes_sampled_outputs(h, M, N, K):
    """The shapes and the operand recipe bench.py times (codes uniform in 0x08..0x4F), default launch
    configuration, both kernels: 64 x 64 sampled outputs (first and last rows and columns included)
    against the oracle's product of the sampled rows."""
    g = torch.Generator(device=dev()).manual_seed(M + N + K)
    ca = torch.randint(8, 0x50, (M, K), generator=g, dtype=torch.int32, device=dev()).to(torch.uint8)
    cb = torch.randint(8, 0x50, (N, K), generator=g, dtype=torch.int32, device=dev()).to(torch.uint8)
    h.hif8_gemm_set_variant(0)
    ld = h.hif8_expanded_ld(K)
    xa = torch.empty(M, ld, dtype=torch.bfloat16, device=dev())
    xb = torch.empty(N, ld, dtype=torch.bfloat16, device=dev())
    h.hif8_expand_bf16(ca, M, K, xa, ld)
    h.hif8_expand_bf16(cb, N, K, xb, ld)
    out_x = torch.full((M, N), float("nan"), dtype=torch.float32, device=dev())
    out_c = torch.full((M, N), float("nan"), dtype=torch.float32, device=dev())
    h.hif8_gemm_expanded_f32(xa, xb, out_x, M, N, K, ld, 4.0, 0.5)
    h.hif8_gemm_f32(ca, cb, out_c, M, N, K, 4.0, 0.5)
    torch.cuda.synchronize()
    # every output was written (the ragged shape is covered by two launches with different tiles), and the
    # two kernels agree everywhere to accumulation-order noise
    assert not bool(torch.isnan(out_x).any()) and not bool(torch.isnan(out_c).any())
    assert float((out_x - out_c).abs().max()) <= 1e-4 * float(out_c.abs().max())
    rng = np.random.default_rng(1)
    rows = np.unique(np.concatenate([[0, 1, 255, 256, M - 1], rng.integers(0, M, 59)]))
    # columns on both sides of the places where a second launch with smaller tiles may take over
    edge = [N - 769, N - 768, N - 767, N - 641, N - 640, N - 129, N - 128, N - 1]
    cols = np.unique(np.concatenate([[0, 31, 32, 257], edge, rng.integers(0, N, 52)]))
    sa, sb = ca[torch.from_numpy(rows).to(dev())].cpu().numpy(), cb[torch.from_numpy(cols).to(dev())].cpu().numpy()
    for out in (out_x, out_c):
        got = out[torch.from_numpy(rows).to(dev())][:, torch.from_numpy(cols).to(dev())].cpu().numpy()
        diff, bound = check(got, sa, sb, 4.0, 0.5)
        assert np.mean(diff) <= 0.05 * K * 2.0 ** -23 * np.mean(bound)


def test_ragged_round_shape_all_outputs_and_sqerr(h):
    """A shape whose 256 x 256 tiles leave a ragged last round (two launches: large tiles, then small tiles
    over the remaining columns), with a short K: every output of both kernels against the fp64 product of the
    oracle-decoded operands (a torch matmul, not this library), and the squared-error epilogues against the error
    of those outputs."""
    M, N, K = 8192, 11008, 64
    g = torch.Generator(device=dev()).manual_seed(77)
    ca = torch.randint(8, 0x50, (M, K), generator=g, dtype=torch.int32, device=dev()).to(torch.uint8)
    cb = torch.randint(8, 0x50, (N, K), generator=g, dtype=torch.int32, device=dev()).to(torch.uint8)
    h.hif8_gemm_set_variant(0)
    ld = h.hif8_expanded_ld(K)
    xa = torch.empty(M, ld, dtype=torch.bfloat16, device=dev())
    xb = torch.empty(N, ld, dtype=torch.bfloat16, device=dev())
    h.hif8_expand_bf16(ca, M, K, xa, ld)
    h.hif8_expand_bf16(cb, N, K, xb, ld)
    out_x = torch.full((M, N), float("nan"), dtype=torch.float32, device=dev())
    out_c = torch.full((M, N), float("nan"), dtype=torch.float32, device=dev())
    h.hif8_gemm_expanded_f32(xa, xb, out_x, M, N, K, ld, 1.0, 1.0)
    h.hif8_gemm_f32(ca, cb, out_c, M, N, K, 1.0, 1.0)
    torch.cuda.synchronize()
    # values of codes 0x08..0x4F lie in a few binades around 1: K = 64 products sum exactly enough for fp64 on the GPU
    # to serve as the exact product of the decoded operands (decode is pinned against the oracle elsewhere)
    dec = torch.from_numpy(orc.decode_f32(np.arange(256, dtype=np.uint8), 1.0).astype(np.float64)).to(dev())
    exact = dec[ca.long()] @ dec[cb.long()].T
    bound = (dec[ca.long()].abs() @ dec[cb.long()].abs().T) * (K * 2.0 ** -23)
    for out in (out_x, out_c):
        assert not bool(torch.isnan(out).any())
        assert bool(((out.double() - exact).abs() <= bound).all())
    ref = torch.randn(M, N, generator=g, device=dev())
    for out, call in ((out_x, lambda e: h.hif8_gemm_expanded_sqerr(xa, xb, ref, M, N, K, ld, 1.0, 1.0, e)),
                      (out_c, lambda e: h.hif8_gemm_sqerr(ca, cb, ref, M, N, K, 1.0, 1.0, e))):
        err = torch.zeros(1, dtype=torch.float64, device=dev())
        call(err)
        torch.cuda.synchronize()
        want = float(((out.double() - ref.double()) ** 2).sum())
        assert abs(err.item() - want) <= 1e-10 * want
