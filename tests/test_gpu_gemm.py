"""GPU parity for the simulated HiF8 GEMM (bf16 MFMA on decoded codes, FP32 accumulation) against
the fp64 oracle.

Tolerance (floating point, derived from the arithmetic): products of two HiF8 values are exact;
an FP32 sum of K terms in any order differs from the exact sum by at most
(K - 1) * 2^-24 * sum_k |a_k b_k| (1 + o(1)); the descale multiply adds 2^-24 relative.  The
tests allow K * 2^-23 * sum_k |a b| * descale per element (twice the bound) and also check
that the typical error is far below it.  BF16 / FP16 outputs add half an ulp of that format.
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
    if kind == "uniform_codes":          # every finite code equally likely: 38 binades of dynamic range
        return rng.choice(FINITE, size=shape).astype(np.uint8)
    x = rng.standard_normal(shape).astype(np.float32)   # cast of N(0,1) data, the usual operand
    return orc.encode_f32(x.reshape(-1), 8.0, orc.RM_TA).reshape(shape)


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


SHAPES = [(32, 32, 16), (128, 128, 64), (100, 70, 48), (257, 129, 80), (1, 1, 16), (64, 300, 1040),
          (256, 256, 32), (300, 520, 4096), (33, 17, 16)]


@pytest.mark.parametrize("variant", [5, 6])
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_f32_matches_oracle(h, variant, M, N, K):
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    h.hif8_gemm_set_variant(variant)
    for kind in ("cast_normal", "uniform_codes"):
        ca, cb = random_codes(rng, (M, K), kind), random_codes(rng, (N, K), kind)
        a, b = torch.from_numpy(ca).to(dev()), torch.from_numpy(cb).to(dev())
        out = torch.full((M, N), 7.0, dtype=torch.float32, device=dev())
        sa, sb = (8.0, 0.5) if kind == "cast_normal" else (1.0, 1.0)
        h.hif8_gemm_f32(a, b, out, M, N, K, sa, sb)
        torch.cuda.synchronize()
        diff, bound = check(out.cpu().numpy(), ca, cb, sa, sb)
        # typical error: a small fraction of the worst-case bound
        assert np.mean(diff) <= 0.05 * K * 2.0 ** -23 * np.mean(bound) + 1e-45


def test_gemm_exact_when_sums_fit_24_bits(h):
    """Small integers as operands: every partial sum is an integer below 2^24, so FP32
    accumulation is exact in any order and the result must equal the oracle bit for bit."""
    rng = np.random.default_rng(5)
    M, N, K = 200, 136, 512
    ints = np.array([0x00, 0x08, 0x10, 0x14, 0x20, 0x88, 0x90, 0x94, 0xA0], np.uint8)   # 0, 1, 2, 3, 4, -1, -2, -3, -4
    assert [orc.decode_value(int(c)) for c in ints] == [0, 1, 2, 3, 4, -1, -2, -3, -4]
    ca, cb = rng.choice(ints, size=(M, K)), rng.choice(ints, size=(N, K))
    a, b = torch.from_numpy(ca).to(dev()), torch.from_numpy(cb).to(dev())
    for variant in (5, 6):
        h.hif8_gemm_set_variant(variant)
        out = torch.zeros(M, N, dtype=torch.float32, device=dev())
        h.hif8_gemm_f32(a, b, out, M, N, K, 1.0, 1.0)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().astype(np.float64), go.gemm_hif8(ca, cb))
        o16 = torch.zeros(M, N, dtype=torch.bfloat16, device=dev())
        h.hif8_gemm_bf16(a, b, o16, M, N, K, 4.0, 0.25)
        oh = torch.zeros(M, N, dtype=torch.float16, device=dev())
        h.hif8_gemm_f16(a, b, oh, M, N, K, 4.0, 0.25)
        torch.cuda.synchronize()
        want = torch.from_numpy(go.gemm_hif8(ca, cb)).to(torch.float32)
        assert torch.equal(o16.cpu(), want.to(torch.bfloat16)) and torch.equal(oh.cpu(), want.to(torch.float16))


def test_gemm_16bit_outputs_and_scales(h):
    rng = np.random.default_rng(6)
    M, N, K = 192, 160, 256
    ca, cb = random_codes(rng, (M, K), "cast_normal"), random_codes(rng, (N, K), "cast_normal")
    a, b = torch.from_numpy(ca).to(dev()), torch.from_numpy(cb).to(dev())
    h.hif8_gemm_set_variant(0)
    for sa, sb in ((8.0, 8.0), (0.37, 1311.7), (2.0 ** -20, 2.0 ** 10)):
        o16 = torch.zeros(M, N, dtype=torch.bfloat16, device=dev())
        oh = torch.zeros(M, N, dtype=torch.float16, device=dev())
        h.hif8_gemm_bf16(a, b, o16, M, N, K, sa, sb)
        h.hif8_gemm_f16(a, b, oh, M, N, K, sa, sb)
        torch.cuda.synchronize()
        check(o16.float().cpu().numpy(), ca, cb, sa, sb, extra_rel=2.0 ** -8)
        want = go.gemm_hif8(ca, cb, sa, sb)
        if np.abs(want).max() < 6.0e4 and np.abs(want)[want != 0].min() > 1e-4:
            check(oh.float().cpu().numpy(), ca, cb, sa, sb, extra_rel=2.0 ** -10)


def test_gemm_special_codes_follow_ieee(h):
    rng = np.random.default_rng(7)
    M, N, K = 64, 64, 64
    ca, cb = random_codes(rng, (M, K), "cast_normal"), random_codes(rng, (N, K), "cast_normal")
    ca[3, 5] = 0x6F       # +Inf
    ca[9, 0] = 0x80       # NaN
    ca[20, 7] = 0xEF      # -Inf, meeting a zero below: Inf * 0 = NaN
    cb[11, 7] = 0x00
    a, b = torch.from_numpy(ca).to(dev()), torch.from_numpy(cb).to(dev())
    for variant in (5, 6):
        h.hif8_gemm_set_variant(variant)
        out = torch.zeros(M, N, dtype=torch.float32, device=dev())
        h.hif8_gemm_f32(a, b, out, M, N, K, 1.0, 1.0)
        torch.cuda.synchronize()
        got, want = out.cpu().numpy(), go.gemm_hif8(ca, cb)
        assert np.array_equal(np.isnan(got), np.isnan(want))
        assert np.array_equal(np.isposinf(got), np.isposinf(want)) and np.array_equal(np.isneginf(got), np.isneginf(want))
        assert np.isnan(want[9]).all() and np.isnan(want[20, 11]) and np.isinf(want[3]).any()


@pytest.mark.parametrize("M,N,K,off", [(40, 24, 17, 0), (5, 9, 100, 0), (64, 64, 64, 1), (3, 2, 1, 0)])
def test_gemm_plain_kernel_for_odd_k_and_alignment(h, M, N, K, off):
    rng = np.random.default_rng(8)
    ca, cb = random_codes(rng, (M, K), "cast_normal"), random_codes(rng, (N, K), "cast_normal")
    abuf = torch.zeros(M * K + 16, dtype=torch.uint8, device=dev())
    abuf[off:off + M * K] = torch.from_numpy(ca.reshape(-1)).to(dev())
    b = torch.from_numpy(cb).to(dev())
    out = torch.zeros(M, N, dtype=torch.float32, device=dev())
    h.hif8_gemm_f32(abuf[off:].data_ptr(), b, out, M, N, K, 2.0, 1.0)
    torch.cuda.synchronize()
    check(out.cpu().numpy(), ca, cb, 2.0, 1.0)


def test_gemm_sqerr_epilogue(h):
    """*d_err += sum (out - ref)^2.  With d = out - ref exact and e the GEMM's rounding error,
    the two sums differ by at most 2 sqrt(S sum e^2) + sum e^2; e is bounded as above."""
    rng = np.random.default_rng(9)
    M, N, K = 300, 200, 512
    x = rng.standard_normal((M, K)).astype(np.float32)
    w = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    ref = (x.astype(np.float64) @ w.astype(np.float64).T).astype(np.float32)
    ca = orc.encode_f32(x.reshape(-1), 4.0, orc.RM_TA).reshape(M, K)
    cb = orc.encode_f32(w.reshape(-1), 64.0, orc.RM_TA).reshape(N, K)
    a, b, r = torch.from_numpy(ca).to(dev()), torch.from_numpy(cb).to(dev()), torch.from_numpy(ref).to(dev())
    want_o = go.gemm_hif8(ca, cb, 4.0, 64.0)
    S = np.sum((want_o - ref.astype(np.float64)) ** 2)
    e = K * 2.0 ** -23 * go.gemm_abs_bound(ca, cb, 4.0, 64.0)
    tol = 2 * np.sqrt(S * np.sum(e ** 2)) + np.sum(e ** 2)
    for variant in (5, 6):
        h.hif8_gemm_set_variant(variant)
        err = torch.zeros(2, dtype=torch.float64, device=dev())
        h.hif8_gemm_sqerr(a, b, r, M, N, K, 4.0, 64.0, err)
        h.hif8_gemm_sqerr(a, b, r, M, N, K, 4.0, 64.0, err)          # accumulates
        torch.cuda.synchronize()
        got = err.cpu().numpy()
        assert got[1] == 0.0 and abs(got[0] - 2 * S) <= 2 * tol, (got, S, tol)
        assert abs(got[0] / (2 * S) - 1) < 1e-4


@pytest.mark.parametrize("kind", ["f32", "bf16", "f16"])
def test_calibrate_layer_matches_algorithm_1_oracle(h, kind):
    """The whole inner loop of Algorithm 1 for one layer: 10 x 10 search square, TA casts,
    error against the high-precision output; error table and chosen (Ea, Ew) against the oracle."""
    rng = np.random.default_rng(12)
    M, N, K = 160, 200, 256
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[rng.random((M, K)) < 0.002] *= 30.0                              # a few activation outliers
    w = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)        # weights far below 1
    tx, tw = torch.from_numpy(x).to(dev()), torch.from_numpy(w).to(dev())
    okind = {"f32": orc.SRC_F32, "bf16": orc.SRC_BF16, "f16": orc.SRC_F16}[kind]
    if kind == "bf16":
        tx, tw = tx.to(torch.bfloat16), tw.to(torch.bfloat16)
        xn, wn = bf16_bits(tx), bf16_bits(tw)
        xf, wf = tx.float().cpu().numpy(), tw.float().cpu().numpy()
    elif kind == "f16":
        tx, tw = tx.to(torch.float16), tw.to(torch.float16)
        xn, wn = tx.view(torch.int16).cpu().numpy().view(np.uint16), tw.view(torch.int16).cpu().numpy().view(np.uint16)
        xf, wf = tx.float().cpu().numpy(), tw.float().cpu().numpy()
    else:
        xn, wn, xf, wf = x, w, x, w
    o_ref = (xf.astype(np.float64) @ wf.astype(np.float64).T).astype(np.float32)   # the layer's high-precision output
    want, want_best = go.calibrate_layer(xn, wn, o_ref, okind, -4, 10, -4, 10)
    nbytes = h.hif8_calibrate_workspace_bytes(M, N, K, 10, 10)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev())
    err = torch.full((10, 10), -1.0, dtype=torch.float64, device=dev())
    best = torch.zeros(2, dtype=torch.int32, device=dev())
    h.hif8_gemm_set_variant(0)
    getattr(h, "hif8_calibrate_layer_" + kind)(tx, tw, torch.from_numpy(o_ref).to(dev()), M, N, K, -4, 10, -4, 10,
                                               orc.RM_TA, ws, nbytes, err, best)
    torch.cuda.synchronize()
    got = err.cpu().numpy()
    fin = np.isfinite(want)
    assert np.array_equal(np.isfinite(got), fin) and fin.sum() >= 60
    np.testing.assert_allclose(got[fin], want[fin], rtol=2e-4)          # FP32 accumulation inside the GEMMs
    assert tuple(best.cpu().tolist()) == want_best
    assert want_best[1] > 0                                              # the small weights want scaling up
    # argument checks
    from paper_2409_16626_amd.hif8 import Hif8Error
    with pytest.raises(Hif8Error):
        getattr(h, "hif8_calibrate_layer_" + kind)(tx, tw, torch.from_numpy(o_ref).to(dev()), M, N, K, -4, 10, -4, 10,
                                                   orc.RM_TA, ws, nbytes - 1, err, best)


@pytest.mark.parametrize("M,N,K", [(100, 70, 50), (257, 129, 80), (300, 520, 4096), (512, 768, 200), (33, 17, 1)])
def test_gemm_with_workspace_matches_oracle_and_expanded_kernel(h, M, N, K):
    """hif8_gemm_ws_*: expand into the workspace, then the expanded-operand kernel.  Any K and alignment; the
    result is that of hif8_gemm_expanded_* bit for bit, and within the summation bound of the oracle."""
    rng = np.random.default_rng(M + 3 * N + 7 * K)
    ca, cb = random_codes(rng, (M, K), "cast_normal"), random_codes(rng, (N, K), "cast_normal")
    pad = torch.zeros(M * K + 1, dtype=torch.uint8, device=dev())
    a = pad[1:]                                              # a code matrix that is not 16-byte aligned
    a.copy_(torch.from_numpy(ca).reshape(-1).to(dev()))
    b = torch.from_numpy(cb).to(dev())
    need = h.hif8_gemm_workspace_bytes(M, N, K)
    ld = h.hif8_expanded_ld(K)
    assert need == 2 * (M + N) * ld
    ws = torch.empty(need, dtype=torch.uint8, device=dev())
    out = torch.full((M, N), 7.0, dtype=torch.float32, device=dev())
    h.hif8_gemm_ws_f32(a, b, out, M, N, K, ws, 8.0, 0.5)
    torch.cuda.synchronize()
    check(out.cpu().numpy(), ca, cb, 8.0, 0.5)
    xa = torch.empty(M, ld, dtype=torch.bfloat16, device=dev())
    xb = torch.empty(N, ld, dtype=torch.bfloat16, device=dev())
    h.hif8_expand_bf16(torch.from_numpy(ca).to(dev()), M, K, xa, ld)
    h.hif8_expand_bf16(b, N, K, xb, ld)
    ref = torch.empty_like(out)
    h.hif8_gemm_expanded_f32(xa, xb, ref, M, N, K, ld, 8.0, 0.5)
    assert torch.equal(out.view(torch.int32), ref.view(torch.int32))
    # the narrower outputs and the error epilogue
    ob = torch.empty(M, N, dtype=torch.bfloat16, device=dev())
    rb = torch.empty_like(ob)
    h.hif8_gemm_ws_bf16(a, b, ob, M, N, K, ws, 8.0, 0.5)
    h.hif8_gemm_expanded_bf16(xa, xb, rb, M, N, K, ld, 8.0, 0.5)
    assert torch.equal(ob.view(torch.int16), rb.view(torch.int16))
    oh = torch.empty(M, N, dtype=torch.float16, device=dev())
    rh = torch.empty_like(oh)
    h.hif8_gemm_ws_f16(a, b, oh, M, N, K, ws, 8.0, 0.5)
    h.hif8_gemm_expanded_f16(xa, xb, rh, M, N, K, ld, 8.0, 0.5)
    assert torch.equal(oh.view(torch.int16), rh.view(torch.int16))
    target = (out * 1.01).contiguous()
    e1 = torch.zeros(1, dtype=torch.float64, device=dev())
    e2 = torch.zeros(1, dtype=torch.float64, device=dev())
    h.hif8_gemm_ws_sqerr(a, b, target, M, N, K, 8.0, 0.5, e1, ws)
    h.hif8_gemm_expanded_sqerr(xa, xb, target, M, N, K, ld, 8.0, 0.5, e2)
    want = float(((out.double() - target.double()) ** 2).sum())
    assert abs(e1.item() - want) <= 1e-9 * want and abs(e1.item() - e2.item()) <= 1e-12 * want


def test_gemm_with_workspace_argument_checks(h):
    M, N, K = 64, 48, 32
    a = torch.zeros(M, K, dtype=torch.uint8, device=dev())
    b = torch.zeros(N, K, dtype=torch.uint8, device=dev())
    out = torch.full((M, N), 3.0, dtype=torch.float32, device=dev())
    need = h.hif8_gemm_workspace_bytes(M, N, K)
    ws = torch.empty(need + 16, dtype=torch.uint8, device=dev())
    assert h.lib.hif8_gemm_ws_f32(a.data_ptr(), b.data_ptr(), out.data_ptr(), M, N, K, 1.0, 1.0, ws.data_ptr(), need - 1, None) == -5
    assert h.lib.hif8_gemm_ws_f32(a.data_ptr(), b.data_ptr(), out.data_ptr(), M, N, K, 1.0, 1.0, None, need, None) == -1
    assert h.lib.hif8_gemm_ws_f32(a.data_ptr(), b.data_ptr(), out.data_ptr(), M, N, K, 1.0, 1.0, ws.data_ptr() + 8, need, None) == -5
    assert h.lib.hif8_gemm_ws_f32(a.data_ptr(), b.data_ptr(), out.data_ptr(), M, N, K, 0.0, 1.0, ws.data_ptr(), need, None) == -3
    torch.cuda.synchronize()
    assert torch.all(out == 3.0)                             # nothing was enqueued by the refused calls
    # K = 0: no workspace needed, the product is a matrix of zeros
    assert h.hif8_gemm_workspace_bytes(M, N, 0) == 0
    h.hif8_gemm_ws_f32(a, b, out, M, N, 0, None)
    torch.cuda.synchronize()
    assert torch.all(out == 0.0)
