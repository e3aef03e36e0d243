"""The entry point that allocates nothing (hif8_quantize_tensor_static: partial maxima in a static device array)
against the workspace form it is a variant of (hif8_quantize_tensor_*), through the C ABI: two calls in a row,
the second on a smaller input, every output bit for bit; sizes beyond the stated maximum are refused."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def h():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2409_16626_amd import hif8
    hif8.hif8_init()
    return hif8


def run_both(h, kind, x, pow2, mode, with_dst, with_codes):
    dev = x.device
    n = x.numel()
    L = h.lib
    st = torch.cuda.current_stream().cuda_stream
    kind_id = {"f32": h.KIND_F32, "bf16": h.KIND_BF16, "f16": h.KIND_F16}[kind]
    res = []
    for static in (False, True):
        am = torch.full((1,), 3.0, dtype=torch.float32, device=dev)
        sc = torch.full((2,), 5.0, dtype=torch.float32, device=dev)
        out = torch.zeros_like(x) if with_dst else None
        codes = torch.zeros(n, dtype=torch.uint8, device=dev) if with_codes else None
        po = out.data_ptr() if with_dst else None
        pc = codes.data_ptr() if with_codes else None
        if static:
            rc = L.hif8_quantize_tensor_static(x.data_ptr(), po, pc, n, kind_id, 32768.0, pow2, mode, am.data_ptr(),
                                               sc.data_ptr(), st)
        else:
            ws = torch.full((1024,), -1, dtype=torch.int32, device=dev)
            rc = getattr(L, "hif8_quantize_tensor_" + kind)(x.data_ptr(), po, pc, n, 32768.0, pow2, mode, am.data_ptr(),
                                                            sc.data_ptr(), ws.data_ptr(), 4096, st)
        assert rc == 0
        torch.cuda.synchronize()
        res.append((am, sc, out, codes))
    (a0, s0, o0, c0), (a1, s1, o1, c1) = res
    assert torch.equal(a0.view(torch.int32), a1.view(torch.int32)) and torch.equal(s0, s1)
    if with_codes:
        assert torch.equal(c0, c1)
    if with_dst:
        assert torch.equal(o0.view(torch.uint8), o1.view(torch.uint8))
    return a1.item()


@pytest.mark.parametrize("kind", ["bf16", "f32", "f16"])
def test_static_scratch_form_equals_workspace_form_twice_in_a_row(h, kind):
    dev = torch.device("cuda:0")
    dt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[kind]
    g = torch.Generator(device=dev).manual_seed(1234)
    big = (torch.randn((5 << 20) + 13, generator=g, device=dev) * 3.0).to(dt)       # several hundred partial maxima
    big[777] = 200.0
    small = (torch.randn(4099, generator=g, device=dev) * 0.01).to(dt)              # one workgroup; amax far below the first call's
    am_big = run_both(h, kind, big, 0, h.RM_TA, True, True)
    am_small = run_both(h, kind, small, 1, h.RM_HR | h.FLAG_SAT, True, True)
    assert am_big == 200.0 and 0.0 < am_small < 1.0          # the second call saw nothing of the first call's maxima
    run_both(h, kind, small[1:], 0, h.RM_TA, False, True)      # unaligned source: element-per-lane path, no scratch
    run_both(h, kind, big[:1 << 20], 0, h.RM_HR, True, False)


def test_static_form_refuses_what_it_cannot_do(h):
    L = h.lib
    p = 0x1000   # never dereferenced: every call below fails validation
    assert L.hif8_quantize_tensor_static(p, p, p, (1 << 32) + 1, h.KIND_BF16, 32768.0, 0, 0, p, p, None) == -5
    assert L.hif8_quantize_tensor_static(p, p, p, 16, 3, 32768.0, 0, 0, p, p, None) == -5
    assert L.hif8_quantize_tensor_static(p, p, p, 16, h.KIND_F32, 32768.0, 0, 9, p, p, None) == -2
    assert L.hif8_quantize_tensor_static(p, p, p, 16, h.KIND_F32, -1.0, 0, 0, p, p, None) == -5
    assert L.hif8_quantize_tensor_static(p, None, None, 16, h.KIND_F16, 32768.0, 0, 0, p, p, None) == -1
    assert L.hif8_quantize_tensor_static(p, p, p, 16, h.KIND_F16, 32768.0, 0, 0, None, p, None) == -1
