"""The library under HIP graph capture: every entry point only enqueues kernels on the caller's
stream (no allocation, no memset, no synchronisation once hif8_init has run), so a whole
amax -> scale -> cast -> expand -> GEMM sequence can be captured once and replayed.

Each replay, with fresh input written between replays by ordinary eager work, is compared bit
for bit with the same sequence run eagerly on the same input, and the casts with the oracle.
"""
import numpy as np
import pytest
import torch

from oracle import hif8_oracle as orc
from gpu_util import bf16_bits, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def h():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2409_16626_amd import hif8
    hif8.hif8_init()
    return hif8


def test_cast_and_gemm_sequence_replays_exactly(h):
    M, N, K = 192, 160, 200
    ld = h.hif8_expanded_ld(K)
    g = torch.Generator(device=dev()).manual_seed(21)
    x = torch.empty(M, K, dtype=torch.bfloat16, device=dev())
    w = (torch.randn(N, K, generator=g, device=dev()) * 0.03).to(torch.bfloat16)

    class Bufs:
        def __init__(self):
            self.amax = torch.zeros(2, dtype=torch.float32, device=dev())
            self.scale = torch.zeros(2, 2, dtype=torch.float32, device=dev())
            self.xq = torch.empty_like(x)
            self.xc = torch.empty(M, K, dtype=torch.uint8, device=dev())
            self.wc = torch.empty(N, K, dtype=torch.uint8, device=dev())
            self.xe = torch.empty(M, ld, dtype=torch.bfloat16, device=dev())
            self.we = torch.empty(N, ld, dtype=torch.bfloat16, device=dev())
            self.out = torch.empty(M, N, dtype=torch.float32, device=dev())
            self.ram = torch.zeros(N, dtype=torch.float32, device=dev())
            self.rsc = torch.zeros(N, 2, dtype=torch.float32, device=dev())
            self.rc = torch.empty(N, K, dtype=torch.uint8, device=dev())
            self.acc = torch.zeros(2, dtype=torch.float32, device=dev())
            self.mc = torch.empty(M * K + N * K, dtype=torch.uint8, device=dev())
            self.items = h.hif8_multi_plan([(x.data_ptr(), self.mc.data_ptr(), M * K),
                                            (w.data_ptr(), self.mc[M * K:].data_ptr(), N * K)], src_is_16bit=True)

    def sequence(b):
        b.amax.zero_()                                                     # a fill kernel, not a memset node
        h.hif8_amax_bf16(x, M * K, b.amax[0:1])
        h.hif8_amax_bf16(w, N * K, b.amax[1:2])
        h.hif8_scale_from_amax_n(b.amax, b.scale, 2, h.MAX_FINITE, 1)
        h.hif8_fake_quant_bf16_ds(x, b.xq, b.xc, M * K, b.scale[0], h.RM_TA)
        h.hif8_encode_bf16_ds(w, b.wc, N * K, b.scale[1], h.RM_HR)
        h.hif8_expand_bf16(b.xc, M, K, b.xe, ld)
        h.hif8_expand_bf16(b.wc, N, K, b.we, ld)
        h.hif8_gemm_expanded_f32(b.xe, b.we, b.out, M, N, K, ld, 1.0, 1.0)
        h.hif8_quantize_rows_bf16(w, b.rc, N, K, b.ram, b.rsc, h.MAX_FINITE, 1, h.RM_TA)      # per-row scaling in one pass
        b.acc.zero_()
        d_items, count, tiles = b.items
        h.hif8_multi_encode_bf16_ds(d_items, count, tiles, b.scale, h.RM_TA, d_amax_accum=b.acc)  # both tensors, one launch

    eager, graphed = Bufs(), Bufs()
    x.copy_(torch.randn(M, K, generator=g, device=dev()).to(torch.bfloat16))
    sequence(graphed)                                                      # warm-up outside the capture: one-time setup happens here
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sequence(graphed)

    for rep in range(4):
        x.copy_((torch.randn(M, K, generator=g, device=dev()) * (0.5 + 3.0 * rep)).to(torch.bfloat16))   # eager work between replays
        torch.cuda.synchronize()
        for t in (graphed.xq, graphed.xc, graphed.wc, graphed.xe, graphed.out):
            t.fill_(0)
        graph.replay()
        sequence(eager)
        torch.cuda.synchronize()
        for name in ("amax", "scale", "xc", "wc", "out", "ram", "rsc", "rc", "acc", "mc"):
            assert torch.equal(getattr(graphed, name), getattr(eager, name)), (rep, name)
        assert torch.equal(graphed.xq.view(torch.int16), eager.xq.view(torch.int16)), rep
        assert torch.equal(graphed.xe.view(torch.int16), eager.xe.view(torch.int16)), rep
        # and against the oracle: amax, scale and codes of the activation cast
        xn = bf16_bits(x)
        w_am = orc.amax_bf16(xn.reshape(-1))
        w_s = orc.scale_from_amax(w_am, 32768.0, True)
        assert graphed.amax[0].item() == float(w_am) and graphed.scale[0, 0].item() == float(w_s)
        assert np.array_equal(graphed.xc.cpu().numpy().reshape(-1), orc.encode_bf16(xn.reshape(-1), w_s, orc.RM_TA))
        assert np.array_equal(graphed.mc[:M * K].cpu().numpy(), orc.encode_bf16(xn.reshape(-1), w_s, orc.RM_TA))
        assert graphed.acc[0].item() == float(w_am)


def test_one_call_entry_points_replay_exactly(h):
    """Per-tensor scaling in one call (workspace and static-scratch forms) and the group-wise
    multi-tensor cast under capture: they enqueue kernels only, so a captured sequence replays
    bit for bit on fresh inputs, and matches the oracle."""
    n0, n1 = 70001 * 16, 4099 * 16            # both multiples of 16 elements: slices stay 16-byte aligned
    n = n0 + n1
    g = torch.Generator(device=dev()).manual_seed(77)
    x = torch.empty(n, dtype=torch.bfloat16, device=dev())
    xf = torch.empty(n1, dtype=torch.float32, device=dev())

    class Bufs:
        def __init__(self):
            self.ws = torch.zeros(h.hif8_quantize_workspace_bytes(), dtype=torch.uint8, device=dev())
            self.am = torch.zeros(4, dtype=torch.float32, device=dev())
            self.sc = torch.zeros(4, 2, dtype=torch.float32, device=dev())
            self.c_ws = torch.empty(n, dtype=torch.uint8, device=dev())
            self.q_ws = torch.empty(n, dtype=torch.bfloat16, device=dev())
            self.c_st = torch.empty(n1, dtype=torch.uint8, device=dev())
            self.c_mc = torch.empty(n, dtype=torch.uint8, device=dev())
            self.plan = h.hif8_multi_plan([(x.data_ptr(), self.c_mc.data_ptr(), n0),
                                           (x[n0:].data_ptr(), self.c_mc[n0:].data_ptr(), n1)], src_is_16bit=True)

    def sequence(b):
        h.hif8_quantize_tensor_bf16(x, b.q_ws, b.c_ws, n, b.am[0:1], b.sc[0], b.ws, h.MAX_FINITE, 1, h.RM_TA)
        h.hif8_quantize_tensor_static(xf, None, b.c_st, n1, h.KIND_F32, b.am[1:2], b.sc[1], h.MAX_FINITE, 0, h.RM_HR)
        d_items, count, tiles = b.plan
        h.hif8_multi_cast_bf16(d_items, count, tiles, b.am[2:4], b.sc[2:4], h.MAX_FINITE, 1, h.RM_TA,
                               host_items=b.plan.host_items)

    eager, graphed = Bufs(), Bufs()
    x.copy_(torch.randn(n, generator=g, device=dev()).to(torch.bfloat16))
    xf.copy_(torch.randn(n1, generator=g, device=dev()))
    sequence(graphed)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sequence(graphed)

    for rep in range(4):
        gain = 0.25 + 5.0 * (3 - rep)                                          # amax shrinks from replay to replay
        x.copy_((torch.randn(n, generator=g, device=dev()) * gain).to(torch.bfloat16))
        xf.copy_(torch.randn(n1, generator=g, device=dev()) * gain)
        torch.cuda.synchronize()
        for t in (graphed.c_ws, graphed.c_st, graphed.c_mc):
            t.fill_(0)
        graph.replay()
        sequence(eager)
        torch.cuda.synchronize()
        for name in ("am", "sc", "c_ws", "c_st", "c_mc"):
            assert torch.equal(getattr(graphed, name), getattr(eager, name)), (rep, name)
        assert torch.equal(graphed.q_ws.view(torch.int16), eager.q_ws.view(torch.int16)), rep
        xn, fn = bf16_bits(x), xf.cpu().numpy()
        am = orc.amax_bf16(xn)
        s = orc.scale_from_amax(am, 32768.0, True)
        assert graphed.am[0].item() == float(am) and graphed.sc[0, 0].item() == float(s)
        assert np.array_equal(graphed.c_ws.cpu().numpy(), orc.encode_bf16(xn, s, orc.RM_TA))
        amf = orc.amax_f32(fn)
        sf = orc.scale_from_amax(amf, 32768.0, False)
        assert graphed.am[1].item() == float(amf) and graphed.sc[1, 0].item() == float(sf)
        assert np.array_equal(graphed.c_st.cpu().numpy(), orc.encode_f32(fn, sf, orc.RM_HR))
        for k, (lo, m) in enumerate(((0, n0), (n0, n1))):
            amk = orc.amax_bf16(xn[lo:lo + m])
            sk = orc.scale_from_amax(amk, 32768.0, True)
            assert graphed.am[2 + k].item() == float(amk)
            assert np.array_equal(graphed.c_mc[lo:lo + m].cpu().numpy(), orc.encode_bf16(xn[lo:lo + m], sk, orc.RM_TA)), (rep, k)
