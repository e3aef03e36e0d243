"""Helpers shared by the GPU parity tests (numpy <-> device plumbing only)."""
import numpy as np
import torch


def dev():
    return torch.device("cuda:0")


def to_gpu(a):
    """numpy array -> device tensor with the same bytes (uint16/uint32 travel as int16/int32)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(dev())
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).to(dev())
    return torch.from_numpy(a).to(dev())


def bf16_bits(t):
    """bfloat16 (or int16) tensor -> numpy uint16 patterns."""
    if t.dtype == torch.bfloat16:
        t = t.view(torch.int16)
    return t.cpu().numpy().view(np.uint16)


def f32_bits(t):
    return t.view(torch.int32).cpu().numpy().view(np.uint32)


def assert_same_bytes(got, want, what=""):
    got = np.asarray(got)
    want = np.asarray(want)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, "%s: %d mismatches, first at %s: got %s want %s" % (
        what, bad.size, bad[:5], got[bad[:5]], want[bad[:5]])
