"""Seeded synthetic input generators for the five benchmark configurations.

This module holds no HiF8 arithmetic: it only draws numbers.  It serves both the
HIP path and the CPU oracle, so that both see byte-identical inputs.  Everything
is built with torch ops on the requested device from a seeded torch.Generator;
bfloat16 tensors are returned as torch.bfloat16 (callers reinterpret as uint16).

The distributions stand in for the tensors of the paper's training / inference
experiments (Sec. 4-5: centralised activations and weights, widely dispersed
gradients, LLM activation outliers), which used public datasets that are not
available here.
"""
import torch

BASE_SEED = 0x48694638  # "HiF8"


def _gen(device, cfg):
    g = torch.Generator(device=device)
    g.manual_seed(BASE_SEED + cfg)
    return g


def all_codes(device="cpu"):
    """C1(i): the 256 HiF8 codes."""
    return torch.arange(256, dtype=torch.int32, device=device).to(torch.uint8)


def all_fp16_as_f32(device="cpu"):
    """C1(ii): all 65,536 FP16 bit patterns widened to FP32 (subnormals, Infs, NaNs included)."""
    bits = torch.arange(65536, dtype=torch.int32, device=device).to(torch.int16)
    return bits.view(torch.float16).to(torch.float32)


def all_bf16(device="cpu"):
    """All 65,536 BF16 bit patterns."""
    bits = torch.arange(65536, dtype=torch.int32, device=device).to(torch.int16)
    return bits.view(torch.bfloat16)


def normal_f32(n=1 << 20, device="cpu"):
    """C1(iii): FP32 ~ N(0, 1)."""
    return torch.randn(n, generator=_gen(device, 1), device=device, dtype=torch.float32)


def dynamic_range_sweep(n=1 << 26, device="cpu", tie_fraction=0.01):
    """C2: random sign * 2^u, u ~ U[-30, 20]; about 1 % of the positions are overwritten
    with short-mantissa values +-2^E * (1 + q/16), E in [-24, 16], q in [0, 15].  Those
    are exactly the numbers with at most four fractional mantissa bits, which include
    every value representable with <= 3 mantissa bits and every midpoint between two
    such neighbours (exact rounding ties)."""
    g = _gen(device, 2)
    u = torch.rand(n, generator=g, device=device, dtype=torch.float32) * 50.0 - 30.0
    x = torch.exp2(u)
    del u
    sign = torch.randint(0, 2, (n,), generator=g, device=device, dtype=torch.int8)
    x = torch.where(sign.bool(), -x, x)
    del sign
    n_tie = int(n * tie_fraction)
    if n_tie > 0:
        pos = torch.randint(0, n, (n_tie,), generator=g, device=device, dtype=torch.int64)
        E = torch.randint(-24, 17, (n_tie,), generator=g, device=device, dtype=torch.int32)
        q = torch.randint(0, 16, (n_tie,), generator=g, device=device, dtype=torch.int32)
        s = torch.randint(0, 2, (n_tie,), generator=g, device=device, dtype=torch.int32)
        t = torch.ldexp(1.0 + q.to(torch.float32) / 16.0, E)
        t = torch.where(s.bool(), -t, t)
        x[pos] = t
    return x


def activation_bf16(rows=8192, cols=8192, device="cpu", outlier_fraction=0.001, outlier_gain=100.0):
    """C3: BF16 [rows, cols] ~ N(0, 1) with a fraction of seeded positions multiplied by 100."""
    g = _gen(device, 3)
    n = rows * cols
    x = torch.randn(n, generator=g, device=device, dtype=torch.float32)
    n_out = int(n * outlier_fraction)
    if n_out > 0:
        pos = torch.randint(0, n, (n_out,), generator=g, device=device, dtype=torch.int64)
        x[pos] = x[pos] * outlier_gain
    return x.to(torch.bfloat16).view(rows, cols)


def gradient_f32(n=1 << 30, device="cpu", zero_fraction=0.05, chunk=1 << 26):
    """C4: log-normal magnitudes, ln|x| ~ Normal(mean -12, std 3), random sign, 5 % exact zeros."""
    g = _gen(device, 4)
    out = torch.empty(n, device=device, dtype=torch.float32)
    for lo in range(0, n, chunk):
        m = min(chunk, n - lo)
        z = torch.randn(m, generator=g, device=device, dtype=torch.float32)
        x = torch.exp(z * 3.0 - 12.0)
        r = torch.rand(m, generator=g, device=device, dtype=torch.float32)
        x = torch.where(r < 0.5, -x, x)
        r = torch.rand(m, generator=g, device=device, dtype=torch.float32)
        x = torch.where(r < zero_fraction, torch.zeros_like(x), x)
        out[lo:lo + m] = x
    return out


def llm_weight_shapes(layers=32, hidden=4096, ffn=11008, vocab=32000):
    """C5: the weight shapes of a decoder-only LLM, in cast order."""
    shapes = []
    for l in range(layers):
        for name in ("wq", "wk", "wv", "wo"):
            shapes.append(("layer%d.%s" % (l, name), (hidden, hidden)))
        shapes.append(("layer%d.w_gate" % l, (ffn, hidden)))
        shapes.append(("layer%d.w_up" % l, (ffn, hidden)))
        shapes.append(("layer%d.w_down" % l, (hidden, ffn)))
    shapes.append(("embedding", (vocab, hidden)))
    return shapes


def llm_weights_bf16(device="cpu", layers=32, hidden=4096, ffn=11008, vocab=32000, std=0.02):
    """C5: one flat BF16 arena ~ N(0, 0.02) plus (name, offset, numel) per tensor.
    Every tensor size is a multiple of 16 elements, so each slice stays 16-byte aligned."""
    g = _gen(device, 5)
    shapes = llm_weight_shapes(layers, hidden, ffn, vocab)
    total = sum(a * b for _, (a, b) in shapes)
    arena = torch.empty(total, device=device, dtype=torch.bfloat16)
    index = []
    off = 0
    for name, (a, b) in shapes:
        m = a * b
        arena[off:off + m] = (torch.randn(m, generator=g, device=device, dtype=torch.float32) * std).to(torch.bfloat16)
        index.append((name, off, m))
        off += m
    return arena, index
