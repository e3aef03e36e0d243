"""Seeded synthetic input generators for the five benchmark configurations.

This module holds no HiF8 arithmetic: it only draws numbers.  It serves both the HIP path and the
CPU oracle, so that both see byte-identical inputs.

Every value is a pure function of (base seed, configuration, element index): a counter-based
generator (splitmix64's output function over the index, keyed per configuration and per word)
evaluated with exact 64-bit integer tensor operations, and values assembled from the hashed bits as
IEEE bit patterns or by single IEEE operations.  No library random-number generator and no
transcendental function takes part, so the bytes do not depend on the device (CPU and GPU give the
same tensor), on the torch version, or on how a tensor is cut into chunks; tests pin a digest of a
reduced instance of every configuration.

The distributions stand in for the tensors of the paper's training / inference experiments (Sec. 4-5:
centralised activations and weights, widely dispersed gradients, LLM activation outliers), which used
public datasets that are not available here.  "Normal" draws are Irwin-Hall sums of twelve 16-bit
uniforms (mean 0, variance 1, support +-6), plus a small uniform dither so that low mantissa bits are
populated.
"""
import torch

BASE_SEED = 0x48694638  # "HiF8"

_M64 = (1 << 64) - 1
_GOLD = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB


def _s64(c):
    """Python integer (mod 2^64) as the signed value an int64 tensor holds."""
    c &= _M64
    return c - (1 << 64) if c >= (1 << 63) else c


def _lsr(x, k):
    """Logical right shift of an int64 tensor."""
    return (x >> k) & ((1 << (64 - k)) - 1)


def _mix(z):
    """splitmix64's output function on an int64 tensor (arithmetic wraps modulo 2^64)."""
    z = (z ^ _lsr(z, 30)) * _s64(_C1)
    z = (z ^ _lsr(z, 27)) * _s64(_C2)
    return z ^ _lsr(z, 31)


def _mix_int(z):
    """The same on a Python integer."""
    z &= _M64
    z = ((z ^ (z >> 30)) * _C1) & _M64
    z = ((z ^ (z >> 27)) * _C2) & _M64
    return z ^ (z >> 31)


def hash_words(cfg, word, idx):
    """64 hashed bits per element: word number `word` of configuration `cfg` for the element indices in
    the int64 tensor `idx`.  h = mix(mix((i + 1) * G + key) ^ key2) with keys derived from the base seed."""
    key = _mix_int(BASE_SEED + cfg * _GOLD)
    key2 = _mix_int(key + (word + 1) * _GOLD)
    return _mix(_mix((idx + 1) * _s64(_GOLD) + _s64(key)) ^ _s64(key2))


def hash_word_int(cfg, word, i):
    """hash_words for one index, in Python integers (used by the tests that pin the generator)."""
    key = _mix_int(BASE_SEED + cfg * _GOLD)
    key2 = _mix_int(key + (word + 1) * _GOLD)
    return _mix_int(_mix_int((i + 1) * _GOLD + key) ^ key2)


def _u16(h, k):
    """16-bit field k (0..3) of hashed words, as int64 in [0, 65535]."""
    return _lsr(h, 16 * k) & 0xFFFF


def _irwin_hall(cfg, word0, idx):
    """Integer d = 2 * (sum of twelve 16-bit uniforms) - 12 * 65535: d * 2^-17 has mean 0 and variance 1 (to
    within 2^-32).  Uses words word0 .. word0 + 2."""
    s = torch.zeros_like(idx)
    for w in range(3):
        h = hash_words(cfg, word0 + w, idx)
        for k in range(4):
            s = s + _u16(h, k)
    return 2 * s - 12 * 65535


def _normal_f32(cfg, word0, idx):
    """FP32 ~ N(0, 1): Irwin-Hall value (a multiple of 2^-17) plus a uniform dither in +-2^-18 (one IEEE add).
    Uses words word0 .. word0 + 3."""
    d = _irwin_hall(cfg, word0, idx)
    z = d.to(torch.float32) * (2.0 ** -17)                                         # exact: |d| < 2^21
    dither = ((hash_words(cfg, word0 + 3, idx) & 0xFFFFFF) - (1 << 23)).to(torch.float32) * (2.0 ** -41)
    return z + dither


def _pattern_view(bits):
    """int64 tensor of 32-bit patterns -> float32 tensor with those patterns."""
    b = bits & 0xFFFFFFFF
    b = torch.where(b >= (1 << 31), b - (1 << 32), b)       # to the signed value of the same 32-bit pattern
    return b.to(torch.int32).view(torch.float32)


def _chunks(n, chunk, device="cpu"):
    """(start, length) pieces of [0, n).  The default piece is 2^26 elements on a GPU (few launches; the int64
    temporaries take a few GiB) and 2^22 on the CPU; the bytes generated do not depend on it."""
    if chunk is None:
        chunk = 1 << 22 if torch.device(device).type == "cpu" else 1 << 26
    for lo in range(0, n, chunk):
        yield lo, min(chunk, n - lo)


def _index(lo, m, device):
    return torch.arange(lo, lo + m, dtype=torch.int64, device=device)


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


def normal_f32(n=1 << 20, device="cpu", chunk=None):
    """C1(iii): FP32 ~ N(0, 1)."""
    out = torch.empty(n, device=device, dtype=torch.float32)
    for lo, m in _chunks(n, chunk, device):
        out[lo:lo + m] = _normal_f32(1, 0, _index(lo, m, device))
    return out


def dynamic_range_sweep(n=1 << 26, device="cpu", tie_fraction=0.01, chunk=None):
    """C2: random sign * 2^E * (1 + m / 2^23) with E uniform over the integers -30 .. 19 and all 23 mantissa bits
    random (every binade from far below the smallest HiF8 denormal to above its largest value, every rounding
    position), and about 1 % of the positions overwritten with exact rounding ties: midpoints between two adjacent
    representable magnitudes, including 2^-23 (between zero and the smallest denormal) and 1.25 * 2^15 (between
    the largest value and the overflow slot).  Placing the ties needs one fact about the format, the number of
    mantissa bits kept per exponent (Table 3: 3 for |E| <= 3, 2 up to 7, 1 up to 15, none in the denormal range
    E = -22 .. -16, Eq. (2)): a midpoint has one more mantissa bit than its binade keeps, and that bit is set."""
    out = torch.empty(n, device=device, dtype=torch.float32)
    thr = int(tie_fraction * 65536)
    for lo, m in _chunks(n, chunk, device):
        idx = _index(lo, m, device)
        h0 = hash_words(2, 0, idx)
        e = -30 + ((_u16(h0, 0) * 50) >> 16)                       # -30 .. 19
        mant = _lsr(h0, 16) & 0x7FFFFF
        sign = _lsr(h0, 63)
        bits = (sign << 31) | ((e + 127) << 23) | mant
        h1 = hash_words(2, 1, idx)
        is_tie = _u16(h1, 0) < thr
        et = -23 + ((_u16(h1, 1) * 39) >> 16)                      # -23 .. 15
        ae = et.abs()
        k = torch.where(ae <= 3, 3, torch.where(ae <= 7, 2, torch.where(ae <= 15, 1, 0)))
        k = torch.where(et < -15, torch.zeros_like(k), k)          # denormal range: powers of two only
        kept = (_u16(h1, 2) & ((1 << k) - 1)) << (23 - k)
        mt = kept | (1 << (22 - k))
        mt = torch.where(et == -23, torch.zeros_like(mt), mt)      # 2^-23 itself: halfway between 0 and 2^-22
        tbits = (_lsr(h1, 63) << 31) | ((et + 127) << 23) | mt
        out[lo:lo + m] = _pattern_view(torch.where(is_tie, tbits, bits))
    return out


def activation_bf16(rows=8192, cols=8192, device="cpu", outlier_fraction=0.001, outlier_gain=100.0, chunk=None):
    """C3: BF16 [rows, cols] ~ N(0, 1) with a fraction of hash-selected positions multiplied by 100."""
    n = rows * cols
    out = torch.empty(n, device=device, dtype=torch.bfloat16)
    thr = int(outlier_fraction * (1 << 32))
    for lo, m in _chunks(n, chunk, device):
        idx = _index(lo, m, device)
        x = _normal_f32(3, 0, idx)
        sel = (hash_words(3, 4, idx) & 0xFFFFFFFF) < thr
        x = torch.where(sel, x * outlier_gain, x)
        out[lo:lo + m] = x.to(torch.bfloat16)
    return out.view(rows, cols)


def gradient_f32(n=1 << 30, device="cpu", zero_fraction=0.05, chunk=None):
    """C4: log-normal magnitudes, ln|x| ~ Normal(mean -12, std 3), random sign, 5 % exact zeros.
    Built in the binary logarithm, in fixed point: log2|x| = (-12 + 3 z) / ln 2 with z the Irwin-Hall normal; its
    integer part is the exponent, its fraction the top 16 mantissa bits (linear within a binade), and the low 7
    mantissa bits are hashed, so every bit of the pattern varies."""
    out = torch.empty(n, device=device, dtype=torch.float32)
    a_fix = -1134566      # round(-12 / ln 2 * 2^16)
    b_fix = 283645        # round(3 / ln 2 * 2^16)
    zthr = int(zero_fraction * 65536)
    for lo, m in _chunks(n, chunk, device):
        idx = _index(lo, m, device)
        d = _irwin_hall(4, 0, idx)                                # z = d * 2^-17
        t = a_fix + ((b_fix * d) >> 17)                            # log2|x| in Q16 (floor)
        e = t >> 16
        frac = t & 0xFFFF
        h = hash_words(4, 3, idx)
        mant = (frac << 7) | (h & 0x7F)
        bits = (_lsr(h, 63) << 31) | ((e + 127) << 23) | mant
        bits = torch.where(_u16(h, 1) < zthr, torch.zeros_like(bits), bits)
        out[lo:lo + m] = _pattern_view(bits)
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


def llm_weights_bf16(device="cpu", layers=32, hidden=4096, ffn=11008, vocab=32000, std=0.02, chunk=None):
    """C5: one flat BF16 arena ~ N(0, 0.02) plus (name, offset, numel) per tensor (element i of the arena is a
    function of i alone).  Every tensor size is a multiple of 16 elements, so each slice stays 16-byte aligned."""
    shapes = llm_weight_shapes(layers, hidden, ffn, vocab)
    total = sum(a * b for _, (a, b) in shapes)
    arena = torch.empty(total, device=device, dtype=torch.bfloat16)
    for lo, m in _chunks(total, chunk, device):
        arena[lo:lo + m] = (_normal_f32(5, 0, _index(lo, m, device)) * std).to(torch.bfloat16)
    index = []
    off = 0
    for name, (a, b) in shapes:
        index.append((name, off, a * b))
        off += a * b
    return arena, index
