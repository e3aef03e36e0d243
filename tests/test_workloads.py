"""The seeded input generators (paper_2409_16626_amd/workloads.py): pinned bytes, device independence and the
distributions the benchmark configurations ask for.  The generators hold no HiF8 arithmetic; these tests make
sure that a change of torch, of the device or of the chunking cannot silently change any workload."""
import hashlib

import numpy as np
import pytest
import torch

from paper_2409_16626_amd import workloads as w

# sha256 (first 32 hex digits) of reduced instances, written once from this module's own generators on the CPU
DIGESTS = {
    "normal": "47e63e36a278279913207c2194168c32",
    "c2": "b111a59c03b6d6b10e82871a52e9b4a6",
    "c3": "833ac3424eaebc7e31cebf4e887a645c",
    "c4": "ff2b365b4e87378eb8d410c1580b7a74",
    "c5": "eede3276f490b8b98aa12ebca13590f3",
}


def reduced(device):
    return {
        "normal": w.normal_f32(100003, device),
        "c2": w.dynamic_range_sweep(100003, device),
        "c3": w.activation_bf16(251, 397, device),
        "c4": w.gradient_f32(100003, device),
        "c5": w.llm_weights_bf16(device, layers=1, hidden=64, ffn=176, vocab=100)[0],
    }


def digest(t):
    return hashlib.sha256(t.contiguous().cpu().view(torch.uint8).numpy().tobytes()).hexdigest()[:32]


def test_generator_matches_its_definition_in_plain_integers():
    idx = torch.tensor([0, 1, 2, 12345, 2 ** 40 + 7, 2 ** 62], dtype=torch.int64)
    for cfg, word in ((1, 0), (2, 0), (2, 1), (4, 3), (5, 1)):
        got = [x & ((1 << 64) - 1) for x in w.hash_words(cfg, word, idx).tolist()]
        assert got == [w.hash_word_int(cfg, word, i) for i in idx.tolist()]
    # splitmix64's output function on a value whose result is easy to check by hand: mix(0) == 0
    assert w._mix_int(0) == 0 and w._mix(torch.zeros(1, dtype=torch.int64)).item() == 0
    assert w._mix_int(1) == 0x5692161D100B05E5     # first output of splitmix64's mixer for z = 1


def test_reduced_instances_have_the_pinned_bytes():
    for name, t in reduced("cpu").items():
        assert digest(t) == DIGESTS[name], name


def test_chunking_does_not_change_the_bytes():
    assert torch.equal(w.gradient_f32(100003, chunk=1 << 12), w.gradient_f32(100003))
    assert torch.equal(w.dynamic_range_sweep(100003, chunk=777), w.dynamic_range_sweep(100003))
    assert torch.equal(w.activation_bf16(251, 397, chunk=1000).view(torch.int16), w.activation_bf16(251, 397).view(torch.int16))


@pytest.mark.gpu
def test_gpu_and_cpu_generate_the_same_bytes():
    assert torch.cuda.is_available()
    for name, t in reduced("cuda:0").items():
        assert digest(t) == DIGESTS[name], name


def test_distributions_match_the_recipes():
    x = w.normal_f32(1 << 20).numpy()
    assert abs(x.mean()) < 5e-3 and abs(x.std() - 1.0) < 5e-3 and 4.0 < np.abs(x).max() < 6.0
    assert np.unique(x.view(np.uint32) & 0x3FFF).size > 16000          # low mantissa bits are populated
    # C2: every binade -30 .. 19 about equally often, both signs, ~1 % exact ties incl. the two edge midpoints
    c2 = w.dynamic_range_sweep(1 << 22).numpy()
    b = c2.view(np.uint32)
    e = ((b >> 23) & 0xFF).astype(int) - 127
    assert e.min() == -30 and e.max() == 19
    counts = np.bincount(e + 30, minlength=50)
    assert counts.min() > 0.9 * c2.size / 50 and counts.max() < 1.2 * c2.size / 50
    assert 0.49 < np.mean(c2 < 0) < 0.51
    assert 0.009 < np.mean((b & 0x7FFFF) == 0) < 0.0115
    mag = b & 0x7FFFFFFF
    assert (mag == np.float32(2.0 ** -23).view(np.uint32)).sum() > 500
    assert (mag == np.float32(40960.0).view(np.uint32)).sum() > 200
    # C3: N(0, 1) in BF16 with 0.1 % x100 outliers
    c3 = w.activation_bf16(1024, 1024).float().numpy().ravel()
    assert 0.0008 < np.mean(np.abs(c3) > 20) < 0.0012 and np.abs(c3).max() > 300
    assert abs(np.std(c3[np.abs(c3) < 6]) - 1.0) < 0.01
    # C4: ln|x| ~ Normal(-12, 3), 5 % exact zeros, random sign
    c4 = w.gradient_f32(1 << 22).numpy()
    nz = c4[c4 != 0]
    ln = np.log(np.abs(nz.astype(np.float64)))
    assert 0.049 < np.mean(c4 == 0) < 0.051 and 0.49 < np.mean(nz < 0) < 0.51
    assert abs(ln.mean() + 12.0) < 0.06 and abs(ln.std() - 3.0) < 0.02
    assert np.unique(c4.view(np.uint32) & 0x3FFF).size > 16000
    # C5: N(0, 0.02) BF16, shapes of the decoder
    arena, index = w.llm_weights_bf16("cpu", layers=2, hidden=256, ffn=688, vocab=2000)
    assert len(index) == 15 and sum(m for _, _, m in index) == arena.numel()
    assert abs(arena.float().std().item() - 0.02) < 2e-4
    assert [m for _, _, m in index[:7]] == [256 * 256] * 4 + [688 * 256] * 3 and index[-1][2] == 2000 * 256
    shapes = w.llm_weight_shapes()
    assert len(shapes) == 225 and sum(a * b for _, (a, b) in shapes) == 6607077376
