"""CPU oracle for the simulated HiF8 GEMM and the layer calibration of Algorithm 1 -- TEST
INFRASTRUCTURE, NOT PRODUCT CODE.  numpy, fp64; shares nothing with the HIP library.

    gemm_hif8        O = (value(A_codes) x value(B_codes)^T) * (1/scale_a) * (1/scale_b): the
                     paper's experiments cast the GEMM inputs to HiF8 and run the GEMM on the
                     represented values (Sec. 4: simulated HiF8); with per-tensor scaling the
                     output is descaled (Sec. 5.1 / Algorithm 1 "MatMul & Restore").
                     A is [M, K], B is [N, K] (both with K contiguous), O is [M, N].
    calibrate_layer  Algorithm 1 for one layer: for every (Ea, Ew) of the search square, scale
                     and cast both inputs with TA, multiply, restore by 2^-(Ea+Ew), and take the
                     squared error against the high-precision output; the pair with the smallest
                     error is the layer's choice.  Returns the sums (MSE = sum / (M N)).
Every product of two HiF8 values is exact in fp64 and sums of K <= 2^20 of them lose at most
K * 2^-53 relative to the sum of magnitudes: the fp64 result stands in for the exact one.
"""
import numpy as np

from . import hif8_oracle as orc

_VALUES = np.array([orc.decode_value(c) for c in range(256)], np.float64)


def decode_values(codes):
    return _VALUES[np.asarray(codes, np.uint8)]


def gemm_hif8(codes_a, codes_b, scale_a=1.0, scale_b=1.0):
    va, vb = decode_values(codes_a), decode_values(codes_b)
    inv = float(np.float32(1.0) / np.float32(scale_a)) * float(np.float32(1.0) / np.float32(scale_b))
    with np.errstate(invalid="ignore", over="ignore"):
        return (va @ vb.T) * inv


def gemm_abs_bound(codes_a, codes_b, scale_a=1.0, scale_b=1.0):
    """sum_k |a_ik b_jk| * |descale|: the scale of the rounding error of any summation order."""
    va, vb = np.abs(decode_values(codes_a)), np.abs(decode_values(codes_b))
    inv = float(np.float32(1.0) / np.float32(scale_a)) * float(np.float32(1.0) / np.float32(scale_b))
    return (va @ vb.T) * inv


_ENC = {orc.SRC_F32: orc.encode_f32, orc.SRC_BF16: orc.encode_bf16, orc.SRC_F16: orc.encode_f16}


def calibrate_layer(a, w, o_ref, kind=orc.SRC_F32, ea_lo=-4, ea_count=10, ew_lo=-4, ew_count=10, mode=orc.RM_TA):
    """a: [M, K], w: [N, K] in the container of `kind`; o_ref: [M, N] float.  Returns
    err[ea_count, ew_count] (fp64 sums of squared output error) and the argmin pair (Ea, Ew)."""
    enc = _ENC[kind]
    o_ref = np.asarray(o_ref, np.float64)
    ca = [enc(a.reshape(-1), np.float32(2.0 ** (ea_lo + i)), mode).reshape(a.shape) for i in range(ea_count)]
    cw = [enc(w.reshape(-1), np.float32(2.0 ** (ew_lo + j)), mode).reshape(w.shape) for j in range(ew_count)]
    err = np.zeros((ea_count, ew_count), np.float64)
    for i in range(ea_count):
        for j in range(ew_count):
            o = gemm_hif8(ca[i], cw[j], 2.0 ** (ea_lo + i), 2.0 ** (ew_lo + j))
            with np.errstate(invalid="ignore", over="ignore"):
                err[i, j] = np.sum((o - o_ref) ** 2)
    best = np.unravel_index(np.nanargmin(np.where(np.isfinite(err), err, np.inf)), err.shape)
    return err, (ea_lo + int(best[0]), ew_lo + int(best[1]))
