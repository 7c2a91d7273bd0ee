"""CPU oracle of the MXFP6 variant of the HALO forward product (numpy, slow, plain).

THIS IS TEST INFRASTRUCTURE (same rules as halo_oracle.py: only tests/, smoke() and bench.py's cpu_baseline leg
may import it; it shares nothing with the HIP library).

The paper evaluates HALO with FP6 E3M2 elements (Section 4 "Setup") and, in the Appendix "MXFP6", with
microscaling: a block of consecutive elements along the reduction dimension shares one power-of-two scale.  It
names the formats and gives no arithmetic, so the element format, the shared-scale rule and the rounding are taken
from the public OCP Microscaling Formats (MX) specification v1.0:

* element E3M2: value = (-1)^s * 2^(e-3) * (1 + m/4) for e in 1..7, (-1)^s * 2^(-2) * (m/4) for e = 0; no Inf/NaN;
  largest magnitude 28; code bits [s | e e e | m m];
* block of 32 elements along K shares X = 2^(floor(log2(max|v|)) - 4) (4 = exponent of the largest E3M2 binade),
  stored as E8M0 = exponent + 127; an all-zero block gets X = 1 (code 127); the exponent is clamped to [-127, 127];
* elements are v / X rounded to the nearest E3M2 value, ties to the even mantissa, magnitudes beyond 28 saturate
  to 28; a result of magnitude zero is stored as +0.

parity unpinned: the values of rotated+quantised tensors (the paper prints none); pinned through the format table,
round trips, tie and saturation cases, hand examples of the shared scale and block independence (tests/).
"""
from __future__ import annotations

import numpy as np

from . import halo_oracle as _h

BLOCK = 32
E3M2_MAX = 28.0
ELEM_EMAX = 4          # floor(log2(28))

__all__ = ["e3m2_decode", "e3m2_encode", "mx_quantize_rows", "mx_dequantize", "pack_fp6", "unpack_fp6",
           "mx_gemm", "forward_mxfp6"]


def e3m2_decode(codes: np.ndarray) -> np.ndarray:
    """6-bit codes -> float64 values."""
    c = np.asarray(codes).astype(np.int64)
    s, e, m = (c >> 5) & 1, (c >> 2) & 7, c & 3
    mag = np.where(e == 0, m * 0.25 * 2.0 ** -2, (1.0 + m * 0.25) * 2.0 ** (e - 3))
    return np.where(s == 1, -mag, mag)


def e3m2_encode(x: np.ndarray) -> np.ndarray:
    """Nearest E3M2 code of each x (ties to even mantissa, saturating at +-28, zero magnitude stored as +0)."""
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    # spacing of the format around a: 2^(floor(log2 a) - 2) for normals, 2^-4 below the smallest normal 0.25
    with np.errstate(divide="ignore"):
        ex = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    ex = np.maximum(ex, -2.0)
    quantum = 2.0 ** (ex - 2)
    q = np.rint(a / quantum) * quantum              # np.rint: round half to even
    q = np.minimum(q, E3M2_MAX)
    # q is representable: find its fields
    e_field = np.where(q < 0.25, 0, np.floor(np.log2(np.where(q > 0, q, 1.0))) + 3).astype(np.int64)
    m_field = np.where(e_field == 0, np.rint(q * 16.0), np.rint((q / 2.0 ** (e_field - 3) - 1.0) * 4.0)).astype(np.int64)
    sign = ((x < 0) & (q > 0)).astype(np.int64)
    return ((sign << 5) | (e_field << 2) | m_field).astype(np.uint8)


def mx_quantize_rows(v: np.ndarray):
    """v fp32 [rows, K] (K a multiple of 32) -> (codes uint8 [rows, K] 6-bit, scales uint8 [rows, K/32] E8M0)."""
    assert v.dtype == np.float32 and v.shape[1] % BLOCK == 0
    rows, K = v.shape
    blk = v.reshape(rows, K // BLOCK, BLOCK)
    amax = np.max(np.abs(blk), axis=2)
    mant, ex = np.frexp(amax.astype(np.float64))              # amax = mant * 2^ex, mant in [0.5, 1): floor(log2) = ex - 1
    shared = np.clip(np.where(amax > 0, ex - 1 - ELEM_EMAX, 0), -127, 127).astype(np.int64)
    scaled = np.ldexp(blk, (-shared)[:, :, None].astype(np.int32)).astype(np.float32)     # exact unless it underflows
    codes = e3m2_encode(scaled.astype(np.float64)).reshape(rows, K)
    return codes, (shared + 127).astype(np.uint8)


def mx_dequantize(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """float64 values of an MX-quantised matrix."""
    rows, K = codes.shape
    vals = e3m2_decode(codes).reshape(rows, K // BLOCK, BLOCK)
    return (vals * 2.0 ** (scales.astype(np.int64) - 127)[:, :, None]).reshape(rows, K)


def pack_fp6(codes: np.ndarray) -> np.ndarray:
    """[rows, K] 6-bit codes -> [rows, K/32 * 24] bytes: element i of a block occupies bits [6i, 6i+6) of the block's
    192 bits, least significant bit first (the operand layout of the CDNA4 scaled MFMA)."""
    rows, K = codes.shape
    c = codes.reshape(rows, K // 4, 4).astype(np.uint32)
    word = c[:, :, 0] | (c[:, :, 1] << 6) | (c[:, :, 2] << 12) | (c[:, :, 3] << 18)      # 4 codes -> 24 bits
    out = np.empty((rows, K // 4, 3), dtype=np.uint8)
    out[:, :, 0] = word & 0xFF
    out[:, :, 1] = (word >> 8) & 0xFF
    out[:, :, 2] = (word >> 16) & 0xFF
    return out.reshape(rows, K // 4 * 3)


def unpack_fp6(packed: np.ndarray, K: int) -> np.ndarray:
    rows = packed.shape[0]
    p = packed.reshape(rows, K // 4, 3).astype(np.uint32)
    word = p[:, :, 0] | (p[:, :, 1] << 8) | (p[:, :, 2] << 16)
    out = np.empty((rows, K // 4, 4), dtype=np.uint8)
    for i in range(4):
        out[:, :, i] = (word >> (6 * i)) & 0x3F
    return out.reshape(rows, K)


def mx_gemm(codes_a, scales_a, codes_b, scales_b) -> np.ndarray:
    """C[i,j] = sum_k a[i,k] b[j,k] on the dequantised values, in float64 (the hardware accumulates in fp32; the
    order of its additions is not specified, so GPU results are compared within a bound, not bit for bit)."""
    return mx_dequantize(codes_a, scales_a) @ mx_dequantize(codes_b, scales_b).T


def forward_mxfp6(X: np.ndarray, W: np.ndarray, had_block_m: int):
    """HALO-1 forward product with MXFP6 operands: (XH)_Q (WH)_Q^T, blocks of 32 along the in-feature axis
    (Table "HALO levels", level 1, F; Appendix "MXFP6")."""
    Xh = _h.fwht(X.astype(np.float32), had_block_m, 1)
    Wh = _h.fwht(W.astype(np.float32), had_block_m, 1)
    xc, xs = mx_quantize_rows(Xh)
    wc, ws = mx_quantize_rows(Wh)
    return dict(Xc=xc, Xs=xs, Wc=wc, Ws=ws, Y=mx_gemm(xc, xs, wc, ws))
