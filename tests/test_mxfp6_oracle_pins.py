"""Pins of the MXFP6 oracle (CPU): format table typed by hand, round trips, ties, saturation, shared-scale hand
examples, block independence, packing."""
import os

import numpy as np

from oracle import halo_oracle as orc
from oracle import mxfp6_oracle as mx

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def table():
    vals = {}
    with open(os.path.join(GOLDEN, "e3m2_values.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            e, rest = line.split(":")
            vals[int(e)] = [float(t) for t in rest.split()]
    return vals


def test_all_64_codes_decode_to_the_hand_typed_table():
    t = table()
    assert sorted(t) == list(range(8))
    for code in range(64):
        s, e, m = code >> 5, (code >> 2) & 7, code & 3
        want = t[e][m] * (-1.0 if s else 1.0)
        assert mx.e3m2_decode(np.array([code]))[0] == want, code
    assert mx.e3m2_decode(np.array([31]))[0] == 28.0 and mx.e3m2_decode(np.array([1]))[0] == 0.0625


def test_every_representable_value_round_trips_and_neighbours_round_to_nearest():
    codes = np.arange(64)
    vals = mx.e3m2_decode(codes)
    back = mx.e3m2_encode(vals)
    keep = codes != 32                                   # -0 is stored as +0
    assert np.array_equal(back[keep], codes[keep]) and back[32] == 0
    pos = np.sort(vals[:32])
    for lo, hi in zip(pos[:-1], pos[1:]):
        mid = (lo + hi) / 2
        assert mx.e3m2_decode(mx.e3m2_encode(np.array([lo + 0.49 * (hi - lo)])))[0] == lo
        assert mx.e3m2_decode(mx.e3m2_encode(np.array([lo + 0.51 * (hi - lo)])))[0] == hi
        tie = mx.e3m2_encode(np.array([mid]))[0]
        assert tie & 1 == 0 and mx.e3m2_decode(np.array([tie]))[0] in (lo, hi)      # ties go to the even mantissa


def test_ties_saturation_and_subnormals_hand_cases():
    enc = lambda x: float(mx.e3m2_decode(mx.e3m2_encode(np.array([x])))[0])
    assert enc(1.125) == 1.0 and enc(1.375) == 1.5 and enc(-1.375) == -1.5        # even mantissas 0 and 2
    assert enc(0.03125) == 0.0 and enc(0.09375) == 0.125 and enc(0.21875) == 0.25  # subnormal ties, carry into normals
    assert enc(28.0) == 28.0 and enc(29.9) == 28.0 and enc(31.0) == 28.0 and enc(1e9) == 28.0 and enc(-40.0) == -28.0
    assert enc(26.0) == 24.0 and enc(26.1) == 28.0 and enc(15.0) == 16.0 and enc(14.9) == 14.0
    assert mx.e3m2_encode(np.array([-0.01]))[0] == 0           # rounds to zero: stored as +0
    assert mx.e3m2_encode(np.array([-0.0]))[0] == 0


def test_shared_scale_hand_examples_and_block_independence():
    v = np.zeros((1, 96), dtype=np.float32)
    v[0, 0] = 28.0            # block 0: floor(log2 28) = 4 -> exponent 0 -> E8M0 127; 28 -> code 31
    v[0, 1] = -3.0
    v[0, 32] = 1.0            # block 1: floor(log2 1) = 0 -> exponent -4 -> 123; 1/2^-4 = 16 -> e=7 m=0 -> code 28
    v[0, 33] = 0.9            # 0.9 * 16 = 14.4 -> 14 -> code 0b110_11 = 27
    v[0, 64] = 0.0            # block 2: all zero -> scale 1 (127), codes 0
    codes, scales = mx.mx_quantize_rows(v)
    assert scales.tolist() == [[127, 123, 127]]
    assert codes[0, 0] == 31 and codes[0, 1] == (32 | (4 << 2) | 2) and codes[0, 32] == 28 and codes[0, 33] == 27
    assert not codes[0, 64:].any()
    back = mx.mx_dequantize(codes, scales)
    assert back[0, 0] == 28.0 and back[0, 1] == -3.0 and back[0, 32] == 1.0 and back[0, 33] == 0.875
    # amax just below a power of two lands in the saturating top binade: 0.99 -> scale 2^-5, 31.68 -> 28
    w = np.full((1, 32), 0.5, dtype=np.float32); w[0, 7] = 0.99
    c, s = mx.mx_quantize_rows(w)
    assert s[0, 0] == 127 - 5 and c[0, 7] == 31 and mx.mx_dequantize(c, s)[0, 7] == 28.0 / 32
    # changing one block leaves the others alone
    rng = np.random.default_rng(0)
    a = rng.standard_normal((3, 128)).astype(np.float32)
    b = a.copy(); b[:, 32:64] *= 1000.0
    ca, sa = mx.mx_quantize_rows(a); cb, sb = mx.mx_quantize_rows(b)
    keep = np.r_[0:32, 64:128]
    assert np.array_equal(ca[:, keep], cb[:, keep]) and np.array_equal(sa[:, [0, 2, 3]], sb[:, [0, 2, 3]])
    assert not np.array_equal(sa[:, 1], sb[:, 1])
    # relative error bound of the format inside a block: half a mantissa step of the top binade relative to amax
    err = np.abs(mx.mx_dequantize(ca, sa) - a)
    amax = np.abs(a.reshape(3, 4, 32)).max(axis=2)
    assert np.all(err.reshape(3, 4, 32) <= amax[:, :, None] * 0.125 + 1e-12)


def test_pack_layout_and_round_trip():
    codes = np.arange(64, dtype=np.uint8).reshape(1, 64) % 64
    p = mx.pack_fp6(codes)
    assert p.shape == (1, 48)
    bits = int.from_bytes(bytes(p[0, :24].tolist()), "little")
    for i in range(32):
        assert (bits >> (6 * i)) & 63 == codes[0, i]
    rng = np.random.default_rng(1)
    c = rng.integers(0, 64, size=(5, 256)).astype(np.uint8)
    assert np.array_equal(mx.unpack_fp6(mx.pack_fp6(c), 256), c)


def test_mx_gemm_is_the_product_of_the_dequantised_matrices_and_close_to_the_plain_product():
    rng = np.random.default_rng(2)
    X = rng.standard_normal((24, 256)).astype(np.float32); W = (rng.standard_normal((40, 256)) * 0.02).astype(np.float32)
    f = mx.forward_mxfp6(X, W, 256)
    A, B = mx.mx_dequantize(f["Xc"], f["Xs"]), mx.mx_dequantize(f["Wc"], f["Ws"])
    brute = np.array([[sum(A[i, k] * B[j, k] for k in range(256)) for j in range(40)] for i in range(0, 24, 6)])
    assert np.allclose(f["Y"][::6], brute, rtol=1e-12, atol=1e-15)
    ref = X.astype(np.float64) @ W.astype(np.float64).T
    assert np.linalg.norm(f["Y"] - ref) / np.linalg.norm(ref) < 0.08
    # the codes are those of the ROTATED operands
    assert not np.array_equal(f["Xc"], mx.mx_quantize_rows(X)[0])
    assert np.array_equal(f["Xc"], mx.mx_quantize_rows(orc.fwht(X, 256, 1))[0])
