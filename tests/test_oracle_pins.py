"""Pins for the CPU oracle: each step is checked against something other than itself
(closed forms, hand-typed fixtures, brute force, plain matrix algebra)."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import halo_oracle as orc
from paper_2501_02625_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers (independent of the oracle)
def dense_hadamard(d):
    """Normalised Sylvester matrix from the closed form H[i][j] = (-1)^popcount(i&j) / sqrt(d), fp64."""
    i = np.arange(d)
    bits = i[:, None] & i[None, :]
    pop = np.zeros_like(bits)
    while np.any(bits):
        pop += bits & 1
        bits >>= 1
    return np.where(pop % 2 == 0, 1.0, -1.0) / np.sqrt(float(d))


def read_sign_fixture():
    mats, name, rows = {}, None, []
    with open(os.path.join(GOLDEN, "sylvester_signs.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("H"):
                if name:
                    mats[name] = rows
                name, rows = line, []
            else:
                rows.append([1.0 if ch == "+" else -1.0 for ch in line])
        mats[name] = rows
    return {int(k[1:]): np.array(v) for k, v in mats.items()}


# ----------------------------------------------------------------------------- O1: Hadamard
def test_closed_form_matches_hand_typed_recursion_and_kronecker():
    fx = read_sign_fixture()
    for d, signs in fx.items():
        assert np.array_equal(np.sign(dense_hadamard(d)), signs)
    h2 = dense_hadamard(2) * np.sqrt(2.0)
    for d in (4, 8, 16, 64):
        hd = dense_hadamard(d) * np.sqrt(d)
        assert np.array_equal(hd, np.kron(h2, dense_hadamard(d // 2) * np.sqrt(d // 2)))


@pytest.mark.parametrize("d", [2, 4, 8, 16, 64, 256])
def test_fwht_equals_dense_matrix_product(d):
    rng = np.random.default_rng(d)
    x = rng.standard_normal((5, d))
    H = dense_hadamard(d)
    got64 = orc.fwht(x.astype(np.float64), d, 1)
    np.testing.assert_allclose(got64, x @ H, rtol=0, atol=1e-13 * np.sqrt(d) * np.abs(x).max() * d)
    got32 = orc.fwht(x.astype(np.float32), d, 1)
    assert got32.dtype == np.float32
    tol = np.log2(d) * 2.0 ** -23 * np.abs(x).sum(axis=1, keepdims=True) / np.sqrt(d) * 2
    assert np.all(np.abs(got32 - x.astype(np.float32).astype(np.float64) @ H) <= tol)


@pytest.mark.parametrize("d", [2, 8, 64, 512])
def test_fwht_of_identity_is_orthonormal_symmetric_and_has_pm_entries(d):
    H = orc.fwht(np.eye(d, dtype=np.float64), d, 1)       # rows e_j H = row j of H
    np.testing.assert_allclose(H @ H.T, np.eye(d), atol=1e-12)   # H H^T = I
    np.testing.assert_allclose(np.abs(H), 1.0 / np.sqrt(d), rtol=1e-14)
    assert np.array_equal(H, H.T)
    if d <= 64:
        np.testing.assert_allclose(H, dense_hadamard(d), atol=1e-15)


def test_fwht_closed_forms():
    d = 128
    ones = np.ones((1, d), dtype=np.float32)
    out = orc.fwht(ones, d, 1)
    expect = np.zeros(d, dtype=np.float32); expect[0] = np.float32(np.sqrt(d))
    np.testing.assert_allclose(out[0], expect, rtol=1e-6, atol=0)
    # alternating signs pick out the last basis vector of stride 1: x_i = (-1)^i -> sqrt(d) e_1
    alt = ((-1.0) ** np.arange(d)).astype(np.float32)[None]
    out = orc.fwht(alt, d, 1)
    expect = np.zeros(d, dtype=np.float32); expect[1] = np.float32(np.sqrt(d))
    np.testing.assert_allclose(out[0], expect, rtol=1e-6, atol=0)
    # x_i = (-1)^(i >= d/2): picks index d/2 (pins the stage <-> index-bit correspondence)
    half = np.where(np.arange(d) >= d // 2, -1.0, 1.0).astype(np.float32)[None]
    out = orc.fwht(half, d, 1)
    expect = np.zeros(d, dtype=np.float32); expect[d // 2] = np.float32(np.sqrt(d))
    np.testing.assert_allclose(out[0], expect, rtol=1e-6, atol=0)


def test_fwht_involution_and_parseval_fp32():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((7, 4096)).astype(np.float32)
    y = orc.fwht(x, 4096, 1)
    np.testing.assert_allclose(np.linalg.norm(y, axis=1), np.linalg.norm(x, axis=1), rtol=1e-5)
    z = orc.fwht(y, 4096, 1)
    assert np.max(np.abs(z - x)) <= 5e-6 * np.max(np.abs(x)) * 12


def test_fwht_block_diagonal_is_per_block_and_leaves_input_alone():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((3, 7 * 64)).astype(np.float32)
    keep = x.copy()
    y = orc.fwht(x, 64, 1)
    assert np.array_equal(x, keep)
    for k in range(7):
        assert np.array_equal(y[:, 64 * k:64 * (k + 1)], orc.fwht(x[:, 64 * k:64 * (k + 1)].copy(), 64, 1))
    assert np.array_equal(orc.fwht(x, 0, 1), x)


def test_left_hadamard_is_transpose_of_right_on_transpose():
    rng = np.random.default_rng(3)
    a = rng.standard_normal((256, 24)).astype(np.float32)
    left = orc.fwht(a, 128, 0)
    right = orc.fwht(np.ascontiguousarray(a.T), 128, 1).T
    assert np.array_equal(left, right)
    H = dense_hadamard(128)
    blk = np.kron(np.eye(2), H)
    np.testing.assert_allclose(left, blk.T @ a.astype(np.float64), atol=1e-4)


def test_fwht_fp32_stage_order_is_ascending_stride():
    """Scalar re-derivation with one fp32 rounding per add/sub, stride 1 first; bit-for-bit."""
    rng = np.random.default_rng(4)
    d = 32
    x = (rng.standard_normal(d) * np.array([1e-3, 1.0, 300.0, 7.0] * 8)).astype(np.float32)
    v = [np.float32(t) for t in x]
    h = 1
    while h < d:
        for i in range(d):
            if i & h == 0:
                a, b = v[i], v[i + h]
                v[i], v[i + h] = np.float32(a + b), np.float32(a - b)
        h *= 2
    c = np.float32(1.0 / np.sqrt(np.float64(d)))
    want = np.array([np.float32(t * c) for t in v], dtype=np.float32)
    got = orc.fwht(x[None].copy(), d, 1)[0]
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # and the order matters: descending stride gives different bits somewhere on such data
    w = [np.float32(t) for t in x]
    h = d // 2
    while h >= 1:
        for i in range(d):
            if i & h == 0:
                a, b = w[i], w[i + h]
                w[i], w[i + h] = np.float32(a + b), np.float32(a - b)
        h //= 2
    other = np.array([np.float32(t * c) for t in w], dtype=np.float32)
    np.testing.assert_allclose(other, want, rtol=1e-4, atol=1e-4)


# ----------------------------------------------------------------------------- O2: quantizer
def test_quantizer_hand_examples():
    with open(os.path.join(GOLDEN, "quantizer_hand_examples.txt")) as f:
        lines = [l.strip() for l in f if l.strip() and not l.startswith("#")]
    assert len(lines) == 4
    for line in lines:
        xs, cs, sc = [p.strip() for p in line.split("|")]
        x = np.array([float(t) for t in xs.split()], dtype=np.float32)[None]
        codes, scale = orc.quantize_rows(x)
        assert codes.dtype == np.int8 and scale.dtype == np.float32
        assert codes[0].tolist() == [int(t) for t in cs.split()]
        num, den = sc.split("/")
        assert scale[0] == np.float32(np.float32(num) / np.float32(den))


def test_quantizer_hadamard_hand_example_d4():
    x = np.ones((1, 4), dtype=np.float32)
    codes, scale = orc.quantize_rows(orc.fwht(x, 4, 1))
    assert codes[0].tolist() == [127, 0, 0, 0]
    assert scale[0] == np.float32(np.float32(2) / np.float32(127))


def test_quantizer_invariants():
    rng = np.random.default_rng(5)
    v = (rng.standard_normal((64, 300)) * rng.lognormal(0, 3, size=(64, 1))).astype(np.float32)
    v[7] = 0
    codes, scale = orc.quantize_rows(v)
    assert np.all(np.abs(codes.astype(np.int32)) <= 127)
    amax_pos = np.argmax(np.abs(v), axis=1)
    for r in range(64):
        if r == 7:
            assert scale[r] == 1 and not codes[r].any()
            continue
        assert abs(int(codes[r, amax_pos[r]])) == 127
        err = np.abs(v[r].astype(np.float64) - codes[r].astype(np.float64) * float(scale[r]))
        assert np.all(err <= 0.5 * float(scale[r]) * (1 + 1e-5))
        # rows are independent
        c1, s1 = orc.quantize_rows(v[r:r + 1])
        assert np.array_equal(c1[0], codes[r]) and s1[0] == scale[r]
    # exact rational check of the rounding decision away from ties
    r = 3
    inv = Fraction(float(np.float32(127) / np.max(np.abs(v[r]))))
    for k in range(0, 300, 17):
        q = Fraction(float(np.float32(Fraction(float(v[r, k])) * inv)))
        assert int(codes[r, k]) == round(q)   # Python's round() is ties-to-even as well


def test_quantizer_no_rounding_mode_is_a_pure_rescale():
    rng = np.random.default_rng(6)
    v = rng.standard_normal((4, 33))
    c, s = orc.quantize_rows(v, rounding=False)
    np.testing.assert_allclose(c * s[:, None], v, rtol=1e-14)
    np.testing.assert_allclose(np.max(np.abs(c), axis=1), 127.0, rtol=1e-14)


def test_quantize_tensor_hand_example_and_reduction_to_rows():
    """One scale for the whole tensor (Section 4 setup).  Hand example; and when every row has the same absmax the
    per-tensor quantizer must give exactly what the per-row one gives."""
    v = np.array([[1.0, -2.0, 0.5, 4.0], [0.25, 0.0, -1.0, 3.0]], dtype=np.float32)
    codes, scale = orc.quantize_tensor(v)
    # 127/4 = 31.75: 1 -> 31.75 -> 32, -2 -> -63.5 -> -64 (tie to even), 0.5 -> 15.875 -> 16, 0.25 -> 7.9375 -> 8, 3 -> 95.25 -> 95
    want = [[32, -64, 16, 127], [8, 0, -32, 95]]
    assert codes.tolist() == want and codes.dtype == np.int8
    assert scale.tolist() == [float(np.float32(4) / np.float32(127))] * 2 and scale.dtype == np.float32
    # per-row would scale the second row by 127/3 instead
    rows_codes, rows_scale = orc.quantize_rows(v)
    assert rows_codes[0].tolist() == want[0] and rows_codes[1].tolist() != want[1]
    rng = np.random.default_rng(31)
    u = rng.standard_normal((9, 40)).astype(np.float32)
    u[:, 0] = 5.0 * rng.choice([-1.0, 1.0], size=9)          # the same absmax in every row
    ct, st = orc.quantize_tensor(u)
    cr, sr = orc.quantize_rows(u)
    assert np.array_equal(ct, cr) and np.array_equal(st, sr)
    z, sz = orc.quantize_tensor(np.zeros((3, 4), dtype=np.float32))
    assert not z.any() and sz.tolist() == [1.0, 1.0, 1.0]


@pytest.mark.parametrize("level", [0, 1, 2])
def test_per_tensor_levels_equal_plain_products_when_rounding_is_off(level):
    """The paper-literal scalar-scale formulas of Table "HALO levels": with Q a pure rescale they reproduce
    X W^T, E W and E^T X at every level (scales factor out, no fold)."""
    rng = np.random.default_rng(40 + level)
    b, m, n = 32, 64, 48
    X = rng.standard_normal((b, m)); W = rng.standard_normal((n, m)) * 0.02; E = rng.standard_t(3, size=(b, n)) * 1e-3
    f = orc.forward(X, W, level, m, rounding=False, real=np.float64, per_tensor=True)
    ex = orc.backward_input(E, f["Wq"], f["s_w"], level, m, b, rounding=False, real=np.float64, per_tensor=True)
    g = orc.backward_weight(E, f["Xq"], f["s_x"], level, m, rounding=False, real=np.float64, per_tensor=True)
    ref = orc.plain_products(X, W, E)
    for got, want in ((f["Y"], ref["Y"]), (ex["EX"], ref["EX"]), (g["G"], ref["G"])):
        assert np.max(np.abs(got - want)) <= 1e-11 * np.max(np.abs(want))
    assert np.all(f["s_x"] == f["s_x"][0]) and np.all(f["s_w"] == f["s_w"][0])
    # the quantised error is E itself (left-rotated at level 2) over one scalar, not a folded tensor
    L = dense_hadamard(b) if level >= 2 else np.eye(b)
    assert np.allclose(ex["Eq"] * ex["s_e"][:, None], L.T @ E, rtol=1e-10, atol=1e-18)
    assert np.all(ex["s_e"] == ex["s_e"][0])


def test_per_tensor_is_worse_than_per_row_on_outlier_rows():
    """Why the build target asks for per-row scales: with heavy-tailed errors one tensor-wide scale wastes most of
    the INT8 range on a few rows (Section 3.2, Step 3 describes those outliers)."""
    X = inputs.bf16_bits_to_f32(inputs.make_activations(128, 512, 0.005, 0))
    W = inputs.bf16_bits_to_f32(inputs.make_weights(256, 512, 0))
    E = inputs.bf16_bits_to_f32(inputs.make_errors(128, 256, 0))
    ref = orc.plain_products(X, W, E)
    err = {}
    for pt in (False, True):
        f = orc.forward(X, W, 1, 512, per_tensor=pt)
        ex = orc.backward_input(E, f["Wq"], f["s_w"], 1, 512, 128, per_tensor=pt)
        err[pt] = np.linalg.norm(ex["EX"].astype(np.float64) - ref["EX"]) / np.linalg.norm(ref["EX"])
    assert err[True] > 1.5 * err[False] and err[False] < 0.1, err


# ----------------------------------------------------------------------------- O3 / O4: GEMM, dequant
def test_gemm_codes_brute_force_int64():
    rng = np.random.default_rng(7)
    a = rng.integers(-127, 128, size=(9, 37), dtype=np.int8)
    b = rng.integers(-127, 128, size=(37, 5), dtype=np.int8)
    got = orc.gemm_codes(a, b)
    assert got.dtype == np.int32
    want = np.zeros((9, 5), dtype=np.int64)
    for i in range(9):
        for j in range(5):
            for k in range(37):
                want[i, j] += int(a[i, k]) * int(b[k, j])
    assert np.array_equal(got.astype(np.int64), want)
    assert np.array_equal(got.astype(np.int64), a.astype(np.int64) @ b.astype(np.int64))


def test_gemm_codes_extreme_values_at_longest_k():
    k = 14336
    a = np.full((2, k), 127, dtype=np.int8); a[1] = -127
    b = np.full((k, 2), 127, dtype=np.int8); b[:, 1] = -127
    got = orc.gemm_codes(a, b)
    big = 127 * 127 * k
    assert big < 2 ** 31
    assert got.tolist() == [[big, -big], [-big, big]]


def test_dequantize_order_and_rounding():
    acc = np.array([[(1 << 24) + 1, -3]], dtype=np.int32)
    s_r = np.array([np.float32(1) / np.float32(3)], dtype=np.float32)
    s_c = np.array([np.float32(0.1), np.float32(7)], dtype=np.float32)
    out = orc.dequantize(acc, s_r, s_c)
    a0 = np.float32(1 << 24)            # 2^24+1 rounds to even
    want0 = np.float32(np.float32(a0 * s_r[0]) * s_c[0])
    want1 = np.float32(np.float32(np.float32(-3) * s_r[0]) * s_c[1])
    assert out.dtype == np.float32 and out[0, 0] == want0 and out[0, 1] == want1


def test_bf16_round_trip_and_ties():
    vals = np.array([1.0, 1.00390625, 1.005859375, 1.001953125, -2.5, 3.0e-5, 65280.0], dtype=np.float32)
    bits = orc.real_to_bf16_bits(vals)
    back = orc.bf16_bits_to_real(bits)
    # 1 + 2^-8 is a tie between 1.0 and 1+2^-7 -> even mantissa (1.0); 1 + 3*2^-9 -> up
    assert back[1] == np.float32(1.0)
    assert back[2] == np.float32(1.0078125)
    assert back[3] == np.float32(1.0)
    assert np.all(np.abs(back - vals) <= np.abs(vals) * 2.0 ** -8)
    assert np.array_equal(orc.real_to_bf16_bits(back), bits)
    assert np.array_equal(inputs.f32_to_bf16_bits(vals), bits)     # the generator's rounding agrees


# ----------------------------------------------------------------------------- O5: placement algebra
@pytest.mark.parametrize("level", [0, 1, 2])
@pytest.mark.parametrize("shape", [(64, 96, 40), (32, 64, 64)])
def test_levels_equal_plain_products_when_rounding_is_off(level, shape):
    """With Q a pure rescale, F, E and G of every level equal X W^T, E W and E^T X: this pins every
    Hadamard placement, the scale fold and both un-rotations (Section 3.1 cases; Section 3.2 Step 2)."""
    b, m, n = shape
    rng = np.random.default_rng(10 * level + b)
    X = rng.standard_normal((b, m)) * (1 + 30 * (rng.random(m) < 0.05))
    W = rng.standard_normal((n, m)) * 0.02 * rng.lognormal(0, 1, size=(n, 1))
    E = rng.standard_t(3, size=(b, n)) * 1e-3
    hm, hb = (m & -m), (b & -b)
    f = orc.forward(X, W, level, hm, rounding=False, real=np.float64)
    ex = orc.backward_input(E, f["Wq"], f["s_w"], level, hm, hb, rounding=False, real=np.float64)
    g = orc.backward_weight(E, f["Xq"], f["s_x"], level, hm, rounding=False, real=np.float64)
    ref = orc.plain_products(X, W, E)
    for got, want in ((f["Y"], ref["Y"]), (ex["EX"], ref["EX"]), (g["G"], ref["G"])):
        assert got.shape == want.shape
        assert np.max(np.abs(got - want)) <= 1e-12 * np.max(np.abs(want)) * 10
    # the codes really are rotated at levels >= 1 and not at level 0
    plain_codes, _ = orc.quantize_rows(X, rounding=False)
    assert np.allclose(f["Xq"], plain_codes) == (level == 0)


def test_planted_mistakes_are_caught_by_the_algebra_pin():
    """The pin above has teeth: dropping the fold or an un-rotation breaks it.  (The left Hadamard of level 2 cancels
    in the product; test_level2_really_left_rotates_the_error_before_quantising pins it.)"""
    rng = np.random.default_rng(11)
    b, m, n = 32, 64, 48
    X = rng.standard_normal((b, m)); W = rng.standard_normal((n, m)) * rng.lognormal(0, 1, size=(n, 1))
    E = rng.standard_normal((b, n))
    ref = orc.plain_products(X, W, E)
    f = orc.forward(X, W, 2, m, rounding=False, real=np.float64)
    ones = np.ones_like(f["s_w"])
    no_fold = orc.backward_input(E, f["Wq"], ones, 2, m, b, rounding=False, real=np.float64)["EX"]
    assert np.max(np.abs(no_fold - ref["EX"])) > 1e-3 * np.max(np.abs(ref["EX"]))
    lvl_mismatch = orc.backward_input(E, f["Wq"], f["s_w"], 0, m, b, rounding=False, real=np.float64)["EX"]
    assert np.max(np.abs(lvl_mismatch - ref["EX"])) > 1e-3 * np.max(np.abs(ref["EX"]))
    g_wrong = orc.backward_weight(E, f["Xq"], f["s_x"], 0, m, rounding=False, real=np.float64)["G"]
    assert np.max(np.abs(g_wrong - ref["G"])) > 1e-3 * np.max(np.abs(ref["G"]))


def _level2_quantises_the_left_rotated_error(backward_input, E, Wq, s_w, m, b, hb):
    """True iff backward_input(level 2)'s quantiser input is (I (x) H_hb)^T E scaled by s_w per column, built here
    from the dense closed-form matrix: with the rounding off, Eq * s_e is exactly the tensor that was quantised."""
    L = np.kron(np.eye(b // hb), dense_hadamard(hb))
    want = (L.T @ E) * s_w[None, :]
    r = backward_input(E, Wq, s_w, 2, m, hb)
    got = r["Eq"] * r["s_e"][:, None]
    return got.shape == want.shape and np.max(np.abs(got - want)) <= 1e-12 * np.max(np.abs(want))


@pytest.mark.parametrize("hb", [32, 8])
def test_level2_really_left_rotates_the_error_before_quantising(hb):
    """Table "HALO levels", HALO-2 row: E = H^T (H E_Y)_Q (WH)_Q H^T.  The two left-hand rotations cancel
    when Q is a pure rescale, so the product pin above cannot see them; this one looks at what is quantised."""
    rng = np.random.default_rng(21)
    b, m, n = 32, 64, 48
    X = rng.standard_normal((b, m)); W = rng.standard_normal((n, m)) * rng.lognormal(0, 1, size=(n, 1))
    E = rng.standard_t(3, size=(b, n))
    f = orc.forward(X, W, 2, m, rounding=False, real=np.float64)
    oracle = lambda E_, Wq, s_w, lvl, m_, hb_: orc.backward_input(E_, Wq, s_w, lvl, m_, hb_, rounding=False, real=np.float64)
    assert _level2_quantises_the_left_rotated_error(oracle, E, f["Wq"], f["s_w"], m, b, hb)
    # planted mistakes: level 2 computed as level 1, level 2 with the left rotation skipped, with a left block
    # of the wrong size, and with the rotation on the wrong (right-hand) side of E
    as_level1 = lambda E_, Wq, s_w, lvl, m_, hb_: oracle(E_, Wq, s_w, 1, m_, hb_)
    no_left = lambda E_, Wq, s_w, lvl, m_, hb_: oracle(E_, Wq, s_w, 2, m_, 0)
    wrong_block = lambda E_, Wq, s_w, lvl, m_, hb_: oracle(E_, Wq, s_w, 2, m_, hb_ // 2)
    right_side = lambda E_, Wq, s_w, lvl, m_, hb_: oracle(orc.fwht(E_, 16, 1), Wq, s_w, 1, m_, hb_)
    for mutant in (as_level1, no_left, wrong_block, right_side):
        assert not _level2_quantises_the_left_rotated_error(mutant, E, f["Wq"], f["s_w"], m, b, hb)
    # and the level-1 quantiser input is the plain E (x) s_w: the two levels differ exactly by L
    r1 = oracle(E, f["Wq"], f["s_w"], 1, m, hb)
    assert np.allclose(r1["Eq"] * r1["s_e"][:, None], E * f["s_w"][None, :], rtol=1e-12, atol=0)
    r2 = oracle(E, f["Wq"], f["s_w"], 2, m, hb)
    assert np.max(np.abs(r2["Eq"] * r2["s_e"][:, None] - r1["Eq"] * r1["s_e"][:, None])) > 1e-3 * np.max(np.abs(E * f["s_w"]))
    # with the rounding on (fp32), the INT8 codes are those of the dense-matrix rotation up to one code step at
    # values that fp32 and fp64 place on different sides of a rounding boundary
    E32 = E.astype(np.float32)
    f32 = orc.forward(X.astype(np.float32), W.astype(np.float32), 2, m)
    got = orc.backward_input(E32, f32["Wq"], f32["s_w"], 2, m, hb)
    L = np.kron(np.eye(b // hb), dense_hadamard(hb))
    ref = (L.T @ E32.astype(np.float64)) * f32["s_w"].astype(np.float64)[None, :]
    ref_codes = np.rint(ref * (127.0 / np.max(np.abs(ref), axis=1))[:, None])
    d = np.abs(got["Eq"].astype(np.int64) - ref_codes.astype(np.int64))
    assert d.max() <= 1 and np.mean(d != 0) < 0.01
    as1 = orc.backward_input(E32, f32["Wq"], f32["s_w"], 1, m, hb)
    assert np.mean(as1["Eq"] != got["Eq"]) > 0.5


def test_fold_reduces_to_scalar_scale_formula_when_all_row_scales_are_equal():
    """Level 0, weight rows that are signed permutations of one vector whose absmax is 127*2^-9:
    every s_w equals 2^-9, so folding it into E only shifts exponents and E_X must equal
    s * s_e * (E_Q W_Q), the paper's single-scale form, bit for bit."""
    rng = np.random.default_rng(12)
    m, n, b = 64, 16, 8
    base = rng.integers(-126, 127, size=m).astype(np.float32)
    base[0] = 127
    W = np.stack([rng.permutation(base) * rng.choice([-1.0, 1.0]) for _ in range(n)]).astype(np.float32) * np.float32(2.0 ** -9)
    E = inputs.bf16_bits_to_f32(inputs.make_errors(b, n, 3))
    X = rng.standard_normal((b, m)).astype(np.float32)
    f = orc.forward(X, W, 0, 0)
    assert np.all(f["s_w"] == np.float32(2.0 ** -9))
    got = orc.backward_input(E, f["Wq"], f["s_w"], 0, 0, 0)
    Eq, s_e = orc.quantize_rows(E)
    assert np.array_equal(got["Eq"], Eq)
    want = orc.dequantize(orc.gemm_codes(Eq, f["Wq"]), s_e * np.float32(2.0 ** -9))
    assert np.array_equal(got["EX"], want)


def test_quantized_path_is_close_and_hadamard_helps_on_outlier_channels():
    """Qualitative claim of Section 3.2 Step 1 / Appendix ablation on levels: with outlier channels in X,
    INT8 without the forward Hadamard is much worse than with it."""
    cfg = inputs.CONFIGS["c1"]
    t = inputs.make_linear_inputs(cfg)
    X = orc.bf16_bits_to_real(t["X"]); W = orc.bf16_bits_to_real(t["W"])
    ref = orc.plain_products(X, W, None)["Y"]
    errs = {}
    for level in (0, 1):
        Y = orc.forward(X, W, level, 512)["Y"].astype(np.float64)
        errs[level] = np.linalg.norm(Y - ref) / np.linalg.norm(ref)
    assert errs[1] < 0.02
    assert errs[0] > 3 * errs[1]


def test_quantized_backward_is_close_to_plain_products():
    rng = np.random.default_rng(13)
    b, m, n = 128, 256, 192
    X = inputs.bf16_bits_to_f32(inputs.make_activations(b, m, 0.01, 5))
    W = inputs.bf16_bits_to_f32(inputs.make_weights(n, m, 5))
    E = inputs.bf16_bits_to_f32(inputs.make_errors(b, n, 5))
    ref = orc.plain_products(X, W, E)
    for level in (1, 2):
        f = orc.forward(X, W, level, 256)
        ex = orc.backward_input(E, f["Wq"], f["s_w"], level, 256, 128)
        g = orc.backward_weight(E, f["Xq"], f["s_x"], level, 256)
        assert f["Xq"].dtype == np.int8 and ex["acc"].dtype == np.int32
        for got, want, tol in ((f["Y"], ref["Y"], 0.03), (ex["EX"], ref["EX"], 0.08), (g["G"], ref["G"], 0.08)):
            rel = np.linalg.norm(got.astype(np.float64) - want) / np.linalg.norm(want)
            assert rel < tol, (level, rel)
