"""Pins for the oracle's Kronecker rotation H_{2^n} (x) H_28 (Section 2, "Hadamard Transformations"): the order-28
factor against the definition of a Hadamard matrix and hand-typed quadratic residues, the transform against a dense
Kronecker product built with a library routine, and the placement algebra of the three products."""
import os

import numpy as np
import pytest
import scipy.linalg

from oracle import halo_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def hand_typed_character():
    with open(os.path.join(GOLDEN, "quadratic_character_mod13.txt")) as f:
        line = [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")][0]
    return [{"0": 0, "+": 1, "-": -1}[ch] for ch in line]


def test_order_28_factor_is_a_symmetric_hadamard_matrix():
    H = orc.paley_hadamard_28()
    assert H.shape == (28, 28)
    assert set(np.unique(H).tolist()) == {-1, 1}
    assert np.array_equal(H @ H.T, 28 * np.eye(28, dtype=np.int64))
    assert np.array_equal(H, H.T)


def test_order_28_factor_follows_the_quadratic_character():
    """Row 1 of the conference matrix is chi(-j) = chi(j) (13 = 1 mod 4); every entry c = +-1 of it stands at the top left
    of a block c * [[1, 1], [1, -1]] and the diagonal zero becomes [[1, -1], [-1, -1]]."""
    chi = hand_typed_character()
    assert len(chi) == 13 and chi[0] == 0
    # the hand-typed line against the definition: a is a square iff a^6 = 1 (mod 13) (Euler's criterion)
    for a in range(1, 13):
        assert chi[a] == (1 if pow(a, 6, 13) == 1 else -1)
    H = orc.paley_hadamard_28()
    for j in range(1, 13):
        blk = H[2:4, 2 + 2 * j:4 + 2 * j]
        assert np.array_equal(blk, chi[j] * np.array([[1, 1], [1, -1]]))
    assert np.array_equal(H[2:4, 2:4], np.array([[1, -1], [-1, -1]]))
    # border of the conference matrix: all ones
    for j in range(1, 14):
        assert np.array_equal(H[0:2, 2 * j:2 * j + 2], np.array([[1, 1], [1, -1]]))
    assert np.array_equal(H[0:2, 0:2], np.array([[1, -1], [-1, -1]]))


def test_block_factorisation_helper():
    assert orc.kron_block_factors(28) == (1, 28)
    assert orc.kron_block_factors(14336) == (512, 28)
    assert orc.kron_block_factors(1792) == (64, 28)
    assert orc.kron_block_factors(2048) is None
    assert orc.kron_block_factors(84) is None        # 3 * 28
    assert orc.kron_block_factors(0) is None


@pytest.mark.parametrize("p", [1, 2, 8, 64])
def test_kronecker_rotation_equals_dense_kronecker_product(p):
    """x -> x (H_p (x) H_28) / sqrt(28 p) with the Walsh-Hadamard factor outermost: element i * 28 + j."""
    d = 28 * p
    rng = np.random.default_rng(p)
    x = rng.standard_normal((5, 2 * d))
    H28 = orc.paley_hadamard_28().astype(np.float64)
    Hp = scipy.linalg.hadamard(p).astype(np.float64) if p > 1 else np.ones((1, 1))
    K = np.kron(Hp, H28) / np.sqrt(float(d))
    want = np.concatenate([x[:, :d] @ K, x[:, d:] @ K], axis=1)
    got = orc.fwht(x, d, 1)
    assert np.max(np.abs(got - want)) <= 1e-13 * np.max(np.abs(want)) * d
    if p > 1:       # the other Kronecker order is a different matrix and must not match
        K_swapped = np.kron(H28, Hp) / np.sqrt(float(d))
        assert np.max(np.abs(got[:, :d] - x[:, :d] @ K_swapped)) > 1e-3
    # left-hand form is the transpose of the right-hand form on the transpose
    xt = np.ascontiguousarray(x.T)
    assert np.array_equal(orc.fwht(xt, d, 0), np.ascontiguousarray(orc.fwht(x, d, 1).T))


def test_kronecker_rotation_is_an_orthonormal_involution_in_fp32():
    d = 28 * 64
    rng = np.random.default_rng(3)
    x = rng.standard_normal((4, d)).astype(np.float32)
    y = orc.fwht(x, d, 1)
    assert y.dtype == np.float32
    assert np.allclose(np.sum(y.astype(np.float64) ** 2, axis=1), np.sum(x.astype(np.float64) ** 2, axis=1), rtol=1e-5)
    back = orc.fwht(y, d, 1)
    assert np.max(np.abs(back - x)) <= 64 * 2.0 ** -24 * np.max(np.abs(x)) * 8
    # fp32 against fp64 within the running-sum bound: (27 + 6 + 2) roundings over sum |x| / sqrt(d)
    y64 = orc.fwht(x.astype(np.float64), d, 1)
    bound = 35 * 2.0 ** -24 * np.sum(np.abs(x.astype(np.float64)), axis=1, keepdims=True) / np.sqrt(d)
    assert np.all(np.abs(y - y64) <= bound)


def test_order_28_factor_sums_in_ascending_index_order_in_fp32():
    """With x = (2^24, 1, 1, ..., 1) the ascending running sum in fp32 absorbs every +1 (a tie that rounds back to the
    even 2^24) but follows every -1 while the sum sits at or below 2^24; summing the ones first gives another value."""
    H = orc.paley_hadamard_28()
    x = np.ones((1, 28), dtype=np.float32)
    x[0, 0] = np.float32(2.0 ** 24)
    got = orc.fwht(x, 28, 1)[0]
    c = np.float32(1.0 / np.sqrt(28.0))
    differs = 0
    for i in range(28):
        acc = np.float32(H[0, i]) * x[0, 0]
        for j in range(1, 28):
            acc = np.float32(acc + np.float32(H[j, i]) * x[0, j])
        assert got[i] == np.float32(acc * c)
        ones_first = np.float32(0.0)
        for j in range(27, 0, -1):
            ones_first = np.float32(ones_first + np.float32(H[j, i]) * x[0, j])
        other = np.float32(np.float32(ones_first + np.float32(H[0, i]) * x[0, 0]) * c)
        differs += int(other != got[i])
    assert differs > 0


@pytest.mark.parametrize("level", [1, 2])
def test_levels_with_a_kronecker_block_equal_plain_products_when_rounding_is_off(level):
    """Placement algebra with had_block_m = 2 * 28 over m = 112 (two blocks): F, E and G equal the plain products."""
    b, m, n = 32, 112, 48
    rng = np.random.default_rng(20 + level)
    X = rng.standard_normal((b, m)) * (1 + 30 * (rng.random(m) < 0.05))
    W = rng.standard_normal((n, m)) * 0.02
    E = rng.standard_t(3, size=(b, n)) * 1e-3
    f = orc.forward(X, W, level, 56, rounding=False, real=np.float64)
    ex = orc.backward_input(E, f["Wq"], f["s_w"], level, 56, 32, rounding=False, real=np.float64)
    g = orc.backward_weight(E, f["Xq"], f["s_x"], level, 56, rounding=False, real=np.float64)
    ref = orc.plain_products(X, W, E)
    for got, want in ((f["Y"], ref["Y"]), (ex["EX"], ref["EX"]), (g["G"], ref["G"])):
        assert np.max(np.abs(got - want)) <= 1e-11 * np.max(np.abs(want))


def test_kronecker_rotation_spreads_an_outlier_channel_over_its_block():
    """One large channel in a block of 28 * 8 lands with equal magnitude on every element of that block only."""
    d = 28 * 8
    x = np.zeros((1, 2 * d), dtype=np.float32)
    x[0, 5] = 100.0
    y = orc.fwht(x, d, 1)[0]
    assert np.allclose(np.abs(y[:d]), 100.0 / np.sqrt(d), rtol=1e-6)
    assert np.all(y[d:] == 0.0)
