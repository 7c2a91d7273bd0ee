"""GPU parity of the Kronecker rotation H_{2^n} (x) H_28 (Section 2, "Hadamard Transformations") against the CPU oracle,
through the C ABI: quantiser codes and scales bit-exact, fp32 un-rotated outputs bit-identical, bf16 within one ulp,
and the whole layer at levels 1 and 2 with a Kronecker block on the in-feature axis."""
import numpy as np
import pytest
import torch

from oracle import halo_oracle as orc
from paper_2501_02625_amd import binding, inputs
from tests import gpu_util as gu
from tests.test_gpu_linear import run_and_check

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("rows,cols,block", [
    (37, 1792, 1792),          # one wavefront per row, no stage across wavefronts
    (64, 3584, 1792),          # two blocks per row
    (33, 7168, 3584),          # one stage across wavefronts
    (24, 14336, 7168),         # two stages
    (16, 14336, 14336),        # the paper's 512 * 28: three stages across eight wavefronts
])
def test_quantiser_with_kronecker_blocks(rows, cols, block):
    xb = inputs.make_activations(rows, cols, 0.01, rows + cols)
    x = orc.bf16_bits_to_real(xb)
    want_q, want_s = orc.quantize_rows(orc.fwht(x, block, 1))
    q, s = binding.halo_hadamard_quant(gu.bits_to_dev(xb), had_block=block)
    gu.assert_codes_equal(q, want_q, "codes")
    gu.assert_f32_identical(s, want_s, "scales")
    # the same launch twice gives the same bits
    q2, s2 = binding.halo_hadamard_quant(gu.bits_to_dev(xb), had_block=block)
    assert torch.equal(q, q2) and torch.equal(s, s2)


def test_quantiser_with_fold_fp32_input_and_a_zero_row():
    rows, cols, block = 19, 3584, 3584
    rng = np.random.default_rng(5)
    x = rng.standard_normal((rows, cols)).astype(np.float32)
    x[3] = 0.0
    fold = (rng.random(cols) + 0.25).astype(np.float32)
    want_q, want_s = orc.quantize_rows(orc.fwht(x, block, 1) * fold[None, :])
    q, s = binding.halo_hadamard_quant(gu.to_dev(x), had_block=block, fold=gu.to_dev(fold))
    gu.assert_codes_equal(q, want_q, "codes")
    gu.assert_f32_identical(s, want_s, "scales")
    assert want_s[3] == 1.0 and not want_q[3].any()


def test_quantiser_with_left_rotation_then_kronecker_block():
    rows, cols = 64, 1792
    xb = inputs.make_errors(rows, cols, 9)
    x = orc.bf16_bits_to_real(xb)
    want_q, want_s = orc.quantize_rows(orc.fwht(orc.fwht(x, 64, 0), 1792, 1))
    q, s = binding.halo_hadamard_quant(gu.bits_to_dev(xb), had_block=1792, had_block_left=64)
    gu.assert_codes_equal(q, want_q, "codes")
    gu.assert_f32_identical(s, want_s, "scales")


@pytest.mark.parametrize("rows,cols,block", [(21, 1792, 1792), (40, 14336, 14336), (12, 7168, 1792)])
def test_unrotation_of_accumulators(rows, cols, block):
    rng = np.random.default_rng(rows)
    acc = rng.integers(-127 * 127 * 64, 127 * 127 * 64, size=(rows, cols), dtype=np.int32)
    s = (rng.random(rows) * 1e-3 + 1e-5).astype(np.float32)
    want = orc.fwht(orc.dequantize(acc, s, None, np.float32), block, 1)
    out = binding.halo_dequant_unrotate(gu.to_dev(acc), gu.to_dev(s), had_block=block, out_dtype=torch.float32)
    gu.assert_f32_identical(out[:, :cols].contiguous(), want, "fp32 un-rotation")
    out16 = binding.halo_dequant_unrotate(gu.to_dev(acc), gu.to_dev(s), had_block=block, out_dtype=torch.bfloat16)
    gu.assert_bf16_within_one_ulp(out16[:, :cols].contiguous(), want, "bf16 un-rotation")


@pytest.mark.parametrize("level", [1, 2])
def test_layer_with_kronecker_block_on_the_in_feature_axis(level):
    b, m, n = 64, 3584, 128
    Xb = inputs.make_activations(b, m, 0.01, 31); Wb = inputs.make_weights(n, m, 31); Eb = inputs.make_errors(b, n, 31)
    run_and_check(b, m, n, level, Xb, Wb, Eb, hm=1792)


def test_layer_at_the_papers_width_14336():
    """m = 14336 = 512 * 28 in one Kronecker block, level 2, every output compared in full."""
    b, m, n = 256, 14336, 256
    Xb = inputs.make_activations(b, m, 0.01, 32); Wb = inputs.make_weights(n, m, 32); Eb = inputs.make_errors(b, n, 32)
    run_and_check(b, m, n, 2, Xb, Wb, Eb, hm=14336, internals=True)
    run_and_check(b, m, n, 1, Xb, Wb, Eb, hm=14336, odt=torch.bfloat16)


def test_config_c6_full_size_level2():
    """Config c6: the shape of c3 (tokens 4096, K = 14336, N = 4096, HALO-2) with one Kronecker block over K,
    every output compared in full."""
    cfg = inputs.CONFIGS["c6"]
    t = inputs.make_linear_inputs(cfg)
    run_and_check(cfg.tokens, 14336, 4096, cfg.level, t["X"], t["W"], t["E"], odt=torch.float32,
                  hm=cfg.had_block_m(14336))


def test_kronecker_rotation_spreads_outliers_like_the_block_diagonal_one():
    """Quantisation error of X at 14336 columns with outlier channels: both rotations beat no rotation by a wide margin."""
    rows, cols = 64, 14336
    xb = inputs.make_activations(rows, cols, 0.01, 77)
    x = orc.bf16_bits_to_real(xb).astype(np.float64)
    errs = {}
    for name, block in (("none", 0), ("blockdiag", 2048), ("kron", 14336)):
        q, s = binding.halo_hadamard_quant(gu.bits_to_dev(xb), had_block=block)
        deq = q.cpu().numpy().astype(np.float64) * s.cpu().numpy().astype(np.float64)[:, None]
        back = orc.fwht(deq, block, 1) if block else deq       # both rotations are symmetric and orthonormal
        errs[name] = np.linalg.norm(back - x) / np.linalg.norm(x)
    assert errs["kron"] < 0.5 * errs["none"] and errs["blockdiag"] < 0.5 * errs["none"]
    assert errs["kron"] < 1.2 * errs["blockdiag"]
