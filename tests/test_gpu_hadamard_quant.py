"""GPU parity: halo_hadamard_quant / halo_dequant_unrotate against the CPU oracle, through the C ABI.
INT8 codes and fp32 scales must match bit for bit."""
import numpy as np
import pytest
import torch

from oracle import halo_oracle as orc
from paper_2501_02625_amd import binding, inputs
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def oracle_row_quant(x_real, had_block, had_block_left=0, fold=None):
    v = x_real
    if had_block_left:
        v = orc.fwht(v, had_block_left, 0)
    v = orc.fwht(v, had_block, 1)
    if fold is not None:
        v = v * fold[None, :]
    return orc.quantize_rows(v)


ROW_CASES = [
    # rows, cols, had_block, outlier fraction
    (128, 512, 512, 0.005),      # config c1 activation shape
    (37, 4096, 4096, 0.001),     # one wavefront per row, ragged row count
    (5, 14336, 2048, 0.001),     # block-diagonal 7 x 2048, seven wavefronts per row
    (64, 1024, 1024, 0.01),
    (33, 2048, 2048, 0.01),
    (16, 1536, 512, 0.01),       # three blocks
    (9, 512, 64, 0.0),           # small blocks inside one segment
    (3, 8, 8, 0.0),
    (4, 16, 2, 0.0),
    (7, 1000, 0, 0.01),          # no rotation, ragged row length
    (130, 4096, 0, 0.001),
    (1, 32768, 4096, 0.0),       # longest supported row
    (21, 4096, 256, 0.001),
]


@pytest.mark.parametrize("rows,cols,hb,frac", ROW_CASES)
def test_row_quant_bf16_bit_exact(rows, cols, hb, frac):
    bits = inputs.make_activations(rows, cols, frac, seed=rows + cols)
    ld = (cols + 7) // 8 * 8
    x = torch.zeros((rows, ld), dtype=torch.bfloat16, device=gu.DEV)
    x[:, :cols] = gu.bits_to_dev(bits)
    ldq = (cols + 15) // 16 * 16
    out_q = torch.full((rows, ldq), 55, dtype=torch.int8, device=gu.DEV)
    q, s = binding.halo_hadamard_quant(x[:, :cols], had_block=hb, out_q=out_q[:, :cols])
    torch.cuda.synchronize()
    wq, ws = oracle_row_quant(orc.bf16_bits_to_real(bits), hb)
    gu.assert_codes_equal(q, wq, "codes")
    gu.assert_f32_identical(s, ws, "scales")
    if ldq > cols:
        assert torch.all(out_q[:, cols:] == 55), "padding columns were overwritten"


def test_row_quant_weights_and_errors_distributions():
    w = inputs.make_weights(96, 4096, 3)
    q, s = binding.halo_hadamard_quant(gu.bits_to_dev(w), had_block=4096)
    wq, ws = oracle_row_quant(orc.bf16_bits_to_real(w), 4096)
    gu.assert_codes_equal(q, wq, "W codes"); gu.assert_f32_identical(s, ws, "W scales")
    e = inputs.make_errors(200, 4096, 3)
    fold = np.abs(np.random.default_rng(0).standard_normal(4096)).astype(np.float32) * 1e-3 + 1e-5
    q, s = binding.halo_hadamard_quant(gu.bits_to_dev(e), had_block=0, fold=gu.to_dev(fold))
    wq, ws = oracle_row_quant(orc.bf16_bits_to_real(e), 0, fold=fold)
    gu.assert_codes_equal(q, wq, "E codes"); gu.assert_f32_identical(s, ws, "E scales")


def test_row_quant_zero_rows_and_extreme_values():
    x = inputs.bf16_bits_to_f32(inputs.make_activations(8, 512, 0.0, 1))
    x[2] = 0
    x[5, 17] = 3.0e38
    x[6] *= 1e-30
    bits = inputs.f32_to_bf16_bits(x)
    q, s = binding.halo_hadamard_quant(gu.bits_to_dev(bits), had_block=0)
    wq, ws = oracle_row_quant(orc.bf16_bits_to_real(bits), 0)
    gu.assert_codes_equal(q, wq, "codes"); gu.assert_f32_identical(s, ws, "scales")
    assert s[2].item() == 1.0 and not q[2].any()
    x[5, 17] = 1.0
    bits = inputs.f32_to_bf16_bits(x)
    q, s = binding.halo_hadamard_quant(gu.bits_to_dev(bits), had_block=512)
    wq, ws = oracle_row_quant(orc.bf16_bits_to_real(bits), 512)
    gu.assert_codes_equal(q, wq, "rotated codes"); gu.assert_f32_identical(s, ws, "rotated scales")


@pytest.mark.parametrize("rows,cols,hb", [(19, 1024, 1024), (6, 4096, 4096), (11, 200, 0), (4, 6144, 2048)])
def test_row_quant_fp32_input(rows, cols, hb):
    rng = np.random.default_rng(rows)
    x = (rng.standard_normal((rows, cols)) * rng.lognormal(0, 2, size=(1, cols))).astype(np.float32)
    q, s = binding.halo_hadamard_quant(gu.to_dev(x), had_block=hb)
    wq, ws = oracle_row_quant(x, hb)
    gu.assert_codes_equal(q, wq, "codes"); gu.assert_f32_identical(s, ws, "scales")


LEFT_CASES = [(256, 192, 256), (64, 520, 64), (2048, 256, 512), (4096, 384, 4096), (8192, 128, 8192), (128, 64, 2)]


@pytest.mark.parametrize("rows,cols,hbl", LEFT_CASES)
def test_left_hadamard_fold_row_quant_bit_exact(rows, cols, hbl):
    """(H E_Y)_Q of level 2: left-hand rotation over tokens, saved weight scales folded in, per-row quantiser."""
    e = inputs.make_errors(rows, cols, rows + cols)
    fold = (np.abs(np.random.default_rng(1).standard_normal(cols)) * 1e-2 + 1e-4).astype(np.float32)
    q, s = binding.halo_hadamard_quant(gu.bits_to_dev(e), had_block_left=hbl, fold=gu.to_dev(fold))
    wq, ws = oracle_row_quant(orc.bf16_bits_to_real(e), 0, hbl, fold)
    gu.assert_codes_equal(q, wq, "codes"); gu.assert_f32_identical(s, ws, "scales")


COLT_CASES = [(256, 384), (128, 128), (130, 200), (2048, 1024), (16, 4096), (1000, 24)]


@pytest.mark.parametrize("rows,cols", COLT_CASES)
def test_col_quant_transposed_bit_exact(rows, cols):
    """(E_Y^T)_Q with the saved activation scales folded in: one scale per column, transposed codes."""
    e = inputs.make_errors(rows, cols, rows * 3 + cols)
    fold = (np.abs(np.random.default_rng(2).standard_normal(rows)) * 0.5 + 0.01).astype(np.float32)
    ld = (cols + 7) // 8 * 8
    x = torch.zeros((rows, ld), dtype=torch.bfloat16, device=gu.DEV)
    x[:, :cols] = gu.bits_to_dev(e)
    ldq = (rows + 15) // 16 * 16
    out_q = torch.full((cols, ldq), 77, dtype=torch.int8, device=gu.DEV)
    q, s = binding.halo_hadamard_quant(x[:, :cols], axis=binding.HALO_QUANT_COLS_T, fold=gu.to_dev(fold),
                                       out_q=out_q[:, :rows])
    et = np.ascontiguousarray((orc.bf16_bits_to_real(e) * fold[:, None]).T)
    wq, ws = orc.quantize_rows(et)
    gu.assert_codes_equal(q, wq, "codes"); gu.assert_f32_identical(s, ws, "scales")
    if ldq > rows:
        assert torch.all(out_q[:, rows:] == 77)
    # and without fold, including an all-zero column
    e2 = e.copy(); e2[:, 3] = 0
    q, s = binding.halo_hadamard_quant(gu.bits_to_dev(e2), axis=binding.HALO_QUANT_COLS_T)
    wq, ws = orc.quantize_rows(np.ascontiguousarray(orc.bf16_bits_to_real(e2).T))
    gu.assert_codes_equal(q, wq, "codes (no fold)"); gu.assert_f32_identical(s, ws, "scales (no fold)")


@pytest.mark.parametrize("rows,cols", [(256, 512), (128, 256), (130, 200), (2048, 1024), (48, 4096), (1000, 24)])
def test_quant_dual_matches_both_single_quantisers(rows, cols):
    """One tiling of E gives (E_Y)_Q (weight scales folded per column) and (E_Y^T)_Q (activation scales per row)."""
    e = inputs.make_errors(rows, cols, rows + 7 * cols)
    fc = (np.abs(np.random.default_rng(3).standard_normal(cols)) * 1e-2 + 1e-4).astype(np.float32)
    fr = (np.abs(np.random.default_rng(4).standard_normal(rows)) * 0.5 + 0.01).astype(np.float32)
    e[:, 1] = 0                      # an all-zero column
    if rows > 5:
        e[5, :] = 0                  # and an all-zero row
    ld = (cols + 7) // 8 * 8
    x = torch.zeros((rows, ld), dtype=torch.bfloat16, device=gu.DEV)
    x[:, :cols] = gu.bits_to_dev(e)
    q, rs, qt, cs = binding.halo_quant_dual(x[:, :cols], fold_cols=gu.to_dev(fc), fold_rows=gu.to_dev(fr))
    er = orc.bf16_bits_to_real(e)
    wq, ws = orc.quantize_rows(er * fc[None, :])
    wqt, wst = orc.quantize_rows(np.ascontiguousarray((er * fr[:, None]).T))
    gu.assert_codes_equal(q, wq, "row codes"); gu.assert_f32_identical(rs, ws, "row scales")
    gu.assert_codes_equal(qt, wqt, "column codes"); gu.assert_f32_identical(cs, wst, "column scales")
    # no folds at all
    q, rs, qt, cs = binding.halo_quant_dual(x[:, :cols])
    wq, ws = orc.quantize_rows(er)
    wqt, wst = orc.quantize_rows(np.ascontiguousarray(er.T))
    gu.assert_codes_equal(q, wq, "row codes (no fold)"); gu.assert_f32_identical(rs, ws, "row scales (no fold)")
    gu.assert_codes_equal(qt, wqt, "column codes (no fold)"); gu.assert_f32_identical(cs, wst, "column scales (no fold)")


UNROT_CASES = [(64, 512, 512, 0), (33, 4096, 4096, 0), (8, 14336, 2048, 0), (256, 1024, 1024, 256),
               (4096, 256, 256, 4096), (50, 96, 0, 0), (2048, 512, 0, 2048)]


@pytest.mark.parametrize("rows,cols,hb,hbl", UNROT_CASES)
@pytest.mark.parametrize("odt", [torch.float32, torch.bfloat16])
def test_dequant_unrotate(rows, cols, hb, hbl, odt):
    rng = np.random.default_rng(rows + cols)
    acc = rng.integers(-(1 << 27), 1 << 27, size=(rows, cols), dtype=np.int32)
    scale = (np.abs(rng.standard_normal(rows)) * 1e-6 + 1e-8).astype(np.float32)
    out = binding.halo_dequant_unrotate(gu.to_dev(acc), gu.to_dev(scale), had_block=hb, had_block_left=hbl, out_dtype=odt)
    T = orc.dequantize(acc, scale)
    T = orc.fwht(T, hbl, 0) if hbl else T          # the left-hand un-rotation comes first (as in the oracle's level 2)
    T = orc.fwht(T, hb, 1)
    if odt == torch.float32:
        gu.assert_f32_identical(out, T, "unrotated fp32 (same stage order => same bits)")
    else:
        gu.assert_bf16_within_one_ulp(out, T, "unrotated bf16")


def test_bf16_outputs_round_to_nearest_even_exactly():
    """bf16 stores go through the hardware conversion: integers that lie exactly between two bf16 values (and random
    ones) must come out as the oracle's round-to-nearest-even, bit for bit."""
    rng = np.random.default_rng(12)
    ties = np.array([257, 259, 261, 263, 513 * 2, 515 * 2, -257, -259, (1 << 16) + 128, (1 << 16) + 384, 3, 0, -1, 1 << 23],
                    dtype=np.int32)
    acc = rng.integers(-(1 << 24), 1 << 24, size=(64, 512), dtype=np.int32)
    acc[0, :ties.size] = ties
    acc[1] = (rng.integers(1, 1 << 15, size=512) * 2 + 1).astype(np.int32) << 7      # odd multiples of 128: all ties
    out = binding.halo_dequant_unrotate(gu.to_dev(acc), None, had_block=0, out_dtype=torch.bfloat16)
    want = orc.real_to_bf16_bits(acc.astype(np.float32))
    got = gu.dev_bf16_to_bits(out[:, :512].contiguous())
    assert np.array_equal(got, want), int(np.sum(got != want))


def test_repeatability_same_bits_twice():
    bits = inputs.make_activations(300, 4096, 0.001, 9)
    x = gu.bits_to_dev(bits)
    q1, s1 = binding.halo_hadamard_quant(x, had_block=4096)
    q2, s2 = binding.halo_hadamard_quant(x, had_block=4096)
    assert torch.equal(q1, q2) and torch.equal(s1, s2)


def test_repeatability_dual_and_left_quantisers_at_config_sizes():
    """Config c2's E through the dual quantiser and config c3's E through the left-rotating quantiser, twice each:
    same bits both times, and the oracle's bits (full size)."""
    b, n = 2048, 4096
    e = inputs.make_errors(b, n, 0)
    fc = (np.abs(np.random.default_rng(5).standard_normal(n)) * 1e-2 + 1e-4).astype(np.float32)
    fr = (np.abs(np.random.default_rng(6).standard_normal(b)) * 0.5 + 0.01).astype(np.float32)
    E, dfc, dfr = gu.bits_to_dev(e), gu.to_dev(fc), gu.to_dev(fr)
    r1 = binding.halo_quant_dual(E, fold_cols=dfc, fold_rows=dfr)
    r2 = binding.halo_quant_dual(E, fold_cols=dfc, fold_rows=dfr)
    assert all(torch.equal(x, y) for x, y in zip(r1, r2)), "two runs of the dual quantiser differ"
    er = orc.bf16_bits_to_real(e)
    wq, ws = orc.quantize_rows(er * fc[None, :])
    wqt, wst = orc.quantize_rows(np.ascontiguousarray((er * fr[:, None]).T))
    gu.assert_codes_equal(r1[0], wq, "row codes"); gu.assert_f32_identical(r1[1], ws, "row scales")
    gu.assert_codes_equal(r1[2], wqt, "column codes"); gu.assert_f32_identical(r1[3], wst, "column scales")
    b = 4096
    e = inputs.make_errors(b, n, 1)
    E = gu.bits_to_dev(e)
    q1, s1 = binding.halo_hadamard_quant(E, had_block_left=b, fold=dfc)
    q2, s2 = binding.halo_hadamard_quant(E, had_block_left=b, fold=dfc)
    assert torch.equal(q1, q2) and torch.equal(s1, s2), "two runs of the left-rotating quantiser differ"
    wq, ws = oracle_row_quant(orc.bf16_bits_to_real(e), 0, b, fc)
    gu.assert_codes_equal(q1, wq, "left-rotated codes"); gu.assert_f32_identical(s1, ws, "left-rotated scales")
