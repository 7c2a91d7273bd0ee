"""GPU parity of the one-scale-per-tensor mode (the paper's own quantiser, Section 4 setup) against the oracle's
per_tensor=True formulas, through the C ABI: codes, scales, accumulator-derived fp32 outputs bit for bit."""
import numpy as np
import pytest
import torch

from oracle import halo_oracle as orc
from paper_2501_02625_amd import binding, inputs
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("rows,cols,hb,hbl", [(128, 512, 512, 0), (37, 4096, 4096, 0), (5, 14336, 2048, 0), (70, 1000, 0, 0),
                                              (256, 192, 0, 256), (2048, 256, 256, 512)])
def test_tensor_quantiser_rows_bit_exact(rows, cols, hb, hbl):
    bits = inputs.make_activations(rows, (cols + 7) // 8 * 8, 0.01, rows + cols)[:, :cols]
    x = torch.zeros((rows, (cols + 7) // 8 * 8), dtype=torch.bfloat16, device=gu.DEV)
    x[:, :cols] = gu.bits_to_dev(np.ascontiguousarray(bits))
    q, s = binding.halo_hadamard_quant_tensor(x[:, :cols], had_block=hb, had_block_left=hbl)
    v = orc.bf16_bits_to_real(np.ascontiguousarray(bits))
    if hbl:
        v = orc.fwht(v, hbl, 0)
    wq, ws = orc.quantize_tensor(orc.fwht(v, hb, 1))
    gu.assert_codes_equal(q, wq, "codes"); gu.assert_f32_identical(s, ws, "scales")


def test_tensor_quantiser_transposed_and_zero_tensor():
    e = inputs.make_errors(200, 136, 5)
    q, s = binding.halo_hadamard_quant_tensor(gu.bits_to_dev(e), axis=binding.HALO_QUANT_COLS_T)
    wq, ws = orc.quantize_tensor(np.ascontiguousarray(orc.bf16_bits_to_real(e).T))
    gu.assert_codes_equal(q, wq, "transposed codes"); gu.assert_f32_identical(s, ws, "transposed scales")
    z = torch.zeros((16, 64), dtype=torch.bfloat16, device=gu.DEV)
    q, s = binding.halo_hadamard_quant_tensor(z, had_block=64)
    assert not q.any() and torch.all(s == 1.0)


def run_per_tensor(b, m, n, level, seed, odt=torch.float32):
    Xb = inputs.make_activations(b, m, 0.01, seed); Wb = inputs.make_weights(n, m, seed); Eb = inputs.make_errors(b, n, seed)
    hm, hb = min(m & -m, 4096), b & -b
    desc = binding.make_desc(b, m, n, level, odt, scale_mode=binding.HALO_SCALE_PER_TENSOR)
    Y, st = binding.halo_linear_fwd(desc, gu.bits_to_dev(Xb), gu.bits_to_dev(Wb))
    f = orc.forward(orc.bf16_bits_to_real(Xb), orc.bf16_bits_to_real(Wb), level, hm, per_tensor=True)
    gu.assert_codes_equal(st.Xq, f["Xq"], "Xq"); gu.assert_f32_identical(st.s_x, f["s_x"], "s_x")
    gu.assert_codes_equal(st.Wq, f["Wq"], "Wq"); gu.assert_f32_identical(st.s_w, f["s_w"], "s_w")
    cmp = gu.assert_f32_identical if odt == torch.float32 else gu.assert_bf16_within_one_ulp
    cmp(Y, f["Y"], "Y")
    EX, G = binding.halo_linear_bwd(desc, gu.bits_to_dev(Eb), st)
    Er = orc.bf16_bits_to_real(Eb)
    cmp(EX, orc.backward_input(Er, f["Wq"], f["s_w"], level, hm, hb, per_tensor=True)["EX"], "E_X")
    cmp(G, orc.backward_weight(Er, f["Xq"], f["s_x"], level, hm, per_tensor=True)["G"], "G")
    return Y, EX, G


@pytest.mark.parametrize("b,m,n", [(64, 128, 96), (256, 1024, 512), (144, 1536, 272)])
@pytest.mark.parametrize("level", [0, 1, 2])
def test_per_tensor_layers_all_levels(b, m, n, level):
    run_per_tensor(b, m, n, level, b + m + n)


def test_config_c7_full_size_per_tensor():
    """Config c7: the shape of c2 (tokens 2048, 4096 x 4096, HALO-1) with one scale per tensor, compared in full; and a
    level-2 layer large enough for the product's epilogue to run the low left-hand strides with the tensor scale."""
    cfg = inputs.CONFIGS["c7"]
    assert cfg.per_tensor
    run_per_tensor(cfg.tokens, 4096, 4096, cfg.level, cfg.seed * 1000)
    run_per_tensor(1024, 2048, 512, 2, 11)


def test_per_tensor_bf16_and_quantisation_error_of_both_modes_on_config_c1():
    """bf16 outputs; and on config c1's data (plus a heavy-tailed E) the error of each mode against the fp64 products:
    the per-row mode must be the more accurate one for the backward product fed by outlier-laden errors."""
    run_per_tensor(256, 512, 384, 2, 3, odt=torch.bfloat16)
    cfg = inputs.CONFIGS["c1"]
    t = inputs.make_linear_inputs(cfg, need_error=True)
    b, m, n = 128, 512, 512
    ref = orc.plain_products(*(orc.bf16_bits_to_real(t[k]) for k in ("X", "W", "E")))
    err = {}
    for mode in (binding.HALO_SCALE_PER_ROW, binding.HALO_SCALE_PER_TENSOR):
        desc = binding.make_desc(b, m, n, 1, torch.float32, scale_mode=mode)
        Y, st = binding.halo_linear_fwd(desc, gu.bits_to_dev(t["X"]), gu.bits_to_dev(t["W"]))
        EX, G = binding.halo_linear_bwd(desc, gu.bits_to_dev(t["E"]), st)
        rel = lambda got, want: float(np.linalg.norm(got.cpu().numpy().astype(np.float64) - want) / np.linalg.norm(want))
        err[mode] = (rel(Y, ref["Y"]), rel(EX, ref["EX"]), rel(G, ref["G"]))
    print("relative error (Y, E_X, G): per-row %s, per-tensor %s" % (err[0], err[1]))
    assert 2 * err[0][1] < err[1][1] and all(e < 0.1 for e in err[0]) and all(e < 0.5 for e in err[1])
