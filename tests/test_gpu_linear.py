"""GPU parity of the whole layer (halo_linear_fwd / halo_linear_bwd) against the CPU oracle, through the C ABI.

Bars: saved INT8 codes, fp32 scales and int32 accumulators bit-exact; fp32 outputs bit-identical to the oracle's
(well inside the 1e-3 relative bar the build target states); bf16 outputs within one bf16 ulp of the rounded
oracle value."""
import numpy as np
import pytest
import torch

from oracle import halo_oracle as orc
from paper_2501_02625_amd import binding, inputs
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def check_internals(b, m, n, level, hb_eff, E, st, f, ex, g):
    """The intermediate tensors of the layer at this size, through the entry points the layer itself uses:
    forward accumulators, both quantisations of E, both backward accumulators (one paired launch)."""
    _, acc = binding.halo_gemm_i8(st.Xq, st.Wq, trans_b=True, out_dtype=None, want_acc=True)
    gu.assert_codes_equal(acc, f["acc"], "forward accumulators")
    del acc
    if level <= 1:
        Eq, s_e, EqT, s_g = binding.halo_quant_dual(E, fold_cols=st.s_w, fold_rows=st.s_x)
    else:
        Eq, s_e = binding.halo_hadamard_quant(E, had_block_left=hb_eff, fold=st.s_w)
        EqT, s_g = binding.halo_hadamard_quant(E, axis=binding.HALO_QUANT_COLS_T, fold=st.s_x)
    gu.assert_codes_equal(Eq, ex["Eq"], "Eq"); gu.assert_f32_identical(s_e, ex["s_e"], "s_e")
    gu.assert_codes_equal(EqT, g["EqT"], "EqT"); gu.assert_f32_identical(s_g, g["s_g"], "s_g")
    acc_x = torch.empty((b, m), dtype=torch.int32, device=gu.DEV)
    acc_g = torch.empty((n, m), dtype=torch.int32, device=gu.DEV)
    binding.halo_gemm_i8_pair(binding.gemm_desc(Eq, st.Wq, trans_b=False, acc_out=acc_x),
                              binding.gemm_desc(EqT, st.Xq, trans_b=False, acc_out=acc_g))
    gu.assert_codes_equal(acc_x, ex["acc"], "E_X accumulators")
    gu.assert_codes_equal(acc_g, g["acc"], "G accumulators")


def run_and_check(b, m, n, level, Xb, Wb, Eb, odt=torch.float32, hm=0, hb=0, state=None, check_fwd=True,
                  internals=False):
    """Saved codes and scales bit-exact; fp32 outputs bit-identical to the oracle's (the kernels keep its stage
    order and its order of multiplications; +0 and -0 compare equal); bf16 outputs within one bf16 ulp."""
    desc = binding.make_desc(b, m, n, level, odt, hm, hb)
    hm_eff = hm or min(m & -m, 4096)
    hb_eff = hb or (b & -b)
    X, W = gu.bits_to_dev(Xb), gu.bits_to_dev(Wb)
    Y, st = binding.halo_linear_fwd(desc, X, W, state=state)
    f = orc.forward(orc.bf16_bits_to_real(Xb), orc.bf16_bits_to_real(Wb), level, hm_eff)
    gu.assert_codes_equal(st.Xq, f["Xq"], "Xq"); gu.assert_f32_identical(st.s_x, f["s_x"], "s_x")
    gu.assert_codes_equal(st.Wq, f["Wq"], "Wq"); gu.assert_f32_identical(st.s_w, f["s_w"], "s_w")
    cmp = gu.assert_f32_identical if odt == torch.float32 else gu.assert_bf16_within_one_ulp
    if check_fwd:
        cmp(Y, f["Y"], "Y")
    if Eb is None:
        return st
    E = gu.bits_to_dev(Eb)
    EX, G = binding.halo_linear_bwd(desc, E, st)
    Er = orc.bf16_bits_to_real(Eb)
    ex = orc.backward_input(Er, f["Wq"], f["s_w"], level, hm_eff, hb_eff)
    cmp(EX, ex["EX"], "E_X")
    ex.pop("EX"); del EX
    g = orc.backward_weight(Er, f["Xq"], f["s_x"], level, hm_eff)
    cmp(G, g["G"], "G")
    g.pop("G"); del G
    if internals:
        check_internals(b, m, n, level, hb_eff, E, st, f, ex, g)
    return st


def test_config_c1_forward_with_and_without_rotation():
    """Config c1: X 128x512 with outlier channels, W 512x512; forward with the 512-point rotation
    (levels 1/2 share it) and the true level 0 (no rotation)."""
    cfg = inputs.CONFIGS["c1"]
    t = inputs.make_linear_inputs(cfg)
    ref = orc.plain_products(orc.bf16_bits_to_real(t["X"]), orc.bf16_bits_to_real(t["W"]), None)["Y"]
    errs = {}
    for level in (1, 0):
        run_and_check(128, 512, 512, level, t["X"], t["W"], None)
        desc = binding.make_desc(128, 512, 512, level, torch.float32)
        Y, _ = binding.halo_linear_fwd(desc, gu.bits_to_dev(t["X"]), gu.bits_to_dev(t["W"]))
        errs[level] = np.linalg.norm(Y.cpu().numpy() - ref) / np.linalg.norm(ref)
    assert errs[1] < 0.02 and errs[0] > 3 * errs[1]


SMALL = [
    # b, m, n
    (64, 128, 96),
    (256, 1024, 512),
    (144, 1536, 272),      # m = 3 x 512 blocks, b and n not powers of two
    (512, 512, 2048),
]


@pytest.mark.parametrize("b,m,n", SMALL)
@pytest.mark.parametrize("level", [0, 1, 2])
def test_small_layers_all_levels(b, m, n, level):
    seed = b + m + n
    Xb = inputs.make_activations(b, m, 0.01, seed)
    Wb = inputs.make_weights(n, m, seed)
    Eb = inputs.make_errors(b, n, seed)
    run_and_check(b, m, n, level, Xb, Wb, Eb)


@pytest.mark.parametrize("b,m,n,hm,hb,odt", [
    (1024, 1024, 256, 0, 0, torch.float32),        # left block 1024: two top strides after the epilogue's eight; right block 1024
    (2048, 2048, 128, 0, 0, torch.bfloat16),       # three top strides, right block 2048
    (4096, 512, 64, 0, 0, torch.float32),          # four top strides, right block 512
    (1024, 1536, 192, 512, 512, torch.float32),    # two left blocks of 512 (one top stride), three right blocks of 512
    (8192, 512, 64, 0, 0, torch.float32),          # left block 8192: five strides left, two rows per wavefront
    (8192, 2048, 64, 0, 0, torch.bfloat16),        # the same with the widest segment that fits (2048)
    (16384, 1024, 64, 0, 8192, torch.float32),     # two left blocks of 8192
    (8192, 4096, 64, 0, 0, torch.float32),         # five strides and a 4096 block: the strided pass takes them
    (768, 1024, 128, 0, 0, torch.float32),         # b = 3 * 256: left block 256, nothing left after the epilogue
    (512, 4096, 64, 0, 0, torch.float32),          # one top stride, right block 4096 (64 values per lane)
    (4096, 4096, 128, 0, 0, torch.bfloat16),       # four top strides, right block 4096
    (2048, 8192, 64, 4096, 1024, torch.float32),   # two left blocks of 1024, two right blocks of 4096
])
def test_level2_output_side_variants(b, m, n, hm, hb, odt):
    """Level 2 with the low left-hand strides in the product's epilogue: every way the rest of the un-rotation can go."""
    Xb = inputs.make_activations(b, m, 0.01, b + m); Wb = inputs.make_weights(n, m, b + m); Eb = inputs.make_errors(b, n, b + m)
    run_and_check(b, m, n, 2, Xb, Wb, Eb, odt=odt, hm=hm, hb=hb)


def test_bf16_outputs_and_explicit_blocks():
    b, m, n = 256, 1024, 384
    Xb = inputs.make_activations(b, m, 0.01, 1); Wb = inputs.make_weights(n, m, 1); Eb = inputs.make_errors(b, n, 1)
    run_and_check(b, m, n, 2, Xb, Wb, Eb, odt=torch.bfloat16)
    run_and_check(b, m, n, 2, Xb, Wb, Eb, hm=256, hb=64)


def test_backward_skipping_one_product_and_reusing_saved_codes():
    b, m, n = 128, 512, 256
    Xb = inputs.make_activations(b, m, 0.01, 2); Wb = inputs.make_weights(n, m, 2); Eb = inputs.make_errors(b, n, 2)
    st = run_and_check(b, m, n, 1, Xb, Wb, Eb)
    desc = binding.make_desc(b, m, n, 1, torch.float32)
    E = gu.bits_to_dev(Eb)
    EX, G = binding.halo_linear_bwd(desc, E, st)
    EX1, none = binding.halo_linear_bwd(desc, E, st, want_g=False)
    none2, G1 = binding.halo_linear_bwd(desc, E, st, want_ex=False)
    assert none is None and none2 is None and torch.equal(EX, EX1) and torch.equal(G, G1)
    # forward again from the saved codes only (X = W = None): same Y
    Y0, _ = binding.halo_linear_fwd(desc, gu.bits_to_dev(Xb), gu.bits_to_dev(Wb))
    Y1, _ = binding.halo_linear_fwd(desc, None, None, state=st)
    assert torch.equal(Y0, Y1)


def test_config_c2_full_size_level1():
    """Config c2 (the benchmarked workload): tokens 2048, 4096 x 4096, HALO-1, every output compared in full."""
    cfg = inputs.CONFIGS["c2"]
    t = inputs.make_linear_inputs(cfg)
    run_and_check(cfg.tokens, 4096, 4096, cfg.level, t["X"], t["W"], t["E"], odt=torch.float32, internals=True)
    run_and_check(cfg.tokens, 4096, 4096, cfg.level, t["X"], t["W"], t["E"], odt=torch.bfloat16)


def test_config_c3_full_size_level2():
    """Config c3: tokens 4096, K = 14336 = 7 x 2048 block-diagonal, N = 4096, HALO-2, compared in full."""
    cfg = inputs.CONFIGS["c3"]
    t = inputs.make_linear_inputs(cfg)
    run_and_check(cfg.tokens, 14336, 4096, cfg.level, t["X"], t["W"], t["E"], odt=torch.float32, internals=True)


def test_config_c4_decoder_layer_linears_level2():
    """Config c4: the seven linears of a Llama-3-8B-shaped decoder layer at 8192 tokens, HALO-2, bf16 outputs.
    q/k/v and gate/up share one quantised activation (only the first of each group quantises X)."""
    cfg = inputs.CONFIGS["c4"]
    b = cfg.tokens
    x_for = {}
    states = {}
    for idx, lin in enumerate(cfg.linears):
        owner = lin.shares_input_with or lin.name
        if owner not in x_for:
            x_for[owner] = inputs.make_activations(b, lin.m, cfg.outlier_frac, 100 + idx)
        Xb = x_for[owner]
        Wb = inputs.make_weights(lin.n, lin.m, 100 + idx)
        Eb = inputs.make_errors(b, lin.n, 100 + idx)
        desc = binding.make_desc(b, lin.m, lin.n, cfg.level, torch.bfloat16)
        if lin.shares_input_with:
            src = states[owner]
            st = binding.LinearState(src.Xq, src.s_x,
                                     torch.empty((lin.n, lin.m), dtype=torch.int8, device=gu.DEV),
                                     torch.empty((lin.n,), dtype=torch.float32, device=gu.DEV))
            Y, st = binding.halo_linear_fwd(desc, None, gu.bits_to_dev(Wb), state=st)
        else:
            Y, st = binding.halo_linear_fwd(desc, gu.bits_to_dev(Xb), gu.bits_to_dev(Wb))
        states[lin.name] = st
        hm = min(lin.m & -lin.m, 4096)
        f = orc.forward(orc.bf16_bits_to_real(Xb), orc.bf16_bits_to_real(Wb), cfg.level, hm)
        gu.assert_codes_equal(st.Xq, f["Xq"], lin.name + " Xq"); gu.assert_f32_identical(st.s_x, f["s_x"], lin.name + " s_x")
        gu.assert_codes_equal(st.Wq, f["Wq"], lin.name + " Wq"); gu.assert_f32_identical(st.s_w, f["s_w"], lin.name + " s_w")
        gu.assert_bf16_within_one_ulp(Y, f["Y"], lin.name + " Y")
        EX, G = binding.halo_linear_bwd(desc, gu.bits_to_dev(Eb), st)
        Er = orc.bf16_bits_to_real(Eb)
        ex = orc.backward_input(Er, f["Wq"], f["s_w"], cfg.level, hm, b)
        gu.assert_bf16_within_one_ulp(EX, ex["EX"], lin.name + " E_X")
        del ex, EX
        g = orc.backward_weight(Er, f["Xq"], f["s_x"], cfg.level, hm)
        gu.assert_bf16_within_one_ulp(G, g["G"], lin.name + " G")
        del g, G, f
        print("c4 linear %s ok" % lin.name, flush=True)
