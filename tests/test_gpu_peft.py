"""GPU parity of the HALO-PEFT module (halo_peft_fwd / halo_peft_bwd) against the CPU oracle, through the C ABI.

The quantised branch keeps the bars of the plain layer (with a zero adapter the outputs are bit-identical to the
oracle's).  The low-rank branch is floating point accumulated in fp32 in an order the hardware picks, against exact
products in the oracle, so it is compared within bounds derived from the arithmetic, u = 2^-24:
  T = X U^T, S = E V          |err| <= (16 + K/16) u (|X| |U|^T)          K = m resp. n (one matrix instruction per 32 terms)
  G_V, G_U                    |err| <= (32 + b/4) u (|E|^T |T|) ...        (a generous count: one rounding per 4 tokens)
  Y                           |err| <= (32 + m/16) u (|Y_q| + (|X||U|^T)|V|^T)
  E_X                         the same with n, plus 64 u (max|E_X,q| + max|S U|): the low-rank term is added before the
                              un-rotation, whose fp32 roundings then act on the sum
bf16 outputs: within one bf16 ulp of the rounded oracle value (or inside the fp32 bound), at most 2 % off by that ulp."""
import numpy as np
import pytest
import torch

from oracle import halo_oracle as orc
from paper_2501_02625_amd import binding, inputs
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

U32 = 2.0 ** -24


def assert_within(got, want, bound, what):
    g = got.float().cpu().numpy().astype(np.float64)
    assert g.shape == want.shape, (what, g.shape, want.shape)
    err = np.abs(g - want)
    bad = err > bound
    if np.any(bad):
        i = tuple(np.argwhere(bad)[0])
        raise AssertionError("%s: %d of %d outside the bound; first at %s: got %r want %r bound %r"
                             % (what, int(bad.sum()), want.size, i, g[i], want[i], bound[i] if np.ndim(bound) else bound))


def assert_bf16_close(got, want, bound, what):
    """Within one bf16 ulp of the rounded oracle value or inside the fp32 bound; few are off at all."""
    gb = gu.dev_bf16_to_bits(got).astype(np.int32)
    wb = orc.real_to_bf16_bits(want.astype(np.float32)).astype(np.int32)
    key = lambda b: np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    d = np.abs(key(gb) - key(wb))
    g = orc.bf16_bits_to_real(gb.astype(np.uint16)).astype(np.float64)
    ok = (d <= 1) | (np.abs(g - want) <= bound)
    assert ok.all(), (what, int((~ok).sum()), int(d.max()))
    assert (d != 0).mean() <= 0.02, (what, float((d != 0).mean()))


def frozen_weight(Wb, hm):
    W = gu.bits_to_dev(Wb)
    Wq, s_w = binding.halo_hadamard_quant(W, had_block=hm)
    return Wq, s_w


def run_peft(b, m, n, rank, level, seed, odt=torch.float32, hm=0, hb=0, zero_v=False, tensors=None):
    hm_eff = (hm or min(m & -m, 4096)) if level >= 1 else 0
    hb_eff = (hb or (b & -b)) if level >= 2 else 0
    if tensors is None:
        Xb = inputs.make_activations(b, m, 0.002, seed)
        Wb = inputs.make_weights(n, m, seed)
        Eb = inputs.make_errors(b, n, seed)
        Ub, Vb = inputs.make_adapters(rank, n, m, seed)
    else:
        Xb, Wb, Eb, Ub, Vb = tensors
    if zero_v:
        Vb = np.zeros_like(Vb)
    Xr, Wr, Er, Ur, Vr = (orc.bf16_bits_to_real(a) for a in (Xb, Wb, Eb, Ub, Vb))
    base = orc.forward(np.zeros((16, m), np.float32), Wr, level, hm_eff)      # the frozen (WH)_Q, made once
    desc = binding.make_desc(b, m, n, level, odt, hm_eff, hb_eff)
    X, E, U, V = (gu.bits_to_dev(a) for a in (Xb, Eb, Ub, Vb))
    Wq, s_w = frozen_weight(Wb, hm_eff)
    gu.assert_codes_equal(Wq, base["Wq"], "frozen Wq"); gu.assert_f32_identical(s_w, base["s_w"], "frozen s_w")

    ws = torch.empty((binding.halo_peft_workspace_bytes(desc, rank),), dtype=torch.uint8, device=gu.DEV)
    Y, T = binding.halo_peft_fwd(desc, X, Wq, s_w, U, V, workspace=ws)
    EX, GU, GV = binding.halo_peft_bwd(desc, E, X, T, Wq, s_w, U, V, workspace=ws)
    torch.cuda.synchronize()

    f = orc.peft_forward(Xr, base["Wq"], base["s_w"], Ur, Vr, level, hm_eff)
    bw = orc.peft_backward(Er, Xr, base["Wq"], base["s_w"], Ur, Vr, level, hm_eff, hb_eff)
    aX, aU, aV, aE = (np.abs(a).astype(np.float64) for a in (Xr, Ur, Vr, Er))
    BT = aX @ aU.T
    BS = aE @ aV
    assert_within(T, f["T"], (16 + m / 16) * U32 * BT, "T")
    assert_within(GV, bw["GV"], (32 + b / 4) * U32 * (aE.T @ BT), "G_V")
    assert_within(GU, bw["GU"], (32 + b / 4 + n / 16) * U32 * (BS.T @ aX), "G_U")
    Yq = f["Y"] - f["T"] @ Vr.astype(np.float64).T
    EXq = bw["EX"] - bw["S"] @ Ur.astype(np.float64)
    bound_y = (32 + m / 16) * U32 * (np.abs(Yq) + BT @ aV.T)
    lr_ex = bw["S"] @ Ur.astype(np.float64)
    bound_ex = (32 + n / 16) * U32 * (np.abs(EXq) + BS @ aU) + 64 * U32 * (np.abs(EXq).max() + np.abs(lr_ex).max())
    if zero_v:
        # LoRA's initial state: the low-rank term is exactly zero and the outputs are those of the plain layer
        cmp = gu.assert_f32_identical if odt == torch.float32 else gu.assert_bf16_within_one_ulp
        cmp(Y, f["Y"].astype(np.float32), "Y with V = 0")
        cmp(EX, bw["EX"].astype(np.float32), "E_X with V = 0")
        assert not torch.any(GU)
    elif odt == torch.float32:
        assert_within(Y, f["Y"], bound_y, "Y")
        assert_within(EX, bw["EX"], bound_ex, "E_X")
    else:
        assert_bf16_close(Y, f["Y"], bound_y, "Y")
        assert_bf16_close(EX, bw["EX"], bound_ex, "E_X")
    # the low-rank term is really there: far outside the bound without it
    if not zero_v and odt == torch.float32:
        assert np.mean(np.abs(Yq - f["Y"]) > 4 * bound_y) > 0.5
        assert np.mean(np.abs(EXq - bw["EX"]) > 4 * bound_ex) > 0.5
    return dict(Y=Y, T=T, EX=EX, GU=GU, GV=GV, args=(desc, X, E, U, V, Wq, s_w, ws))


# (tokens, in-features, out-features, rank, level, right block, left block)
SHAPES = [
    (128, 512, 512, 16, 2, 0, 0),          # 128x128 tiles; left block 128: plain epilogue, all left strides afterwards
    (512, 1024, 768, 8, 2, 0, 0),          # rank 8; left block 512: low strides in the epilogue
    (768, 512, 1024, 16, 2, 512, 256),     # left block 256 = the tile: nothing left for the strided passes
    (272, 640, 448, 32, 1, 128, 0),        # ragged row tile, rank 32, block-diagonal rotation
    (304, 576, 320, 64, 0, 0, 0),          # level 0 (no rotation), rank 64, product stored straight from the epilogue
    (96, 192, 64, 24, 2, 64, 32),          # rank 24 (a masked half tile), small blocks
    (256, 1792, 256, 16, 2, 1792, 256),    # Kronecker rotation H_64 (x) H_28
    (2048, 4096, 4096, 16, 2, 0, 0),       # 256x128 forward tiles, 256x256 backward tiles, four top left strides
    (32768, 64, 64, 8, 2, 64, 32768),      # left block too long for the small rotation kernel: strided passes for H S
    (512, 14336, 128, 16, 2, 14336, 512),  # one Kronecker block H_512 (x) H_28 over 14336
    (1024, 2048, 192, 64, 2, 2048, 1024),  # rank 64 (four rank tiles), right block 2048
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_peft_module_fp32_outputs(shape):
    b, m, n, rank, level, hm, hb = shape
    run_peft(b, m, n, rank, level, seed=b + rank, hm=hm, hb=hb)


@pytest.mark.parametrize("shape", [SHAPES[1], SHAPES[3], SHAPES[4]], ids=lambda s: "x".join(map(str, s)))
def test_peft_module_bf16_outputs(shape):
    b, m, n, rank, level, hm, hb = shape
    run_peft(b, m, n, rank, level, seed=7 * b + rank, odt=torch.bfloat16, hm=hm, hb=hb)


@pytest.mark.parametrize("shape,odt", [(SHAPES[1], torch.float32), (SHAPES[2], torch.bfloat16), (SHAPES[3], torch.float32),
                                       (SHAPES[4], torch.float32)], ids=lambda s: str(s).replace(" ", ""))
def test_zero_adapter_is_the_plain_layer(shape, odt):
    b, m, n, rank, level, hm, hb = shape
    run_peft(b, m, n, rank, level, seed=3 * b, odt=odt, hm=hm, hb=hb, zero_v=True)


def test_repeat_calls_are_identical_and_partial_outputs_match():
    b, m, n, rank, level, hm, hb = SHAPES[1]
    r = run_peft(b, m, n, rank, level, seed=11, hm=hm, hb=hb)
    desc, X, E, U, V, Wq, s_w, ws = r["args"]
    ws.fill_(0x5A)                                       # nothing in the workspace is carried between calls
    Y2, T2 = binding.halo_peft_fwd(desc, X, Wq, s_w, U, V, workspace=ws)
    EX2, GU2, GV2 = binding.halo_peft_bwd(desc, E, X, T2, Wq, s_w, U, V, workspace=ws)
    for a, c, what in ((r["Y"], Y2, "Y"), (r["T"], T2, "T"), (r["EX"], EX2, "E_X"), (r["GU"], GU2, "G_U"), (r["GV"], GV2, "G_V")):
        assert torch.equal(a, c), what
    ex_only, none_u, none_v = binding.halo_peft_bwd(desc, E, X, T2, Wq, s_w, U, V, want_gu=False, want_gv=False, workspace=ws)
    assert none_u is None and none_v is None and torch.equal(ex_only, EX2)
    _, gu_only, gv_only = binding.halo_peft_bwd(desc, E, X, T2, Wq, s_w, U, V, want_ex=False, workspace=ws)
    assert torch.equal(gu_only, GU2) and torch.equal(gv_only, GV2)


def test_config_c8_full_size():
    """Config c8 at full size (4096 tokens, 4096 x 4096, rank 16, level 2, bf16 outputs), every output element."""
    cfg = inputs.CONFIGS["c8"]
    lin = cfg.linears[0]
    t = inputs.make_linear_inputs(cfg)
    run_peft(cfg.tokens, lin.m, lin.n, cfg.peft_rank, cfg.level, seed=0, odt=torch.bfloat16,
             hm=cfg.had_block_m(lin.m), hb=cfg.had_block_b(), tensors=(t["X"], t["W"], t["E"], t["U"], t["V"]))
