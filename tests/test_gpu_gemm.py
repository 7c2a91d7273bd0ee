"""GPU parity: halo_gemm_i8 int32 accumulators bit-exact against the oracle's exact integer product."""
import numpy as np
import pytest
import torch

from oracle import halo_oracle as orc
from paper_2501_02625_amd import binding
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, scope="module")
def forced_config():
    """HALO_TEST_GEMM_CFG=<n> runs this module with one GEMM tile configuration forced (development aid)."""
    import os
    cfg = int(os.environ.get("HALO_TEST_GEMM_CFG", "-1"))
    binding.halo_gemm_i8_set_config(cfg)
    yield
    binding.halo_gemm_i8_set_config(-1)

# M, N, K -- chosen to hit each macro-tile configuration, ragged edges and a K tail
SHAPES = [
    (128, 512, 512),       # config c1 forward
    (32, 32, 16),
    (1, 1, 64),
    (300, 200, 272),       # ragged M, N; K not a multiple of the K step
    (257, 129, 1040),
    (2048, 4096, 256),     # 256x128 tiles
    (4096, 4096, 128),     # 256x256 tiles
    (4100, 3900, 80),      # 256x256 tiles with ragged edges
    (512, 14336, 64),
]


def rand_codes(rng, shape, extreme=False):
    if extreme:
        return rng.choice(np.array([-127, 127], dtype=np.int8), size=shape)
    return rng.integers(-127, 128, size=shape, dtype=np.int8)


@pytest.mark.parametrize("M,N,K", SHAPES)
@pytest.mark.parametrize("trans_b", [True, False])
def test_gemm_accumulators_bit_exact(M, N, K, trans_b):
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    a = rand_codes(rng, (M, K))
    b = rand_codes(rng, (N, K) if trans_b else (K, N))
    ldb = (b.shape[1] + 15) // 16 * 16
    bd = torch.zeros((b.shape[0], ldb), dtype=torch.int8, device=gu.DEV)
    bd[:, :b.shape[1]] = gu.to_dev(b)
    _, acc = binding.halo_gemm_i8(gu.to_dev(a), bd[:, :b.shape[1]], trans_b=trans_b, out_dtype=None, want_acc=True,
                                  acc_out=torch.full((M, (N + 3) // 4 * 4), -7, dtype=torch.int32, device=gu.DEV)[:, :N])
    want = orc.gemm_codes(a, b.T if trans_b else b)
    gu.assert_codes_equal(acc, want, "accumulators")


@pytest.mark.parametrize("trans_b", [True, False])
def test_gemm_extreme_codes_longest_k(trans_b):
    """All +-127 at K = 14336: the largest magnitude the layer can produce, no int32 overflow."""
    rng = np.random.default_rng(5)
    M, N, K = 96, 160, 14336
    a = rand_codes(rng, (M, K), extreme=True)
    b = rand_codes(rng, (N, K) if trans_b else (K, N), extreme=True)
    a[0] = 127
    if trans_b:
        b[0] = 127
    else:
        b[:, 0] = 127
    _, acc = binding.halo_gemm_i8(gu.to_dev(a), gu.to_dev(b), trans_b=trans_b, out_dtype=None, want_acc=True)
    want = orc.gemm_codes(a, b.T if trans_b else b)
    assert want[0, 0] == 127 * 127 * K
    gu.assert_codes_equal(acc, want, "accumulators")


@pytest.mark.parametrize("odt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("trans_b", [True, False])
def test_gemm_scaled_epilogue(odt, trans_b):
    rng = np.random.default_rng(6)
    M, N, K = 200, 328, 512
    a = rand_codes(rng, (M, K)); b = rand_codes(rng, (N, K) if trans_b else (K, N))
    rs = (np.abs(rng.standard_normal(M)) * 1e-2 + 1e-4).astype(np.float32)
    cs = (np.abs(rng.standard_normal(N)) * 1e-3 + 1e-5).astype(np.float32)
    ldc = (N + 7) // 8 * 8
    out = torch.zeros((M, ldc), dtype=odt, device=gu.DEV)
    ldb = (b.shape[1] + 15) // 16 * 16
    bd = torch.zeros((b.shape[0], ldb), dtype=torch.int8, device=gu.DEV)
    bd[:, :b.shape[1]] = gu.to_dev(b)
    bd = bd[:, :b.shape[1]]
    c, acc = binding.halo_gemm_i8(gu.to_dev(a), bd, trans_b=trans_b, row_scale=gu.to_dev(rs),
                                  col_scale=gu.to_dev(cs), out=out[:, :N], want_acc=True)
    want_acc = orc.gemm_codes(a, b.T if trans_b else b)
    want = orc.dequantize(want_acc, rs, cs)
    gu.assert_codes_equal(acc, want_acc, "accumulators")
    if odt == torch.float32:
        gu.assert_f32_identical(c, want, "scaled output")
    else:
        gu.assert_bf16_within_one_ulp(c, want, "scaled bf16 output")
    # row scale only / no scales
    c2, _ = binding.halo_gemm_i8(gu.to_dev(a), bd, trans_b=trans_b, row_scale=gu.to_dev(rs))
    gu.assert_f32_identical(c2, orc.dequantize(want_acc, rs), "row-scaled output")


def test_gemm_k_zero_writes_zeros_and_empty_is_noop():
    a = torch.empty((8, 0), dtype=torch.int8, device=gu.DEV)
    b = torch.empty((8, 0), dtype=torch.int8, device=gu.DEV)
    c, acc = binding.halo_gemm_i8(a, b, trans_b=True, want_acc=True)
    assert not c.any() and not acc.any()
    a = torch.empty((0, 64), dtype=torch.int8, device=gu.DEV)
    b = torch.empty((16, 64), dtype=torch.int8, device=gu.DEV)
    c, _ = binding.halo_gemm_i8(a, b, trans_b=True)
    assert c.shape == (0, 16)


def test_gemm_pair_matches_two_single_launches():
    """Both backward products in one launch give the same bits as two launches (config c2's shapes scaled down,
    ragged edges, one scaled bf16 output and one raw accumulator output)."""
    rng = np.random.default_rng(9)
    b, m, n = 384, 512, 640
    Eq = rand_codes(rng, (b, n)); Wq = rand_codes(rng, (n, m)); EqT = rand_codes(rng, (n, b)); Xq = rand_codes(rng, (b, m))
    s_e = (np.abs(rng.standard_normal(b)) * 1e-3 + 1e-5).astype(np.float32)
    dEq, dWq, dEqT, dXq = map(gu.to_dev, (Eq, Wq, EqT, Xq))
    ex = torch.zeros((b, m), dtype=torch.bfloat16, device=gu.DEV)
    acc_g = torch.zeros((n, m), dtype=torch.int32, device=gu.DEV)
    g1 = binding.gemm_desc(dEq, dWq, trans_b=False, row_scale=gu.to_dev(s_e), out=ex)
    g2 = binding.gemm_desc(dEqT, dXq, trans_b=False, acc_out=acc_g)
    binding.halo_gemm_i8_pair(g1, g2)
    want_ex = orc.dequantize(orc.gemm_codes(Eq, Wq), s_e)
    gu.assert_bf16_within_one_ulp(ex, want_ex, "paired E_X")
    gu.assert_codes_equal(acc_g, orc.gemm_codes(EqT, Xq), "paired G accumulators")
    ex1, _ = binding.halo_gemm_i8(dEq, dWq, trans_b=False, row_scale=gu.to_dev(s_e), out_dtype=torch.bfloat16)
    assert torch.equal(ex.view(torch.int16), ex1.contiguous().view(torch.int16))
    # a pair the shared configuration cannot take (K-contiguous B, ragged K) still works
    a = rand_codes(rng, (70, 80)); bb = rand_codes(rng, (50, 80))
    acc1 = torch.zeros((70, 52), dtype=torch.int32, device=gu.DEV)[:, :50]
    acc2 = torch.zeros((n, m), dtype=torch.int32, device=gu.DEV)
    binding.halo_gemm_i8_pair(binding.gemm_desc(gu.to_dev(a), gu.to_dev(bb), trans_b=True, acc_out=acc1),
                              binding.gemm_desc(dEqT, dXq, trans_b=False, acc_out=acc2))
    gu.assert_codes_equal(acc1, orc.gemm_codes(a, bb.T), "fallback pair, first")
    gu.assert_codes_equal(acc2, orc.gemm_codes(EqT, Xq), "fallback pair, second")
