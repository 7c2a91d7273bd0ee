"""GPU parity: halo_gemm_i8 int32 accumulators bit-exact against the oracle's exact integer product."""
import numpy as np
import pytest
import torch

from oracle import halo_oracle as orc
from paper_2501_02625_amd import binding
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


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


# Every tile configuration on shapes its K step divides (ragged M and N, several trips through the ring), through
# halo_gemm_i8_desc: the configurations differ in speed only.
@pytest.mark.parametrize("name", sorted(binding.HALO_GEMM_CONFIGS))
@pytest.mark.parametrize("trans_b", [True, False])
def test_every_tile_configuration_gives_the_same_accumulators(name, trans_b):
    cfg = binding.HALO_GEMM_CONFIGS[name]
    rng = np.random.default_rng(cfg + 10 * int(trans_b))
    M, N, K = 600, 520, 1024 + (16 if name.startswith("staged") else 0)
    a = rand_codes(rng, (M, K))
    b = rand_codes(rng, (N, K) if trans_b else (K, N))
    ldb = (b.shape[1] + 15) // 16 * 16
    bd = torch.zeros((b.shape[0], ldb), dtype=torch.int8, device=gu.DEV)
    bd[:, :b.shape[1]] = gu.to_dev(b)
    acc = torch.full((M, N), -7, dtype=torch.int32, device=gu.DEV)
    binding.halo_gemm_i8_desc(binding.gemm_desc(gu.to_dev(a), bd[:, :b.shape[1]], trans_b=trans_b, acc_out=acc, config=cfg))
    gu.assert_codes_equal(acc, orc.gemm_codes(a, b.T if trans_b else b), "accumulators, configuration " + name)


def test_tile_configuration_argument_errors():
    a = torch.zeros((64, 80), dtype=torch.int8, device=gu.DEV)
    b = torch.zeros((64, 80), dtype=torch.int8, device=gu.DEV)
    acc = torch.zeros((64, 64), dtype=torch.int32, device=gu.DEV)
    with pytest.raises(binding.HaloError) as e:       # K = 80 is not a multiple of the 64-byte K step
        binding.halo_gemm_i8_desc(binding.gemm_desc(a, b, trans_b=True, acc_out=acc, config=0))
    assert e.value.status == binding.HALO_ESHAPE
    with pytest.raises(binding.HaloError) as e:
        binding.halo_gemm_i8_desc(binding.gemm_desc(a, b, trans_b=True, acc_out=acc, config=9))
    assert e.value.status == binding.HALO_EINVAL
    binding.halo_gemm_i8_desc(binding.gemm_desc(a, b, trans_b=True, acc_out=acc, config=4))


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


# Full-size products of configs c2 and c3 in the tile configuration the library picks for them: the steady state of
# the global->LDS ring (64..224 trips) on the large macro tiles.  Each runs twice into separate buffers: same bits
# both times, and the oracle's bits.
FULL = [
    ("c2 forward", 2048, 4096, 4096, True),
    ("c3 forward", 4096, 4096, 14336, True),
    ("c2 E_X", 2048, 4096, 4096, False),
    ("c2 G", 4096, 4096, 2048, False),
    ("c3 E_X / G", 4096, 14336, 4096, False),
]


@pytest.mark.parametrize("what,M,N,K,trans_b", FULL, ids=[f[0] for f in FULL])
def test_gemm_full_size_accumulators_bit_exact_and_repeatable(what, M, N, K, trans_b):
    rng = np.random.default_rng(M + 3 * N + 7 * K + int(trans_b))
    a = rand_codes(rng, (M, K))
    b = rand_codes(rng, (N, K) if trans_b else (K, N))
    da, db = gu.to_dev(a), gu.to_dev(b)
    _, acc1 = binding.halo_gemm_i8(da, db, trans_b=trans_b, out_dtype=None, want_acc=True)
    _, acc2 = binding.halo_gemm_i8(da, db, trans_b=trans_b, out_dtype=None, want_acc=True)
    assert torch.equal(acc1, acc2), "two runs of the same product differ"
    del acc2
    gu.assert_codes_equal(acc1, orc.gemm_codes(a, b.T if trans_b else b), what + " accumulators")


@pytest.mark.parametrize("b,m,n", [(2048, 4096, 4096), (4096, 14336, 4096)], ids=["c2", "c3"])
def test_gemm_pair_full_size_bit_exact_and_repeatable(b, m, n):
    """The paired backward launch at the sizes of configs c2 and c3: E_X = Eq Wq and G = EqT Xq accumulators."""
    rng = np.random.default_rng(b + m + n)
    Eq = rand_codes(rng, (b, n)); Wq = rand_codes(rng, (n, m)); EqT = rand_codes(rng, (n, b)); Xq = rand_codes(rng, (b, m))
    dEq, dWq, dEqT, dXq = map(gu.to_dev, (Eq, Wq, EqT, Xq))
    accs = []
    for _ in range(2):
        ax = torch.empty((b, m), dtype=torch.int32, device=gu.DEV)
        ag = torch.empty((n, m), dtype=torch.int32, device=gu.DEV)
        binding.halo_gemm_i8_pair(binding.gemm_desc(dEq, dWq, trans_b=False, acc_out=ax),
                                  binding.gemm_desc(dEqT, dXq, trans_b=False, acc_out=ag))
        accs.append((ax, ag))
    assert torch.equal(accs[0][0], accs[1][0]) and torch.equal(accs[0][1], accs[1][1]), "two runs differ"
    ax, ag = accs[0]
    del accs
    gu.assert_codes_equal(ax, orc.gemm_codes(Eq, Wq), "paired E_X accumulators")
    gu.assert_codes_equal(ag, orc.gemm_codes(EqT, Xq), "paired G accumulators")
