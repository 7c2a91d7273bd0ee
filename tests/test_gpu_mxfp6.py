"""GPU parity of the MXFP6 variant (FP6 E3M2 elements, E8M0 scale per 32 along K) through the C ABI: packed codes
and scale bytes bit for bit against the oracle; the scaled-MFMA product within fp32 accumulation error of the
oracle's exact (float64) product of the dequantised operands."""
import numpy as np
import pytest
import torch

from oracle import halo_oracle as orc
from oracle import mxfp6_oracle as mx
from paper_2501_02625_amd import binding, inputs
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def quant_and_check(bits, hb):
    rows, cols = bits.shape
    codes, scales = binding.halo_mx6_quant(gu.bits_to_dev(bits), had_block=hb)
    want_c, want_s = mx.mx_quantize_rows(orc.fwht(orc.bf16_bits_to_real(bits), hb, 1))
    got_s = scales.cpu().numpy()
    assert np.array_equal(got_s, want_s), "scale bytes differ: %d of %d" % ((got_s != want_s).sum(), want_s.size)
    got_p = codes.cpu().numpy()
    want_p = mx.pack_fp6(want_c)
    if not np.array_equal(got_p, want_p):
        got_c = mx.unpack_fp6(got_p, cols)
        bad = np.argwhere(got_c != want_c)
        raise AssertionError("%d of %d codes differ; first at %s: got %d want %d"
                             % (len(bad), want_c.size, tuple(bad[0]), got_c[tuple(bad[0])], want_c[tuple(bad[0])]))
    return codes, scales, want_c, want_s


@pytest.mark.parametrize("rows,cols,hb,frac", [(128, 512, 512, 0.005), (37, 4096, 4096, 0.001), (5, 14336, 2048, 0.001),
                                               (64, 1024, 0, 0.01), (9, 96, 32, 0.0), (33, 2048, 256, 0.01)])
def test_mx6_quantiser_codes_and_scales_bit_exact(rows, cols, hb, frac):
    quant_and_check(inputs.make_activations(rows, cols, frac, rows + cols), hb)


def test_mx6_quantiser_zero_blocks_tiny_and_huge_values():
    x = inputs.bf16_bits_to_f32(inputs.make_activations(8, 256, 0.0, 1))
    x[1, 32:64] = 0
    x[2] *= 1e-30
    x[3, 5] = 3.0e38
    x[4] = 0
    x[5, 64:96] = np.float32(2.0 ** -130)       # subnormal fp32 (flushes to zero in bf16 or stays tiny)
    quant_and_check(inputs.f32_to_bf16_bits(x), 0)
    w = inputs.make_weights(40, 512, 2)
    quant_and_check(w, 512)


@pytest.mark.parametrize("M,N,K", [(128, 128, 128), (200, 136, 512), (64, 300, 4096), (512, 512, 1024),
                                   (4000, 3100, 256),      # ragged, enough 256 x 256 tiles for the DMA kernel
                                   (3584, 3584, 128),      # one K step: the ring never fills
                                   (3600, 3330, 1024),     # ragged, K a multiple of 512: scale bytes of four K steps per request
                                   (4096, 3072, 512)])     # one group of four K steps
def test_mx6_gemm_against_exact_product(M, N, K):
    Xb = inputs.make_activations(M, K, 0.01, M + N); Wb = inputs.make_weights(N, K, M + N)
    hb = K & -K if K <= 4096 else 0
    a, sa, xc, xs = quant_and_check(Xb, hb)
    b, sb, wc, ws = quant_and_check(Wb, hb)
    want = mx.mx_gemm(xc, xs, wc, ws)
    got = binding.halo_gemm_mx6(a, sa, b, sb).cpu().numpy().astype(np.float64)
    # fp32 accumulation in an order the hardware does not specify (the products of a block are aligned to a common
    # exponent before they are added): the error stays below 2^-16 of the sum of the magnitudes of the products
    bound = np.abs(mx.mx_dequantize(xc, xs)) @ np.abs(mx.mx_dequantize(wc, ws)).T * 2.0 ** -16 + 1e-30
    assert np.all(np.abs(got - want) <= bound), float(np.max(np.abs(got - want) / bound))
    assert np.max(np.abs(got - want)) <= 1e-3 * np.max(np.abs(want))
    out16 = binding.halo_gemm_mx6(a, sa, b, sb, out_dtype=torch.bfloat16)
    gu.assert_bf16_within_one_ulp(out16, got.astype(np.float32), "bf16 output")


def test_mx6_forward_on_config_c5_shape_sampled():
    """Config c5: X 8192 x 4096, W 4096 x 4096, FWHT over K = 4096, MXFP6, fp32 accumulation.  Codes and scales of both
    operands in full; the product on sampled rows and columns (each output element is an independent dot product)."""
    b, m, n = 8192, 4096, 4096
    Xb = inputs.make_activations(b, m, 0.001, 50); Wb = inputs.make_weights(n, m, 50)
    a, sa, xc, xs = quant_and_check(Xb, 4096)
    w, sw, wc, ws = quant_and_check(Wb, 4096)
    Y = binding.halo_gemm_mx6(a, sa, w, sw)
    rng = np.random.default_rng(0)
    ri, ci = np.sort(rng.choice(b, 96, replace=False)), np.sort(rng.choice(n, 160, replace=False))
    want = mx.mx_gemm(xc[ri], xs[ri], wc[ci], ws[ci])
    got = Y[torch.as_tensor(ri, device=gu.DEV)][:, torch.as_tensor(ci, device=gu.DEV)].cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got - want)) <= 1e-3 * np.max(np.abs(want))
    ref = orc.bf16_bits_to_real(Xb[ri]).astype(np.float64) @ orc.bf16_bits_to_real(Wb[ci]).astype(np.float64).T
    assert np.linalg.norm(got - ref) / np.linalg.norm(ref) < 0.08       # FP6 with Hadamard stays close to the plain product
