"""Helpers for the GPU parity tests: host <-> device moves and the comparison bars."""
import numpy as np
import torch

DEV = "cuda:0"


def bits_to_dev(bits: np.ndarray) -> torch.Tensor:
    """bf16 bit patterns (uint16) -> bf16 device tensor."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(DEV).view(torch.bfloat16)


def dev_bf16_to_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def to_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def assert_codes_equal(got: torch.Tensor, want: np.ndarray, what: str):
    g = got.cpu().numpy()
    assert g.shape == want.shape, (what, g.shape, want.shape)
    if not np.array_equal(g, want):
        bad = np.argwhere(g != want)
        i = tuple(bad[0])
        raise AssertionError("%s: %d of %d codes differ; first at %s: got %d want %d"
                             % (what, len(bad), want.size, i, g[i], want[i]))


def assert_f32_identical(got: torch.Tensor, want: np.ndarray, what: str):
    g = got.cpu().numpy()
    assert g.dtype == np.float32 and want.dtype == np.float32 and g.shape == want.shape, what
    # value equality: +0.0 and -0.0 are the same number (the kernels carry signs separately)
    if not np.array_equal(g, want):
        bad = np.argwhere(g != want)
        i = tuple(bad[0])
        raise AssertionError("%s: %d of %d fp32 values differ; first at %s: got %r want %r"
                             % (what, len(bad), want.size, i, g[i], want[i]))


def assert_close_1e3(got: torch.Tensor, want: np.ndarray, what: str):
    """Dequantised fp32 outputs: max-abs error and Frobenius error both within 1e-3 relative."""
    g = got.float().cpu().numpy().astype(np.float64)
    w = want.astype(np.float64)
    assert g.shape == w.shape, (what, g.shape, w.shape)
    scale = np.max(np.abs(w))
    assert np.max(np.abs(g - w)) <= 1e-3 * scale, (what, np.max(np.abs(g - w)) / scale)
    assert np.linalg.norm(g - w) <= 1e-3 * np.linalg.norm(w), what


def assert_bf16_within_one_ulp(got: torch.Tensor, want_f32: np.ndarray, what: str):
    """bf16 outputs: at most one bf16 ulp away from the rounded oracle value."""
    from oracle import halo_oracle as orc
    gb = dev_bf16_to_bits(got).astype(np.int32)
    wb = orc.real_to_bf16_bits(want_f32).astype(np.int32)
    # compare as sign-magnitude integers
    key = lambda b: np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    d = np.abs(key(gb) - key(wb))
    assert d.max() <= 1, (what, int(d.max()))
