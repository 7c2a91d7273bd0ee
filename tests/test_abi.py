"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, and rejects bad
arguments on the host before anything is launched (no device needed for any call made here)."""
import ctypes
import os
import re

import pytest

from paper_2501_02625_amd import _build, binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(_build.LIB_PATH):
        _build.build()
    return binding.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "halo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(halo_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(binding.EXPORTED_SYMBOLS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings(lib):
    assert lib.halo_version() >= 1
    seen = {binding.status_string(s) for s in range(7)}
    assert len(seen) == 7 and "ok" in seen


def _p(v):
    return ctypes.c_void_p(v)


def test_hadamard_quant_argument_errors(lib):
    f = lib.halo_hadamard_quant
    good = dict(rows=64, cols=512, ld=512)
    A, Q, S = _p(0x1000), _p(0x2000), _p(0x3000)
    # null pointers
    assert f(None, 0, 64, 512, 512, 0, 512, 0, None, Q, 512, S, None, 0, None) == binding.HALO_EINVAL
    # negative size, bad enums
    assert f(A, 0, -1, 512, 512, 0, 0, 0, None, Q, 512, S, None, 0, None) == binding.HALO_EINVAL
    assert f(A, 7, 64, 512, 512, 0, 0, 0, None, Q, 512, S, None, 0, None) == binding.HALO_EINVAL
    assert f(A, 0, 64, 512, 512, 9, 0, 0, None, Q, 512, S, None, 0, None) == binding.HALO_EINVAL
    # block not a power of two / does not divide / too large
    assert f(A, 0, 64, 512, 512, 0, 48, 0, None, Q, 512, S, None, 0, None) == binding.HALO_ESHAPE
    assert f(A, 0, 64, 768, 768, 0, 512, 0, None, Q, 768, S, None, 0, None) == binding.HALO_ESHAPE
    assert f(A, 0, 64, 8192, 8192, 0, 8192, 0, None, Q, 8192, S, None, 0, None) == binding.HALO_EUNSUPPORTED
    # leading dimension too small, misaligned pointer / ld
    assert f(A, 0, 64, 512, 256, 0, 0, 0, None, Q, 512, S, None, 0, None) == binding.HALO_ESHAPE
    assert f(_p(0x1004), 0, 64, 512, 512, 0, 0, 0, None, Q, 512, S, None, 0, None) == binding.HALO_EALIGN
    assert f(A, 0, 64, 500, 500, 0, 0, 0, None, Q, 512, S, None, 0, None) == binding.HALO_EALIGN
    # left-hand rotation without workspace
    assert f(A, 0, 64, 512, 512, 0, 0, 64, None, Q, 512, S, None, 0, None) == binding.HALO_EWORKSPACE
    need = lib.halo_hadamard_quant_workspace_bytes(64, 512, 0, 64)
    assert need >= 64 * 512 * 4
    assert f(A, 0, 64, 512, 512, 0, 0, 64, None, Q, 512, S, _p(0x4000), need - 1, None) == binding.HALO_EWORKSPACE
    # transposed-output axis has no rotation
    need = lib.halo_hadamard_quant_workspace_bytes(64, 512, 1, 0)
    assert f(A, 0, 64, 512, 512, 1, 512, 0, None, Q, 64, S, _p(0x4000), need, None) == binding.HALO_EUNSUPPORTED
    # empty input is a no-op
    assert f(None, 0, 0, 512, 512, 0, 0, 0, None, None, 512, None, None, 0, None) == binding.HALO_OK
    assert good


def test_kronecker_block_argument_errors(lib):
    """Blocks of the form 28 * 2^n: the Walsh-Hadamard factor must lie in [64, 512], the block must divide the row and
    the row may hold at most 14336 elements; the microscaling quantiser takes power-of-two blocks only."""
    f = lib.halo_hadamard_quant
    A, Q, S = _p(0x1000), _p(0x2000), _p(0x3000)
    assert f(A, 0, 64, 896, 896, 0, 896, 0, None, Q, 896, S, None, 0, None) == binding.HALO_EUNSUPPORTED       # 32 * 28
    assert f(A, 0, 64, 28672, 28672, 0, 28672, 0, None, Q, 28672, S, None, 0, None) == binding.HALO_EUNSUPPORTED
    assert f(A, 0, 64, 28672, 28672, 0, 14336, 0, None, Q, 28672, S, None, 0, None) == binding.HALO_EUNSUPPORTED
    assert f(A, 0, 64, 2048, 2048, 0, 1792, 0, None, Q, 2048, S, None, 0, None) == binding.HALO_ESHAPE         # does not divide
    assert f(A, 0, 64, 5376, 5376, 0, 5376, 0, None, Q, 5376, S, None, 0, None) == binding.HALO_ESHAPE         # 3 * 64 * 28
    u = lib.halo_dequant_unrotate
    assert u(A, 2048, 16, 2048, None, None, 1792, 0, Q, 1, 2048, None, 0, None) == binding.HALO_ESHAPE
    assert lib.halo_mx6_quant(A, 64, 1792, 1792, 1792, Q, 1344, S, 64, None) == binding.HALO_ESHAPE
    d = binding.make_desc(64, 28672, 128, 1, had_block_m=14336)
    P = _p(0x1000)
    assert lib.halo_linear_fwd(ctypes.byref(d), P, P, P, P, P, P, P, None, 0, None) == binding.HALO_EUNSUPPORTED


def test_quant_dual_argument_errors(lib):
    f = lib.halo_quant_dual
    A, Q, S, T, U, W = _p(0x1000), _p(0x2000), _p(0x3000), _p(0x4000), _p(0x5000), _p(0x6000)
    need = lib.halo_quant_dual_workspace_bytes(64, 512)
    assert need >= 4 * 64 * 2
    assert f(None, 64, 512, 512, None, None, Q, 512, S, T, 64, U, W, need, None) == binding.HALO_EINVAL
    assert f(A, 64, 512, 256, None, None, Q, 512, S, T, 64, U, W, need, None) == binding.HALO_ESHAPE
    assert f(A, 64, 512, 512, None, None, Q, 512, S, T, 48, U, W, need, None) == binding.HALO_ESHAPE
    assert f(A, 64, 512, 512, None, None, Q, 520, S, T, 64, U, W, need, None) == binding.HALO_EALIGN
    assert f(A, 64, 512, 512, None, None, Q, 512, S, T, 64, U, W, need - 1, None) == binding.HALO_EWORKSPACE
    assert f(A, 64, 512, 512, None, None, Q, 512, S, T, 64, U, None, 0, None) == binding.HALO_EWORKSPACE
    assert f(None, 0, 512, 512, None, None, None, 512, None, None, 64, None, None, 0, None) == binding.HALO_OK


def test_gemm_argument_errors(lib):
    f = lib.halo_gemm_i8
    A, B, C = _p(0x1000), _p(0x2000), _p(0x3000)
    assert f(A, 64, B, 64, 1, 32, 32, 64, None, None, None, 1, 32, None, 0, None) == binding.HALO_EINVAL
    assert f(None, 64, B, 64, 1, 32, 32, 64, None, None, C, 1, 32, None, 0, None) == binding.HALO_EINVAL
    assert f(A, 64, B, 64, 1, 32, 32, 40, None, None, C, 1, 32, None, 0, None) == binding.HALO_ESHAPE     # K % 16
    assert f(A, 32, B, 64, 1, 32, 32, 64, None, None, C, 1, 32, None, 0, None) == binding.HALO_ESHAPE     # lda < K
    assert f(A, 64, B, 16, 0, 32, 32, 64, None, None, C, 1, 32, None, 0, None) == binding.HALO_ESHAPE     # ldb < N
    assert f(A, 72, B, 64, 1, 32, 32, 64, None, None, C, 1, 32, None, 0, None) == binding.HALO_EALIGN
    assert f(A, 64, B, 64, 1, 32, 32, 64, None, None, C, 0, 36, None, 0, None) == binding.HALO_EALIGN     # bf16 ldc
    assert f(A, 64, B, 64, 1, 32, 32, 64, None, None, C, 5, 32, None, 0, None) == binding.HALO_EINVAL
    k_too_long = 1 << 18   # 127*127*K would overflow int32
    assert f(A, k_too_long, B, k_too_long, 1, 32, 32, k_too_long, None, None, C, 1, 32, None, 0, None) == binding.HALO_ESHAPE
    assert f(None, 0, None, 0, 1, 0, 32, 64, None, None, None, 1, 32, None, 0, None) == binding.HALO_OK


def test_gemm_pair_argument_errors(lib):
    A, B, C = 0x1000, 0x2000, 0x3000
    good = binding.GemmDesc(A, 64, B, 64, 0, 32, 64, 64, None, None, C, binding.HALO_F32, 64, None, 0, -1)
    bad_k = binding.GemmDesc(A, 64, B, 64, 0, 32, 64, 40, None, None, C, binding.HALO_F32, 64, None, 0, -1)
    no_out = binding.GemmDesc(A, 64, B, 64, 0, 32, 64, 64, None, None, None, binding.HALO_F32, 64, None, 0, -1)
    empty = binding.GemmDesc(None, 0, None, 0, 0, 0, 64, 64, None, None, None, binding.HALO_F32, 0, None, 0, -1)
    bad_cfg = binding.GemmDesc(A, 64, B, 64, 0, 32, 64, 64, None, None, C, binding.HALO_F32, 64, None, 0, 7)
    k_step = binding.GemmDesc(A, 64, B, 64, 0, 32, 64, 64, None, None, C, binding.HALO_F32, 64, None, 0, 1)   # K % 128
    assert lib.halo_gemm_i8_desc(ctypes.byref(bad_cfg), None) == binding.HALO_EINVAL
    assert lib.halo_gemm_i8_desc(ctypes.byref(k_step), None) == binding.HALO_ESHAPE
    assert lib.halo_gemm_i8_desc(None, None) == binding.HALO_EINVAL
    assert lib.halo_gemm_i8_desc(ctypes.byref(empty), None) == binding.HALO_OK
    assert lib.halo_mfma_i8_probe(None, 1, None, None) == binding.HALO_EINVAL
    assert lib.halo_mfma_i8_probe(ctypes.c_void_p(0x1000), -1, None, None) == binding.HALO_EINVAL
    assert lib.halo_mfma_i8_probe(ctypes.c_void_p(0x1004), 1, None, None) == binding.HALO_EALIGN
    assert lib.halo_mfma_i8_probe(ctypes.c_void_p(0x1000), 0, None, None) == binding.HALO_OK
    f = lib.halo_gemm_i8_pair
    assert f(None, ctypes.byref(good), None) == binding.HALO_EINVAL
    assert f(ctypes.byref(good), ctypes.byref(bad_k), None) == binding.HALO_ESHAPE
    assert f(ctypes.byref(no_out), ctypes.byref(good), None) == binding.HALO_EINVAL
    assert f(ctypes.byref(empty), ctypes.byref(empty), None) == binding.HALO_OK


def test_linear_desc_errors_and_workspace(lib):
    d = binding.make_desc(2048, 4096, 4096, 1)
    ws1 = binding.halo_linear_workspace_bytes(d)
    assert ws1 >= 2048 * 4096 * 2 + 4096 * 4096 * 4
    d2 = binding.make_desc(2048, 4096, 4096, 2)
    assert binding.halo_linear_workspace_bytes(d2) >= ws1 + 2048 * 4096 * 4
    P = _p(0x1000)
    bad_level = binding.make_desc(64, 64, 64, 3)
    assert lib.halo_linear_fwd(ctypes.byref(bad_level), P, P, P, P, P, P, P, None, 0, None) == binding.HALO_EINVAL
    odd = binding.make_desc(60, 64, 64, 1)
    assert lib.halo_linear_fwd(ctypes.byref(odd), P, P, P, P, P, P, P, None, 0, None) == binding.HALO_ESHAPE
    blk = binding.make_desc(64, 96, 64, 1, had_block_m=64)
    assert lib.halo_linear_fwd(ctypes.byref(blk), P, P, P, P, P, P, P, None, 0, None) == binding.HALO_ESHAPE
    # tokens are the reduction length of G = E^T X: 127*127*b must fit the int32 accumulator (b <= 133,136)
    long_b = binding.make_desc(133152, 64, 64, 1)
    assert lib.halo_linear_fwd(ctypes.byref(long_b), P, P, P, P, P, P, P, None, 0, None) == binding.HALO_ESHAPE
    assert lib.halo_linear_bwd(ctypes.byref(long_b), P, P, P, P, P, P, P, P, 1 << 40, None) == binding.HALO_ESHAPE
    assert binding.halo_linear_workspace_bytes(long_b) == 0
    assert binding.halo_linear_workspace_bytes(binding.make_desc(133136, 64, 64, 1)) > 0
    ok = binding.make_desc(64, 64, 64, 1)
    assert lib.halo_linear_fwd(ctypes.byref(ok), P, P, None, P, P, P, P, None, 0, None) == binding.HALO_EINVAL
    assert lib.halo_linear_bwd(ctypes.byref(ok), P, P, P, P, P, None, None, P, 1 << 30, None) == binding.HALO_EINVAL
    assert lib.halo_linear_bwd(ctypes.byref(ok), P, P, P, P, P, P, P, P, 16, None) == binding.HALO_EWORKSPACE
    assert lib.halo_linear_bwd(ctypes.byref(ok), P, P, P, P, P, P, P, None, 0, None) == binding.HALO_EWORKSPACE


def test_peft_argument_errors(lib):
    P = _p(0x1000)
    ok = binding.make_desc(64, 128, 64, 2)
    need = binding.halo_peft_workspace_bytes(ok, 16)
    assert need >= 64 * 128 * 5 + 64 * 64
    fwd, bwd = lib.halo_peft_fwd, lib.halo_peft_bwd
    assert fwd(ctypes.byref(ok), 16, P, P, P, P, P, P, P, P, 16, None) == binding.HALO_EWORKSPACE
    assert fwd(ctypes.byref(ok), 16, P, P, P, P, None, P, P, P, need, None) == binding.HALO_EINVAL
    assert fwd(ctypes.byref(ok), 0, P, P, P, P, P, P, P, P, need, None) == binding.HALO_EINVAL
    assert fwd(ctypes.byref(ok), 12, P, P, P, P, P, P, P, P, need, None) == binding.HALO_ESHAPE
    assert fwd(ctypes.byref(ok), 72, P, P, P, P, P, P, P, P, need, None) == binding.HALO_EUNSUPPORTED
    assert fwd(ctypes.byref(ok), 16, _p(0x1008), P, P, P, P, P, P, P, need, None) == binding.HALO_EALIGN
    assert binding.halo_peft_workspace_bytes(ok, 12) == 0
    # both widths are reduction lengths of a K-step product: multiples of 64
    narrow = binding.make_desc(64, 96, 64, 0)
    assert fwd(ctypes.byref(narrow), 16, P, P, P, P, P, P, P, P, 1 << 30, None) == binding.HALO_ESHAPE
    tensor = binding.make_desc(64, 128, 64, 2, scale_mode=binding.HALO_SCALE_PER_TENSOR)
    assert fwd(ctypes.byref(tensor), 16, P, P, P, P, P, P, P, P, 1 << 30, None) == binding.HALO_EUNSUPPORTED
    # backward: something must be wanted, and each output needs its own inputs
    assert bwd(ctypes.byref(ok), 16, P, P, P, P, P, P, P, None, None, None, P, need, None) == binding.HALO_EINVAL
    assert bwd(ctypes.byref(ok), 16, None, P, P, P, P, P, P, P, P, P, P, need, None) == binding.HALO_EINVAL
    assert bwd(ctypes.byref(ok), 16, P, None, P, P, P, P, P, None, P, None, P, need, None) == binding.HALO_EINVAL   # G_U reads X
    assert bwd(ctypes.byref(ok), 16, P, P, None, P, P, P, P, None, None, P, P, need, None) == binding.HALO_EINVAL   # G_V reads T
    assert bwd(ctypes.byref(ok), 16, P, P, P, None, P, P, P, P, None, None, P, need, None) == binding.HALO_EINVAL   # E_X reads Wq
    assert bwd(ctypes.byref(ok), 16, P, P, P, P, P, P, P, P, P, P, P, need - 1, None) == binding.HALO_EWORKSPACE
    assert bwd(ctypes.byref(ok), 16, P, P, P, P, P, P, P, P, P, P, None, 0, None) == binding.HALO_EWORKSPACE
    # empty problem: nothing to do, nothing touched
    empty = binding.make_desc(0, 128, 64, 2)
    assert fwd(ctypes.byref(empty), 16, P, P, P, P, P, P, P, None, 0, None) == binding.HALO_OK


def test_dequant_unrotate_argument_errors(lib):
    f = lib.halo_dequant_unrotate
    A, O = _p(0x1000), _p(0x2000)
    assert f(None, 64, 16, 64, None, None, 64, 0, O, 1, 64, None, 0, None) == binding.HALO_EINVAL
    assert f(A, 64, 16, 64, None, None, 48, 0, O, 1, 64, None, 0, None) == binding.HALO_ESHAPE
    assert f(A, 64, 16, 64, None, None, 64, 16, O, 1, 64, None, 0, None) == binding.HALO_EWORKSPACE
    assert f(A, 32, 16, 64, None, None, 64, 0, O, 1, 64, None, 0, None) == binding.HALO_ESHAPE
    assert f(A, 64, 16, 64, None, None, 64, 0, O, 0, 68, None, 0, None) == binding.HALO_EALIGN


def test_hadamard_quant_tensor_argument_errors(lib):
    f = lib.halo_hadamard_quant_tensor
    A, Q, S, W = _p(0x1000), _p(0x2000), _p(0x3000), _p(0x4000)
    need = lib.halo_hadamard_quant_tensor_workspace_bytes(64, 512, 0, 0)
    assert need >= (64 + 1) * 4
    assert lib.halo_hadamard_quant_tensor_workspace_bytes(64, 512, 0, 64) >= need + 64 * 512 * 4
    assert f(None, 0, 64, 512, 512, 0, 512, 0, Q, 512, S, W, need, None) == binding.HALO_EINVAL
    assert f(A, 0, 64, 512, 512, 0, 48, 0, Q, 512, S, W, need, None) == binding.HALO_ESHAPE
    assert f(A, 0, 64, 512, 512, 0, 512, 0, Q, 512, S, None, 0, None) == binding.HALO_EWORKSPACE
    assert f(A, 0, 64, 512, 512, 0, 512, 0, Q, 512, S, W, need - 1, None) == binding.HALO_EWORKSPACE
    assert f(A, 0, 64, 512, 512, 1, 512, 0, Q, 64, S, W, 1 << 20, None) == binding.HALO_EUNSUPPORTED
    assert f(A, 0, 64, 512, 512, 0, 0, 0, Q, 520, S, W, need, None) == binding.HALO_EALIGN
    assert f(None, 0, 0, 512, 512, 0, 0, 0, None, 512, None, None, 0, None) == binding.HALO_OK
    bad_mode = binding.make_desc(64, 64, 64, 1, scale_mode=5)
    P = _p(0x1000)
    assert lib.halo_linear_fwd(ctypes.byref(bad_mode), P, P, P, P, P, P, P, None, 0, None) == binding.HALO_EINVAL
    per_tensor = binding.make_desc(64, 64, 64, 1, scale_mode=binding.HALO_SCALE_PER_TENSOR)
    assert lib.halo_linear_fwd(ctypes.byref(per_tensor), P, P, P, P, P, P, P, None, 0, None) == binding.HALO_EWORKSPACE
    assert binding.halo_linear_workspace_bytes(per_tensor) > binding.halo_linear_workspace_bytes(binding.make_desc(64, 64, 64, 1))


def test_mx6_argument_errors(lib):
    q, g = lib.halo_mx6_quant, lib.halo_gemm_mx6
    A, Cq, S, B, C = _p(0x1000), _p(0x2000), _p(0x3000), _p(0x4000), _p(0x5000)
    assert q(None, 64, 512, 512, 512, Cq, 384, S, 16, None) == binding.HALO_EINVAL
    assert q(A, 64, 500, 512, 0, Cq, 384, S, 16, None) == binding.HALO_ESHAPE          # cols % 32
    assert q(A, 64, 512, 512, 0, Cq, 380, S, 16, None) == binding.HALO_ESHAPE          # ld_codes < cols/32*24
    assert q(A, 64, 512, 512, 0, Cq, 388, S, 16, None) == binding.HALO_EALIGN          # ld_codes % 8
    assert q(A, 64, 512, 512, 48, Cq, 384, S, 16, None) == binding.HALO_ESHAPE         # block not a power of two
    assert q(None, 0, 512, 512, 0, None, 384, None, 16, None) == binding.HALO_OK
    assert g(A, 96, S, 4, B, 96, S, 4, 64, 64, 128, None, 1, 64, None) == binding.HALO_EINVAL
    assert g(A, 96, S, 4, B, 96, S, 4, 64, 64, 96, C, 1, 64, None) == binding.HALO_ESHAPE      # K % 128
    assert g(A, 90, S, 4, B, 96, S, 4, 64, 64, 128, C, 1, 64, None) == binding.HALO_ESHAPE     # lda too small
    assert g(A, 104, S, 4, B, 96, S, 4, 64, 64, 128, C, 1, 64, None) == binding.HALO_EALIGN    # lda % 16
    assert g(A, 96, S, 6, B, 96, S, 4, 64, 64, 128, C, 1, 64, None) == binding.HALO_EALIGN     # scale pitch % 4
    assert g(A, 96, S, 4, B, 96, S, 4, 64, 64, 128, C, 7, 64, None) == binding.HALO_EINVAL
    assert g(None, 0, None, 0, None, 0, None, 0, 0, 64, 128, None, 1, 64, None) == binding.HALO_OK


def test_binding_refuses_missing_library(tmp_path):
    with pytest.raises(RuntimeError):
        binding.load_library(str(tmp_path / "nope.so"))


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: bench.py --gpus N with N > 1 exits with a message before it touches a device."""
    import subprocess, sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr


def test_inputs_are_deterministic_and_shaped():
    import numpy as np
    from paper_2501_02625_amd import inputs
    cfg = inputs.CONFIGS["c1"]
    a = inputs.make_linear_inputs(cfg)
    b = inputs.make_linear_inputs(cfg)
    assert a["X"].shape == (128, 512) and a["W"].shape == (512, 512) and "E" not in a
    assert np.array_equal(a["X"], b["X"]) and np.array_equal(a["W"], b["W"])
    X = inputs.bf16_bits_to_f32(a["X"])
    cols = inputs.outlier_columns(512, 0.005, 0)
    assert len(cols) == 3
    rms = np.sqrt((X.astype(np.float64) ** 2).mean(axis=0))
    assert np.all(rms[cols] > 25) and np.median(rms) < 1.5
    assert abs(np.std(inputs.bf16_bits_to_f32(a["W"])) - 0.02) < 2e-3
    E = inputs.bf16_bits_to_f32(inputs.make_errors(256, 64, 1))
    assert np.max(np.abs(E)) > 8 * np.median(np.abs(E))     # heavy tails
    assert inputs.CONFIGS["c2"].gemm_ops() == 6 * 2048 * 4096 * 4096
    assert inputs.CONFIGS["c3"].had_block_m(14336) == 2048
    assert inputs.CONFIGS["c6"].had_block_m(14336) == 14336 and inputs.CONFIGS["c6"].had_block_m(4096) == 4096
    assert inputs.CONFIGS["c7"].per_tensor and not inputs.CONFIGS["c2"].per_tensor
