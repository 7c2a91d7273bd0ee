"""Thin ctypes binding of libhalo's C ABI (include/halo.h).

Argument marshalling only: every step of the HALO linear layer runs in the HIP kernels of libhalo.so.
torch is used for device memory and the current stream, nothing else.  There is no CPU fallback: if the
shared library is missing, importing a function from here raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Tuple

import torch

from . import _build

HALO_OK = 0
HALO_EINVAL, HALO_ESHAPE, HALO_EALIGN, HALO_EWORKSPACE, HALO_EUNSUPPORTED, HALO_EHIP = 1, 2, 3, 4, 5, 6
HALO_BF16, HALO_F32 = 0, 1
HALO_QUANT_ROWS, HALO_QUANT_COLS_T = 0, 1
HALO_SCALE_PER_ROW, HALO_SCALE_PER_TENSOR = 0, 1
HALO_GEMM_AUTO = -1
HALO_GEMM_CONFIGS = {"256x256x64": 0, "256x256x128": 1, "256x128x128": 2, "128x128x64": 3, "staged_128x128x64": 4}

EXPORTED_SYMBOLS = (
    "halo_status_string", "halo_version",
    "halo_hadamard_quant_workspace_bytes", "halo_hadamard_quant",
    "halo_hadamard_quant_tensor_workspace_bytes", "halo_hadamard_quant_tensor",
    "halo_quant_dual_workspace_bytes", "halo_quant_dual",
    "halo_quant_dual_static_max_workspace_bytes", "halo_quant_dual_static",
    "halo_gemm_i8", "halo_gemm_i8_desc", "halo_gemm_i8_pair", "halo_mfma_i8_probe",
    "halo_mx6_quant", "halo_gemm_mx6",
    "halo_dequant_unrotate_workspace_bytes", "halo_dequant_unrotate",
    "halo_linear_workspace_bytes", "halo_linear_fwd", "halo_linear_bwd",
    "halo_peft_workspace_bytes", "halo_peft_fwd", "halo_peft_bwd",
)


class HaloError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (status %d)" % (where, status_string(status), status))


class GemmDesc(ctypes.Structure):
    _fields_ = [("A", ctypes.c_void_p), ("lda", ctypes.c_int64), ("B", ctypes.c_void_p), ("ldb", ctypes.c_int64),
                ("transB", ctypes.c_int32), ("M", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64),
                ("row_scale", ctypes.c_void_p), ("col_scale", ctypes.c_void_p), ("C", ctypes.c_void_p),
                ("c_dt", ctypes.c_int32), ("ldc", ctypes.c_int64), ("acc_out", ctypes.c_void_p),
                ("ld_acc", ctypes.c_int64), ("config", ctypes.c_int32)]


class LinearDesc(ctypes.Structure):
    _fields_ = [("b", ctypes.c_int64), ("m", ctypes.c_int64), ("n", ctypes.c_int64),
                ("level", ctypes.c_int32), ("had_block_m", ctypes.c_int32),
                ("had_block_b", ctypes.c_int32), ("out_dt", ctypes.c_int32), ("scale_mode", ctypes.c_int32)]


_lib: Optional[ctypes.CDLL] = None


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Load libhalo.so (built in-tree by _build.build()).  Raises if it is not there."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or _build.LIB_PATH
    if not os.path.exists(path):
        raise RuntimeError(
            "libhalo.so is not built (%s). Run `python -c 'import __graft_entry__ as g; g.build()'`; "
            "there is no fallback path." % path)
    lib = ctypes.CDLL(path)
    c = ctypes
    vp, i64, i32, sz = c.c_void_p, c.c_int64, c.c_int32, c.c_size_t
    lib.halo_status_string.restype = c.c_char_p
    lib.halo_status_string.argtypes = [c.c_int]
    lib.halo_version.restype = c.c_int
    lib.halo_version.argtypes = []
    lib.halo_hadamard_quant_workspace_bytes.restype = sz
    lib.halo_hadamard_quant_workspace_bytes.argtypes = [i64, i64, c.c_int, i32]
    lib.halo_hadamard_quant.restype = c.c_int
    lib.halo_hadamard_quant.argtypes = [vp, c.c_int, i64, i64, i64, c.c_int, i32, i32, vp, vp, i64, vp, vp, sz, vp]
    lib.halo_hadamard_quant_tensor_workspace_bytes.restype = sz
    lib.halo_hadamard_quant_tensor_workspace_bytes.argtypes = [i64, i64, c.c_int, i32]
    lib.halo_hadamard_quant_tensor.restype = c.c_int
    lib.halo_hadamard_quant_tensor.argtypes = [vp, c.c_int, i64, i64, i64, c.c_int, i32, i32, vp, i64, vp, vp, sz, vp]
    lib.halo_quant_dual_workspace_bytes.restype = sz
    lib.halo_quant_dual_workspace_bytes.argtypes = [i64, i64]
    lib.halo_quant_dual.restype = c.c_int
    lib.halo_quant_dual.argtypes = [vp, i64, i64, i64, vp, vp, vp, i64, vp, vp, i64, vp, vp, sz, vp]
    lib.halo_quant_dual_static_max_workspace_bytes.restype = sz
    lib.halo_quant_dual_static_max_workspace_bytes.argtypes = []
    lib.halo_quant_dual_static.restype = c.c_int
    lib.halo_quant_dual_static.argtypes = [vp, i64, i64, i64, vp, vp, vp, i64, vp, vp, i64, vp, vp]
    lib.halo_gemm_i8.restype = c.c_int
    lib.halo_gemm_i8.argtypes = [vp, i64, vp, i64, c.c_int, i64, i64, i64, vp, vp, vp, c.c_int, i64, vp, i64, vp]
    lib.halo_gemm_i8_pair.restype = c.c_int
    lib.halo_gemm_i8_pair.argtypes = [c.POINTER(GemmDesc), c.POINTER(GemmDesc), vp]
    lib.halo_gemm_i8_desc.restype = c.c_int
    lib.halo_gemm_i8_desc.argtypes = [c.POINTER(GemmDesc), vp]
    lib.halo_mfma_i8_probe.restype = c.c_int
    lib.halo_mfma_i8_probe.argtypes = [vp, i32, vp, vp]
    lib.halo_mx6_quant.restype = c.c_int
    lib.halo_mx6_quant.argtypes = [vp, i64, i64, i64, i32, vp, i64, vp, i64, vp]
    lib.halo_gemm_mx6.restype = c.c_int
    lib.halo_gemm_mx6.argtypes = [vp, i64, vp, i64, vp, i64, vp, i64, i64, i64, i64, vp, c.c_int, i64, vp]
    lib.halo_dequant_unrotate_workspace_bytes.restype = sz
    lib.halo_dequant_unrotate_workspace_bytes.argtypes = [i64, i64, i32]
    lib.halo_dequant_unrotate.restype = c.c_int
    lib.halo_dequant_unrotate.argtypes = [vp, i64, i64, i64, vp, vp, i32, i32, vp, c.c_int, i64, vp, sz, vp]
    lib.halo_linear_workspace_bytes.restype = sz
    lib.halo_linear_workspace_bytes.argtypes = [c.POINTER(LinearDesc)]
    lib.halo_linear_fwd.restype = c.c_int
    lib.halo_linear_fwd.argtypes = [c.POINTER(LinearDesc), vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.halo_linear_bwd.restype = c.c_int
    lib.halo_linear_bwd.argtypes = [c.POINTER(LinearDesc), vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.halo_peft_workspace_bytes.restype = sz
    lib.halo_peft_workspace_bytes.argtypes = [c.POINTER(LinearDesc), i32]
    lib.halo_peft_fwd.restype = c.c_int
    lib.halo_peft_fwd.argtypes = [c.POINTER(LinearDesc), i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.halo_peft_bwd.restype = c.c_int
    lib.halo_peft_bwd.argtypes = [c.POINTER(LinearDesc), i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    if path == _build.LIB_PATH:
        _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().halo_status_string(int(status)).decode()


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dt(dtype: torch.dtype) -> int:
    if dtype == torch.bfloat16:
        return HALO_BF16
    if dtype == torch.float32:
        return HALO_F32
    raise TypeError("HALO tensors are bf16 or fp32, got %s" % dtype)


def _check(status: int, where: str):
    if status != HALO_OK:
        raise HaloError(status, where)


def _empty_padded(rows: int, cols: int, dtype: torch.dtype, device) -> torch.Tensor:
    """[rows, cols] view of a buffer whose row pitch is a multiple of 16 bytes (the ABI's alignment rule)."""
    per16 = 16 // torch.empty((), dtype=dtype).element_size()
    ld = (cols + per16 - 1) // per16 * per16
    return torch.empty((rows, max(ld, per16)), dtype=dtype, device=device)[:, :cols]


def _need_cuda(*ts):
    for t in ts:
        if t is not None and not t.is_cuda:
            raise ValueError("libhalo takes device tensors only")


# ------------------------------------------------------------------------------------------------ entry points
def halo_hadamard_quant(x: torch.Tensor, *, axis: int = HALO_QUANT_ROWS, had_block: int = 0,
                        had_block_left: int = 0, fold: Optional[torch.Tensor] = None,
                        out_q: Optional[torch.Tensor] = None, out_scale: Optional[torch.Tensor] = None,
                        workspace: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """rotate -> fold -> absmax -> INT8.  Returns (codes int8, scales fp32)."""
    lib = load_library()
    _need_cuda(x, fold, out_q, out_scale, workspace)
    assert x.dim() == 2 and x.stride(1) == 1
    rows, cols = x.shape
    if axis == HALO_QUANT_ROWS:
        qshape, nscale = (rows, cols), rows
    else:
        qshape, nscale = (cols, rows), cols
    if out_q is None:
        out_q = _empty_padded(qshape[0], qshape[1], torch.int8, x.device)
    if out_scale is None:
        out_scale = torch.empty((nscale,), dtype=torch.float32, device=x.device)
    need = lib.halo_hadamard_quant_workspace_bytes(rows, cols, axis, had_block_left)
    if workspace is None and need:
        workspace = torch.empty((need,), dtype=torch.uint8, device=x.device)
    st = lib.halo_hadamard_quant(_ptr(x), _dt(x.dtype), rows, cols, x.stride(0) if rows else cols, axis,
                                 had_block, had_block_left, _ptr(fold), _ptr(out_q),
                                 out_q.stride(0) if out_q.numel() else qshape[1], _ptr(out_scale), _ptr(workspace),
                                 workspace.numel() if workspace is not None else 0, _stream())
    _check(st, "halo_hadamard_quant")
    return out_q, out_scale


def halo_hadamard_quant_tensor(x: torch.Tensor, *, axis: int = HALO_QUANT_ROWS, had_block: int = 0,
                               had_block_left: int = 0, out_q: Optional[torch.Tensor] = None,
                               out_scale: Optional[torch.Tensor] = None,
                               workspace: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """rotate -> absmax of the whole tensor -> INT8.  Returns (codes int8, scales fp32: the one scale in every entry)."""
    lib = load_library()
    _need_cuda(x, out_q, out_scale, workspace)
    assert x.dim() == 2 and x.stride(1) == 1
    rows, cols = x.shape
    qshape, nscale = ((rows, cols), rows) if axis == HALO_QUANT_ROWS else ((cols, rows), cols)
    if out_q is None:
        out_q = _empty_padded(qshape[0], qshape[1], torch.int8, x.device)
    if out_scale is None:
        out_scale = torch.empty((nscale,), dtype=torch.float32, device=x.device)
    need = lib.halo_hadamard_quant_tensor_workspace_bytes(rows, cols, axis, had_block_left)
    if workspace is None:
        workspace = torch.empty((max(need, 16),), dtype=torch.uint8, device=x.device)
    st = lib.halo_hadamard_quant_tensor(_ptr(x), _dt(x.dtype), rows, cols, x.stride(0) if rows else cols, axis, had_block,
                                        had_block_left, _ptr(out_q), out_q.stride(0) if out_q.numel() else qshape[1],
                                        _ptr(out_scale), _ptr(workspace), workspace.numel(), _stream())
    _check(st, "halo_hadamard_quant_tensor")
    return out_q, out_scale


def halo_quant_dual(x: torch.Tensor, *, fold_cols: Optional[torch.Tensor] = None,
                    fold_rows: Optional[torch.Tensor] = None, out_q: Optional[torch.Tensor] = None,
                    row_scale: Optional[torch.Tensor] = None, out_qt: Optional[torch.Tensor] = None,
                    col_scale: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None):
    """Row-wise codes of x*fold_cols and transposed column-wise codes of x*fold_rows in one go.
    Returns (codes [rows,cols], row_scale, codesT [cols,rows], col_scale)."""
    lib = load_library()
    _need_cuda(x, fold_cols, fold_rows, out_q, row_scale, out_qt, col_scale, workspace)
    assert x.dim() == 2 and x.stride(1) == 1 and x.dtype == torch.bfloat16
    rows, cols = x.shape
    if out_q is None:
        out_q = _empty_padded(rows, cols, torch.int8, x.device)
    if out_qt is None:
        out_qt = _empty_padded(cols, rows, torch.int8, x.device)
    if row_scale is None:
        row_scale = torch.empty((rows,), dtype=torch.float32, device=x.device)
    if col_scale is None:
        col_scale = torch.empty((cols,), dtype=torch.float32, device=x.device)
    need = lib.halo_quant_dual_workspace_bytes(rows, cols)
    if workspace is None:
        workspace = torch.empty((max(need, 16),), dtype=torch.uint8, device=x.device)
    st = lib.halo_quant_dual(_ptr(x), rows, cols, x.stride(0) if rows else cols, _ptr(fold_cols), _ptr(fold_rows),
                             _ptr(out_q), out_q.stride(0) if out_q.numel() else max(cols, 16), _ptr(row_scale),
                             _ptr(out_qt), out_qt.stride(0) if out_qt.numel() else max(rows, 16), _ptr(col_scale),
                             _ptr(workspace), workspace.numel(), _stream())
    _check(st, "halo_quant_dual")
    return out_q, row_scale, out_qt, col_scale


def halo_quant_dual_static(x: torch.Tensor, *, fold_cols: Optional[torch.Tensor], fold_rows: Optional[torch.Tensor],
                           out_q: torch.Tensor, row_scale: torch.Tensor, out_qt: torch.Tensor,
                           col_scale: torch.Tensor) -> None:
    """halo_quant_dual without a workspace and without any allocation: every output is passed in."""
    _need_cuda(x, fold_cols, fold_rows, out_q, row_scale, out_qt, col_scale)
    assert x.dim() == 2 and x.stride(1) == 1 and x.dtype == torch.bfloat16
    rows, cols = x.shape
    st = load_library().halo_quant_dual_static(_ptr(x), rows, cols, x.stride(0), _ptr(fold_cols), _ptr(fold_rows),
                                               _ptr(out_q), out_q.stride(0), _ptr(row_scale), _ptr(out_qt),
                                               out_qt.stride(0), _ptr(col_scale), _stream())
    _check(st, "halo_quant_dual_static")


def halo_gemm_i8(a: torch.Tensor, b: torch.Tensor, *, trans_b: bool, row_scale: Optional[torch.Tensor] = None,
                 col_scale: Optional[torch.Tensor] = None, out_dtype: Optional[torch.dtype] = torch.float32,
                 want_acc: bool = False, out: Optional[torch.Tensor] = None,
                 acc_out: Optional[torch.Tensor] = None):
    """C = diag(row_scale) (A op(B)) diag(col_scale); returns (C or None, acc or None)."""
    lib = load_library()
    _need_cuda(a, b, row_scale, col_scale, out, acc_out)
    assert a.dtype == torch.int8 and b.dtype == torch.int8 and a.dim() == 2 and b.dim() == 2
    M, K = a.shape
    N = b.shape[0] if trans_b else b.shape[1]
    assert (b.shape[1] if trans_b else b.shape[0]) == K
    if out is None and out_dtype is not None:
        out = _empty_padded(M, N, out_dtype, a.device)
    if acc_out is None and want_acc:
        acc_out = _empty_padded(M, N, torch.int32, a.device)
    st = lib.halo_gemm_i8(_ptr(a), a.stride(0) if M else K, _ptr(b), b.stride(0) if b.shape[0] else b.shape[1],
                          1 if trans_b else 0, M, N, K, _ptr(row_scale), _ptr(col_scale), _ptr(out),
                          _dt(out.dtype) if out is not None else HALO_F32,
                          (out.stride(0) if M else N) if out is not None else 0, _ptr(acc_out),
                          (acc_out.stride(0) if M else N) if acc_out is not None else 0, _stream())
    _check(st, "halo_gemm_i8")
    return out, acc_out


def gemm_desc(a: torch.Tensor, b: torch.Tensor, *, trans_b: bool, row_scale: Optional[torch.Tensor] = None,
              col_scale: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
              acc_out: Optional[torch.Tensor] = None, config: int = HALO_GEMM_AUTO) -> GemmDesc:
    """Marshal one product for halo_gemm_i8_desc / halo_gemm_i8_pair (the caller keeps the tensors alive)."""
    _need_cuda(a, b, row_scale, col_scale, out, acc_out)
    M, K = a.shape
    N = b.shape[0] if trans_b else b.shape[1]
    dp = lambda t: None if t is None else t.data_ptr()
    return GemmDesc(dp(a), a.stride(0), dp(b), b.stride(0), 1 if trans_b else 0, M, N, K, dp(row_scale), dp(col_scale),
                    dp(out), _dt(out.dtype) if out is not None else HALO_F32, out.stride(0) if out is not None else 0,
                    dp(acc_out), acc_out.stride(0) if acc_out is not None else 0, int(config))


def halo_gemm_i8_pair(g1: GemmDesc, g2: GemmDesc) -> None:
    """Two independent products in one launch."""
    st = load_library().halo_gemm_i8_pair(ctypes.byref(g1), ctypes.byref(g2), _stream())
    _check(st, "halo_gemm_i8_pair")


def halo_gemm_i8_desc(g: GemmDesc) -> None:
    """One product from a descriptor (tile configuration included)."""
    st = load_library().halo_gemm_i8_desc(ctypes.byref(g), _stream())
    _check(st, "halo_gemm_i8_desc")


def halo_mfma_i8_probe(operands: torch.Tensor, iters: int, sink: Optional[torch.Tensor] = None) -> float:
    """Launch the MFMA ceiling probe; returns the number of integer operations it performs."""
    _need_cuda(operands, sink)
    assert operands.dtype == torch.int8 and operands.numel() >= 4096 and operands.is_contiguous()
    st = load_library().halo_mfma_i8_probe(_ptr(operands), int(iters), _ptr(sink), _stream())
    _check(st, "halo_mfma_i8_probe")
    return 256.0 * 8 * iters * 16 * 65536.0


def halo_mx6_quant(x: torch.Tensor, *, had_block: int = 0, out_codes: Optional[torch.Tensor] = None,
                   out_scales: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """rotate -> E8M0 scale per 32 elements -> packed FP6 E3M2.  Returns (codes uint8 [rows, cols/32*24],
    scales uint8 [rows, cols/32])."""
    _need_cuda(x, out_codes, out_scales)
    assert x.dim() == 2 and x.stride(1) == 1 and x.dtype == torch.bfloat16
    rows, cols = x.shape
    if out_codes is None:
        out_codes = torch.empty((rows, cols // 32 * 24), dtype=torch.uint8, device=x.device)
    if out_scales is None:
        out_scales = torch.empty((rows, cols // 32), dtype=torch.uint8, device=x.device)
    st = load_library().halo_mx6_quant(_ptr(x), rows, cols, x.stride(0) if rows else cols, had_block, _ptr(out_codes),
                                       out_codes.stride(0) if rows else 24, _ptr(out_scales),
                                       out_scales.stride(0) if rows else 1, _stream())
    _check(st, "halo_mx6_quant")
    return out_codes, out_scales


def halo_gemm_mx6(a: torch.Tensor, sa: torch.Tensor, b: torch.Tensor, sb: torch.Tensor, *,
                  out_dtype: torch.dtype = torch.float32, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """C = A B^T on packed MXFP6 operands (codes [rows, K/32*24] uint8, scales [rows, K/32] uint8)."""
    _need_cuda(a, sa, b, sb, out)
    M, N, K = a.shape[0], b.shape[0], sa.shape[1] * 32
    assert a.shape[1] == K // 32 * 24 and b.shape[1] == K // 32 * 24 and sb.shape[1] * 32 == K
    if out is None:
        out = _empty_padded(M, N, out_dtype, a.device)
    st = load_library().halo_gemm_mx6(_ptr(a), a.stride(0) if M else 24, _ptr(sa), sa.stride(0) if M else 4, _ptr(b),
                                      b.stride(0) if N else 24, _ptr(sb), sb.stride(0) if N else 4, M, N, K, _ptr(out),
                                      _dt(out.dtype), out.stride(0) if M else N, _stream())
    _check(st, "halo_gemm_mx6")
    return out


def halo_dequant_unrotate(acc: torch.Tensor, row_scale: Optional[torch.Tensor], *, had_block: int = 0,
                          had_block_left: int = 0, out_dtype: torch.dtype = torch.float32,
                          out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                          tensor_scale: Optional[torch.Tensor] = None) -> torch.Tensor:
    lib = load_library()
    _need_cuda(acc, row_scale, out, workspace, tensor_scale)
    assert acc.dtype == torch.int32 and acc.dim() == 2
    rows, cols = acc.shape
    if out is None:
        out = _empty_padded(rows, cols, out_dtype, acc.device)
    need = lib.halo_dequant_unrotate_workspace_bytes(rows, cols, had_block_left)
    if workspace is None and need:
        workspace = torch.empty((need,), dtype=torch.uint8, device=acc.device)
    st = lib.halo_dequant_unrotate(_ptr(acc), acc.stride(0) if rows else cols, rows, cols, _ptr(row_scale),
                                   _ptr(tensor_scale), had_block, had_block_left, _ptr(out), _dt(out.dtype), out.stride(0) if rows else cols,
                                   _ptr(workspace), workspace.numel() if workspace is not None else 0, _stream())
    _check(st, "halo_dequant_unrotate")
    return out


@dataclass
class LinearState:
    """What the layer keeps between forward and backward (Section 3.2, Step 2): codes and scales only."""
    Xq: torch.Tensor
    s_x: torch.Tensor
    Wq: torch.Tensor
    s_w: torch.Tensor


def make_desc(b: int, m: int, n: int, level: int, out_dtype: torch.dtype = torch.bfloat16,
              had_block_m: int = 0, had_block_b: int = 0, scale_mode: int = HALO_SCALE_PER_ROW) -> LinearDesc:
    return LinearDesc(b, m, n, level, had_block_m, had_block_b, _dt(out_dtype), scale_mode)


def halo_linear_workspace_bytes(desc: LinearDesc) -> int:
    return int(load_library().halo_linear_workspace_bytes(ctypes.byref(desc)))


def halo_linear_fwd(desc: LinearDesc, X: Optional[torch.Tensor], W: Optional[torch.Tensor], *,
                    state: Optional[LinearState] = None, Y: Optional[torch.Tensor] = None,
                    workspace: Optional[torch.Tensor] = None):
    """Forward product; returns (Y, LinearState).  Pass X=None / W=None with a `state` that already holds
    the corresponding codes to reuse them."""
    lib = load_library()
    dev = (X if X is not None else state.Xq).device
    odt = torch.bfloat16 if desc.out_dt == HALO_BF16 else torch.float32
    if state is None:
        state = LinearState(torch.empty((desc.b, desc.m), dtype=torch.int8, device=dev),
                            torch.empty((desc.b,), dtype=torch.float32, device=dev),
                            torch.empty((desc.n, desc.m), dtype=torch.int8, device=dev),
                            torch.empty((desc.n,), dtype=torch.float32, device=dev))
    if Y is None:
        Y = torch.empty((desc.b, desc.n), dtype=odt, device=dev)
    _need_cuda(X, W, Y, state.Xq, state.Wq)
    for t in (X, W):
        assert t is None or (t.dtype == torch.bfloat16 and t.is_contiguous())
    if workspace is None and desc.scale_mode == HALO_SCALE_PER_TENSOR:
        workspace = torch.empty((max(halo_linear_workspace_bytes(desc), 16),), dtype=torch.uint8, device=dev)
    st = lib.halo_linear_fwd(ctypes.byref(desc), _ptr(X), _ptr(W), _ptr(Y), _ptr(state.Xq), _ptr(state.s_x),
                             _ptr(state.Wq), _ptr(state.s_w), _ptr(workspace),
                             workspace.numel() if workspace is not None else 0, _stream())
    _check(st, "halo_linear_fwd")
    return Y, state


def halo_linear_bwd(desc: LinearDesc, E: torch.Tensor, state: LinearState, *, want_ex: bool = True,
                    want_g: bool = True, workspace: Optional[torch.Tensor] = None,
                    EX: Optional[torch.Tensor] = None, G: Optional[torch.Tensor] = None):
    """Both backward products; returns (E_X or None, G or None)."""
    lib = load_library()
    _need_cuda(E, workspace, EX, G)
    assert E.dtype == torch.bfloat16 and E.is_contiguous()
    odt = torch.bfloat16 if desc.out_dt == HALO_BF16 else torch.float32
    if want_ex and EX is None:
        EX = torch.empty((desc.b, desc.m), dtype=odt, device=E.device)
    if want_g and G is None:
        G = torch.empty((desc.n, desc.m), dtype=odt, device=E.device)
    need = halo_linear_workspace_bytes(desc)
    if workspace is None:
        workspace = torch.empty((max(need, 1),), dtype=torch.uint8, device=E.device)
    st = lib.halo_linear_bwd(ctypes.byref(desc), _ptr(E), _ptr(state.Xq), _ptr(state.s_x), _ptr(state.Wq),
                             _ptr(state.s_w), _ptr(EX) if want_ex else None, _ptr(G) if want_g else None,
                             _ptr(workspace), workspace.numel(), _stream())
    _check(st, "halo_linear_bwd")
    return (EX if want_ex else None), (G if want_g else None)


def halo_peft_workspace_bytes(desc: LinearDesc, rank: int) -> int:
    return int(load_library().halo_peft_workspace_bytes(ctypes.byref(desc), int(rank)))


def halo_peft_fwd(desc: LinearDesc, X: torch.Tensor, Wq: torch.Tensor, s_w: torch.Tensor, U: torch.Tensor,
                  V: torch.Tensor, *, workspace: Optional[torch.Tensor] = None, Y: Optional[torch.Tensor] = None,
                  T: Optional[torch.Tensor] = None):
    """Forward pass of the LoRA-style module on a frozen quantised weight; returns (Y, T = X U^T in fp32)."""
    lib = load_library()
    _need_cuda(X, Wq, s_w, U, V, workspace, Y, T)
    rank = U.shape[0]
    assert X.dtype == torch.bfloat16 and U.dtype == torch.bfloat16 and V.dtype == torch.bfloat16
    assert X.is_contiguous() and U.is_contiguous() and V.is_contiguous() and Wq.is_contiguous()
    assert tuple(V.shape) == (desc.n, rank) and tuple(U.shape) == (rank, desc.m)
    odt = torch.bfloat16 if desc.out_dt == HALO_BF16 else torch.float32
    if Y is None:
        Y = torch.empty((desc.b, desc.n), dtype=odt, device=X.device)
    if T is None:
        T = torch.empty((desc.b, rank), dtype=torch.float32, device=X.device)
    if workspace is None:
        workspace = torch.empty((max(halo_peft_workspace_bytes(desc, rank), 1),), dtype=torch.uint8, device=X.device)
    st = lib.halo_peft_fwd(ctypes.byref(desc), rank, _ptr(X), _ptr(Wq), _ptr(s_w), _ptr(U), _ptr(V), _ptr(Y), _ptr(T),
                           _ptr(workspace), workspace.numel(), _stream())
    _check(st, "halo_peft_fwd")
    return Y, T


def halo_peft_bwd(desc: LinearDesc, E: torch.Tensor, X: torch.Tensor, T: torch.Tensor, Wq: torch.Tensor,
                  s_w: torch.Tensor, U: torch.Tensor, V: torch.Tensor, *, want_ex: bool = True, want_gu: bool = True,
                  want_gv: bool = True, workspace: Optional[torch.Tensor] = None, EX: Optional[torch.Tensor] = None,
                  GU: Optional[torch.Tensor] = None, GV: Optional[torch.Tensor] = None):
    """Backward pass of the module; returns (E_X, G_U [rank x m] fp32, G_V [n x rank] fp32), None where not wanted."""
    lib = load_library()
    _need_cuda(E, X, T, Wq, s_w, U, V, workspace, EX, GU, GV)
    rank = U.shape[0]
    assert E.dtype == torch.bfloat16 and E.is_contiguous()
    odt = torch.bfloat16 if desc.out_dt == HALO_BF16 else torch.float32
    if want_ex and EX is None:
        EX = torch.empty((desc.b, desc.m), dtype=odt, device=E.device)
    if want_gu and GU is None:
        GU = torch.empty((rank, desc.m), dtype=torch.float32, device=E.device)
    if want_gv and GV is None:
        GV = torch.empty((desc.n, rank), dtype=torch.float32, device=E.device)
    if workspace is None:
        workspace = torch.empty((max(halo_peft_workspace_bytes(desc, rank), 1),), dtype=torch.uint8, device=E.device)
    st = lib.halo_peft_bwd(ctypes.byref(desc), rank, _ptr(E), _ptr(X), _ptr(T), _ptr(Wq), _ptr(s_w), _ptr(U), _ptr(V),
                           _ptr(EX) if want_ex else None, _ptr(GU) if want_gu else None, _ptr(GV) if want_gv else None,
                           _ptr(workspace), workspace.numel(), _stream())
    _check(st, "halo_peft_bwd")
    return (EX if want_ex else None), (GU if want_gu else None), (GV if want_gv else None)
