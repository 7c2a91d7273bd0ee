"""GPU: halo_quant_dual_static (the allocation-free entry point, scratch in a device array built into the library)
against halo_quant_dual, bit for bit, on two calls in a row, the second with a smaller input."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2501_02625_amd import binding, inputs
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _both(rows, cols, seed):
    e = inputs.make_errors(rows, (cols + 7) // 8 * 8, seed)[:, :cols]
    e[:, 2] = 0
    fc = (np.abs(np.random.default_rng(seed).standard_normal(cols)) * 1e-2 + 1e-4).astype(np.float32)
    fr = (np.abs(np.random.default_rng(seed + 1).standard_normal(rows)) * 0.5 + 0.01).astype(np.float32)
    ld = (cols + 7) // 8 * 8
    Ef = torch.zeros((rows, ld), dtype=torch.bfloat16, device=gu.DEV)
    Ef[:, :cols] = gu.bits_to_dev(np.ascontiguousarray(e))
    E, dfc, dfr = Ef[:, :cols], gu.to_dev(fc), gu.to_dev(fr)
    want = binding.halo_quant_dual(E, fold_cols=dfc, fold_rows=dfr)
    pad16 = lambda v: (v + 15) // 16 * 16       # leading dimensions of the code matrices: multiples of 16 bytes
    got = (torch.full((rows, pad16(cols)), 99, dtype=torch.int8, device=gu.DEV)[:, :cols],
           torch.full((rows,), -1.0, device=gu.DEV),
           torch.full((cols, pad16(rows)), 99, dtype=torch.int8, device=gu.DEV)[:, :rows],
           torch.full((cols,), -1.0, device=gu.DEV))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    binding.halo_quant_dual_static(E, fold_cols=dfc, fold_rows=dfr, out_q=got[0], row_scale=got[1], out_qt=got[2],
                                   col_scale=got[3])
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for g, w, what in zip(got, want, ("row codes", "row scales", "column codes", "column scales")):
        assert torch.equal(g, w), "%s differ between halo_quant_dual_static and halo_quant_dual (%dx%d)" % (what, rows, cols)


def test_static_scratch_entry_point_matches_the_workspace_one_twice_in_a_row():
    _both(2048, 4096, 11)        # config c2's E
    _both(130, 200, 12)          # smaller and ragged: the array still holds the first call's partial maxima
    _both(1024, 1536, 13)


def test_static_scratch_entry_point_refuses_sizes_beyond_its_array():
    lib = binding.load_library()
    cap = lib.halo_quant_dual_static_max_workspace_bytes()
    assert cap == 8 << 20
    rows, cols = 8192, 14336
    assert lib.halo_quant_dual_workspace_bytes(rows, cols) > cap
    P = ctypes.c_void_p(0x1000)
    st = lib.halo_quant_dual_static(P, rows, cols, cols, None, None, P, cols, P, P, rows, P, None)
    assert st == binding.HALO_EWORKSPACE
