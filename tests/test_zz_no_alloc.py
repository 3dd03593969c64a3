"""The workspace-free backward entry point (for callers that cannot allocate device memory) against
the ordinary one, through the C ABI: same dx bit for bit, same ds bit for bit (same kernel, same
grid, same reduction order), on two calls in a row, the second with a smaller input, so that
whatever the first call left in the library's device array cannot leak into the second."""
from __future__ import annotations

import ctypes
import os

import numpy as np
import pytest
import torch

from paper_2512_14481_amd import binding as B

pytestmark = pytest.mark.gpu

i64 = ctypes.c_int64


def _call_static(lib, x, dy, s, dx, ds, bits, dt):
    rows, cols = x.shape
    lib.sasq_fakequant_bwd_static.argtypes = [ctypes.c_void_p] * 5 + [i64, i64, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    return lib.sasq_fakequant_bwd_static(x.data_ptr(), dy.data_ptr(), s.data_ptr(), dx.data_ptr() if dx is not None else None,
                                         ds.data_ptr(), rows, cols, bits, dt,
                                         ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))


def _call_ws(lib, x, dy, s, dx, ds, ws, bits, dt):
    rows, cols = x.shape
    lib.sasq_fakequant_bwd.argtypes = [ctypes.c_void_p] * 5 + [i64, i64, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                                                ctypes.c_size_t, ctypes.c_void_p]
    return lib.sasq_fakequant_bwd(x.data_ptr(), dy.data_ptr(), s.data_ptr(), dx.data_ptr() if dx is not None else None,
                                  ds.data_ptr(), rows, cols, bits, dt, ws.data_ptr(), ws.numel(),
                                  ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_static_backward_matches_workspace_backward_twice(dtype):
    lib = ctypes.CDLL(B.LIB_PATH)
    dt = B.SASQ_F16 if dtype == torch.float16 else B.SASQ_BF16
    gen = torch.Generator(device="cuda").manual_seed(1234)
    ws = B.new_workspace(B.sasq_fakequant_bwd_workspace(1, 1))
    # a large input (every block busy, several chunks per block, ragged tail), then a small one
    # (fewer blocks than the first call used), then the large one again
    for rows, cols in ((3001, 1027), (37, 251), (3001, 1027)):
        x = (torch.randn((rows, cols), device="cuda", generator=gen) * 3.0).to(dtype)
        dy = torch.randn((rows, cols), device="cuda", generator=gen).to(dtype)
        s = torch.tensor([0.0371], dtype=torch.float32, device="cuda")
        dx_a, dx_b = torch.full_like(x, 7.0), torch.full_like(x, -7.0)
        ds_a = torch.full((1,), 123.0, dtype=torch.float32, device="cuda")
        ds_b = torch.full((1,), -123.0, dtype=torch.float32, device="cuda")
        assert _call_ws(lib, x, dy, s, dx_a, ds_a, ws, 8, dt) == 0
        assert _call_static(lib, x, dy, s, dx_b, ds_b, 8, dt) == 0
        torch.cuda.synchronize()
        assert torch.equal(dx_a.view(torch.int16), dx_b.view(torch.int16)), (rows, cols)
        assert np.array_equal(ds_a.cpu().numpy().view(np.uint32), ds_b.cpu().numpy().view(np.uint32)), (rows, cols)
        # ds only (dx = NULL) takes the other kernel instantiation
        ds_c = torch.zeros(1, dtype=torch.float32, device="cuda")
        assert _call_static(lib, x, dy, s, None, ds_c, 8, dt) == 0
        torch.cuda.synchronize()
        assert np.array_equal(ds_a.cpu().numpy().view(np.uint32), ds_c.cpu().numpy().view(np.uint32)), (rows, cols)


def test_static_backward_rejects_bad_arguments():
    lib = ctypes.CDLL(B.LIB_PATH)
    x = torch.zeros((8, 8), dtype=torch.float16, device="cuda")
    s = torch.ones(1, dtype=torch.float32, device="cuda")
    ds = torch.zeros(1, dtype=torch.float32, device="cuda")
    f = lib.sasq_fakequant_bwd_static
    f.argtypes = [ctypes.c_void_p] * 5 + [i64, i64, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    assert f(None, x.data_ptr(), s.data_ptr(), None, ds.data_ptr(), 8, 8, 8, 0, None) == 1          # NULL
    assert f(x.data_ptr(), x.data_ptr(), s.data_ptr(), None, ds.data_ptr(), 0, 8, 8, 0, None) == 2  # shape
    assert f(x.data_ptr(), x.data_ptr(), s.data_ptr(), None, ds.data_ptr(), 1 << 21, 1 << 20, 8, 0, None) == 2   # above the maximum
    assert f(x.data_ptr(), x.data_ptr(), s.data_ptr(), None, ds.data_ptr(), 8, 8, 9, 0, None) == 4  # bits
    assert f(x.data_ptr() + 2, x.data_ptr(), s.data_ptr(), None, ds.data_ptr(), 8, 4, 8, 0, None) == 3   # alignment
