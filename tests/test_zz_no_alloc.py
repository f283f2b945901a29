"""The entry point that allocates nothing (deinfer_lowrank_linear_static: scratch in a static device
array of the library) against deinfer_lowrank_linear with a caller's workspace, through the C ABI:
same kernels, so the outputs must be identical bit for bit, and both must meet the oracle's bar.
Two calls in a row, the second with a smaller input (the array keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest

import oracle
import synth_inputs as si
from gpu_util import TOL, max_err, pair, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dn():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2604_17709_amd as dn
    dn.lib()
    return dn


def _both(dn, seed, T, d_in, r, d_out):
    import torch
    x = si.make(seed, 1, (T, d_in), 1.0, "bf16")
    U = si.make(seed, 2, (d_in, r), 1.0 / np.sqrt(d_in), "bf16")
    V = si.make(seed, 3, (r, d_out), 1.0 / np.sqrt(r), "bf16")
    p, keep = pair(dn, U, V, packed=True)
    xd = to_dev(x)
    L = dn.lib()
    y_static = torch.full((T, d_out), 7.0, dtype=torch.bfloat16, device="cuda")
    torch.cuda.synchronize()
    rc = L.deinfer_lowrank_linear_static(xd.data_ptr(), T, xd.stride(0), ctypes.byref(p.desc),
                                         y_static.data_ptr(), y_static.stride(0), None)
    assert rc == dn.OK, dn.last_error()
    torch.cuda.synchronize()
    ws = dn.Workspace(dn.deinfer_workspace_bytes(T, [p]))
    y_ws = torch.full((T, d_out), 3.0, dtype=torch.bfloat16, device="cuda")
    rc = L.deinfer_lowrank_linear(xd.data_ptr(), T, xd.stride(0), ctypes.byref(p.desc),
                                  y_ws.data_ptr(), y_ws.stride(0), ws.buf.data_ptr(), ws.nbytes, None)
    assert rc == dn.OK, dn.last_error()
    ws.check()
    assert torch.equal(y_static.view(torch.int16), y_ws.view(torch.int16))
    ref = oracle.lowrank_linear(x.values, U.values, V.values)
    assert max_err(to_host(y_static), ref) <= TOL["bf16"]
    return p, keep


def test_static_scratch_entry_point_matches_the_workspace_one(dn):
    import torch
    # every schedule: T <= 8 (tile kernels), <= 32 / <= 128 (streaming kernels with partial sums), > 128 (large tiles with a k-split)
    for seed, (T, d_in, r, d_out) in enumerate([(128, 1024, 300, 2048), (40, 1024, 300, 2048), (200, 2048, 96, 512),
                                                 (8, 512, 100, 640), (1, 512, 100, 640)]):
        _both(dn, 40 + seed, T, d_in, r, d_out)
    # a second pass in the opposite order: a larger call after smaller ones
    _both(dn, 50, 3, 256, 40, 96)
    p, keep = _both(dn, 51, 100, 2048, 520, 1024)
    # sizes beyond the static array are refused with a clear error and nothing is enqueued
    L = dn.lib()
    big_T = 1 << 20
    FP = ctypes.POINTER(dn.Factors)
    assert dn.deinfer_workspace_bytes(big_T, [p]) > dn.STATIC_SCRATCH_BYTES
    rc = L.deinfer_lowrank_linear_static(0x1000, big_T, 2048, ctypes.byref(p.desc), 0x2000, 1024, None)
    assert rc == dn.ERR_WORKSPACE and "static scratch" in dn.last_error()
    # T == 0 is a no-op
    assert L.deinfer_lowrank_linear_static(0x1000, 0, 2048, ctypes.byref(p.desc), 0x2000, 1024, None) == dn.OK
    torch.cuda.synchronize()
