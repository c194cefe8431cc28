"""The entry point that allocates nothing, fno_spectral_conv_fwd_static, against the entry point it
is a variant of, fno_spectral_conv_fwd: same kernels, the workspace in the library's static device
array instead of a caller's buffer.  Two calls in a row, the second on a smaller input (the array
keeps the first call's contents), each bit-equal to the workspace variant and within the layer's
tolerance of the oracle; shapes beyond the array are refused before anything is launched.
"""
import numpy as np
import pytest
import torch

from oracle import fno_oracle as O
from paper_2204_01205_amd import binding as B
from paper_2204_01205_amd import synth

pytestmark = pytest.mark.gpu
TOL = 1e-5


def rel(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return float(np.linalg.norm((a - b).ravel()) / np.linalg.norm(b.ravel()))


def run_pair(seed, batch, width, grid, modes):
    counts = tuple(len(k) for k in O.mode_lists(O.LayerSpec(grid, modes, 0)))
    x = synth.normal_field(seed, synth.T_X, batch, width, grid)
    R = synth.spectral_weights(seed, width, width, counts)
    desc = B.make_desc(batch, width, width, grid, modes, 0, B.FNO_ACT_IDENTITY)
    assert B.fno_workspace_bytes(desc, B.FNO_OP_SPECTRAL_CONV_FWD) <= B.FNO_STATIC_SCRATCH_BYTES
    dx, dR = torch.from_numpy(x).cuda(), torch.from_numpy(R).cuda()
    y_static = torch.full_like(dx, float("nan"))
    xh_static = torch.full((batch, width) + counts, float("nan"), dtype=torch.complex64, device="cuda")
    before = torch.cuda.memory_allocated()
    B.fno_spectral_conv_fwd_static(desc, dx, dR, y_static, xh_static)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    ws = B.alloc_workspace(desc, B.FNO_OP_SPECTRAL_CONV_FWD)
    y_ws = torch.empty_like(dx)
    xh_ws = torch.empty_like(xh_static)
    B.fno_spectral_conv_fwd(desc, dx, dR, y_ws, xh_ws, ws)
    torch.cuda.synchronize()
    assert torch.equal(y_static, y_ws)
    assert torch.equal(torch.view_as_real(xh_static), torch.view_as_real(xh_ws))
    want, xhat = O.spectral_conv_fwd(x, R, O.LayerSpec(grid, modes, 0), return_xhat=True)
    assert rel(y_static.cpu().numpy(), want) <= TOL
    got_xh = xh_static.cpu().numpy()
    assert float(np.linalg.norm((got_xh - xhat).ravel()) / np.linalg.norm(xhat.ravel())) <= TOL


def test_static_scratch_entry_point_two_calls_second_smaller():
    run_pair(21, 2, 8, (32, 32, 32, 16), (8, 8, 8, 8))      # 36.5 MB of the array
    run_pair(22, 1, 8, (16, 16, 16, 8), (4, 4, 4, 3))       # then 1.3 MB of it


def test_static_scratch_entry_point_refuses_shapes_beyond_the_array():
    grid, modes, width, batch = (64, 64, 64, 16), (12, 12, 12, 8), 20, 2
    desc = B.make_desc(batch, width, width, grid, modes, 0, B.FNO_ACT_IDENTITY)
    assert B.fno_workspace_bytes(desc, B.FNO_OP_SPECTRAL_CONV_FWD) > B.FNO_STATIC_SCRATCH_BYTES
    counts = tuple(len(k) for k in O.mode_lists(O.LayerSpec(grid, modes, 0)))
    x = torch.zeros((batch, width) + grid, device="cuda")
    R = torch.zeros((width, width) + counts, dtype=torch.complex64, device="cuda")
    y = torch.full_like(x, 7.0)
    with pytest.raises(B.FnoError) as err:
        B.fno_spectral_conv_fwd_static(desc, x, R, y, None)
    assert err.value.status == B.FNO_ENOSPC
    assert "static array" in str(err.value)
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())
