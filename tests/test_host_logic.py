"""CPU-only checks of the C-ABI library's host side: it loads, exports every symbol the header
declares, lists kept modes bit-for-bit like the oracle, sizes workspaces and rejects bad
arguments without touching a device."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import fno_oracle as O
from paper_2204_01205_amd import binding as B
from paper_2204_01205_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "fno.h")).read()
    declared = set(re.findall(r"\b(fno_[a-z0-9_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    lib = B.lib()
    for name in declared:
        assert hasattr(lib, name), name


def test_no_product_module_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2204_01205_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
    oracle_src = open(os.path.join(ROOT, "oracle", "fno_oracle.py")).read()
    assert "paper_2204_01205_amd" not in oracle_src.replace("the product package", "")


@pytest.mark.parametrize("grid,modes,rule", [
    ((16, 16, 16, 8), (4, 4, 4, 3), 0), ((64, 64, 64, 16), (12, 12, 12, 8), 0),
    ((128, 128, 64, 32), (16, 16, 12, 9), 0), ((256, 256, 128, 32), (24, 24, 16, 9), 0),
    ((128, 128, 128, 16), (16, 16, 16, 9), 0), ((9, 7, 5, 11), (4, 3, 2, 6), 1),
    ((6, 6, 6, 6), (3, 3, 3, 4), 0), ((5, 5, 5, 5), (0, 0, 0, 1), 1)])
def test_mode_indices_bit_exact_against_oracle(grid, modes, rule):
    d = B.make_desc(1, 4, 4, grid, modes, rule)
    want = O.mode_lists(O.LayerSpec(grid, modes, rule))
    for axis in range(4):
        assert B.fno_mode_indices(d, axis) == want[axis]


def test_workspace_sizes_and_config_table():
    for name, c in synth.CONFIGS.items():
        d = B.make_desc(c["batch"], c["width"], c["width"], c["grid"], c["modes"])
        sizes = [B.fno_workspace_bytes(d, op) for op in range(4)]
        assert all(s > 0 and s % 256 == 0 for s in sizes)
        assert sizes[3] > sizes[2] >= sizes[0]
        assert list(B.kept_counts(d)) == [len(k) for k in O.mode_lists(O.LayerSpec(c["grid"], c["modes"], 0))]
    # the largest workload's forward workspace stays far below one activation
    c = synth.CONFIGS["cfg4"]
    d = B.make_desc(1, 20, 20, c["grid"], c["modes"])
    act_bytes = 4 * 20 * int(np.prod(c["grid"]))
    assert B.fno_workspace_bytes(d, B.FNO_OP_BLOCK_FWD) < 0.25 * act_bytes


def _status(fn, *args):
    return fn(*args)


def test_argument_errors_return_codes_without_a_device():
    lib = B.lib()
    good = B.make_desc(1, 4, 4, (8, 8, 8, 8), (2, 2, 2, 3))
    n = ctypes.c_size_t(0)
    assert lib.fno_workspace_bytes(None, 0, ctypes.byref(n)) == B.FNO_EINVAL
    assert lib.fno_workspace_bytes(ctypes.byref(good), 9, ctypes.byref(n)) == B.FNO_EINVAL
    assert lib.fno_workspace_bytes(ctypes.byref(good), 0, None) == B.FNO_EINVAL
    bad = [
        B.make_desc(0, 4, 4, (8, 8, 8, 8), (2, 2, 2, 3)),          # batch
        B.make_desc(1, 4, 4, (8, 8, 8, 8), (5, 2, 2, 3)),          # L = 10 > N = 8
        B.make_desc(1, 4, 4, (8, 8, 8, 8), (2, 2, 2, 6)),          # mt > Nt/2+1
        B.make_desc(1, 4, 4, (8, 8, 8, 8), (2, 2, 2, 0)),          # mt = 0
        B.make_desc(1, 4, 4, (8, 8, 0, 8), (2, 2, 2, 3)),          # empty axis
        B.make_desc(1, 4, 4, (8, 8, 8, 8), (2, 2, 2, 3), 2),       # mode rule
        B.make_desc(1, 4, 4, (8, 8, 8, 8), (2, 2, 2, 3), 0, 7),    # activation
        B.make_desc(1, 4, 4, (8, 8, 8, 8), (2, 2, 2, 3), 0, 1, 64),  # flags
        B.make_desc(1, 4, 4, (8, 8, 8, 8), (0, 2, 2, 3), 0),       # L = 0 under rule 0
    ]
    for d in bad:
        assert lib.fno_workspace_bytes(ctypes.byref(d), 0, ctypes.byref(n)) == B.FNO_EINVAL
        assert len(B.fno_status_string(B.FNO_EINVAL)) > 0
    # block calls need equal widths; spectral conv does not
    uneven = B.make_desc(1, 3, 5, (8, 8, 8, 8), (2, 2, 2, 3))
    assert lib.fno_workspace_bytes(ctypes.byref(uneven), B.FNO_OP_SPECTRAL_CONV_FWD, ctypes.byref(n)) == B.FNO_OK
    assert lib.fno_workspace_bytes(ctypes.byref(uneven), B.FNO_OP_BLOCK_FWD, ctypes.byref(n)) == B.FNO_EINVAL
    wide = B.make_desc(1, 40, 40, (8, 8, 8, 8), (2, 2, 2, 3))
    assert lib.fno_workspace_bytes(ctypes.byref(wide), 0, ctypes.byref(n)) == B.FNO_EUNSUPPORTED
    # null data pointers and a missing workspace are refused before any launch
    z = ctypes.c_void_p(0)
    one = ctypes.c_void_p(256)
    sz = ctypes.c_size_t(1 << 40)
    assert lib.fno_spectral_conv_fwd(ctypes.byref(good), z, one, one, z, one, sz, z) == B.FNO_EINVAL
    assert lib.fno_spectral_conv_fwd(ctypes.byref(good), one, one, one, z, z, sz, z) == B.FNO_EINVAL
    assert lib.fno_spectral_conv_fwd(ctypes.byref(good), one, one, one, z, one, ctypes.c_size_t(16), z) == B.FNO_ENOSPC
    assert lib.fno_spectral_conv_fwd(ctypes.byref(good), one, one, one, z, ctypes.c_void_p(260), sz, z) == B.FNO_ENOSPC
    assert lib.fno_block_fwd(ctypes.byref(good), one, one, z, z, one, z, z, one, sz, z) == B.FNO_EINVAL
    assert lib.fno_block_bwd(ctypes.byref(good), one, one, one, z, z, one, one, one, one, one, one, sz, z) == B.FNO_EINVAL
    assert lib.fno_spectral_conv_bwd(ctypes.byref(good), z, z, one, one, one, one, one, sz, z) == B.FNO_EINVAL
    assert lib.fno_pointwise_linear(1, 4, 40, ctypes.c_int64(10), one, one, z, one, z) == B.FNO_EUNSUPPORTED
    assert lib.fno_pointwise_mlp2(1, 4, 8, 9, ctypes.c_int64(10), one, one, z, one, z, one, z) == B.FNO_EUNSUPPORTED
    assert B.fno_status_string(0) == "ok"


def test_binding_refuses_cpu_tensors():
    import torch
    d = B.make_desc(1, 2, 2, (4, 4, 4, 4), (1, 1, 1, 2))
    x = torch.zeros(1, 2, 4, 4, 4, 4)
    with pytest.raises(ValueError):
        B.fno_spectral_conv_fwd(d, x, x, x, None, torch.zeros(1024, dtype=torch.uint8))


def test_synthetic_inputs_are_reproducible_and_exact():
    a = synth.normal_field(3, synth.T_X, 2, 2, (4, 3, 2, 5))
    b = synth.normal_field(3, synth.T_X, 2, 2, (4, 3, 2, 5))
    assert a.dtype == np.float32 and np.array_equal(a, b)
    f = synth.separable_factors(1, 2, 3, (6, 5, 4, 8))
    field = synth.rank_one_field(f)
    exact = (f[0].astype(np.float64)[:, :, :, None, None, None] * f[1].astype(np.float64)[:, :, None, :, None, None]
             * f[2].astype(np.float64)[:, :, None, None, :, None] * f[3].astype(np.float64)[:, :, None, None, None, :])
    assert np.array_equal(field.astype(np.float64), exact)
    r = synth.spectral_weights(0, 4, 4, (2, 2, 2, 3))
    assert r.dtype == np.complex64 and abs(np.std(r.real) - 0.25) < 0.05


def test_binding_rejects_tensors_whose_size_does_not_match_the_descriptor():
    """The kernels index by the descriptor alone; the binding refuses a mis-sized tensor on the host
    (checked here with CPU tensors: the size check comes before the device check)."""
    import pytest
    import torch
    desc = B.make_desc(1, 2, 2, (4, 4, 4, 4), (1, 1, 1, 2))
    npts, kept = B._sizes(desc)
    assert (npts, kept) == (256, 2 * 2 * 2 * 2)
    good = torch.zeros((1, 2, 4, 4, 4, 4))
    B._check_layer_tensors(desc, x=good, y=good, R=torch.zeros((2, 2, 2, 2, 2, 2), dtype=torch.complex64))
    with pytest.raises(ValueError, match="x holds"):
        B._check_layer_tensors(desc, x=torch.zeros((1, 2, 4, 4, 4, 3)), y=good)
    with pytest.raises(ValueError, match="R holds"):
        B._check_layer_tensors(desc, x=good, R=torch.zeros((2, 2, 2, 2, 2, 1), dtype=torch.complex64))
    with pytest.raises(ValueError, match="xhat holds"):
        B._check_layer_tensors(desc, x=good, xhat=torch.zeros((1, 2, 2, 2, 2, 3), dtype=torch.complex64))


def test_plan_tables_checks_its_arguments_on_the_host():
    import ctypes
    desc = B.make_desc(1, 2, 2, (4, 4, 4, 4), (1, 1, 1, 2))
    n = ctypes.c_size_t(B.fno_workspace_bytes(desc, B.FNO_OP_BLOCK_FWD))
    null = ctypes.c_void_p(0)
    assert B.lib().fno_plan_tables(ctypes.byref(desc), ctypes.c_int(B.FNO_OP_BLOCK_FWD), null, n, null) == B.FNO_EINVAL
    assert B.lib().fno_plan_tables(ctypes.byref(desc), ctypes.c_int(9), null, n, null) == B.FNO_EINVAL
    bad = B.make_desc(1, 2, 2, (4, 4, 4, 4), (3, 1, 1, 2))          # 6 kept modes on an axis of 4
    assert B.lib().fno_plan_tables(ctypes.byref(bad), ctypes.c_int(B.FNO_OP_BLOCK_FWD), null, n, null) == B.FNO_EINVAL
    misaligned = ctypes.c_void_p(64)
    assert B.lib().fno_plan_tables(ctypes.byref(desc), ctypes.c_int(B.FNO_OP_BLOCK_FWD), misaligned, n, null) == B.FNO_ENOSPC
