"""The slab-by-slab evaluation of the oracle (tests/fullsize_oracle.py, used for parity at the
full sizes of the large workloads) returns what the oracle's whole-tensor functions return.
Small grids, even and odd sizes, both through the worker pool."""
import numpy as np
import pytest

from oracle import fno_oracle as O
from paper_2204_01205_amd import synth
from tests import fullsize_oracle as F

TIGHT = 1e-12


@pytest.fixture(scope="module")
def pool():
    with F.SlabPool(nproc=2, threads=1) as p:
        yield p


def problem(seed, batch, width, grid, modes):
    spec = O.LayerSpec(grid, modes, 0)
    counts = tuple(len(k) for k in O.mode_lists(spec))
    x = synth.normal_field(seed, synth.T_X, batch, width, grid)
    r = synth.spectral_weights(seed, width, width, counts)
    w = synth.linear_weights(seed, width, width)
    b = synth.bias(seed, width)
    return spec, x, r, w, b


@pytest.mark.parametrize("batch,width,grid,modes", [(2, 3, (8, 6, 8, 8), (2, 2, 3, 4)), (1, 4, (9, 5, 6, 7), (2, 1, 2, 3))])
def test_streamed_block_forward_and_backward_equal_the_whole_tensor_oracle(pool, batch, width, grid, modes):
    spec, x, r, w, b = problem(3, batch, width, grid, modes)
    out, z, xhat = O.block_fwd(x, r, w, b, spec)
    s_out, s_z, s_xhat = F.block_fwd_streamed(pool, x, r, w, b, spec)
    assert F.rel_l2(s_xhat, xhat) <= TIGHT
    assert F.rel_l2(F.stack_slabs(s_z, batch, width), z) <= TIGHT
    assert F.rel_l2(F.stack_slabs(s_out, batch, width), out) <= TIGHT
    # a subset of output slabs only
    some = [(batch - 1, 1), (0, width - 1)]
    p_out, _, _ = F.block_fwd_streamed(pool, x, r, w, b, spec, which=some)
    assert sorted(p_out) == sorted(some)
    for (bb, o) in some:
        assert F.rel_l2(p_out[(bb, o)], out[bb, o]) <= TIGHT

    target = synth.normal_field(3, synth.T_TARGET, batch, width, grid)
    gout = O.mse_grad(out, target)
    ref = O.block_bwd(x, r, w, b, gout, spec)
    got = F.block_bwd_streamed(pool, x, r, w, z, xhat, gout, spec)
    for key in ("gx", "gR", "gW", "gb"):
        assert F.rel_l2(got[key], ref[key]) <= TIGHT, key

    # batch entries one at a time, the cotangent of the whole-batch mean: sums over the batch add up
    acc = {k: 0.0 for k in ("gR", "gW", "gb")}
    for bb in range(batch):
        sl = slice(bb, bb + 1)
        o1, z1, xh1 = O.block_fwd(x[sl], r, w, b, spec)
        g1 = O.mse_grad(o1, target[sl]) / batch
        part = F.block_bwd_streamed(pool, x[sl], r, w, z1, xh1, g1, spec)
        assert F.rel_l2(part["gx"], ref["gx"][sl]) <= TIGHT
        for k in acc:
            acc[k] = acc[k] + part[k]
    for k in acc:
        assert F.rel_l2(acc[k], ref[k]) <= TIGHT, k


def test_streamed_network_forward_equals_the_whole_tensor_oracle(pool):
    grid, modes, width = (8, 8, 4, 8), (2, 2, 1, 3), 4
    spec = O.LayerSpec(grid, modes, 0)
    counts = tuple(len(k) for k in O.mode_lists(spec))
    a = synth.normal_field(1, synth.T_X, 1, 5, grid)
    lw, lb = synth.linear_weights(0, width, 5, synth.T_LIFT), synth.bias(0, width, synth.T_LIFT)
    blocks = [(synth.spectral_weights(10 + k, width, width, counts), synth.linear_weights(10 + k, width, width),
               synth.bias(10 + k, width)) for k in range(3)]
    proj = (synth.linear_weights(1, 16, width, synth.T_PROJ), synth.bias(1, 16, synth.T_PROJ),
            synth.linear_weights(2, 1, 16, synth.T_PROJ), synth.bias(2, 1, synth.T_PROJ))
    want = O.fno_forward(a, lw, lb, blocks, proj, spec)
    got = F.fno_forward_streamed(pool, a, lw, lb, blocks, proj, spec)
    assert F.rel_l2(got, want) <= TIGHT


def test_seeded_worker_slabs_are_the_generator_slabs(pool):
    grid, modes = (6, 4, 8, 8), (1, 1, 2, 3)
    spec = O.LayerSpec(grid, modes, 0)
    keys = [(7, synth.T_X, 1, 2), (7, synth.T_X, 0, 0)]
    got = pool.forward_seeded_async(keys, spec).get()
    x = synth.normal_field(7, synth.T_X, 2, 3, grid)
    assert F.rel_l2(got[0], O.forward_spectrum(x[1, 2], spec)) <= TIGHT
    assert F.rel_l2(got[1], O.forward_spectrum(x[0, 0], spec)) <= TIGHT
