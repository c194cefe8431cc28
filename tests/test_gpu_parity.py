"""GPU parity: the HIP path through the C ABI against the float64 oracle on the same seeded
inputs.  Floating point bar: relative L2 error <= 1e-5 per output tensor (fp32 arithmetic);
mode bookkeeping is covered bit-exactly in test_host_logic.py."""
import numpy as np
import pytest
import torch

from oracle import fno_oracle as O
from paper_2204_01205_amd import binding as B
from paper_2204_01205_amd import synth

pytestmark = pytest.mark.gpu
TOL = 1e-5


def rel(a, b):
    a = np.asarray(a)
    b = np.asarray(b)
    return float(np.linalg.norm((a - b).ravel()) / max(np.linalg.norm(b.ravel()), 1e-300))


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.cpu().numpy()


class Layer:
    """Seeded inputs of one layer, on both sides."""

    def __init__(self, batch, c_in, c_out, grid, modes, rule=0, seed=0, activation=B.FNO_ACT_GELU):
        self.spec = O.LayerSpec(tuple(grid), tuple(modes), rule)
        self.counts = tuple(len(k) for k in O.mode_lists(self.spec))
        self.batch, self.c_in, self.c_out = batch, c_in, c_out
        self.act = activation
        self.x = synth.normal_field(seed, synth.T_X, batch, c_in, grid)
        self.R = synth.spectral_weights(seed, c_in, c_out, self.counts)
        self.W = synth.linear_weights(seed, c_out, c_in)
        self.b = synth.bias(seed, c_out)
        self.desc = B.make_desc(batch, c_in, c_out, grid, modes, rule, activation)

    def act_name(self):
        return "gelu" if self.act == B.FNO_ACT_GELU else "identity"


def gpu_spectral_fwd(L, x=None):
    x = dev(L.x if x is None else x)
    y = torch.empty((L.batch, L.c_out) + L.spec.grid, device="cuda")
    xh = torch.empty((L.batch, L.c_in) + L.counts, dtype=torch.complex64, device="cuda")
    ws = B.alloc_workspace(L.desc, B.FNO_OP_SPECTRAL_CONV_FWD)
    B.fno_spectral_conv_fwd(L.desc, x, dev(L.R), y, xh, ws)
    torch.cuda.synchronize()
    return host(y), host(xh)


def gpu_block_fwd(L):
    out = torch.empty((L.batch, L.c_out) + L.spec.grid, device="cuda")
    z = torch.empty_like(out)
    xh = torch.empty((L.batch, L.c_in) + L.counts, dtype=torch.complex64, device="cuda")
    ws = B.alloc_workspace(L.desc, B.FNO_OP_BLOCK_FWD)
    B.fno_block_fwd(L.desc, dev(L.x), dev(L.R), dev(L.W), dev(L.b), out, z, xh, ws)
    torch.cuda.synchronize()
    return host(out), host(z), host(xh)


SMALL = [
    # batch, cin, cout, grid, modes, rule
    (1, 8, 8, (16, 16, 16, 8), (4, 4, 4, 3), 0),       # the small workload
    (2, 3, 3, (6, 5, 12, 6), (2, 2, 3, 4), 0),         # no power of two on x,y: dense path, Nyquist kept
    (1, 2, 3, (4, 6, 8, 7), (1, 2, 2, 4), 1),          # symmetric rule, odd Nt, Cin != Cout
    (1, 4, 4, (32, 24, 64, 16), (6, 5, 12, 8), 0),     # several tiles, ragged column tails
    (5, 2, 2, (8, 8, 8, 4), (2, 2, 2, 3), 0),          # batch above the mix kernel's register tile
    (1, 2, 2, (8, 8, 8, 8), (4, 4, 4, 5), 0),          # every mode kept (L = N, mt = Nt/2+1)
    (1, 2, 2, (8, 4, 8, 8), (1, 1, 1, 1), 0),          # a single t mode
    (1, 1, 1, (1, 1, 1, 1), (0, 0, 0, 1), 1),          # one-point grid
    (1, 3, 2, (10, 3, 20, 5), (2, 1, 4, 2), 1),        # mixed radix z (20 = 5*4)
    (1, 3, 3, (2, 3, 32, 16), (1, 1, 4, 5), 0),        # matrix-core inverse kernel, 6 columns, padded channels
    (2, 2, 3, (3, 2, 32, 16), (1, 1, 6, 9), 0),        # same, two residue classes per block, Cin != Cout
    (1, 20, 20, (2, 2, 32, 32), (1, 1, 8, 9), 0),      # same, width 20, Nt = 32
    (1, 24, 24, (2, 2, 32, 16), (1, 1, 4, 4), 0),      # same, width 24 (eight channel tiles)
    (1, 8, 8, (2, 3, 128, 32), (1, 1, 16, 9), 0),      # column kernel (Nt = 32): four steps per column
    (2, 3, 5, (3, 2, 64, 32), (1, 1, 6, 5), 0),        # same, padded channel tiles, Cin != Cout
    (1, 4, 4, (2, 2, 32, 32), (1, 1, 16, 17), 0),      # same, one step, every z and t mode kept
    (1, 20, 20, (2, 3, 128, 16), (1, 1, 16, 9), 0),    # column kernel (Nt = 16): width 20 in two passes, two steps
    (2, 20, 20, (2, 2, 64, 16), (1, 1, 12, 8), 0),     # same, one step, 24 kept z frequencies and 8 t bins
    (1, 8, 8, (2, 3, 64, 16), (1, 1, 8, 5), 0),        # same, width 8: one pass
    (2, 3, 5, (3, 2, 128, 16), (1, 1, 10, 7), 0),      # same, padded channel tiles, Cin != Cout
    (1, 6, 6, (2, 2, 64, 16), (1, 1, 5, 4), 0),        # same, padded channel tiles in a block
    (1, 2, 2, (2, 2, 16, 64), (1, 1, 4, 9), 0),        # 64-point t axis (forward: the in-register 64-point real transform)
    (1, 2, 2, (2, 2, 256, 16), (1, 1, 20, 5), 0),      # 256-point z axis: one plane fills the forward block, 16 residue classes
    (2, 2, 2, (2, 2, 8, 32), (1, 1, 4, 17), 0),        # 8-point z axis under 32 t points: the forward tile's row stride (17) exceeds N + 1
    (1, 8, 8, (3, 2, 32, 30), (1, 1, 4, 8), 0),        # matrix-core inverse kernel, t axis padded 30 -> 32
    (2, 3, 3, (2, 3, 32, 12), (1, 1, 6, 4), 0),        # same, 12 -> 16, padded channel tiles
    (1, 20, 20, (2, 2, 64, 30), (1, 1, 12, 8), 0),     # same, width 20, the z and t lengths of the paper's samples
    (1, 3, 3, (4, 3, 21, 6), (1, 1, 5, 3), 0),         # odd z length: dense z stage of the inverse on 16x16x4 tiles
    (2, 5, 4, (2, 2, 37, 16), (1, 1, 9, 8), 0),        # same, prime z length, ragged last row group, Cin != Cout
    (1, 2, 2, (3, 3, 35, 4), (1, 1, 6, 2), 1),         # same, three row tiles per block, symmetric rule
    (1, 2, 2, (2, 2, 135, 8), (1, 1, 30, 3), 0),       # dense forward z stage: two sweeps of row tiles, 15 of 16 columns
    (1, 4, 4, (3, 5, 6, 7), (1, 2, 2, 3), 0),          # width 4 with 630 points (not a multiple of 64): the generic
                                                       # backward pointwise kernel (erff / expf), where case 3 of the
                                                       # same width takes the matrix-core one (rational erf)
]


@pytest.mark.parametrize("case", SMALL)
def test_spectral_conv_fwd_matches_oracle(case):
    L = Layer(*case)
    y, xh = gpu_spectral_fwd(L)
    yo, xho = O.spectral_conv_fwd(L.x, L.R, L.spec, return_xhat=True)
    assert rel(xh, xho) <= TOL
    assert rel(y, yo) <= TOL


@pytest.mark.parametrize("case", SMALL)
def test_spectral_conv_bwd_matches_oracle(case):
    L = Layer(*case)
    gy = synth.normal_field(1, synth.T_GOUT, L.batch, L.c_out, L.spec.grid)
    gxo, gRo = O.spectral_conv_bwd(L.x, L.R, gy, L.spec)
    ws = B.alloc_workspace(L.desc, B.FNO_OP_SPECTRAL_CONV_BWD)
    gx = torch.empty((L.batch, L.c_in) + L.spec.grid, device="cuda")
    gR = torch.empty((L.c_in, L.c_out) + L.counts, dtype=torch.complex64, device="cuda")
    B.fno_spectral_conv_bwd(L.desc, dev(L.x), None, dev(L.R), dev(gy), gx, gR, ws)
    torch.cuda.synchronize()
    assert rel(host(gx), gxo) <= TOL
    assert rel(host(gR), gRo) <= TOL
    # with the saved spectrum instead of x, and with only one of the two outputs requested
    _, xh = gpu_spectral_fwd(L)
    gR2 = torch.empty_like(gR)
    B.fno_spectral_conv_bwd(L.desc, None, dev(xh), dev(L.R), dev(gy), None, gR2, ws)
    gx2 = torch.empty_like(gx)
    B.fno_spectral_conv_bwd(L.desc, None, None, dev(L.R), dev(gy), gx2, None, ws)
    torch.cuda.synchronize()
    assert rel(host(gR2), gRo) <= TOL
    assert rel(host(gx2), gxo) <= TOL


BLOCKS = [c for c in SMALL if c[1] == c[2]]


@pytest.mark.parametrize("case", BLOCKS)
@pytest.mark.parametrize("activation", [B.FNO_ACT_GELU, B.FNO_ACT_IDENTITY])
def test_block_fwd_and_bwd_match_oracle(case, activation):
    L = Layer(*case, activation=activation)
    out, z, xh = gpu_block_fwd(L)
    oo, zo, xho = O.block_fwd(L.x, L.R, L.W, L.b, L.spec, L.act_name())
    assert rel(out, oo) <= TOL and rel(z, zo) <= TOL and rel(xh, xho) <= TOL

    target = synth.normal_field(2, synth.T_TARGET, L.batch, L.c_out, L.spec.grid)
    gout = synth.normal_field(3, synth.T_GOUT, L.batch, L.c_out, L.spec.grid)
    ws = B.alloc_workspace(L.desc, B.FNO_OP_BLOCK_BWD)
    for mse in (False, True):
        desc = B.make_desc(L.batch, L.c_in, L.c_out, L.spec.grid, L.spec.modes, L.spec.rule,
                           activation, B.FNO_FLAG_MSE_TARGET if mse else 0)
        g_in = target if mse else gout
        # the oracle differentiates its own forward; the GPU gets the z it saved itself
        g_ref = O.mse_grad(oo, target) if mse else gout
        ref = O.block_bwd(L.x, L.R, L.W, L.b, g_ref, L.spec, L.act_name())
        gx = torch.empty((L.batch, L.c_in) + L.spec.grid, device="cuda")
        gR = torch.empty((L.c_in, L.c_out) + L.counts, dtype=torch.complex64, device="cuda")
        gW = torch.empty((L.c_out, L.c_in), device="cuda")
        gb = torch.empty((L.c_out,), device="cuda")
        B.fno_block_bwd(desc, dev(L.x), dev(L.R), dev(L.W), dev(z), dev(xh) if mse else None,
                        dev(g_in), gx, gR, gW, gb, ws)
        torch.cuda.synchronize()
        assert rel(host(gx), ref["gx"]) <= TOL
        assert rel(host(gR), ref["gR"]) <= TOL
        assert rel(host(gW), ref["gW"]) <= TOL
        # gb is a sum of terms of either sign: where they cancel, the error is bounded by the
        # size of the summands (root-sum-square), elsewhere by the sum itself
        gb_scale = np.abs(ref["gb"]) + np.sqrt(np.sum(ref["gz"] ** 2, axis=(0, 2, 3, 4, 5)))
        assert np.max(np.abs(host(gb) - ref["gb"]) / np.maximum(gb_scale, 1e-300)) <= TOL
        assert rel(host(gb), ref["gb"]) <= TOL          # and the criterion of every other tensor, as a vector
        # identical bits on a second run (fixed reduction order)
        gW2 = torch.empty_like(gW)
        gb2 = torch.empty_like(gb)
        gx2 = torch.empty_like(gx)
        B.fno_block_bwd(desc, dev(L.x), dev(L.R), dev(L.W), dev(z), dev(xh) if mse else None,
                        dev(g_in), gx2, None, gW2, gb2, ws)
        torch.cuda.synchronize()
        assert torch.equal(gW, gW2) and torch.equal(gb, gb2) and torch.equal(gx, gx2)


def test_accumulate_flag_adds_parameter_gradients_of_successive_calls():
    """FNO_FLAG_ACCUMULATE_GRADS: gR, gW, gb of a second call are added to those of the first (the
    gradient of a broadcast weight is a sum, Sec. 2.1), gx is overwritten; compared with the sum of
    the oracle's gradients for the two cotangents."""
    L = Layer(2, 4, 4, (8, 6, 16, 8), (2, 2, 4, 4), 0)
    _, z, xh = gpu_block_fwd(L)
    g1 = synth.normal_field(3, synth.T_GOUT, L.batch, L.c_out, L.spec.grid)
    g2 = synth.normal_field(4, synth.T_GOUT, L.batch, L.c_out, L.spec.grid)
    r1 = O.block_bwd(L.x, L.R, L.W, L.b, g1, L.spec, "gelu")
    r2 = O.block_bwd(L.x, L.R, L.W, L.b, g2, L.spec, "gelu")
    ws = B.alloc_workspace(L.desc, B.FNO_OP_BLOCK_BWD)
    gx = torch.empty((L.batch, L.c_in) + L.spec.grid, device="cuda")
    gR = torch.empty((L.c_in, L.c_out) + L.counts, dtype=torch.complex64, device="cuda")
    gW = torch.empty((L.c_out, L.c_in), device="cuda")
    gb = torch.empty((L.c_out,), device="cuda")
    acc = B.make_desc(L.batch, L.c_in, L.c_out, L.spec.grid, L.spec.modes, L.spec.rule, B.FNO_ACT_GELU,
                      B.FNO_FLAG_ACCUMULATE_GRADS)
    B.fno_block_bwd(L.desc, dev(L.x), dev(L.R), dev(L.W), dev(z), dev(xh), dev(g1), gx, gR, gW, gb, ws)
    B.fno_block_bwd(acc, dev(L.x), dev(L.R), dev(L.W), dev(z), dev(xh), dev(g2), gx, gR, gW, gb, ws)
    torch.cuda.synchronize()
    assert rel(host(gx), r2["gx"]) <= TOL
    for name, got in (("gR", gR), ("gW", gW), ("gb", gb)):
        assert rel(host(got), r1[name] + r2[name]) <= TOL, name
    # the spectral convolution's own adjoint: gR accumulates, gx does not
    ws2 = B.alloc_workspace(L.desc, B.FNO_OP_SPECTRAL_CONV_BWD)
    gx1o, gR1o = O.spectral_conv_bwd(L.x, L.R, g1, L.spec)
    gx2o, gR2o = O.spectral_conv_bwd(L.x, L.R, g2, L.spec)
    B.fno_spectral_conv_bwd(L.desc, dev(L.x), None, dev(L.R), dev(g1), gx, gR, ws2)
    B.fno_spectral_conv_bwd(acc, dev(L.x), None, dev(L.R), dev(g2), gx, gR, ws2)
    torch.cuda.synchronize()
    assert rel(host(gx), gx2o) <= TOL
    assert rel(host(gR), gR1o + gR2o) <= TOL


def test_planned_tables_give_the_same_bits_as_rebuilt_ones():
    """fno_plan_tables + FNO_FLAG_TABLES_READY: the calls skip their table kernels and return the
    same bits, forward and backward, also after other calls used the workspace in between."""
    L = Layer(2, 4, 4, (8, 6, 16, 8), (2, 2, 4, 4), 0)
    out0, z0, xh0 = gpu_block_fwd(L)
    flags = B.FNO_FLAG_TABLES_READY
    ready = B.make_desc(L.batch, L.c_in, L.c_out, L.spec.grid, L.spec.modes, L.spec.rule, B.FNO_ACT_GELU, flags)
    ws = B.alloc_workspace(ready, B.FNO_OP_BLOCK_BWD)
    ws.fill_(0xFF)                                   # nothing usable in it before the plan
    B.fno_plan_tables(ready, B.FNO_OP_BLOCK_BWD, ws)
    out = torch.empty((L.batch, L.c_out) + L.spec.grid, device="cuda")
    z = torch.empty_like(out)
    xh = torch.empty((L.batch, L.c_in) + L.counts, dtype=torch.complex64, device="cuda")
    gout = synth.normal_field(3, synth.T_GOUT, L.batch, L.c_out, L.spec.grid)
    gx, gR = torch.empty_like(out), torch.empty((L.c_in, L.c_out) + L.counts, dtype=torch.complex64, device="cuda")
    gW, gb = torch.empty((L.c_out, L.c_in), device="cuda"), torch.empty((L.c_out,), device="cuda")
    ref = {}
    for name, desc in (("rebuilt", L.desc), ("planned", ready), ("planned again", ready)):
        B.fno_block_fwd(desc, dev(L.x), dev(L.R), dev(L.W), dev(L.b), out, z, xh, ws)
        B.fno_block_bwd(desc, dev(L.x), dev(L.R), dev(L.W), z, xh, dev(gout), gx, gR, gW, gb, ws)
        torch.cuda.synchronize()
        got = [t.clone() for t in (out, z, torch.view_as_real(xh), gx, torch.view_as_real(gR), gW, gb)]
        if not ref:
            ref = got
            assert np.array_equal(host(out), out0) and np.array_equal(host(z), z0)
        else:
            assert all(torch.equal(a, b) for a, b in zip(got, ref)), name


@pytest.mark.parametrize("case", [(1, 8, 8, (2, 3, 128, 32), (1, 1, 16, 9), 0),      # column kernel
                                  (1, 20, 20, (2, 3, 128, 16), (1, 1, 16, 9), 0),   # column kernel, Nt = 16
                                  (2, 3, 3, (6, 5, 12, 6), (2, 2, 3, 4), 0)])        # generic kernels
def test_block_forward_and_backward_replay_identically_from_a_hip_graph(case):
    """The calls only enqueue kernels on the caller's stream (no allocation, no memset, no
    synchronisation), so a caller may capture them in a HIP graph: three replays, with eager work and
    synchronisations in between, each give the bits of the eager call."""
    L = Layer(*case)
    dx, dR, dW, db = dev(L.x), dev(L.R), dev(L.W), dev(L.b)
    gout = dev(synth.normal_field(3, synth.T_GOUT, L.batch, L.c_out, L.spec.grid))
    ws = B.alloc_workspace(L.desc, B.FNO_OP_BLOCK_BWD)
    out = torch.empty((L.batch, L.c_out) + L.spec.grid, device="cuda")
    z = torch.empty_like(out)
    xh = torch.empty((L.batch, L.c_in) + L.counts, dtype=torch.complex64, device="cuda")
    gx = torch.empty_like(out)
    gR = torch.empty((L.c_in, L.c_out) + L.counts, dtype=torch.complex64, device="cuda")
    gW, gb = torch.empty((L.c_out, L.c_in), device="cuda"), torch.empty((L.c_out,), device="cuda")
    outs = (out, z, gx, gW, gb)

    def step():
        B.fno_block_fwd(L.desc, dx, dR, dW, db, out, z, xh, ws)
        B.fno_block_bwd(L.desc, dx, dR, dW, z, xh, gout, gx, gR, gW, gb, ws)

    step()
    torch.cuda.synchronize()
    eager = [t.clone() for t in outs] + [torch.view_as_real(xh).clone(), torch.view_as_real(gR).clone()]
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        step()
    for _ in range(3):
        for t in outs:
            t.fill_(float("nan"))                    # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = list(outs) + [torch.view_as_real(xh), torch.view_as_real(gR)]
        assert all(torch.equal(a, b) for a, b in zip(got, eager))


def test_spectral_branch_alone_is_not_masked_by_the_linear_term():
    """The spectral term is much smaller than W x + b; zero W and b isolate it inside the block."""
    L = Layer(1, 4, 4, (16, 16, 32, 8), (4, 4, 8, 4))
    L.W[:] = 0
    L.b[:] = 0
    L.act = B.FNO_ACT_IDENTITY
    L.desc = B.make_desc(1, 4, 4, L.spec.grid, L.spec.modes, 0, B.FNO_ACT_IDENTITY)
    out, z, _ = gpu_block_fwd(L)
    yo = O.spectral_conv_fwd(L.x, L.R, L.spec)
    assert rel(out, yo) <= TOL and np.array_equal(out, z)


def test_one_hot_frequency_is_exactly_truncated():
    """A plane wave outside the kept set gives a spectral output at rounding level only."""
    grid, modes = (16, 16, 16, 8), (4, 4, 4, 3)
    L = Layer(1, 1, 1, grid, modes)
    L.R[:] = 1.0
    n = np.meshgrid(*[np.arange(g) for g in grid], indexing="ij")
    for k4, kept in [((3, -4, 2, 2), True), ((5, 0, 0, 0), False), ((4, 0, 0, 1), False), ((-4, 0, 0, 1), True), ((0, 0, 5, 1), False), ((1, 1, 1, 3), False),
                     ((-4, -4, -4, 0), True)]:
        th = 2 * np.pi * sum(k4[a] * n[a] / grid[a] for a in range(4))
        x = np.cos(th)[None, None].astype(np.float32)
        y, _ = gpu_spectral_fwd(L, x)
        yo = O.spectral_conv_fwd(x, L.R, L.spec)
        if kept:
            assert rel(y, yo) <= TOL and np.max(np.abs(yo)) > 0.1
        else:
            assert np.max(np.abs(yo)) < 1e-7 and np.max(np.abs(y)) < 2e-6   # float32 rounding of the input leaks a little


def test_cfg2_block_forward_full_size_elementwise():
    c = synth.CONFIGS["cfg2"]
    L = Layer(c["batch"], c["width"], c["width"], c["grid"], c["modes"])
    out, z, xh = gpu_block_fwd(L)
    ys, _ = gpu_spectral_fwd(L)
    # oracle one batch entry at a time (the layer does not couple batch entries)
    for b in range(L.batch):
        oo, zo, xho = O.block_fwd(L.x[b:b + 1], L.R, L.W, L.b, L.spec)
        assert rel(out[b:b + 1], oo) <= TOL
        assert rel(xh[b:b + 1], xho) <= TOL
        yso = zo - O.channel_affine(L.x[b:b + 1], L.W, L.b)
        assert rel(ys[b:b + 1], yso) <= TOL


def test_pointwise_lift_and_projection_and_small_network():
    """Lift 5->20, four blocks, projection 20->128->1 on a reduced grid of the cfg3 structure."""
    grid, modes = (16, 16, 8, 8), (4, 4, 2, 3)
    spec = O.LayerSpec(grid, modes, 0)
    counts = tuple(len(k) for k in O.mode_lists(spec))
    npts = int(np.prod(grid))
    a = np.concatenate([synth.smooth_gaussian_field(0, grid, 3.0)[None], synth.coordinate_channels(grid)])[None]
    lw, lb = synth.linear_weights(0, 20, 5, synth.T_LIFT), synth.bias(0, 20, synth.T_LIFT)
    blocks = [(synth.spectral_weights(10 + k, 20, 20, counts), synth.linear_weights(10 + k, 20, 20),
               synth.bias(10 + k, 20)) for k in range(4)]
    w1, b1 = synth.linear_weights(1, 128, 20, synth.T_PROJ), synth.bias(1, 128, synth.T_PROJ)
    w2, b2 = synth.linear_weights(2, 1, 128, synth.T_PROJ), synth.bias(2, 1, synth.T_PROJ)
    want = O.fno_forward(a, lw, lb, blocks, (w1, b1, w2, b2), spec)

    desc = B.make_desc(1, 20, 20, grid, modes)
    ws = B.alloc_workspace(desc, B.FNO_OP_BLOCK_FWD)
    v = torch.empty((1, 20) + grid, device="cuda")
    B.fno_pointwise_linear(1, 5, 20, npts, dev(a.astype(np.float32)), dev(lw), dev(lb), v)
    torch.cuda.synchronize()
    assert rel(host(v), O.pointwise_linear(a, lw, lb)) <= TOL
    for (r, w, b) in blocks:
        nxt = torch.empty_like(v)
        B.fno_block_fwd(desc, v, dev(r), dev(w), dev(b), nxt, None, None, ws)
        v = nxt
    u = torch.empty((1, 1) + grid, device="cuda")
    B.fno_pointwise_mlp2(1, 20, 128, 1, npts, v, dev(w1), dev(b1), dev(w2), dev(b2), u)
    torch.cuda.synchronize()
    assert rel(host(u), want) <= TOL


@pytest.mark.parametrize("npts,ci,co", [(630, 5, 20), (632, 5, 20), (1024, 20, 1), (1026, 20, 1), (256, 3, 32)])
def test_pointwise_linear_point_counts_and_widths(npts, ci, co):
    """Point counts that are and are not multiples of 4 (16-byte and scalar kernels), all width classes."""
    rng = np.random.default_rng(npts + co)
    x = rng.standard_normal((2, ci, npts)).astype(np.float32)
    w = synth.linear_weights(3, co, ci, synth.T_LIFT)
    b = synth.bias(3, co, synth.T_LIFT)
    y = torch.empty((2, co, npts), device="cuda")
    B.fno_pointwise_linear(2, ci, co, npts, dev(x), dev(w), dev(b), y)
    torch.cuda.synchronize()
    want = O.pointwise_linear(x.reshape(2, ci, npts, 1, 1, 1), w, b).reshape(2, co, npts)
    assert rel(host(y), want) <= TOL


def test_block_against_the_stored_oracle_fixture():
    """The HIP path reproduces tests/golden/block_small.txt, values the float64 oracle wrote once.

    The inputs are regenerated here from the fixture's seed (float64 draws rounded to float32 for
    the GPU, which moves the results by a few 1e-8 relative to their scale); the expected values
    are read from the text file and never recomputed.
    """
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    want = {}
    for line in open(os.path.join(here, "golden", "block_small.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, val = line.rstrip("\n").split("\t")
        want[name] = float(val)
    grid, modes = (6, 4, 8, 6), (2, 1, 2, 3)
    spec = O.LayerSpec(grid, modes, 0)
    rng = np.random.default_rng([2204, 1205])
    lx, ly, lz, lt = [len(k) for k in O.mode_lists(spec)]
    x = rng.standard_normal((2, 3) + grid)
    r = (rng.standard_normal((3, 3, lx, ly, lz, lt)) + 1j * rng.standard_normal((3, 3, lx, ly, lz, lt))) / 3.0
    w = rng.standard_normal((3, 3)) / np.sqrt(3.0)
    b = 0.1 * rng.standard_normal(3)
    target = rng.standard_normal(x.shape)

    desc = B.make_desc(2, 3, 3, grid, modes, 0, B.FNO_ACT_GELU, B.FNO_FLAG_MSE_TARGET)
    ws = B.alloc_workspace(desc, B.FNO_OP_BLOCK_BWD)
    dx, dr = dev(x.astype(np.float32)), dev(r.astype(np.complex64))
    dw, db, dt = dev(w.astype(np.float32)), dev(b.astype(np.float32)), dev(target.astype(np.float32))
    out = torch.empty((2, 3) + grid, device="cuda")
    z = torch.empty_like(out)
    xh = torch.empty((2, 3, lx, ly, lz, lt), dtype=torch.complex64, device="cuda")
    B.fno_block_fwd(desc, dx, dr, dw, db, out, z, xh, ws)
    gx = torch.empty_like(out)
    gR = torch.empty_like(dr)
    gW = torch.empty_like(dw)
    gb = torch.empty_like(db)
    B.fno_block_bwd(desc, dx, dr, dw, z, xh, dt, gx, gR, gW, gb, ws)
    torch.cuda.synchronize()
    out, z, xh, gx, gR, gW, gb = [host(t) for t in (out, z, xh, gx, gR, gW, gb)]

    # each value against the scale of the tensor it belongs to (single entries can be near zero)
    def close(got, name, scale):
        assert abs(float(got) - want[name]) <= TOL * scale, (name, float(got), want[name])

    for p in [(0, 0, 0, 0, 0, 0), (1, 2, 5, 3, 7, 5), (0, 1, 2, 1, 3, 4), (1, 0, 4, 2, 6, 1)]:
        close(out[p], "out" + str(p), np.abs(out).max())
        close(z[p], "z" + str(p), np.abs(z).max())
        close(gx[p], "gx" + str(p), np.abs(gx).max())
    close(xh[1, 2, 3, 1, 2, 1].real, "xhat_re", np.abs(xh).max())
    close(xh[1, 2, 3, 1, 2, 1].imag, "xhat_im", np.abs(xh).max())
    close(gR[2, 1, 1, 0, 3, 2].real, "gR_re", np.abs(gR).max())
    close(gR[2, 1, 1, 0, 3, 2].imag, "gR_im", np.abs(gR).max())
    close(gR[0, 2, 3, 1, 1, 0].real, "gR_kt0_re", np.abs(gR).max())
    for o in range(3):
        close(gb[o], f"gb[{o}]", np.abs(gb).max())
        for i in range(3):
            close(gW[o, i], f"gW[{o}][{i}]", np.abs(gW).max())


@pytest.mark.parametrize("shape", [
    # batch, c_in, c_out, spatial grid, nt
    (2, 2, 20, (6, 5, 4), 30),        # the paper's two input channels, nt not a multiple of 4
    (1, 3, 8, (4, 4, 8), 16),         # whole float4 rows
    (1, 1, 24, (3, 2, 5), 7),         # odd nt, one input channel, width above 20
    (1, 2, 20, (60, 60, 64), 30),     # a training sample of the paper (Sec. 4), full size
])
def test_time_lift_matches_oracle(shape):
    batch, c_in, c_out, grid, nt = shape
    rng = np.random.default_rng([7, batch, c_in, c_out, nt])
    a = rng.standard_normal((batch, c_in) + grid + (1,)).astype(np.float32)
    wt = rng.standard_normal(nt).astype(np.float32)
    bt = rng.standard_normal(nt).astype(np.float32)
    wc = (rng.standard_normal((c_out, c_in)) / np.sqrt(c_in)).astype(np.float32)
    bc = (0.1 * rng.standard_normal(c_out)).astype(np.float32)
    nspace = int(np.prod(grid))
    out = torch.empty((batch, c_out) + grid + (nt,), device="cuda")
    B.fno_time_lift(batch, c_in, c_out, nspace, nt, dev(a), dev(wt), dev(bt), dev(wc), dev(bc), out)
    torch.cuda.synchronize()
    assert rel(host(out), O.time_lift(a, wt, bt, wc, bc)) <= TOL
    # without the biases
    B.fno_time_lift(batch, c_in, c_out, nspace, nt, dev(a), dev(wt), None, dev(wc), None, out)
    torch.cuda.synchronize()
    assert rel(host(out), O.time_lift(a, wt, np.zeros(nt), wc, np.zeros(c_out))) <= TOL


@pytest.mark.parametrize("shape", [
    # batch, c_in, c_out, spatial grid, nt
    (2, 2, 20, (6, 5, 4), 30),        # the paper's two input channels, one chunk per batch entry
    (1, 3, 8, (4, 4, 8), 16),         # three input channels on the four-channel register tile
    (3, 1, 24, (3, 2, 5), 7),         # odd nt, one input channel, pairs that do not fill the last block
    (1, 5, 4, (7, 9, 11), 4),         # five input channels, a ragged tail of positions
    (1, 2, 20, (60, 60, 64), 30),     # a training sample of the paper (Sec. 4), full size: 450 chunks
])
def test_time_lift_adjoint_matches_oracle(shape):
    batch, c_in, c_out, grid, nt = shape
    rng = np.random.default_rng([23, batch, c_in, c_out, nt])
    a = rng.standard_normal((batch, c_in) + grid + (1,)).astype(np.float32)
    wt = rng.standard_normal(nt).astype(np.float32)
    bt = rng.standard_normal(nt).astype(np.float32)
    wc = (rng.standard_normal((c_out, c_in)) / np.sqrt(c_in)).astype(np.float32)
    g = rng.standard_normal((batch, c_out) + grid + (nt,)).astype(np.float32)
    nspace = int(np.prod(grid))
    ws = torch.empty(B.fno_time_lift_bwd_workspace_bytes(c_in, c_out, nt) // 4 + 2, dtype=torch.float32,
                     device="cuda")
    gwt, gbt = torch.empty(nt, device="cuda"), torch.empty(nt, device="cuda")
    gwc, gbc = torch.empty((c_out, c_in), device="cuda"), torch.empty(c_out, device="cuda")
    B.fno_time_lift_bwd(batch, c_in, c_out, nspace, nt, dev(a), dev(wt), dev(bt), dev(wc), dev(g),
                        gwt, gbt, gwc, gbc, ws)
    torch.cuda.synchronize()
    want = O.time_lift_bwd(a, wt, bt, wc, g)
    for name, got in (("gWt", gwt), ("gbt", gbt), ("gWc", gwc), ("gbc", gbc)):
        assert rel(host(got), want[name]) <= TOL, name
    # same bits on a second run; without the time bias; a subset of the outputs
    gwt2, gwc2 = torch.empty_like(gwt), torch.empty_like(gwc)
    B.fno_time_lift_bwd(batch, c_in, c_out, nspace, nt, dev(a), dev(wt), dev(bt), dev(wc), dev(g),
                        gwt2, None, gwc2, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(gwt, gwt2) and torch.equal(gwc, gwc2)
    B.fno_time_lift_bwd(batch, c_in, c_out, nspace, nt, dev(a), dev(wt), None, dev(wc), dev(g),
                        None, None, gwc2, None, ws)
    torch.cuda.synchronize()
    assert rel(host(gwc2), O.time_lift_bwd(a, wt, np.zeros(nt), wc, g)["gWc"]) <= TOL


@pytest.mark.parametrize("n", [7, 100003, 60 * 60 * 64 * 30])
def test_relative_l2_loss_and_gradient_match_oracle(n):
    rng = np.random.default_rng([11, n])
    target = rng.standard_normal(n).astype(np.float32)
    pred = (target + 0.3 * rng.standard_normal(n)).astype(np.float32)
    ws = torch.empty(B.fno_rel_l2_workspace_bytes() // 4, dtype=torch.float32, device="cuda")
    loss = torch.empty(1, device="cuda")
    grad = torch.empty(n, device="cuda")
    B.fno_rel_l2_loss(n, dev(pred), dev(target), loss, grad, ws)
    torch.cuda.synchronize()
    want = O.rel_l2_loss(pred, target)
    assert abs(float(loss.cpu()) - want) <= TOL * want
    assert rel(host(grad), O.rel_l2_grad(pred, target)) <= TOL
    # same bits on a second run; loss alone; a perfect prediction has loss 0 and a zero gradient
    loss2 = torch.empty(1, device="cuda")
    B.fno_rel_l2_loss(n, dev(pred), dev(target), loss2, None, ws)
    B.fno_rel_l2_loss(n, dev(target), dev(target), loss, grad, ws)
    torch.cuda.synchronize()
    assert abs(float(loss2.cpu()) - want) <= TOL * want
    assert float(loss.cpu()) == 0.0 and not bool(grad.any())


def test_adam_steps_match_oracle_for_real_and_complex_parameters():
    rng = np.random.default_rng(13)
    w = rng.standard_normal((20, 20)).astype(np.float32)
    r = (rng.standard_normal((3, 3, 4, 4, 4, 3)) + 1j * rng.standard_normal((3, 3, 4, 4, 4, 3))).astype(np.complex64)
    for p0 in (w, r):
        as_real = p0.view(np.float32).ravel() if np.iscomplexobj(p0) else p0.ravel()
        n = as_real.size
        p = dev(as_real.copy())
        m = torch.zeros(n, device="cuda")
        v = torch.zeros(n, device="cuda")
        po, mo, vo = as_real.astype(np.float64), np.zeros(n), np.zeros(n)
        for step in (1, 2, 3):
            g = (rng.standard_normal(n) * (10.0 ** rng.integers(-3, 2))).astype(np.float32)
            B.fno_adam_step(n, p, dev(g), m, v, 1e-3, 0.9, 0.999, 1e-8, step)
            before = po
            po, mo, vo = O.adam_step(po, g, mo, vo, step)
            torch.cuda.synchronize()
            assert rel(host(m), mo) <= TOL and rel(host(v), vo) <= TOL
            assert rel(host(p), po) <= TOL
            # the update itself, not only the updated parameter
            assert rel(host(p).astype(np.float64) - before, po - before) <= 1e-3


@pytest.mark.parametrize("shape", [
    # batch, c_in, hidden, c_out, points
    (2, 3, 5, 2, 77),                 # ragged tile, hidden below one chunk
    (1, 20, 128, 1, 3000),            # the projection of the benchmark network, several tiles
    (2, 5, 20, 4, 1024),              # whole tiles, four outputs
    (2, 5, 32, 1, 200),               # one 32-row block of hidden units on the matrix cores, ragged tile
    (2, 9, 64, 3, 1000),              # two blocks, three outputs, two batch elements
    (1, 24, 192, 4, 333),             # more than 21 input channels, six blocks
    (1, 20, 128, 1, 64 * 512 * 17 + 7),  # every block flushes its weight-gradient accumulator once and goes on
])
def test_pointwise_adjoints_match_oracle(shape):
    batch, c_in, hidden, c_out, npts = shape
    rng = np.random.default_rng([19, c_in, hidden, c_out, npts])
    grid = (npts, 1, 1, 1)
    x = rng.standard_normal((batch, c_in) + grid).astype(np.float32)
    w1 = (rng.standard_normal((hidden, c_in)) / np.sqrt(c_in)).astype(np.float32)
    b1 = (0.1 * rng.standard_normal(hidden)).astype(np.float32)
    w2 = (rng.standard_normal((c_out, hidden)) / np.sqrt(hidden)).astype(np.float32)
    gu = rng.standard_normal((batch, c_out) + grid).astype(np.float32)
    nbytes = max(B.fno_pointwise_bwd_workspace_bytes(c_in, hidden, c_out),
                 B.fno_pointwise_bwd_workspace_bytes(c_in, 0, min(hidden, 32)))
    ws = torch.empty(nbytes // 4 + 2, dtype=torch.float32, device="cuda")
    # the linear map (lift): hidden plays the output width
    gh_in = rng.standard_normal((batch, hidden) + grid).astype(np.float32)
    gx = torch.empty((batch, c_in) + grid, device="cuda")
    gW = torch.empty((hidden, c_in), device="cuda")
    gb = torch.empty(hidden, device="cuda")
    if hidden <= 32:
        B.fno_pointwise_linear_bwd(batch, c_in, hidden, npts, dev(x), dev(w1), dev(gh_in), gx, gW, gb, ws)
        torch.cuda.synchronize()
        want = O.pointwise_linear_bwd(x, w1, gh_in)
        assert rel(host(gx), want["gx"]) <= TOL and rel(host(gW), want["gW"]) <= TOL
        assert rel(host(gb), want["gb"]) <= TOL
    # the two-layer projection: forward, then its adjoint
    b2 = (0.1 * rng.standard_normal(c_out)).astype(np.float32)
    u = torch.empty((batch, c_out) + grid, device="cuda")
    B.fno_pointwise_mlp2(batch, c_in, hidden, c_out, npts, dev(x), dev(w1), dev(b1), dev(w2), dev(b2), u)
    torch.cuda.synchronize()
    assert rel(host(u), O.pointwise_mlp2(x, w1, b1, w2, b2)) <= TOL
    B.fno_pointwise_mlp2(batch, c_in, hidden, c_out, npts, dev(x), dev(w1), None, dev(w2), None, u)
    torch.cuda.synchronize()
    assert rel(host(u), O.pointwise_mlp2(x, w1, np.zeros(hidden), w2, np.zeros(c_out))) <= TOL
    gW1 = torch.empty((hidden, c_in), device="cuda")
    gb1 = torch.empty(hidden, device="cuda")
    gW2 = torch.empty((c_out, hidden), device="cuda")
    gb2 = torch.empty(c_out, device="cuda")
    B.fno_pointwise_mlp2_bwd(batch, c_in, hidden, c_out, npts, dev(x), dev(w1), dev(b1), dev(w2), dev(gu),
                             gx, gW1, gb1, gW2, gb2, ws)
    torch.cuda.synchronize()
    want = O.pointwise_mlp2_bwd(x, w1, b1, w2, gu)
    for name, got in (("gx", gx), ("gW1", gW1), ("gb1", gb1), ("gW2", gW2), ("gb2", gb2)):
        assert rel(host(got), want[name]) <= TOL, name
    # identical bits on a second run
    gW1b, gW2b = torch.empty_like(gW1), torch.empty_like(gW2)
    B.fno_pointwise_mlp2_bwd(batch, c_in, hidden, c_out, npts, dev(x), dev(w1), dev(b1), dev(w2), dev(gu),
                             None, gW1b, None, gW2b, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(gW1, gW1b) and torch.equal(gW2, gW2b)
    # without the hidden bias
    B.fno_pointwise_mlp2_bwd(batch, c_in, hidden, c_out, npts, dev(x), dev(w1), None, dev(w2), dev(gu),
                             gx, gW1b, gb1, gW2b, gb2, ws)
    torch.cuda.synchronize()
    want0 = O.pointwise_mlp2_bwd(x, w1, np.zeros(hidden), w2, gu)
    for name, got in (("gx", gx), ("gW1", gW1b), ("gb1", gb1), ("gW2", gW2b), ("gb2", gb2)):
        assert rel(host(got), want0[name]) <= TOL, name


def test_whole_network_training_step_matches_oracle():
    """Lift, two blocks, projection; relative L2 loss; backward through all of it; one Adam step.

    Every stage runs through the C ABI; the float64 oracle differentiates its own forward."""
    grid, modes, c_in, width, hidden, nblocks = (8, 8, 8, 8), (2, 2, 2, 3), 3, 8, 16, 2
    spec = O.LayerSpec(grid, modes, 0)
    counts = tuple(len(k) for k in O.mode_lists(spec))
    npts = int(np.prod(grid))
    a = synth.normal_field(0, synth.T_X, 1, c_in, grid)
    y = synth.normal_field(1, synth.T_TARGET, 1, 1, grid)
    lw, lb = synth.linear_weights(0, width, c_in, synth.T_LIFT), synth.bias(0, width, synth.T_LIFT)
    blocks = [(synth.spectral_weights(k, width, width, counts), synth.linear_weights(10 + k, width, width),
               synth.bias(10 + k, width)) for k in range(nblocks)]
    w1, b1 = synth.linear_weights(1, hidden, width, synth.T_PROJ), synth.bias(1, hidden, synth.T_PROJ)
    w2, b2 = synth.linear_weights(2, 1, hidden, synth.T_PROJ), synth.bias(2, 1, synth.T_PROJ)

    # ---- GPU: forward
    desc = B.make_desc(1, width, width, grid, modes, 0, B.FNO_ACT_GELU)
    ws = B.alloc_workspace(desc, B.FNO_OP_BLOCK_BWD)
    d = {k: dev(v) for k, v in dict(a=a, y=y, lw=lw, lb=lb, w1=w1, b1=b1, w2=w2, b2=b2).items()}
    dblocks = [tuple(dev(t) for t in blk) for blk in blocks]
    vs = [torch.empty((1, width) + grid, device="cuda")]
    B.fno_pointwise_linear(1, c_in, width, npts, d["a"], d["lw"], d["lb"], vs[0])
    zs, xhs = [], []
    for (R, W, b) in dblocks:
        out = torch.empty_like(vs[0])
        z = torch.empty_like(vs[0])
        xh = torch.empty((1, width) + counts, dtype=torch.complex64, device="cuda")
        B.fno_block_fwd(desc, vs[-1], R, W, b, out, z, xh, ws)
        vs.append(out); zs.append(z); xhs.append(xh)
    u = torch.empty((1, 1) + grid, device="cuda")
    B.fno_pointwise_mlp2(1, width, hidden, 1, npts, vs[-1], d["w1"], d["b1"], d["w2"], d["b2"], u)
    # ---- loss and its gradient
    lws = torch.empty(B.fno_rel_l2_workspace_bytes() // 4, dtype=torch.float32, device="cuda")
    loss = torch.empty(1, device="cuda")
    gu = torch.empty_like(u)
    B.fno_rel_l2_loss(npts, u, d["y"], loss, gu, lws)
    # ---- backward
    pws = torch.empty(max(B.fno_pointwise_bwd_workspace_bytes(width, hidden, 1),
                          B.fno_pointwise_bwd_workspace_bytes(c_in, 0, width)) // 4 + 2,
                      dtype=torch.float32, device="cuda")
    gv = torch.empty_like(vs[0])
    g = {"w1": torch.empty_like(d["w1"]), "b1": torch.empty_like(d["b1"]), "w2": torch.empty_like(d["w2"]),
         "b2": torch.empty_like(d["b2"]), "lw": torch.empty_like(d["lw"]), "lb": torch.empty_like(d["lb"])}
    B.fno_pointwise_mlp2_bwd(1, width, hidden, 1, npts, vs[-1], d["w1"], d["b1"], d["w2"], gu, gv,
                             g["w1"], g["b1"], g["w2"], g["b2"], pws)
    gblocks = [None] * nblocks
    for k in reversed(range(nblocks)):
        R, W, b = dblocks[k]
        gx = torch.empty_like(vs[0])
        gR, gW, gb = torch.empty_like(R), torch.empty_like(W), torch.empty_like(b)
        B.fno_block_bwd(desc, vs[k], R, W, zs[k], xhs[k], gv, gx, gR, gW, gb, ws)
        gblocks[k] = (gR, gW, gb)
        gv = gx
    B.fno_pointwise_linear_bwd(1, c_in, width, npts, d["a"], d["lw"], gv, None, g["lw"], g["lb"], pws)
    torch.cuda.synchronize()

    # ---- oracle
    uo = O.fno_forward(a, lw, lb, blocks, (w1, b1, w2, b2), spec)
    assert rel(host(u), uo) <= TOL
    assert abs(float(loss.cpu()) - O.rel_l2_loss(uo, y)) <= TOL * O.rel_l2_loss(uo, y)
    ref = O.fno_backward(a, lw, lb, blocks, (w1, b1, w2, b2), spec, O.rel_l2_grad(uo, y))
    GT = 5 * TOL     # gradients pass through 2 blocks and 3 pointwise stages
    assert rel(host(g["w1"]), ref["proj"]["gW1"]) <= GT and rel(host(g["b1"]), ref["proj"]["gb1"]) <= GT
    assert rel(host(g["w2"]), ref["proj"]["gW2"]) <= GT and rel(host(g["b2"]), ref["proj"]["gb2"]) <= GT
    for k in range(nblocks):
        gR, gW, gb = gblocks[k]
        assert rel(host(gR), ref["blocks"][k]["gR"]) <= GT, k
        assert rel(host(gW), ref["blocks"][k]["gW"]) <= GT, k
        assert rel(host(gb), ref["blocks"][k]["gb"]) <= GT, k
    assert rel(host(g["lw"]), ref["lift"]["gW"]) <= GT and rel(host(g["lb"]), ref["lift"]["gb"]) <= GT

    # ---- one Adam step on every parameter (complex weights as pairs of floats)
    params = [(d["lw"], g["lw"], lw, ref["lift"]["gW"]), (d["w1"], g["w1"], w1, ref["proj"]["gW1"])]
    R0 = dblocks[0][0]
    params.append((torch.view_as_real(R0).reshape(-1), torch.view_as_real(gblocks[0][0]).reshape(-1),
                   np.ascontiguousarray(blocks[0][0]).view(np.float32).ravel(),
                   np.ascontiguousarray(ref["blocks"][0]["gR"].astype(np.complex128)).view(np.float64).ravel()))
    for p, grad, p_host, g_ref in params:
        n = p.numel()
        m = torch.zeros(n, device="cuda")
        v = torch.zeros(n, device="cuda")
        B.fno_adam_step(n, p, grad, m, v, 1e-3, 0.9, 0.999, 1e-8, 1)
        torch.cuda.synchronize()
        po, _, _ = O.adam_step(p_host.astype(np.float64).ravel(), np.asarray(g_ref).ravel(), np.zeros(n), np.zeros(n), 1)
        assert rel(host(p).ravel(), po) <= TOL


def test_network_with_time_lift_training_gradients_match_oracle():
    """The paper's input stage (eqs. (8)-(9)) in front of the network: time + channel lift of an
    input without a time axis, one block, projection, relative L2 loss, and the gradients of all
    four lift parameters through the whole chain."""
    sgrid, nt, modes, c_in, width, hidden = (6, 4, 8), 8, (2, 2, 2, 3), 2, 8, 32
    grid = sgrid + (nt,)
    spec = O.LayerSpec(grid, modes, 0)
    counts = tuple(len(k) for k in O.mode_lists(spec))
    nspace, npts = int(np.prod(sgrid)), int(np.prod(grid))
    rng = np.random.default_rng(41)
    a = rng.standard_normal((1, c_in) + sgrid + (1,)).astype(np.float32)
    wt, bt = rng.standard_normal(nt).astype(np.float32), (0.3 * rng.standard_normal(nt)).astype(np.float32)
    wc = (rng.standard_normal((width, c_in)) / np.sqrt(c_in)).astype(np.float32)
    bc = (0.1 * rng.standard_normal(width)).astype(np.float32)
    y = synth.normal_field(1, synth.T_TARGET, 1, 1, grid)
    R, W, b = (synth.spectral_weights(3, width, width, counts), synth.linear_weights(13, width, width),
               synth.bias(13, width))
    w1, b1 = synth.linear_weights(1, hidden, width, synth.T_PROJ), synth.bias(1, hidden, synth.T_PROJ)
    w2, b2 = synth.linear_weights(2, 1, hidden, synth.T_PROJ), synth.bias(2, 1, synth.T_PROJ)

    desc = B.make_desc(1, width, width, grid, modes, 0, B.FNO_ACT_GELU)
    ws = B.alloc_workspace(desc, B.FNO_OP_BLOCK_BWD)
    d = {k: dev(v) for k, v in dict(a=a, wt=wt, bt=bt, wc=wc, bc=bc, y=y, R=R, W=W, b=b, w1=w1, b1=b1, w2=w2,
                                    b2=b2).items()}
    v0 = torch.empty((1, width) + grid, device="cuda")
    B.fno_time_lift(1, c_in, width, nspace, nt, d["a"], d["wt"], d["bt"], d["wc"], d["bc"], v0)
    v1, z = torch.empty_like(v0), torch.empty_like(v0)
    xh = torch.empty((1, width) + counts, dtype=torch.complex64, device="cuda")
    B.fno_block_fwd(desc, v0, d["R"], d["W"], d["b"], v1, z, xh, ws)
    u = torch.empty((1, 1) + grid, device="cuda")
    B.fno_pointwise_mlp2(1, width, hidden, 1, npts, v1, d["w1"], d["b1"], d["w2"], d["b2"], u)
    lws = torch.empty(B.fno_rel_l2_workspace_bytes() // 4, dtype=torch.float32, device="cuda")
    loss, gu = torch.empty(1, device="cuda"), torch.empty_like(u)
    B.fno_rel_l2_loss(npts, u, d["y"], loss, gu, lws)
    pws = torch.empty(B.fno_pointwise_bwd_workspace_bytes(width, hidden, 1) // 4 + 2, dtype=torch.float32,
                      device="cuda")
    gv1, gv0 = torch.empty_like(v0), torch.empty_like(v0)
    B.fno_pointwise_mlp2_bwd(1, width, hidden, 1, npts, v1, d["w1"], d["b1"], d["w2"], gu, gv1,
                             None, None, None, None, pws)
    B.fno_block_bwd(desc, v0, d["R"], d["W"], z, xh, gv1, gv0, torch.empty_like(d["R"]), torch.empty_like(d["W"]),
                    torch.empty_like(d["b"]), ws)
    tws = torch.empty(B.fno_time_lift_bwd_workspace_bytes(c_in, width, nt) // 4 + 2, dtype=torch.float32,
                      device="cuda")
    gwt, gbt = torch.empty(nt, device="cuda"), torch.empty(nt, device="cuda")
    gwc, gbc = torch.empty((width, c_in), device="cuda"), torch.empty(width, device="cuda")
    B.fno_time_lift_bwd(1, c_in, width, nspace, nt, d["a"], d["wt"], d["bt"], d["wc"], gv0, gwt, gbt, gwc, gbc, tws)
    torch.cuda.synchronize()

    # oracle: the same chain in float64
    v0o = O.time_lift(a, wt, bt, wc, bc)
    v1o = O.block_fwd(v0o, R, W, b, spec, "gelu")[0]
    uo = O.pointwise_mlp2(v1o, w1, b1, w2, b2)
    assert rel(host(v0), v0o) <= TOL and rel(host(u), uo) <= TOL
    gvo = O.pointwise_mlp2_bwd(v1o, w1, b1, w2, O.rel_l2_grad(uo, y))["gx"]
    gvo = O.block_bwd(v0o, R, W, b, gvo, spec, "gelu")["gx"]
    ref = O.time_lift_bwd(a, wt, bt, wc, gvo)
    GT = 5 * TOL
    for name, got in (("gWt", gwt), ("gbt", gbt), ("gWc", gwc), ("gbc", gbc)):
        assert rel(host(got), ref[name]) <= GT, name
