"""GPU parity at the full sizes of the three large workloads ON THEIR OWN SEEDED INPUTS
(N(0,1) fields drawn slab by slab, the smooth field plus coordinate channels for the network),
against the float64 oracle evaluated slab by slab (tests/fullsize_oracle.py), whole tensors or
whole output slabs, relative L2 <= 1e-5 per tensor with float64 norms.

  cfg4  block forward, 256x256x128x32: kept spectrum in full; y_s and out for two whole output
        channels (2 x 268 M values each).
  cfg5  training step of a block (GELU, MSE against a seeded target), batch 4, 128^3 x 16: out, z
        and gx of every batch entry in full, gR, gW, gb (sums over the batch) in full.
  cfg3  lift, four blocks, projection chained at 128x128x64x32: the whole output tensor.

The launch configuration is the one bench.py times (same descriptors, same workspace sizes).
"""
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from oracle import fno_oracle as O
from paper_2204_01205_amd import binding as B
from paper_2204_01205_amd import synth
from tests import fullsize_oracle as F

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]
TOL = 1e-5


@pytest.fixture
def log(capsys):
    """progress lines that reach the terminal while the test runs (these tests take minutes)"""
    def say(msg):
        with capsys.disabled():
            print(f"[{time.strftime('%H:%M:%S')}] {msg}", flush=True)
    return say


def draw_field(seed, tensor_id, batch, channels, grid, threads=8):
    """synth.normal_field, its slabs drawn by several threads (same values)."""
    out = np.empty((batch, channels) + tuple(grid), np.float32)

    def one(bc):
        b, c = bc
        out[b, c] = synth.normal_slab(seed, tensor_id, b, c, grid)

    with ThreadPoolExecutor(threads) as tp:
        list(tp.map(one, [(b, c) for b in range(batch) for c in range(channels)]))
    return out


def upload(a):
    """host array -> GPU tensor, one (batch, channel) slab at a time (no second host copy)"""
    t = torch.empty(a.shape, dtype=torch.float32, device="cuda")
    for b in range(a.shape[0]):
        for c in range(a.shape[1]):
            t[b, c].copy_(torch.from_numpy(a[b, c]))
    return t


def layer(name, seed):
    c = synth.CONFIGS[name]
    grid, modes, width, batch = tuple(c["grid"]), tuple(c["modes"]), c["width"], c["batch"]
    spec = O.LayerSpec(grid, modes, 0)
    counts = tuple(len(k) for k in O.mode_lists(spec))
    R = synth.spectral_weights(seed, width, width, counts)
    W = synth.linear_weights(seed, width, width)
    b = synth.bias(seed, width)
    return grid, modes, width, batch, spec, counts, R, W, b


def test_cfg4_block_forward_own_input_whole_output_slabs(log):
    seed = 4
    grid, modes, width, batch, spec, counts, R, W, b = layer("cfg4", seed)
    chans = [(0, 3), (0, 17)]                    # the two output slabs compared in full
    with F.SlabPool(nproc=5, threads=3) as pool:
        # the workers draw the same slabs from the same keys and transform them while the GPU runs
        pending = pool.forward_seeded_async([(seed, synth.T_X, 0, c) for c in range(width)], spec)
        log("cfg4: drawing x")
        x = draw_field(seed, synth.T_X, batch, width, grid, threads=4)
        dx = upload(x)
        dR, dW, db = torch.from_numpy(R).cuda(), torch.from_numpy(W).cuda(), torch.from_numpy(b).cuda()
        desc = B.make_desc(batch, width, width, grid, modes, 0, B.FNO_ACT_GELU)
        ws = B.alloc_workspace(desc, B.FNO_OP_BLOCK_FWD)
        out = torch.empty_like(dx)
        xh = torch.empty((batch, width) + counts, dtype=torch.complex64, device="cuda")
        log("cfg4: GPU block forward and spectral convolution")
        B.fno_block_fwd(desc, dx, dR, dW, db, out, None, xh, ws)
        torch.cuda.synchronize()
        got_out = {k: out[k].cpu().numpy() for k in chans}
        assert bool(torch.isfinite(out).all())
        B.fno_spectral_conv_fwd(desc, dx, dR, out, None, ws)       # spectral branch alone, same buffers
        torch.cuda.synchronize()
        got_ys = {k: out[k].cpu().numpy() for k in chans}
        got_xh = xh.cpu().numpy()
        del out, dx, ws
        torch.cuda.empty_cache()

        log("cfg4: oracle spectra")
        xhat = np.stack(pending.get()).reshape((batch, width) + counts)
        e = F.rel_l2(got_xh, xhat)
        log(f"cfg4: xhat rel-L2 {e:.3e}")
        assert e <= TOL
        log("cfg4: oracle inverse + pointwise for two output channels")
        ys = F.inverse_spectrum_streamed(pool, O.mix_modes(xhat, R), spec, chans)
    for k in chans:
        e = F.rel_l2(got_ys[k], ys[k])
        log(f"cfg4: y_s{k} rel-L2 {e:.3e}")
        assert e <= TOL
    os_ = [o for (_, o) in chans]
    lin = F.pointwise_chunked(lambda xc: O.channel_affine(xc, W[os_], b[os_]), [x], nchunk=16)
    for j, k in enumerate(chans):
        want = O.gelu(ys[k] + lin[0, j])
        e = F.rel_l2(got_out[k], want)
        log(f"cfg4: out{k} rel-L2 {e:.3e}")
        assert e <= TOL


def test_cfg5_training_step_own_input_every_gradient_against_the_oracle(log):
    seed = 5
    grid, modes, width, batch, spec, counts, R, W, b = layer("cfg5", seed)
    log("cfg5: drawing x and target")
    x = draw_field(seed, synth.T_X, batch, width, grid)
    target = draw_field(seed, synth.T_TARGET, batch, width, grid)
    dx, dt = upload(x), upload(target)
    dR, dW, db = torch.from_numpy(R).cuda(), torch.from_numpy(W).cuda(), torch.from_numpy(b).cuda()
    desc = B.make_desc(batch, width, width, grid, modes, 0, B.FNO_ACT_GELU, B.FNO_FLAG_MSE_TARGET)
    ws = B.alloc_workspace(desc, B.FNO_OP_BLOCK_BWD)
    out, z, gx = torch.empty_like(dx), torch.empty_like(dx), torch.empty_like(dx)
    xh = torch.empty((batch, width) + counts, dtype=torch.complex64, device="cuda")
    gR, gW, gb = torch.empty_like(dR), torch.empty_like(dW), torch.empty_like(db)
    log("cfg5: GPU forward + backward")
    B.fno_block_fwd(desc, dx, dR, dW, db, out, z, xh, ws)
    B.fno_block_bwd(desc, dx, dR, dW, z, xh, dt, gx, gR, gW, gb, ws)
    torch.cuda.synchronize()
    got = {"out": out.cpu().numpy(), "z": z.cpu().numpy(), "gx": gx.cpu().numpy(), "xh": xh.cpu().numpy(),
           "gR": gR.cpu().numpy(), "gW": gW.cpu().numpy(), "gb": gb.cpu().numpy()}
    del dx, dt, out, z, gx, ws
    torch.cuda.empty_cache()

    acc = {"gR": 0.0, "gW": 0.0, "gb": 0.0}
    with F.SlabPool(nproc=8, threads=2) as pool:
        for bb in range(batch):
            sl = slice(bb, bb + 1)
            log(f"cfg5: oracle batch entry {bb}: forward")
            o_d, z_d, xhat = F.block_fwd_streamed(pool, x[sl], R, W, b, spec)
            zo = F.stack_slabs(z_d, 1, width)
            oo = F.stack_slabs(o_d, 1, width)
            del o_d, z_d
            for name, want in (("xh", xhat), ("z", zo), ("out", oo)):
                e = F.rel_l2(got[name][sl], want)
                log(f"cfg5: {name}[{bb}] rel-L2 {e:.3e}")
                assert e <= TOL
            # the loss is the mean over the whole batch: an entry's cotangent is that of its own mean / B
            gout = O.mse_grad(oo, target[sl]) / batch
            del oo
            log(f"cfg5: oracle batch entry {bb}: backward")
            ref = F.block_bwd_streamed(pool, x[sl], R, W, zo, xhat, gout, spec)
            e = F.rel_l2(got["gx"][sl], ref["gx"])
            log(f"cfg5: gx[{bb}] rel-L2 {e:.3e}")
            assert e <= TOL
            for k in acc:
                acc[k] = acc[k] + ref[k]
            del ref, zo, gout
    for k in acc:
        e = F.rel_l2(got[k], acc[k])
        log(f"cfg5: {k} rel-L2 {e:.3e}")
        assert e <= TOL


def test_cfg3_network_forward_own_input_whole_output(log):
    c = synth.CONFIGS["cfg3"]
    grid, modes, width = tuple(c["grid"]), tuple(c["modes"]), c["width"]
    spec = O.LayerSpec(grid, modes, 0)
    counts = tuple(len(k) for k in O.mode_lists(spec))
    npts = int(np.prod(grid))
    log("cfg3: input field")
    a = np.concatenate([synth.smooth_gaussian_field(0, grid)[None], synth.coordinate_channels(grid)])[None]
    lw, lb = synth.linear_weights(0, width, 5, synth.T_LIFT), synth.bias(0, width, synth.T_LIFT)
    blocks = [(synth.spectral_weights(10 + k, width, width, counts), synth.linear_weights(10 + k, width, width),
               synth.bias(10 + k, width)) for k in range(c["blocks"])]
    proj = (synth.linear_weights(1, c["hidden"], width, synth.T_PROJ), synth.bias(1, c["hidden"], synth.T_PROJ),
            synth.linear_weights(2, 1, c["hidden"], synth.T_PROJ), synth.bias(2, 1, synth.T_PROJ))
    dev = lambda v: torch.from_numpy(np.ascontiguousarray(v)).cuda()
    desc = B.make_desc(1, width, width, grid, modes)
    ws = B.alloc_workspace(desc, B.FNO_OP_BLOCK_FWD)
    log("cfg3: GPU lift, blocks, projection")
    v = torch.empty((1, width) + grid, device="cuda")
    B.fno_pointwise_linear(1, 5, width, npts, dev(a), dev(lw), dev(lb), v)
    for (r, w, b) in blocks:
        nxt = torch.empty_like(v)
        B.fno_block_fwd(desc, v, dev(r), dev(w), dev(b), nxt, None, None, ws)
        v = nxt
    u = torch.empty((1, 1) + grid, device="cuda")
    B.fno_pointwise_mlp2(1, width, c["hidden"], 1, npts, v, dev(proj[0]), dev(proj[1]), dev(proj[2]), dev(proj[3]), u)
    torch.cuda.synchronize()
    got = u.cpu().numpy()
    got_last = v.cpu().numpy()
    log("cfg3: oracle chain")
    with F.SlabPool(nproc=8, threads=2) as pool:
        want = F.fno_forward_streamed(pool, a, lw, lb, blocks, proj, spec, progress=lambda m: log("cfg3: " + m))
    e = F.rel_l2(got, want)
    log(f"cfg3: network output rel-L2 {e:.3e}")
    assert np.isfinite(got_last).all()
    assert e <= TOL
