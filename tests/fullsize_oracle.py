"""The float64 oracle evaluated slab by slab, for parity at the full sizes of the large workloads.

TEST INFRASTRUCTURE ONLY (like oracle/): it imports the oracle and the seeded input generators,
never the HIP binding.  The oracle's functions act on whole tensors; at 256x256x128x32 with width
20 one float64 activation is 43 GB, so here the same functions are called on one (batch, channel)
slab at a time (the transforms act on each slab independently; the channel map and the activation
act on each grid point independently, so they are called on chunks of the x axis), with the slab
transforms dealt to a pool of worker processes.  Every arithmetic step is a call of an oracle
function; the few lines that join them (the scale c_kt / N of the adjoint, the sums over the batch)
repeat the bodies of oracle.block_fwd / block_bwd / spectral_conv_bwd / fno_forward, and
tests/test_fullsize_oracle.py checks on small grids that the joined result equals what those
functions return on the whole tensor.
"""
from __future__ import annotations

import multiprocessing as mp
import os

import numpy as np

from oracle import fno_oracle as O
from paper_2204_01205_amd import synth


# ---- worker side (runs in spawned processes; numpy, torch-CPU and the oracle only) ---------------
def _w_forward(args):
    slab, grid, modes, rule = args
    return O.forward_spectrum(np.asarray(slab)[None, None], O.LayerSpec(tuple(grid), tuple(modes), rule))[0, 0]


def _w_forward_seeded(args):
    seed, tensor_id, b, c, grid, modes, rule = args
    slab = synth.normal_slab(seed, tensor_id, b, c, grid)
    return O.forward_spectrum(slab[None, None], O.LayerSpec(tuple(grid), tuple(modes), rule))[0, 0]


def _w_inverse(args):
    spectrum, grid, modes, rule = args
    return O.inverse_spectrum(np.asarray(spectrum)[None, None], O.LayerSpec(tuple(grid), tuple(modes), rule))[0, 0]


class SlabPool:
    """Worker processes for slab transforms.  Spawned (never forked: the parent may hold a GPU
    context), each with a few BLAS threads."""

    def __init__(self, nproc: int = 5, threads: int = 3):
        saved = {k: os.environ.get(k) for k in ("OMP_NUM_THREADS", "OPENBLAS_NUM_THREADS", "MKL_NUM_THREADS")}
        for k in saved:
            os.environ[k] = str(threads)
        try:
            self.pool = mp.get_context("spawn").Pool(nproc)
            self.pool.map(abs, range(nproc))        # workers are up (and have read the thread limits)
        finally:
            for k, v in saved.items():
                if v is None:
                    os.environ.pop(k, None)
                else:
                    os.environ[k] = v

    def close(self):
        self.pool.terminate()
        self.pool.join()

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def forward(self, slabs, spec):
        """kept spectrum of each real slab (Nx,Ny,Nz,Nt) -> list of (Lx,Ly,Lz,mt) complex128"""
        return self.pool.map(_w_forward, [(s, spec.grid, spec.modes, spec.rule) for s in slabs], chunksize=1)

    def forward_seeded_async(self, keys, spec):
        """the same for slabs the workers draw themselves: keys = (seed, tensor_id, b, c)"""
        return self.pool.map_async(_w_forward_seeded,
                                   [tuple(k) + (spec.grid, spec.modes, spec.rule) for k in keys], chunksize=1)

    def inverse(self, spectra, spec):
        """(1/N) Re sum c_kt Yhat e^{+i theta} of each spectrum slab -> list of float64 (Nx,Ny,Nz,Nt)"""
        return self.pool.map(_w_inverse, [(s, spec.grid, spec.modes, spec.rule) for s in spectra], chunksize=1)


def x_chunks(nx: int, nchunk: int):
    step = max(1, (nx + nchunk - 1) // nchunk)
    return [slice(s, min(s + step, nx)) for s in range(0, nx, step)]


def pointwise_chunked(fn, arrays, nchunk: int = 8):
    """fn applied to matching x-axis chunks of (B, C, Nx, ...) arrays; results joined along x.
    For functions that act on every grid point independently."""
    parts = [fn(*[a[:, :, sl] for a in arrays]) for sl in x_chunks(arrays[0].shape[2], nchunk)]
    if isinstance(parts[0], dict):
        return parts
    return np.concatenate(parts, axis=2)


# ---- joined evaluations -----------------------------------------------------------------------------
def forward_spectrum_streamed(pool: SlabPool, x, spec):
    B, C = x.shape[:2]
    spectra = pool.forward([x[b, c] for b in range(B) for c in range(C)], spec)
    return np.stack(spectra).reshape((B, C) + spectra[0].shape)


def inverse_spectrum_streamed(pool: SlabPool, yhat, spec, which=None):
    """inverse transform of the listed (b, o) slabs (default: all) -> dict {(b, o): float64 slab}"""
    B, C = yhat.shape[:2]
    which = which if which is not None else [(b, o) for b in range(B) for o in range(C)]
    slabs = pool.inverse([yhat[b, o] for (b, o) in which], spec)
    return dict(zip(which, slabs))


def block_fwd_streamed(pool: SlabPool, x, r, w, b, spec, activation="gelu", which=None, xhat=None):
    """oracle.block_fwd evaluated slab by slab.  Returns (out, z, xhat): out and z are dicts
    {(batch, channel): float64 slab} for the listed output slabs (default: all)."""
    if xhat is None:
        xhat = forward_spectrum_streamed(pool, x, spec)
    ys = inverse_spectrum_streamed(pool, O.mix_modes(xhat, r), spec, which)
    out, z = {}, {}
    for bb in sorted({k[0] for k in ys}):
        chans = [o for (b2, o) in ys if b2 == bb]
        bias = None if b is None else b[chans]
        lin = pointwise_chunked(lambda xc: O.channel_affine(xc, w[chans], bias), [x[bb:bb + 1]])
        for j, o in enumerate(chans):
            z[(bb, o)] = ys[(bb, o)] + lin[0, j]
            out[(bb, o)] = O.gelu(z[(bb, o)]) if activation == "gelu" else z[(bb, o)]
    return out, z, xhat


def stack_slabs(d, B, C):
    return np.stack([np.stack([d[(b, c)] for c in range(C)]) for b in range(B)])


def block_bwd_streamed(pool: SlabPool, x, r, w, z, xhat, gout, spec, activation="gelu"):
    """oracle.block_bwd evaluated slab by slab, given the forward's z and xhat (whole arrays) and
    gout = dL/dout.  Returns dict(gx, gR, gW, gb) like the oracle."""
    B, C = x.shape[:2]
    gz = pointwise_chunked(lambda g, zz: g * (O.gelu_prime(zz) if activation == "gelu" else 1.0), [gout, z])
    # gW, gb and the W^T gz part of gx: the adjoint of the channel map, point by point, summed
    parts = pointwise_chunked(lambda xc, gc: O.pointwise_linear_bwd(xc, w, gc), [x, gz])
    g_w = sum(p["gW"] for p in parts)
    g_b = sum(p["gb"] for p in parts)
    gx_lin = np.concatenate([p["gx"] for p in parts], axis=2)
    # spectral part, as in oracle.spectral_conv_bwd
    c = O.hermitian_weights(spec.grid[3], O.mode_lists(spec)[3])
    gyh = forward_spectrum_streamed(pool, gz, spec) * (c / float(spec.npoints))
    rc = np.asarray(r, np.complex128)
    g_r = np.einsum("bixyzt,boxyzt->ioxyzt", np.conj(xhat), gyh)
    g_xh = np.einsum("ioxyzt,boxyzt->bixyzt", np.conj(rc), gyh)
    gx_s = inverse_spectrum_streamed(pool, g_xh / c, spec)
    gx = stack_slabs(gx_s, B, x.shape[1]) * float(spec.npoints) + gx_lin
    return {"gx": gx, "gR": g_r, "gW": g_w, "gb": g_b, "gz": gz}


def fno_forward_streamed(pool: SlabPool, a, lift_w, lift_b, blocks, proj, spec, progress=None):
    """oracle.fno_forward evaluated slab by slab: lift, blocks of eq. (2), projection."""
    v = pointwise_chunked(lambda ac: O.pointwise_linear(ac, lift_w, lift_b), [a])
    B, C = v.shape[:2]
    for k, (r, w, b) in enumerate(blocks):
        if progress is not None:
            progress(f"oracle block {k}")
        out, _, _ = block_fwd_streamed(pool, v, r, w, b, spec, "gelu")
        v = stack_slabs(out, B, C)
    if progress is not None:
        progress("oracle projection")
    return pointwise_chunked(lambda vc: O.pointwise_mlp2(vc, *proj), [v], nchunk=32)


def rel_l2(got, want) -> float:
    """||got - want||_2 / ||want||_2 with float64 (complex128) accumulation."""
    want = np.asarray(want)
    cplx = np.iscomplexobj(want) or np.iscomplexobj(got)
    tp = np.complex128 if cplx else np.float64
    d = np.asarray(got).astype(tp) - want.astype(tp)
    return float(np.sqrt(np.vdot(d, d).real) / max(np.sqrt(np.vdot(want.astype(tp), want.astype(tp)).real), 1e-300))
