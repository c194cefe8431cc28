"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module draws numbers and names workloads; it contains none of the layer's
arithmetic (no transform, no mode bookkeeping, no channel mix) and imports neither the
HIP binding nor the CPU oracle.  The tensors stand in for the paper's data sets
(Sec. 3.1: subsurface CO2-flow samples in NCXYZT layout, width 20, four blocks), which
are not available: only their shapes are kept.

Every tensor is produced slab by slab from numpy.random.default_rng([seed, tensor_id,
b, c]) so any (batch, channel) slab can be regenerated without holding the whole tensor.
"""
from __future__ import annotations

import numpy as np

# tensor ids used in the rng key
T_X, T_R, T_W, T_B, T_TARGET, T_GOUT, T_FACT, T_LIFT, T_PROJ, T_Z = range(10)

# The five workloads (grid = Nx,Ny,Nz,Nt ; modes = per-side count on x,y,z and count on t).
CONFIGS = {
    "cfg1": dict(batch=1, width=8, grid=(16, 16, 16, 8), modes=(4, 4, 4, 3), op="spectral_conv_fwd"),
    "cfg2": dict(batch=2, width=20, grid=(64, 64, 64, 16), modes=(12, 12, 12, 8), op="block_fwd"),
    "cfg3": dict(batch=1, width=20, grid=(128, 128, 64, 32), modes=(16, 16, 12, 9), op="fno4_fwd",
                 in_channels=5, hidden=128, blocks=4),
    "cfg4": dict(batch=1, width=20, grid=(256, 256, 128, 32), modes=(24, 24, 16, 9), op="block_fwd"),
    "cfg5": dict(batch=4, width=20, grid=(128, 128, 128, 16), modes=(16, 16, 16, 9), op="block_fwd_bwd"),
    # the grid shapes of the paper's own workloads (Sec. 4: training samples and the full Sleipner
    # model); the mode counts are not stated there and are chosen here
    "sleipner_train": dict(batch=1, width=20, grid=(60, 60, 64, 30), modes=(12, 12, 12, 8), op="block_fwd"),
    "sleipner_full": dict(batch=1, width=20, grid=(68, 118, 263, 16), modes=(12, 16, 24, 8), op="block_fwd"),
}


def normal_slab(seed: int, tensor_id: int, b: int, c: int, grid, std: float = 1.0) -> np.ndarray:
    """float32 (Nx, Ny, Nz, Nt) ~ N(0, std^2): the (b, c) slab of normal_field(), on its own."""
    rng = np.random.default_rng([seed, tensor_id, b, c])
    return (std * rng.standard_normal(tuple(grid))).astype(np.float32)


def normal_field(seed: int, tensor_id: int, batch: int, channels: int, grid, std: float = 1.0) -> np.ndarray:
    """float32 (B, C, Nx, Ny, Nz, Nt) ~ N(0, std^2)."""
    out = np.empty((batch, channels) + tuple(grid), np.float32)
    for b in range(batch):
        for c in range(channels):
            out[b, c] = normal_slab(seed, tensor_id, b, c, grid, std)
    return out


def spectral_weights(seed: int, c_in: int, c_out: int, counts, tensor_id: int = T_R) -> np.ndarray:
    """complex64 (Cin, Cout, Lx, Ly, Lz, mt); Re and Im independent N(0, 1/(Cin*Cout))."""
    std = 1.0 / np.sqrt(float(c_in * c_out))
    out = np.empty((c_in, c_out) + tuple(counts), np.complex64)
    for i in range(c_in):
        rng = np.random.default_rng([seed, tensor_id, i, 0])
        re = rng.standard_normal((c_out,) + tuple(counts))
        im = rng.standard_normal((c_out,) + tuple(counts))
        out[i] = (std * (re + 1j * im)).astype(np.complex64)
    return out


def linear_weights(seed: int, c_out: int, c_in: int, tensor_id: int = T_W) -> np.ndarray:
    """float32 (Cout, Cin) ~ N(0, 1/Cin)."""
    rng = np.random.default_rng([seed, tensor_id, 0, 0])
    return (rng.standard_normal((c_out, c_in)) / np.sqrt(float(c_in))).astype(np.float32)


def bias(seed: int, c_out: int, tensor_id: int = T_B) -> np.ndarray:
    """float32 (Cout,) ~ N(0, 0.01)."""
    rng = np.random.default_rng([seed, tensor_id, 0, 0])
    return (0.1 * rng.standard_normal(c_out)).astype(np.float32)


def separable_factors(seed: int, batch: int, channels: int, grid, tensor_id: int = T_FACT):
    """Four float32 arrays (B, C, N_a) of multiples of 1/8 in [-15/8, 15/8].

    The product of one value from each has at most 16 significant bits, so the rank-one
    field fx*fy*fz*ft is exactly representable in float32: a full-size tensor built from
    these on the device equals, bit for bit, the field a float64 routine reasons about.
    """
    out = []
    for a, n in enumerate(grid):
        rng = np.random.default_rng([seed, tensor_id, a, 0])
        v = rng.integers(-15, 16, size=(batch, channels, n)).astype(np.float32) / np.float32(8.0)
        out.append(v)
    return out


def rank_one_field(factors) -> np.ndarray:
    """float32 (B, C, Nx, Ny, Nz, Nt) outer product of separable_factors() (exact)."""
    fx, fy, fz, ft = factors
    return (fx[:, :, :, None, None, None] * fy[:, :, None, :, None, None]
            * fz[:, :, None, None, :, None] * ft[:, :, None, None, None, :]).astype(np.float32)


def smooth_gaussian_field(seed: int, grid, k0: float = 8.0) -> np.ndarray:
    """float32 (Nx,Ny,Nz,Nt): white noise low-passed by exp(-|k/k0|^2/2), unit variance.

    Stands in for a permeability-like input channel; built with the library FFT because
    it is input synthesis, not part of the layer.
    """
    rng = np.random.default_rng([seed, T_X, 0, 0])
    white = rng.standard_normal(tuple(grid))
    spec = np.fft.fftn(white)
    k2 = np.zeros(tuple(grid))
    for a, n in enumerate(grid):
        k = np.fft.fftfreq(n) * n
        shape = [1] * len(grid)
        shape[a] = n
        k2 = k2 + (k.reshape(shape) / k0) ** 2
    f = np.fft.ifftn(spec * np.exp(-0.5 * k2)).real
    f = f / f.std()
    return f.astype(np.float32)


def coordinate_channels(grid) -> np.ndarray:
    """float32 (4, Nx,Ny,Nz,Nt): channel a holds n_a/(N_a-1) broadcast over the other axes."""
    out = np.empty((4,) + tuple(grid), np.float32)
    for a, n in enumerate(grid):
        shape = [1] * 4
        shape[a] = n
        v = (np.arange(n, dtype=np.float64) / max(n - 1, 1)).reshape(shape)
        out[a] = np.broadcast_to(v, tuple(grid)).astype(np.float32)
    return out


def sample_points(seed: int, grid, count: int) -> np.ndarray:
    """int64 (count, 4) grid points, always including the first and last point."""
    rng = np.random.default_rng([seed, 77, 0, 0])
    pts = np.stack([rng.integers(0, n, size=count) for n in grid], axis=1).astype(np.int64)
    pts[0] = 0
    pts[-1] = np.asarray(grid) - 1
    return pts
