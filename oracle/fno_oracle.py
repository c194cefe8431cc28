"""Float64 CPU oracle for the 4D (x,y,z,t) FNO spectral convolution and FNO block.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the
HIP path is checked against.  Only tests, the smoke check and the cpu_baseline
leg of the benchmark may import it; the product path never does, and this
module imports nothing from the product package.

What it computes (all in float64 / complex128, layout NCXYZT, t contiguous):

* iterative update of the neural operator, eq. (2) of the paper:
      nu_{k+1} = sigma( W nu_k + K(phi) nu_k )
* spectral convolution, eq. (3):  K(phi) nu = F^{-1}( R_phi . F nu ), where
  R_phi keeps a user-chosen number of low-frequency modes per dimension and
  multiplies them by a learned complex weight (Sec. 1.4, Fig. 5 caption:
  "R_phi is sparse, nonzero only in the low-frequency modes").
* pointwise affine map along channels, eq. (4)  y = W x + b  (Sec. 2.2).
* the adjoint of all of the above (the paper relies on autograd and on
  F^T being the adjoint DFFT, eq. (7) and Fig. 5 caption).

The method reaches these definitions exactly (a truncated spectral convolution
is a finite linear map), so the oracle is the definition written out: explicit
truncated DFT matrices applied axis by axis (the transform is separable,
Sec. 2.3), no blocking, fusion or fast transform.

Readings taken where the paper is silent (each pinned in tests/test_oracle_pins.py
or marked there as unpinned):
  A1  "keep m modes" on a spatial axis: signed frequencies 0..m-1 and -m..-1
      (rule 0, L = 2m) or -m..m (rule 1, L = 2m+1); on the real-FFT axis t the
      first mt non-negative frequencies 0..mt-1.     [parity unpinned by the paper]
  A2  the inverse takes the complex inverse over x,y,z and a complex-to-real
      transform over t last, i.e. Re( sum_k c_kt Yhat e^{+i theta} ) / N.
  A3  forward unnormalised, inverse carries 1/N.
  A4  sigma = GELU in its exact erf form.
  A5  weight tensor R[Cin][Cout][Lx][Ly][Lz][mt], mode axes in mode-list order.
  A8  complex gradient gR = dL/dRe R + i dL/dIm R.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Sequence

import numpy as np
import torch


def _erf(v: np.ndarray) -> np.ndarray:
    """erf in float64 (PyTorch's CPU routine: same values as scipy's to 1 ulp, multi-threaded)."""
    return torch.erf(torch.from_numpy(np.ascontiguousarray(v, dtype=np.float64))).numpy()

__all__ = [
    "LayerSpec", "spatial_modes", "temporal_modes", "mode_lists", "hermitian_weights",
    "dft_matrix", "forward_spectrum", "mix_modes", "inverse_spectrum",
    "spectral_conv_fwd", "spectral_conv_bwd", "channel_affine", "gelu", "gelu_prime",
    "block_fwd", "block_bwd", "mse_loss", "mse_grad",
    "brute_forward_spectrum", "brute_inverse_spectrum", "brute_spectral_conv",
    "separable_forward_spectrum", "inverse_at_points", "separable_weight_grads",
    "pointwise_linear", "pointwise_mlp2", "fno_forward",
]


# ----------------------------------------------------------------------------------------
# Mode sets (restriction part of R_phi, Sec. 1.4 below eq. (3))
# ----------------------------------------------------------------------------------------
def spatial_modes(n: int, m: int, rule: int = 0) -> list[int]:
    """Signed frequencies kept on a complex-transform axis of length n.

    rule 0: 0..m-1 then -m..-1 (L = 2m);  rule 1: 0..m then -m..-1 (L = 2m+1).
    Order is the order of the weight tensor's mode axis (reading A5).
    """
    if rule == 0:
        ks = list(range(0, m)) + list(range(-m, 0))
    elif rule == 1:
        ks = list(range(0, m + 1)) + list(range(-m, 0))
    else:
        raise ValueError("mode rule must be 0 or 1")
    if m < 0 or len(ks) > n or len(ks) == 0:
        raise ValueError(f"cannot keep {len(ks)} modes on an axis of length {n}")
    return ks


def temporal_modes(nt: int, mt: int) -> list[int]:
    """Frequencies kept on the real-FFT axis: 0..mt-1, at most floor(nt/2)+1 of them."""
    if mt < 1 or mt > nt // 2 + 1:
        raise ValueError(f"cannot keep {mt} rFFT modes on a t axis of length {nt}")
    return list(range(mt))


@dataclass(frozen=True)
class LayerSpec:
    """Shape statement of one layer: grid, modes kept per axis, mode rule."""
    grid: tuple[int, int, int, int]          # Nx, Ny, Nz, Nt
    modes: tuple[int, int, int, int]         # mx, my, mz (per side) ; mt (count on t)
    rule: int = 0

    @property
    def npoints(self) -> int:
        return int(np.prod(self.grid))


def mode_lists(spec: LayerSpec) -> list[list[int]]:
    nx, ny, nz, nt = spec.grid
    mx, my, mz, mt = spec.modes
    return [spatial_modes(nx, mx, spec.rule), spatial_modes(ny, my, spec.rule),
            spatial_modes(nz, mz, spec.rule), temporal_modes(nt, mt)]


def hermitian_weights(nt: int, kt: Sequence[int]) -> np.ndarray:
    """c_kt of the inverse real transform: 1 for kt = 0 and (nt even) kt = nt/2, else 2."""
    c = np.full(len(kt), 2.0)
    for j, k in enumerate(kt):
        if k == 0 or (nt % 2 == 0 and k == nt // 2):
            c[j] = 1.0
    return c


# ----------------------------------------------------------------------------------------
# The transform F of eq. (3), restricted to the kept modes, and its inverse
# ----------------------------------------------------------------------------------------
def dft_matrix(n: int, ks: Sequence[int], sign: float) -> np.ndarray:
    """M[j, p] = exp(sign * 2 pi i * ks[j] * p / n), shape (len(ks), n), complex128.

    The integer product ks[j]*p is reduced mod n before the division so the angle is
    exact to the last bit of 2*pi*r/n.
    """
    k = np.asarray(ks, dtype=np.int64)[:, None]
    p = np.arange(n, dtype=np.int64)[None, :]
    r = np.mod(k * p, n).astype(np.float64)
    ang = sign * 2.0 * math.pi * r / float(n)
    return np.cos(ang) + 1j * np.sin(ang)


def _apply_last(a: np.ndarray, m: np.ndarray) -> np.ndarray:
    """out[..., j] = sum_p a[..., p] * m[j, p]   (a real or complex, m complex)"""
    if np.iscomplexobj(a):
        return np.matmul(a, m.T)
    mt_ = np.ascontiguousarray(m.T)
    return np.matmul(a, mt_.real) + 1j * np.matmul(a, mt_.imag)


def _apply_axis(a: np.ndarray, m: np.ndarray, axis: int) -> np.ndarray:
    """Same contraction along another axis: out[.., j, ..] = sum_p a[.., p, ..] * m[j, p]."""
    out = np.tensordot(a, m, axes=([axis], [1]))      # contracted axis reappears last
    return np.moveaxis(out, -1, axis)


def forward_spectrum(x: np.ndarray, spec: LayerSpec) -> np.ndarray:
    """Xhat[..., jx, jy, jz, jt] = sum_n x[..., n] exp(-i theta(k, n)) for kept k only.

    x: real, shape (..., Nx, Ny, Nz, Nt).  Unnormalised forward transform (reading A3),
    applied axis by axis, t first (separability, Sec. 2.3).
    """
    x = np.asarray(x, dtype=np.float64)
    if tuple(x.shape[-4:]) != tuple(spec.grid):
        raise ValueError("grid mismatch")
    kx, ky, kz, kt = mode_lists(spec)
    nx, ny, nz, nt = spec.grid
    a = _apply_last(x, dft_matrix(nt, kt, -1.0))
    a = _apply_axis(a, dft_matrix(nz, kz, -1.0), -2)
    a = _apply_axis(a, dft_matrix(ny, ky, -1.0), -3)
    a = _apply_axis(a, dft_matrix(nx, kx, -1.0), -4)
    return a


def mix_modes(xhat: np.ndarray, r: np.ndarray) -> np.ndarray:
    """Yhat[b,o,k] = sum_i Xhat[b,i,k] R[i,o,k]  (learned pointwise weight multiplication)."""
    return np.einsum("bixyzt,ioxyzt->boxyzt", xhat, np.asarray(r, dtype=np.complex128))


def inverse_spectrum(yhat: np.ndarray, spec: LayerSpec) -> np.ndarray:
    """y[..., n] = (1/N) Re sum_{k kept} c_kt Yhat[..., k] exp(+i theta(k, n)).

    Complex inverse over x, y, z, then the complex-to-real step over t last (reading A2).
    """
    kx, ky, kz, kt = mode_lists(spec)
    nx, ny, nz, nt = spec.grid
    a = np.asarray(yhat, dtype=np.complex128)
    a = _apply_axis(a, dft_matrix(nx, kx, +1.0).T, -4)
    a = _apply_axis(a, dft_matrix(ny, ky, +1.0).T, -3)
    a = _apply_axis(a, dft_matrix(nz, kz, +1.0).T, -2)
    c = hermitian_weights(nt, kt)
    e = dft_matrix(nt, kt, +1.0) * c[:, None]           # e[j, n] = c_kt exp(+2 pi i kt n / Nt)
    # real part of sum_j a[..., j] e[j, n]
    y = np.matmul(a.real, e.real) - np.matmul(a.imag, e.imag)
    return y / float(spec.npoints)


def spectral_conv_fwd(x: np.ndarray, r: np.ndarray, spec: LayerSpec, return_xhat: bool = False):
    """K(phi) x of eq. (3).  x: (B,Cin,Nx,Ny,Nz,Nt) real; r: (Cin,Cout,Lx,Ly,Lz,mt) complex."""
    xhat = forward_spectrum(x, spec)
    y = inverse_spectrum(mix_modes(xhat, r), spec)
    return (y, xhat) if return_xhat else y


# ----------------------------------------------------------------------------------------
# Pointwise pieces: eq. (4) affine map along channels and sigma
# ----------------------------------------------------------------------------------------
def channel_affine(x: np.ndarray, w: np.ndarray, b: np.ndarray | None) -> np.ndarray:
    """y[b,o,n] = sum_i W[o,i] x[b,i,n] + b[o]   (eq. (4), contraction along channels)."""
    y = np.tensordot(np.asarray(w, np.float64), np.asarray(x, np.float64), axes=([1], [1]))   # (o, b, grid)
    y = np.moveaxis(y, 0, 1)
    if b is not None:
        y = y + np.asarray(b, np.float64)[None, :, None, None, None, None]
    return y


def gelu(z: np.ndarray) -> np.ndarray:
    """sigma(z) = z * Phi(z), Phi the standard normal CDF (exact erf form, reading A4)."""
    z = np.asarray(z, np.float64)
    return z * 0.5 * (1.0 + _erf(z / math.sqrt(2.0)))


def gelu_prime(z: np.ndarray) -> np.ndarray:
    """sigma'(z) = Phi(z) + z * phi(z)."""
    z = np.asarray(z, np.float64)
    return 0.5 * (1.0 + _erf(z / math.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi)


def _act(z, activation):
    if activation == "gelu":
        return gelu(z)
    if activation == "identity":
        return np.asarray(z, np.float64)
    raise ValueError(activation)


def _act_prime(z, activation):
    if activation == "gelu":
        return gelu_prime(z)
    if activation == "identity":
        return np.ones_like(np.asarray(z, np.float64))
    raise ValueError(activation)


def block_fwd(x, r, w, b, spec: LayerSpec, activation: str = "gelu"):
    """One FNO block, eq. (2) / Sec. 2.4:  out = sigma(W x + b + K(phi) x).

    Returns (out, z, xhat) with z the pre-activation and xhat the kept forward spectrum.
    """
    ys, xhat = spectral_conv_fwd(x, r, spec, return_xhat=True)
    z = ys + channel_affine(x, w, b)
    return _act(z, activation), z, xhat


# ----------------------------------------------------------------------------------------
# Adjoint pass
# ----------------------------------------------------------------------------------------
def spectral_conv_bwd(x, r, gy, spec: LayerSpec):
    """Adjoint of y = K(phi) x with respect to x and R, given gy = dL/dy.

    Ghat  = forward transform of gy on the kept modes; GY = (c_kt/N) Ghat is dL/dYhat in
    the sense dL = Re sum conj(GY) dYhat.  Then
        gR[i,o,k] = sum_b conj(Xhat[b,i,k]) GY[b,o,k]        (= dL/dRe R + i dL/dIm R)
        GX[b,i,k] = sum_o conj(R[i,o,k]) GY[b,o,k]
        gx[b,i,n] = Re sum_k GX[b,i,k] exp(+i theta(k,n))
    """
    kt = mode_lists(spec)[3]
    c = hermitian_weights(spec.grid[3], kt)
    xhat = forward_spectrum(x, spec)
    gyh = forward_spectrum(gy, spec) * (c / float(spec.npoints))
    rc = np.asarray(r, np.complex128)
    g_r = np.einsum("bixyzt,boxyzt->ioxyzt", np.conj(xhat), gyh)
    g_xh = np.einsum("ioxyzt,boxyzt->bixyzt", np.conj(rc), gyh)
    # Re sum_k GX e^{+i theta}: the inverse routine computes (1/N) Re sum c_kt (.) e^{+i theta}
    gx = inverse_spectrum(g_xh / c, spec) * float(spec.npoints)
    return gx, g_r


def block_bwd(x, r, w, b, gout, spec: LayerSpec, activation: str = "gelu"):
    """Gradients of a scalar L through one block, given gout = dL/dout.

    Returns dict(gx, gR, gW, gb).  gW and gb are sums over every point and batch entry
    (the adjoint of broadcasting W and b to all points is a sum-reduction, Sec. 2.1).
    """
    _, z, _ = block_fwd(x, r, w, b, spec, activation)
    gz = np.asarray(gout, np.float64) * _act_prime(z, activation)
    gb = gz.sum(axis=(0, 2, 3, 4, 5))
    gw = np.einsum("boxyzt,bixyzt->oi", gz, np.asarray(x, np.float64))
    gx_s, g_r = spectral_conv_bwd(x, r, gz, spec)
    gx = gx_s + np.einsum("oi,boxyzt->bixyzt", np.asarray(w, np.float64), gz)
    return {"gx": gx, "gR": g_r, "gW": gw, "gb": gb, "gz": gz}


def mse_loss(out, target) -> float:
    d = np.asarray(out, np.float64) - np.asarray(target, np.float64)
    return float(np.mean(d * d))


def mse_grad(out, target) -> np.ndarray:
    d = np.asarray(out, np.float64) - np.asarray(target, np.float64)
    return 2.0 * d / d.size


# ----------------------------------------------------------------------------------------
# Brute force: the n-dimensional sums of eq. (3) written literally (tiny grids only)
# ----------------------------------------------------------------------------------------
def _theta(spec: LayerSpec, k4) -> np.ndarray:
    """theta(k, n) = 2 pi (kx nx/Nx + ky ny/Ny + kz nz/Nz + kt nt/Nt) on the whole grid."""
    nx, ny, nz, nt = spec.grid
    gx, gy, gz, gt = np.meshgrid(np.arange(nx), np.arange(ny), np.arange(nz), np.arange(nt), indexing="ij")
    return 2.0 * math.pi * (k4[0] * gx / nx + k4[1] * gy / ny + k4[2] * gz / nz + k4[3] * gt / nt)


def brute_forward_spectrum(x, spec: LayerSpec) -> np.ndarray:
    x = np.asarray(x, np.float64)
    kx, ky, kz, kt = mode_lists(spec)
    out = np.zeros(x.shape[:-4] + (len(kx), len(ky), len(kz), len(kt)), np.complex128)
    for a, fa in enumerate(kx):
        for b_, fb in enumerate(ky):
            for c_, fc in enumerate(kz):
                for d, fd in enumerate(kt):
                    th = _theta(spec, (fa, fb, fc, fd))
                    out[..., a, b_, c_, d] = np.sum(x * (np.cos(th) - 1j * np.sin(th)), axis=(-4, -3, -2, -1))
    return out


def brute_inverse_spectrum(yhat, spec: LayerSpec) -> np.ndarray:
    yhat = np.asarray(yhat, np.complex128)
    kx, ky, kz, kt = mode_lists(spec)
    c = hermitian_weights(spec.grid[3], kt)
    out = np.zeros(yhat.shape[:-4] + tuple(spec.grid), np.float64)
    for a, fa in enumerate(kx):
        for b_, fb in enumerate(ky):
            for c_, fc in enumerate(kz):
                for d, fd in enumerate(kt):
                    th = _theta(spec, (fa, fb, fc, fd))
                    coef = yhat[..., a, b_, c_, d][..., None, None, None, None]
                    out += c[d] * (coef.real * np.cos(th) - coef.imag * np.sin(th))
    return out / float(spec.npoints)


def brute_spectral_conv(x, r, spec: LayerSpec) -> np.ndarray:
    xhat = brute_forward_spectrum(x, spec)
    r = np.asarray(r, np.complex128)
    bsz, cin = xhat.shape[:2]
    cout = r.shape[1]
    yhat = np.zeros((bsz, cout) + xhat.shape[2:], np.complex128)
    for bb in range(bsz):
        for o in range(cout):
            for i in range(cin):
                yhat[bb, o] += xhat[bb, i] * r[i, o]
    return brute_inverse_spectrum(yhat, spec)


# ----------------------------------------------------------------------------------------
# Full-size helpers: the same definitions evaluated where the input's structure or the
# small number of requested outputs makes them cheap
# ----------------------------------------------------------------------------------------
def separable_forward_spectrum(fx, fy, fz, ft, spec: LayerSpec) -> np.ndarray:
    """Kept spectrum of the rank-one field x[n] = fx[nx] fy[ny] fz[nz] ft[nt].

    The n-dimensional sum of eq. (3) over a product of one-dimensional factors is the
    product of the one-dimensional sums, so this is forward_spectrum() of the outer product
    without forming it.  Leading axes of the four factors must agree (e.g. (B, C)).
    """
    kx, ky, kz, kt = mode_lists(spec)
    nx, ny, nz, nt = spec.grid
    ax = _apply_last(np.asarray(fx, np.float64).astype(np.complex128), dft_matrix(nx, kx, -1.0))
    ay = _apply_last(np.asarray(fy, np.float64).astype(np.complex128), dft_matrix(ny, ky, -1.0))
    az = _apply_last(np.asarray(fz, np.float64).astype(np.complex128), dft_matrix(nz, kz, -1.0))
    at = _apply_last(np.asarray(ft, np.float64).astype(np.complex128), dft_matrix(nt, kt, -1.0))
    return (ax[..., :, None, None, None] * ay[..., None, :, None, None]
            * az[..., None, None, :, None] * at[..., None, None, None, :])


def inverse_at_points(yhat, spec: LayerSpec, points: np.ndarray) -> np.ndarray:
    """inverse_spectrum() evaluated only at the listed grid points.

    yhat: (..., Lx, Ly, Lz, mt); points: int array (P, 4) of (nx, ny, nz, nt).
    Returns (..., P).
    """
    kx, ky, kz, kt = mode_lists(spec)
    nx, ny, nz, nt = spec.grid
    c = hermitian_weights(nt, kt)
    yhat = np.asarray(yhat, np.complex128)
    pts = np.asarray(points, np.int64)
    out = np.zeros(yhat.shape[:-4] + (pts.shape[0],), np.float64)
    for p, (px, py, pz, pt) in enumerate(pts):
        ex = dft_matrix(nx, kx, +1.0)[:, px]
        ey = dft_matrix(ny, ky, +1.0)[:, py]
        ez = dft_matrix(nz, kz, +1.0)[:, pz]
        et = dft_matrix(nt, kt, +1.0)[:, pt] * c
        v = np.einsum("...xyzt,x,y,z,t->...", yhat, ex, ey, ez, et)
        out[..., p] = v.real / float(spec.npoints)
    return out


def separable_weight_grads(gz_factors, x_factors):
    """gW and gb of block_bwd() when both gz and x are rank-one fields (identity activation).

    gW[o,i] = sum_{b,n} gz[b,o,n] x[b,i,n] and gb[o] = sum_{b,n} gz[b,o,n]; for products of
    one-dimensional factors the sum over the grid is the product of the per-axis sums.
    Factors: four arrays (B, C, N_a) each.
    """
    gw = None
    gb = None
    for ga, xa in zip(gz_factors, x_factors):
        ga = np.asarray(ga, np.float64)
        xa = np.asarray(xa, np.float64)
        pair = np.einsum("bon,bin->boi", ga, xa)
        single = ga.sum(axis=2)
        gw = pair if gw is None else gw * pair
        gb = single if gb is None else gb * single
    return gw.sum(axis=0), gb.sum(axis=0)


# ----------------------------------------------------------------------------------------
# Lift / projection (Sec. 2.4, eqs. (10)-(11) and the final projection) and a whole network
# ----------------------------------------------------------------------------------------
def pointwise_linear(x, w, b=None):
    """Channel lift nu = W_c a + b_c (Sec. 2.4); same contraction as eq. (4)."""
    return channel_affine(x, w, b)


def time_lift(a, wt, bt, wc, bc):
    """The two input lifts of Sec. 2.4 (eqs. (8)-(9)), applied one after the other as written.

    a (B, Cin, Nx, Ny, Nz, 1): input with a time axis of length one.
    a_1 = W_t a + b_t along the time axis (W_t: (nt, 1), b_t: (nt,)) gives (B, Cin, Nx, Ny, Nz, nt);
    nu  = W_c a_1 + b_c along the channel axis (W_c: (C, Cin), b_c: (C,)) gives (B, C, ..., nt).
    """
    a = np.asarray(a, np.float64)
    wt = np.asarray(wt, np.float64).reshape(-1, 1)
    bt = np.asarray(bt, np.float64).reshape(-1)
    a1 = np.tensordot(a, wt, axes=([5], [1])) + bt              # contraction over the unit time axis
    return channel_affine(a1, wc, bc)


def time_lift_bwd(a, wt, bt, wc, g):
    """Adjoint of time_lift for a cotangent g of its output, the two lifts of eqs. (8)-(9) taken
    backwards one after the other: first through nu = W_c a_1 + b_c (channel axis), then through
    a_1 = W_t a + b_t (time axis).  Sums over broadcast axes are the adjoint of the broadcast
    (Sec. 2.1).  Returns ga (shape of a), gWt (nt,), gbt (nt,), gWc (C, Cin), gbc (C,)."""
    a = np.asarray(a, np.float64)
    wt = np.asarray(wt, np.float64).reshape(-1)
    bt = np.asarray(bt, np.float64).reshape(-1)
    a1 = np.tensordot(a, wt.reshape(-1, 1), axes=([5], [1])) + bt
    chan = pointwise_linear_bwd(a1, wc, g)                 # through W_c: g_{a_1}, gWc, gbc
    ga1 = chan["gx"]                                       # (B, Cin, Nx, Ny, Nz, nt)
    lead = tuple(range(ga1.ndim - 1))
    gwt = np.sum(ga1 * a, axis=lead)                       # a broadcasts along the time axis
    gbt = np.sum(ga1, axis=lead)
    ga = np.tensordot(ga1, wt, axes=([5], [0]))[..., None]
    return {"ga": ga, "gWt": gwt, "gbt": gbt, "gWc": chan["gW"], "gbc": chan["gb"]}


def rel_l2_loss(pred, target):
    """Relative L2 misfit of Sec. 4: ||pred - target||_2 / ||target||_2 over all entries."""
    pred = np.asarray(pred, np.float64)
    target = np.asarray(target, np.float64)
    return float(np.sqrt(np.sum((pred - target) ** 2)) / np.sqrt(np.sum(target ** 2)))


def rel_l2_grad(pred, target):
    """d(rel_l2_loss)/d(pred) = (pred - target) / (||pred - target||_2 ||target||_2); zero where pred == target everywhere."""
    pred = np.asarray(pred, np.float64)
    target = np.asarray(target, np.float64)
    d = pred - target
    nd = np.sqrt(np.sum(d ** 2))
    if nd == 0.0:
        return np.zeros_like(d)
    return d / (nd * np.sqrt(np.sum(target ** 2)))


def adam_step(param, grad, m, v, step, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8):
    """One update of Adam (Kingma & Ba, Algorithm 1; the optimiser of Sec. 4, learning rate 1e-3).

    step counts from 1.  Complex parameters are updated as pairs of reals.  Returns (param, m, v).
    """
    param, grad = np.asarray(param, np.float64), np.asarray(grad, np.float64)
    m = beta1 * np.asarray(m, np.float64) + (1.0 - beta1) * grad
    v = beta2 * np.asarray(v, np.float64) + (1.0 - beta2) * grad * grad
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    return param - lr * mhat / (np.sqrt(vhat) + eps), m, v


def pointwise_mlp2(x, w1, b1, w2, b2):
    """Projection to the output channels through one hidden layer: W2 sigma(W1 x + b1) + b2."""
    return channel_affine(gelu(channel_affine(x, w1, b1)), w2, b2)


def pointwise_linear_bwd(x, w, g):
    """Adjoint of y = W x + b along channels: gx = W^T g; gW and gb are sums over batch and points
    (the adjoint of broadcasting W and b, Sec. 2.1)."""
    x, w, g = np.asarray(x, np.float64), np.asarray(w, np.float64), np.asarray(g, np.float64)
    gx = np.moveaxis(np.tensordot(w, g, axes=([0], [1])), 0, 1)            # (b, i, grid)
    axes = [0] + list(range(2, g.ndim))
    gw = np.tensordot(g, x, axes=(axes, axes))                              # (o, i)
    return {"gx": gx, "gW": gw, "gb": g.sum(axis=tuple(axes))}


def pointwise_mlp2_bwd(x, w1, b1, w2, g):
    """Adjoint of u = W2 sigma(W1 x + b1) + b2 for a cotangent g of u, by the chain rule."""
    h = channel_affine(x, w1, b1)
    outer = pointwise_linear_bwd(gelu(h), w2, g)          # through W2: gives g_a, gW2, gb2
    gh = outer["gx"] * gelu_prime(h)
    inner = pointwise_linear_bwd(x, w1, gh)               # through W1: gives gx, gW1, gb1
    return {"gx": inner["gx"], "gW1": inner["gW"], "gb1": inner["gb"], "gW2": outer["gW"], "gb2": outer["gb"]}


def fno_backward(a, lift_w, lift_b, blocks, proj, spec: LayerSpec, gu):
    """Gradients of the whole network (lift, blocks of eq. (2), projection) for a cotangent gu of
    its output: the forward is replayed keeping each block's input, then the chain runs backwards."""
    w1, b1, w2, _ = proj
    vs = [pointwise_linear(a, lift_w, lift_b)]
    for (r, w, b) in blocks:
        vs.append(block_fwd(vs[-1], r, w, b, spec, "gelu")[0])
    gp = pointwise_mlp2_bwd(vs[-1], w1, b1, w2, gu)
    grads = {"proj": gp, "blocks": []}
    gv = gp["gx"]
    for (r, w, b), vin in zip(reversed(blocks), reversed(vs[:-1])):
        gb_ = block_bwd(vin, r, w, b, gv, spec, "gelu")
        grads["blocks"].insert(0, gb_)
        gv = gb_["gx"]
    grads["lift"] = pointwise_linear_bwd(a, lift_w, gv)
    return grads


def fno_forward(a, lift_w, lift_b, blocks, proj, spec: LayerSpec):
    """Lift, K blocks of eq. (2), projection.  blocks: list of (R, W, b); proj: (w1,b1,w2,b2)."""
    v = pointwise_linear(a, lift_w, lift_b)
    for (r, w, b) in blocks:
        v, _, _ = block_fwd(v, r, w, b, spec, "gelu")
    return pointwise_mlp2(v, *proj)
