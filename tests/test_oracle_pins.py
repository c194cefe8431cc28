"""Pins of the float64 oracle against things other than itself (CPU only).

Nothing here calls the HIP path.  Each test names what fixes the expected value:
brute-force sums of eq. (3), numpy's FFT as the textbook special case, closed forms of
single-mode inputs, invariants (linearity, Parseval, shift equivariance, adjoint identity)
and central finite differences for every gradient.
"""
import math

import numpy as np
import pytest

from oracle import fno_oracle as O


def _rng(*key):
    return np.random.default_rng(list(key))


def _rand_layer(seed, spec, b=2, cin=2, cout=3):
    rng = _rng(seed, 1)
    lx, ly, lz, lt = [len(k) for k in O.mode_lists(spec)]
    x = rng.standard_normal((b, cin) + spec.grid)
    r = rng.standard_normal((cin, cout, lx, ly, lz, lt)) + 1j * rng.standard_normal((cin, cout, lx, ly, lz, lt))
    return x, r


def _rel(a, b):
    return np.linalg.norm(np.ravel(a - b)) / max(np.linalg.norm(np.ravel(b)), 1e-300)


TINY = [
    O.LayerSpec((6, 4, 4, 6), (2, 1, 2, 3), 0),     # even sizes, mt below Nyquist
    O.LayerSpec((4, 6, 4, 4), (2, 2, 1, 3), 0),     # mt = Nt/2+1: Nyquist bin kept
    O.LayerSpec((5, 3, 4, 5), (2, 1, 1, 3), 0),     # odd sizes, odd Nt (no Nyquist bin exists)
    O.LayerSpec((5, 4, 3, 6), (1, 1, 1, 2), 1),     # symmetric rule -m..m
    O.LayerSpec((4, 4, 6, 7), (2, 2, 3, 4), 0),     # full spatial sets, odd Nt full half-spectrum
]


# ------------------------------------------------------------------ mode sets (A1, A5)
def test_mode_lists_literal():
    assert O.spatial_modes(16, 4, 0) == [0, 1, 2, 3, -4, -3, -2, -1]
    assert O.spatial_modes(16, 4, 1) == [0, 1, 2, 3, 4, -4, -3, -2, -1]
    assert O.temporal_modes(8, 3) == [0, 1, 2]
    assert O.temporal_modes(16, 9) == list(range(9))
    with pytest.raises(ValueError):
        O.temporal_modes(16, 10)
    with pytest.raises(ValueError):
        O.spatial_modes(6, 4, 0)
    # the five workloads' retained counts
    for grid, modes, want in [((16, 16, 16, 8), (4, 4, 4, 3), (8, 8, 8, 3)),
                              ((64, 64, 64, 16), (12, 12, 12, 8), (24, 24, 24, 8)),
                              ((128, 128, 64, 32), (16, 16, 12, 9), (32, 32, 24, 9)),
                              ((256, 256, 128, 32), (24, 24, 16, 9), (48, 48, 32, 9)),
                              ((128, 128, 128, 16), (16, 16, 16, 9), (32, 32, 32, 9))]:
        got = tuple(len(k) for k in O.mode_lists(O.LayerSpec(grid, modes, 0)))
        assert got == want


def test_hermitian_weights_literal():
    assert O.hermitian_weights(8, [0, 1, 2, 3, 4]).tolist() == [1, 2, 2, 2, 1]
    assert O.hermitian_weights(7, [0, 1, 2, 3]).tolist() == [1, 2, 2, 2]
    assert O.hermitian_weights(16, [0, 1, 2]).tolist() == [1, 2, 2]


# ------------------------------------------------------------------ P1 brute force
@pytest.mark.parametrize("spec", TINY)
def test_P1_definition_equals_brute_force(spec):
    x, r = _rand_layer(11, spec)
    assert _rel(O.forward_spectrum(x, spec), O.brute_forward_spectrum(x, spec)) < 1e-12
    yh = O.mix_modes(O.forward_spectrum(x, spec), r)
    assert _rel(O.inverse_spectrum(yh, spec), O.brute_inverse_spectrum(yh, spec)) < 1e-12
    assert _rel(O.spectral_conv_fwd(x, r, spec), O.brute_spectral_conv(x, r, spec)) < 1e-12


# ------------------------------------------------------------------ P2 library FFT special case
def _lib_spectral_conv(x, r, spec):
    """rfftn -> gather kept modes -> mix -> scatter into zeros -> irfftn (numpy only)."""
    kx, ky, kz, kt = O.mode_lists(spec)
    nx, ny, nz, nt = spec.grid
    full = np.fft.rfftn(x, axes=(-4, -3, -2, -1))
    ix = np.mod(kx, nx)
    iy = np.mod(ky, ny)
    iz = np.mod(kz, nz)
    it = np.asarray(kt)
    kept = full[:, :, ix][:, :, :, iy][:, :, :, :, iz][:, :, :, :, :, it]
    yh = np.einsum("bixyzt,ioxyzt->boxyzt", kept, r)
    big = np.zeros((x.shape[0], r.shape[1], nx, ny, nz, nt // 2 + 1), complex)
    big[np.ix_(range(x.shape[0]), range(r.shape[1]), ix, iy, iz, it)] = yh
    return np.fft.irfftn(big, s=spec.grid, axes=(-4, -3, -2, -1)), kept


@pytest.mark.parametrize("spec", TINY + [O.LayerSpec((16, 16, 16, 8), (4, 4, 4, 3), 0),
                                          O.LayerSpec((12, 10, 9, 11), (3, 2, 4, 5), 1)])
def test_P2_equals_numpy_fft_route(spec):
    x, r = _rand_layer(12, spec)
    want, kept = _lib_spectral_conv(x, r, spec)
    got, xhat = O.spectral_conv_fwd(x, r, spec, return_xhat=True)
    assert _rel(xhat, kept) < 1e-12
    assert _rel(got, want) < 1e-12


# ------------------------------------------------------------------ P3 linearity
def test_P3_linear_in_input_and_weights():
    spec = TINY[0]
    x1, r1 = _rand_layer(13, spec)
    x2, r2 = _rand_layer(14, spec)
    a, b = 0.7, -1.9
    lhs = O.spectral_conv_fwd(a * x1 + b * x2, r1, spec)
    rhs = a * O.spectral_conv_fwd(x1, r1, spec) + b * O.spectral_conv_fwd(x2, r1, spec)
    assert _rel(lhs, rhs) < 1e-12
    lhs = O.spectral_conv_fwd(x1, a * r1 + b * r2, spec)
    rhs = a * O.spectral_conv_fwd(x1, r1, spec) + b * O.spectral_conv_fwd(x1, r2, spec)
    assert _rel(lhs, rhs) < 1e-12


# ------------------------------------------------------------------ P4 identity and Parseval
@pytest.mark.parametrize("grid", [(4, 6, 4, 8), (6, 4, 2, 6)])
def test_P4_full_mode_set_is_identity_and_parseval(grid):
    spec = O.LayerSpec(grid, (grid[0] // 2, grid[1] // 2, grid[2] // 2, grid[3] // 2 + 1), 0)
    rng = _rng(15)
    x = rng.standard_normal((1, 1) + grid)
    r = np.ones((1, 1) + tuple(len(k) for k in O.mode_lists(spec)), complex)
    assert _rel(O.spectral_conv_fwd(x, r, spec), x) < 1e-12
    xhat = O.forward_spectrum(x, spec)
    c = O.hermitian_weights(grid[3], O.mode_lists(spec)[3])
    assert abs(np.sum(x * x) - np.sum(c * np.abs(xhat) ** 2) / spec.npoints) < 1e-10 * np.sum(x * x)


def test_P4_identity_odd_sizes_symmetric_rule():
    grid = (5, 3, 7, 5)
    spec = O.LayerSpec(grid, (2, 1, 3, 3), 1)
    x = _rng(16).standard_normal((1, 1) + grid)
    r = np.ones((1, 1) + tuple(len(k) for k in O.mode_lists(spec)), complex)
    assert _rel(O.spectral_conv_fwd(x, r, spec), x) < 1e-12


# ------------------------------------------------------------------ P5 single-mode closed forms
def _theta(spec, k4):
    nx, ny, nz, nt = spec.grid
    g = np.meshgrid(*[np.arange(n) for n in spec.grid], indexing="ij")
    return 2 * math.pi * (k4[0] * g[0] / nx + k4[1] * g[1] / ny + k4[2] * g[2] / nz + k4[3] * g[3] / nt)


def _one_hot_r(spec, k4, val):
    lists = O.mode_lists(spec)
    r = np.zeros((1, 1) + tuple(len(k) for k in lists), complex)
    idx = tuple(lists[a].index(k4[a]) for a in range(4))
    r[(0, 0) + idx] = val
    return r


def test_P5a_interior_mode_rotates_and_scales_a_cosine():
    spec = O.LayerSpec((8, 6, 8, 8), (3, 2, 3, 4), 0)
    rw = 0.8 * np.exp(1j * 0.6)
    for k4 in [(2, -1, 1, 2), (-3, 1, -2, 1), (0, 0, 0, 3), (1, 1, -3, 3)]:
        phi = 0.37
        x = np.cos(_theta(spec, k4) + phi)[None, None]
        y = O.spectral_conv_fwd(x, _one_hot_r(spec, k4, rw), spec)
        want = abs(rw) * np.cos(_theta(spec, k4) + phi + np.angle(rw))
        assert np.max(np.abs(y[0, 0] - want)) < 1e-13


def test_P5b_kt0_mode_is_halved_unless_partner_carries_conjugate():
    spec = O.LayerSpec((8, 6, 8, 8), (3, 2, 3, 4), 0)
    rw = 1.3 * np.exp(-1j * 1.1)
    k4 = (2, -1, 1, 0)
    neg = (-2, 1, -1, 0)
    phi = -0.52
    x = np.cos(_theta(spec, k4) + phi)[None, None]
    y = O.spectral_conv_fwd(x, _one_hot_r(spec, k4, rw), spec)
    want = 0.5 * abs(rw) * np.cos(_theta(spec, k4) + phi + np.angle(rw))
    assert np.max(np.abs(y[0, 0] - want)) < 1e-13
    r = _one_hot_r(spec, k4, rw) + _one_hot_r(spec, neg, np.conj(rw))
    y = O.spectral_conv_fwd(x, r, spec)
    assert np.max(np.abs(y[0, 0] - 2 * want)) < 1e-13
    # DC: a constant field is scaled by Re(r)
    y = O.spectral_conv_fwd(np.full((1, 1) + spec.grid, 1.7), _one_hot_r(spec, (0, 0, 0, 0), rw), spec)
    assert np.max(np.abs(y - rw.real * 1.7)) < 1e-13


def test_P5c_nyquist_mode():
    # kt = Nt/2 kept: cos(pi*nt + spatial phase) behaves like a kt=0 plane (weight c = 1)
    spec = O.LayerSpec((4, 4, 4, 6), (2, 2, 2, 4), 0)
    rw = 0.9 * np.exp(1j * 0.4)
    k4 = (1, 0, -1, 3)
    x = np.cos(_theta(spec, k4) + 0.2)[None, None]
    y = O.spectral_conv_fwd(x, _one_hot_r(spec, k4, rw), spec)
    want = 0.5 * abs(rw) * np.cos(_theta(spec, k4) + 0.2 + np.angle(rw))
    assert np.max(np.abs(y[0, 0] - want)) < 1e-13


# ------------------------------------------------------------------ P6 truncation exactness
def test_P6_only_kept_frequencies_pass():
    spec = O.LayerSpec((6, 4, 4, 6), (2, 1, 1, 2), 0)
    lists = O.mode_lists(spec)
    kept = {(a, b, c, d) for a in lists[0] for b in lists[1] for c in lists[2] for d in lists[3]}
    r = np.ones((1, 1) + tuple(len(k) for k in lists), complex)
    nx, ny, nz, nt = spec.grid

    for ax in range(nx):
        for ay in range(ny):
            for az in range(nz):
                for at in range(nt // 2 + 1):
                    x = np.cos(_theta(spec, (ax, ay, az, at)))[None, None]
                    y = O.spectral_conv_fwd(x, r, spec)
                    reps = []
                    for s in (+1, -1):
                        kt_ = s * at
                        if kt_ % nt > nt // 2:
                            continue
                        kk = ((s * ax) % nx, (s * ay) % ny, (s * az) % nz, kt_ % nt)
                        reps.append(kk)
                    hit = False
                    for kk in reps:
                        for cand in kept:
                            if (cand[0] % nx, cand[1] % ny, cand[2] % nz, cand[3]) == kk:
                                hit = True
                    if hit:
                        assert np.max(np.abs(y)) > 1e-3
                    else:
                        assert np.max(np.abs(y)) < 1e-12


def test_one_hot_weight_lights_the_matching_frequency():
    # A5: entry (jx,jy,jz,jt) of R acts on frequency (kx[jx], ky[jy], kz[jz], kt[jt])
    spec = O.LayerSpec((8, 8, 8, 8), (2, 2, 2, 3), 0)
    lists = O.mode_lists(spec)
    j = (3, 1, 2, 2)                       # -> k = (-1, 1, -2, 2)
    k4 = tuple(lists[a][j[a]] for a in range(4))
    assert k4 == (-1, 1, -2, 2)
    r = np.zeros((1, 1, 4, 4, 4, 3), complex)
    r[(0, 0) + j] = 1.0
    x = _rng(21).standard_normal((1, 1) + spec.grid)
    y = O.spectral_conv_fwd(x, r, spec)
    spec_full = np.fft.fftn(y[0, 0])
    mag = np.abs(spec_full)
    peak = np.unravel_index(np.argmax(mag), mag.shape)
    want_a = tuple(np.mod(k4, spec.grid))
    want_b = tuple(np.mod([-v for v in k4], spec.grid))
    assert peak in (want_a, want_b)
    mask = np.ones_like(mag, bool)
    mask[want_a] = False
    mask[want_b] = False
    assert np.max(mag[mask]) < 1e-9 * mag[peak]


# ------------------------------------------------------------------ P7 zero weights
def test_P7_zero_weights_give_zero_and_block_reduces_to_pointwise():
    spec = TINY[1]
    x, r = _rand_layer(17, spec, cin=3, cout=3)
    assert np.all(O.spectral_conv_fwd(x, 0 * r, spec) == 0.0)
    rng = _rng(18)
    w = rng.standard_normal((3, 3))
    b = rng.standard_normal(3)
    out, z, _ = O.block_fwd(x, 0 * r, w, b, spec)
    zz = np.zeros_like(x)
    for bb in range(x.shape[0]):
        for o in range(3):
            zz[bb, o] = b[o] + sum(w[o, i] * x[bb, i] for i in range(3))
    assert _rel(z, zz) < 1e-14
    from scipy.stats import norm
    assert _rel(out, zz * norm.cdf(zz)) < 1e-13


def test_gelu_textbook_values():
    # Phi(1) = 0.8413447460685429 (standard normal table); sigma(z) - sigma(-z) = z
    assert abs(O.gelu(np.array(1.0)) - 0.8413447460685429) < 1e-15
    assert abs(O.gelu(np.array(-1.0)) + 0.15865525393145707) < 1e-15
    assert O.gelu(np.array(0.0)) == 0.0
    z = np.linspace(-6, 6, 101)
    assert np.max(np.abs(O.gelu(z) - O.gelu(-z) - z)) < 1e-14
    h = 1e-6
    fd = (O.gelu(z + h) - O.gelu(z - h)) / (2 * h)
    assert np.max(np.abs(fd - O.gelu_prime(z))) < 1e-9


# ------------------------------------------------------------------ P8 Hermitian weights -> real inverse
def test_P8_hermitian_weights_make_complex_inverse_real():
    spec = O.LayerSpec((6, 5, 4, 6), (2, 2, 1, 2), 1)
    lists = O.mode_lists(spec)
    x, r = _rand_layer(19, spec, b=1, cin=1, cout=1)
    # enforce R(-k_xyz, kt=0) = conj(R(k_xyz, kt=0))
    for ax, fa in enumerate(lists[0]):
        for ay, fb in enumerate(lists[1]):
            for az, fc in enumerate(lists[2]):
                pa, pb, pc = lists[0].index(-fa), lists[1].index(-fb), lists[2].index(-fc)
                r[0, 0, pa, pb, pc, 0] = np.conj(r[0, 0, ax, ay, az, 0])
    r[0, 0, 0, 0, 0, 0] = r[0, 0, 0, 0, 0, 0].real        # the self-paired DC entry must be real
    yh = O.mix_modes(O.forward_spectrum(x, spec), r)[0, 0, :, :, :, 0]
    ex = O.dft_matrix(6, lists[0], +1.0)
    ey = O.dft_matrix(5, lists[1], +1.0)
    ez = O.dft_matrix(4, lists[2], +1.0)
    v = np.einsum("xyz,xa,yb,zc->abc", yh, ex, ey, ez)
    assert np.max(np.abs(v.imag)) < 1e-12 * np.max(np.abs(v.real))


# ------------------------------------------------------------------ P9 shift equivariance / convolution theorem
def test_P9_shift_equivariance():
    spec = TINY[2]
    x, r = _rand_layer(20, spec)
    y = O.spectral_conv_fwd(x, r, spec)
    for axis, s in [(-4, 2), (-3, 1), (-2, 3), (-1, 2)]:
        ys = O.spectral_conv_fwd(np.roll(x, s, axis=axis), r, spec)
        assert _rel(ys, np.roll(y, s, axis=axis)) < 1e-12


def test_P9_circular_convolution_with_kernel():
    spec = O.LayerSpec((4, 3, 4, 6), (1, 1, 2, 3), 0)
    x, r = _rand_layer(22, spec, b=1, cin=1, cout=1)
    y = O.spectral_conv_fwd(x, r, spec)[0, 0]
    delta = np.zeros((1, 1) + spec.grid)
    delta[0, 0, 0, 0, 0, 0] = 1.0
    kappa = O.spectral_conv_fwd(delta, r, spec)[0, 0]
    nx, ny, nz, nt = spec.grid
    want = np.zeros(spec.grid)
    for a in range(nx):
        for b in range(ny):
            for c in range(nz):
                for d in range(nt):
                    want += x[0, 0, a, b, c, d] * np.roll(kappa, (a, b, c, d), axis=(0, 1, 2, 3))
    assert _rel(y, want) < 1e-12


# ------------------------------------------------------------------ P10 adjoint identity
@pytest.mark.parametrize("spec", TINY)
def test_P10_adjoint_is_layer_with_conjugate_transposed_weights(spec):
    x, r = _rand_layer(23, spec, b=2, cin=2, cout=3)
    y = _rng(24).standard_normal((2, 3) + spec.grid)
    rh = np.conj(np.swapaxes(r, 0, 1))
    lhs = np.sum(O.spectral_conv_fwd(x, r, spec) * y)
    rhs = np.sum(x * O.spectral_conv_fwd(y, rh, spec))
    assert abs(lhs - rhs) < 1e-12 * abs(lhs)
    gx, _ = O.spectral_conv_bwd(x, r, y, spec)
    assert _rel(gx, O.spectral_conv_fwd(y, rh, spec)) < 1e-12


# ------------------------------------------------------------------ P11 gradients by finite differences
@pytest.mark.parametrize("spec,activation", [(TINY[0], "gelu"), (TINY[1], "gelu"), (TINY[2], "gelu"),
                                              (TINY[3], "identity")])
def test_P11_block_gradients_match_central_differences(spec, activation):
    rng = _rng(25)
    x, r = _rand_layer(26, spec, b=2, cin=2, cout=2)
    w = rng.standard_normal((2, 2))
    b = rng.standard_normal(2)
    target = rng.standard_normal(x.shape)

    def loss(x_, r_, w_, b_):
        out, _, _ = O.block_fwd(x_, r_, w_, b_, spec, activation)
        return O.mse_loss(out, target)

    out, _, _ = O.block_fwd(x, r, w, b, spec, activation)
    g = O.block_bwd(x, r, w, b, O.mse_grad(out, target), spec, activation)
    h = 1e-6
    pick = _rng(27)

    def check(arr, grad, rebuild, n=12, complex_part=None):
        flat_idx = pick.choice(arr.size, size=min(n, arr.size), replace=False)
        for fi in flat_idx:
            idx = np.unravel_index(fi, arr.shape)
            d = np.zeros_like(arr)
            d[idx] = h if complex_part != "im" else 1j * h
            fd = (loss(*rebuild(arr + d)) - loss(*rebuild(arr - d))) / (2 * h)
            an = grad[idx] if complex_part is None else (grad[idx].real if complex_part == "re" else grad[idx].imag)
            assert abs(fd - an) < 1e-9 + 1e-6 * abs(an), (idx, fd, an)

    check(x, g["gx"], lambda v: (v, r, w, b))
    check(w, g["gW"], lambda v: (x, r, v, b))
    check(b, g["gb"], lambda v: (x, r, w, v))
    check(r, g["gR"], lambda v: (x, v, w, b), complex_part="re")
    check(r, g["gR"], lambda v: (x, v, w, b), complex_part="im")
    # entries on the kt = 0 plane explicitly (they carry the half weight)
    r0 = r.copy()
    idx0 = (0, 1, 1, 0, 1, 0)
    for part in ("re", "im"):
        d = np.zeros_like(r0)
        d[idx0] = h if part == "re" else 1j * h
        fd = (loss(x, r0 + d, w, b) - loss(x, r0 - d, w, b)) / (2 * h)
        an = g["gR"][idx0].real if part == "re" else g["gR"][idx0].imag
        assert abs(fd - an) < 1e-9 + 1e-6 * abs(an)


# ------------------------------------------------------------------ full-size helpers equal the plain routines
def test_separable_spectrum_and_point_sampled_inverse_match_plain_routines():
    spec = O.LayerSpec((6, 5, 8, 6), (2, 2, 3, 3), 0)
    rng = _rng(28)
    f = [rng.integers(-15, 16, size=(2, 3, n)) / 8.0 for n in spec.grid]
    x = (f[0][:, :, :, None, None, None] * f[1][:, :, None, :, None, None]
         * f[2][:, :, None, None, :, None] * f[3][:, :, None, None, None, :])
    assert _rel(O.separable_forward_spectrum(*f, spec), O.forward_spectrum(x, spec)) < 1e-12
    yh = O.forward_spectrum(x, spec)
    full = O.inverse_spectrum(yh, spec)
    pts = np.array([[0, 0, 0, 0], [5, 4, 7, 5], [2, 3, 1, 4], [3, 0, 6, 2]])
    got = O.inverse_at_points(yh, spec, pts)
    for p, (a, b, c, d) in enumerate(pts):
        assert np.max(np.abs(got[..., p] - full[..., a, b, c, d])) < 1e-13


def test_network_pieces():
    spec = O.LayerSpec((4, 4, 4, 4), (1, 1, 1, 2), 0)
    rng = _rng(29)
    a = rng.standard_normal((1, 3) + spec.grid)
    lw, lb = rng.standard_normal((4, 3)), rng.standard_normal(4)
    v = O.pointwise_linear(a, lw, lb)
    assert abs(v[0, 2, 1, 2, 3, 0] - (lb[2] + lw[2] @ a[0, :, 1, 2, 3, 0])) < 1e-13
    w1, b1 = rng.standard_normal((6, 4)), rng.standard_normal(6)
    w2, b2 = rng.standard_normal((1, 6)), rng.standard_normal(1)
    u = O.pointwise_mlp2(v, w1, b1, w2, b2)
    hvec = w1 @ v[0, :, 3, 1, 0, 2] + b1
    from scipy.stats import norm
    assert abs(u[0, 0, 3, 1, 0, 2] - (w2 @ (hvec * norm.cdf(hvec)) + b2)[0]) < 1e-13


def test_separable_weight_grads_match_block_bwd():
    spec = O.LayerSpec((4, 5, 6, 4), (1, 2, 2, 2), 0)
    rng = _rng(30)
    fx = [rng.integers(-15, 16, size=(2, 3, n)) / 8.0 for n in spec.grid]
    fg = [rng.integers(-15, 16, size=(2, 3, n)) / 8.0 for n in spec.grid]

    def outer(f):
        return (f[0][:, :, :, None, None, None] * f[1][:, :, None, :, None, None]
                * f[2][:, :, None, None, :, None] * f[3][:, :, None, None, None, :])

    x, g = outer(fx), outer(fg)
    _, r = _rand_layer(31, spec, b=2, cin=3, cout=3)
    w = rng.standard_normal((3, 3))
    ref = O.block_bwd(x, r, w, np.zeros(3), g, spec, "identity")
    gw, gb = O.separable_weight_grads(fg, fx)
    assert _rel(gw, ref["gW"]) < 1e-13 and _rel(gb, ref["gb"]) < 1e-13


def test_oracle_reproduces_its_frozen_fixture():
    """tests/golden/block_small.txt was written by tests/golden/make_golden.py from the oracle alone."""
    import importlib.util
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    spec_ = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec_)
    spec_.loader.exec_module(mod)
    stored = {}
    for line in open(os.path.join(here, "golden", "block_small.txt")):
        if not line.startswith("#"):
            name, val = line.rstrip("\n").split("\t")
            stored[name] = float(val)
    got = dict(mod.values())
    assert set(got) == set(stored)
    for name, v in got.items():
        assert abs(float(v) - stored[name]) <= 1e-12 * max(1.0, abs(stored[name])), name


def test_time_lift_against_loops_closed_forms_and_the_channel_lift():
    """Sec. 2.4, eqs. (8)-(9): a_1 = W_t a + b_t along time, nu = W_c a_1 + b_c along channels."""
    rng = np.random.default_rng(31)
    B, Cin, C, grid, nt = 2, 3, 4, (2, 3, 2), 5
    a = rng.standard_normal((B, Cin) + grid + (1,))
    wt, bt = rng.standard_normal(nt), rng.standard_normal(nt)
    wc, bc = rng.standard_normal((C, Cin)), rng.standard_normal(C)
    got = O.time_lift(a, wt, bt, wc, bc)
    assert got.shape == (B, C) + grid + (nt,)
    # plain loops over every index
    want = np.zeros_like(got)
    for b in range(B):
        for c in range(C):
            for x in range(grid[0]):
                for y in range(grid[1]):
                    for z in range(grid[2]):
                        for t in range(nt):
                            acc = bc[c]
                            for j in range(Cin):
                                acc += wc[c, j] * (wt[t] * a[b, j, x, y, z, 0] + bt[t])
                            want[b, c, x, y, z, t] = acc
    assert np.max(np.abs(got - want)) <= 1e-13
    # zero input: nu[c, t] = b_t[t] * sum_j W_c[c, j] + b_c[c] at every point
    zero = O.time_lift(np.zeros_like(a), wt, bt, wc, bc)
    closed = bt[None, :] * wc.sum(axis=1)[:, None] + bc[:, None]
    assert np.max(np.abs(zero - closed[None, :, None, None, None, :])) <= 1e-13
    # W_t = 1, b_t = 0: every time slice is the channel lift of the input
    ones = O.time_lift(a, np.ones(nt), np.zeros(nt), wc, bc)
    lifted = O.pointwise_linear(a, wc, bc)
    assert np.max(np.abs(ones - np.repeat(lifted, nt, axis=5))) <= 1e-13
    # affine in a: differences are linear and lose both biases
    a2 = rng.standard_normal(a.shape)
    d = O.time_lift(a + a2, wt, bt, wc, bc) - O.time_lift(a2, wt, bt, wc, bc)
    lin = O.time_lift(a, wt, np.zeros(nt), wc, np.zeros(C))
    assert np.max(np.abs(d - lin)) <= 1e-12


def test_time_lift_adjoint_against_loops_and_finite_differences():
    """The adjoint of the two lifts of eqs. (8)-(9): every gradient against plain loops over all
    indices and against central differences of L = <g, time_lift(...)>."""
    rng = np.random.default_rng(37)
    B, Cin, C, grid, nt = 2, 3, 4, (2, 2, 3), 5
    a = rng.standard_normal((B, Cin) + grid + (1,))
    wt, bt = rng.standard_normal(nt), rng.standard_normal(nt)
    wc, bc = rng.standard_normal((C, Cin)), rng.standard_normal(C)
    g = rng.standard_normal((B, C) + grid + (nt,))
    got = O.time_lift_bwd(a, wt, bt, wc, g)
    # loops: d nu[b,c,p,t] / d each parameter, from nu = sum_j wc[c,j] (wt[t] a[b,j,p] + bt[t]) + bc[c]
    gwt, gbt, gwc, gbc, ga = np.zeros(nt), np.zeros(nt), np.zeros((C, Cin)), np.zeros(C), np.zeros(a.shape)
    for b in range(B):
        for c in range(C):
            for x in range(grid[0]):
                for y in range(grid[1]):
                    for z in range(grid[2]):
                        for t in range(nt):
                            gv = g[b, c, x, y, z, t]
                            gbc[c] += gv
                            for j in range(Cin):
                                av = a[b, j, x, y, z, 0]
                                gwc[c, j] += gv * (wt[t] * av + bt[t])
                                gwt[t] += gv * wc[c, j] * av
                                gbt[t] += gv * wc[c, j]
                                ga[b, j, x, y, z, 0] += gv * wc[c, j] * wt[t]
    for name, want in (("gWt", gwt), ("gbt", gbt), ("gWc", gwc), ("gbc", gbc), ("ga", ga)):
        assert np.max(np.abs(got[name] - want)) <= 1e-12 * max(1.0, np.max(np.abs(want))), name
    # central differences (the map is affine in each argument: exact up to rounding)
    def L(a_, wt_, bt_, wc_, bc_):
        return float(np.sum(g * O.time_lift(a_, wt_, bt_, wc_, bc_)))
    h = 1e-3
    for name, idx, arg in (("gWt", (2,), 1), ("gbt", (4,), 2), ("gWc", (1, 2), 3), ("gbc", (3,), 4),
                           ("ga", (1, 2, 1, 0, 2, 0), 0)):
        args = [a, wt, bt, wc, bc]
        plus = [v.copy() for v in args]
        minus = [v.copy() for v in args]
        plus[arg][idx] += h
        minus[arg][idx] -= h
        fd = (L(*plus) - L(*minus)) / (2 * h)
        assert abs(fd - got[name][idx]) <= 1e-8 * max(1.0, abs(fd)), name
    # W_t = 1, b_t = 0 reduces the channel part to the adjoint of the channel lift summed over time
    ones = O.time_lift_bwd(a, np.ones(nt), np.zeros(nt), wc, g)
    lin = O.pointwise_linear_bwd(a, wc, g.sum(axis=5, keepdims=True))
    assert np.max(np.abs(ones["gWc"] - lin["gW"])) <= 1e-12
    assert np.max(np.abs(ones["ga"] - lin["gx"])) <= 1e-12


def test_relative_l2_loss_and_its_gradient():
    """Sec. 4: L(y, yhat) = ||y - yhat||_2 / ||yhat||_2."""
    # a 3-4-5 example by hand: difference (3, 4, 0), target (0, 0, 10) -> 5 / 10
    target = np.array([0.0, 0.0, 10.0])
    pred = target + np.array([3.0, 4.0, 0.0])
    assert abs(O.rel_l2_loss(pred, target) - 0.5) <= 1e-15
    g = O.rel_l2_grad(pred, target)
    assert np.max(np.abs(g - np.array([3.0, 4.0, 0.0]) / 50.0)) <= 1e-16
    rng = np.random.default_rng(5)
    y = rng.standard_normal((2, 1, 3, 4, 2, 3))
    u = rng.standard_normal(y.shape)
    # pred = (1 + alpha) target gives |alpha|; a common positive factor cancels
    assert abs(O.rel_l2_loss(1.25 * y, y) - 0.25) <= 1e-14
    assert abs(O.rel_l2_loss(3.0 * u, 3.0 * y) - O.rel_l2_loss(u, y)) <= 1e-14
    # against plain loops
    sd = sum((a - b) ** 2 for a, b in zip(u.ravel(), y.ravel()))
    sy = sum(b * b for b in y.ravel())
    assert abs(O.rel_l2_loss(u, y) - math.sqrt(sd) / math.sqrt(sy)) <= 1e-14
    # the gradient: central differences, and <grad, pred - target> = loss (degree-one homogeneity)
    g = O.rel_l2_grad(u, y)
    for idx in [(0, 0, 0, 0, 0, 0), (1, 0, 2, 3, 1, 2), (0, 0, 1, 2, 0, 1)]:
        e = np.zeros_like(u)
        e[idx] = 1e-6
        fd = (O.rel_l2_loss(u + e, y) - O.rel_l2_loss(u - e, y)) / 2e-6
        assert abs(fd - g[idx]) <= 1e-9
    assert abs(np.sum(g * (u - y)) - O.rel_l2_loss(u, y)) <= 1e-14
    assert np.all(O.rel_l2_grad(y, y) == 0.0)


def test_adam_step_against_closed_forms():
    """Kingma & Ba, Algorithm 1 (Sec. 4 trains with Adam, learning rate 1e-3)."""
    rng = np.random.default_rng(9)
    p0 = rng.standard_normal(50)
    g = rng.standard_normal(50)
    zeros = np.zeros(50)
    # first step from zero moments: mhat = g, vhat = g^2, the step is lr * g / (|g| + eps)
    p1, m1, v1 = O.adam_step(p0, g, zeros, zeros, 1, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8)
    assert np.max(np.abs(m1 - 0.1 * g)) <= 1e-16 and np.max(np.abs(v1 - 0.001 * g * g)) <= 1e-16
    assert np.max(np.abs(p1 - (p0 - 1e-3 * g / (np.abs(g) + 1e-8)))) <= 1e-15
    # a constant gradient keeps mhat = g and vhat = g^2 at every step
    p, m, v = p0, zeros, zeros
    for t in range(1, 8):
        p, m, v = O.adam_step(p, g, m, v, t)
    assert np.max(np.abs(p - (p0 - 7 * 1e-3 * g / (np.abs(g) + 1e-8)))) <= 1e-14
    # zero gradient: the moments decay, the parameter moves by lr * mhat / (sqrt(vhat) + eps)
    p2, m2, v2 = O.adam_step(p1, zeros, m1, v1, 2)
    assert np.max(np.abs(m2 - 0.9 * m1)) <= 1e-17 and np.max(np.abs(v2 - 0.999 * v1)) <= 1e-18
    mhat, vhat = m2 / (1 - 0.9 ** 2), v2 / (1 - 0.999 ** 2)
    assert np.max(np.abs(p2 - (p1 - 1e-3 * mhat / (np.sqrt(vhat) + 1e-8)))) <= 1e-15
    # element by element with scalar arithmetic
    q, mq, vq = O.adam_step(p0, g, m1, v1, 3, lr=2e-3, beta1=0.8, beta2=0.99, eps=1e-6)
    for i in (0, 17, 49):
        mi = 0.8 * m1[i] + 0.2 * g[i]
        vi = 0.99 * v1[i] + 0.01 * g[i] ** 2
        want = p0[i] - 2e-3 * (mi / (1 - 0.8 ** 3)) / (math.sqrt(vi / (1 - 0.99 ** 3)) + 1e-6)
        assert abs(q[i] - want) <= 1e-14 and abs(mq[i] - mi) <= 1e-15 and abs(vq[i] - vi) <= 1e-15


def test_pointwise_adjoints_against_loops_and_finite_differences():
    rng = np.random.default_rng(17)
    B_, Ci, H, Co, grid = 2, 3, 5, 2, (2, 1, 2, 3)
    x = rng.standard_normal((B_, Ci) + grid)
    w = rng.standard_normal((H, Ci))
    g = rng.standard_normal((B_, H) + grid)
    got = O.pointwise_linear_bwd(x, w, g)
    # plain loops
    gw = np.zeros((H, Ci)); gb = np.zeros(H); gx = np.zeros_like(x)
    for b in range(B_):
        for idx in np.ndindex(*grid):
            for o in range(H):
                gb[o] += g[(b, o) + idx]
                for i in range(Ci):
                    gw[o, i] += g[(b, o) + idx] * x[(b, i) + idx]
                    gx[(b, i) + idx] += w[o, i] * g[(b, o) + idx]
    assert np.max(np.abs(got["gW"] - gw)) <= 1e-13 and np.max(np.abs(got["gb"] - gb)) <= 1e-13
    assert np.max(np.abs(got["gx"] - gx)) <= 1e-13
    # two-layer projection: directional derivatives of S = <gu, mlp2(x; w1, b1, w2, b2)>
    w1, b1 = rng.standard_normal((H, Ci)), rng.standard_normal(H)
    w2, b2 = rng.standard_normal((Co, H)), rng.standard_normal(Co)
    gu = rng.standard_normal((B_, Co) + grid)
    grads = O.pointwise_mlp2_bwd(x, w1, b1, w2, gu)
    S = lambda x_, w1_, b1_, w2_, b2_: float(np.sum(gu * O.pointwise_mlp2(x_, w1_, b1_, w2_, b2_)))
    eps = 1e-6
    for name, base, grad in (("x", x, grads["gx"]), ("w1", w1, grads["gW1"]), ("b1", b1, grads["gb1"]),
                             ("w2", w2, grads["gW2"]), ("b2", b2, grads["gb2"])):
        d = rng.standard_normal(base.shape)
        args_p = {"x": x, "w1": w1, "b1": b1, "w2": w2, "b2": b2}
        args_m = dict(args_p)
        args_p[name] = base + eps * d
        args_m[name] = base - eps * d
        fd = (S(args_p["x"], args_p["w1"], args_p["b1"], args_p["w2"], args_p["b2"])
              - S(args_m["x"], args_m["w1"], args_m["b1"], args_m["w2"], args_m["b2"])) / (2 * eps)
        an = float(np.sum(grad * d))
        assert abs(fd - an) <= 1e-8 + 1e-7 * abs(an), name


def test_whole_network_gradient_by_finite_differences():
    """fno_backward against central differences of S = <gu, fno_forward(...)> in random directions."""
    rng = np.random.default_rng(23)
    spec = O.LayerSpec((4, 4, 4, 4), (1, 1, 1, 2), 0)
    counts = tuple(len(k) for k in O.mode_lists(spec))
    Cin, C, H = 2, 3, 4
    a = rng.standard_normal((1, Cin) + spec.grid)
    lw, lb = rng.standard_normal((C, Cin)), rng.standard_normal(C)
    blocks = []
    for _ in range(2):
        r = (rng.standard_normal((C, C) + counts) + 1j * rng.standard_normal((C, C) + counts)) / C
        blocks.append((r, rng.standard_normal((C, C)) / np.sqrt(C), 0.1 * rng.standard_normal(C)))
    proj = (rng.standard_normal((H, C)), rng.standard_normal(H), rng.standard_normal((1, H)), rng.standard_normal(1))
    gu = rng.standard_normal((1, 1) + spec.grid)
    grads = O.fno_backward(a, lw, lb, blocks, proj, spec, gu)
    S = lambda lw_, blocks_, proj_: float(np.sum(gu * O.fno_forward(a, lw_, lb, blocks_, proj_, spec)))
    eps = 1e-6
    # lift weight
    d = rng.standard_normal(lw.shape)
    fd = (S(lw + eps * d, blocks, proj) - S(lw - eps * d, blocks, proj)) / (2 * eps)
    an = float(np.sum(grads["lift"]["gW"] * d))
    assert abs(fd - an) <= 1e-8 + 1e-6 * abs(an)
    # the first block's spectral weight (real and imaginary directions) and pointwise weight
    r0, w0, b0 = blocks[0]
    dr = rng.standard_normal(r0.shape) + 1j * rng.standard_normal(r0.shape)
    bp = [(r0 + eps * dr, w0, b0), blocks[1]]
    bm = [(r0 - eps * dr, w0, b0), blocks[1]]
    fd = (S(lw, bp, proj) - S(lw, bm, proj)) / (2 * eps)
    gR = grads["blocks"][0]["gR"]
    an = float(np.sum(gR.real * dr.real + gR.imag * dr.imag))
    assert abs(fd - an) <= 1e-8 + 1e-6 * abs(an)
    dw = rng.standard_normal(w0.shape)
    fd = (S(lw, [(r0, w0 + eps * dw, b0), blocks[1]], proj) - S(lw, [(r0, w0 - eps * dw, b0), blocks[1]], proj)) / (2 * eps)
    an = float(np.sum(grads["blocks"][0]["gW"] * dw))
    assert abs(fd - an) <= 1e-8 + 1e-6 * abs(an)
    # projection, first layer
    d1 = rng.standard_normal(proj[0].shape)
    fd = (S(lw, blocks, (proj[0] + eps * d1,) + proj[1:]) - S(lw, blocks, (proj[0] - eps * d1,) + proj[1:])) / (2 * eps)
    an = float(np.sum(grads["proj"]["gW1"] * d1))
    assert abs(fd - an) <= 1e-8 + 1e-6 * abs(an)


def test_fno_forward_is_the_chain_of_its_pinned_pieces():
    """fno_forward against the chain written out with the separately pinned pieces (lift by explicit
    sums, every block by block_fwd, projection by explicit sums): a dropped, repeated or reordered
    block, or a block applied with another block's weights, changes the result."""
    rng = np.random.default_rng(41)
    grid, modes, width, hidden = (4, 3, 4, 6), (1, 1, 1, 3), 3, 5
    spec = O.LayerSpec(grid, modes, 0)
    counts = tuple(len(k) for k in O.mode_lists(spec))
    a = rng.standard_normal((2, 2) + grid)
    lw, lb = rng.standard_normal((width, 2)), rng.standard_normal(width)
    blocks = [(rng.standard_normal((width, width) + counts) + 1j * rng.standard_normal((width, width) + counts),
               rng.standard_normal((width, width)), rng.standard_normal(width)) for _ in range(3)]
    w1, b1 = rng.standard_normal((hidden, width)), rng.standard_normal(hidden)
    w2, b2 = rng.standard_normal((1, hidden)), rng.standard_normal(1)
    got = O.fno_forward(a, lw, lb, blocks, (w1, b1, w2, b2), spec)

    v = np.zeros((2, width) + grid)
    for o in range(width):
        v[:, o] = lb[o] + sum(lw[o, i] * a[:, i] for i in range(2))
    for (r, w, b) in blocks:
        v = O.block_fwd(v, r, w, b, spec, "gelu")[0]
    h = np.zeros((2, hidden) + grid)
    for k in range(hidden):
        h[:, k] = b1[k] + sum(w1[k, i] * v[:, i] for i in range(width))
    h = O.gelu(h)
    want = b2[0] + sum(w2[0, k] * h[:, k] for k in range(hidden))
    assert got.shape == (2, 1) + grid
    assert np.max(np.abs(got[:, 0] - want)) <= 1e-12 * np.max(np.abs(want))
    # the chain is sensitive to each block: leaving one out, or swapping two, moves the output
    for other in (blocks[:2], [blocks[1], blocks[0], blocks[2]]):
        alt = O.fno_forward(a, lw, lb, other, (w1, b1, w2, b2), spec)
        assert np.max(np.abs(alt - got)) > 1e-3 * np.max(np.abs(got))
