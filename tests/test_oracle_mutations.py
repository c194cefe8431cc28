"""Plausible mistakes planted in the oracle (on the CPU, by patching its functions) must each be
caught by at least one pin.  This guards the pins, not the oracle."""
import numpy as np
import pytest

from oracle import fno_oracle as O
import test_oracle_pins as P


def _pins():
    """A representative subset of the pins, as zero-argument callables."""
    spec0, spec1, spec2, spec3 = P.TINY[0], P.TINY[1], P.TINY[2], P.TINY[3]
    return [
        P.test_mode_lists_literal,
        P.test_hermitian_weights_literal,
        lambda: P.test_P1_definition_equals_brute_force(spec0),
        lambda: P.test_P1_definition_equals_brute_force(spec2),
        lambda: P.test_P2_equals_numpy_fft_route(spec1),
        lambda: P.test_P2_equals_numpy_fft_route(spec3),
        lambda: P.test_P4_full_mode_set_is_identity_and_parseval((4, 6, 4, 8)),
        P.test_P5a_interior_mode_rotates_and_scales_a_cosine,
        P.test_P5b_kt0_mode_is_halved_unless_partner_carries_conjugate,
        P.test_P7_zero_weights_give_zero_and_block_reduces_to_pointwise,
        P.test_gelu_textbook_values,
        P.test_one_hot_weight_lights_the_matching_frequency,
        lambda: P.test_P10_adjoint_is_layer_with_conjugate_transposed_weights(spec0),
        lambda: P.test_P11_block_gradients_match_central_differences(spec0, "gelu"),
        P.test_separable_spectrum_and_point_sampled_inverse_match_plain_routines,
        P.test_separable_weight_grads_match_block_bwd,
        P.test_network_pieces,
    ]


def _caught():
    for pin in _pins():
        try:
            pin()
        except (AssertionError, ValueError, IndexError):
            return True
    return False


def test_unmutated_oracle_passes_the_subset():
    assert not _caught()


_orig = {name: getattr(O, name) for name in dir(O)}

MUTATIONS = {
    "all hermitian weights 2": ("hermitian_weights", lambda nt, kt: np.full(len(kt), 2.0)),
    "forward sign flipped": ("dft_matrix", lambda n, ks, sign: _orig["dft_matrix"](n, ks, -sign)),
    "negative modes dropped": ("spatial_modes", lambda n, m, rule=0: list(range(0, m)) + list(range(0, m))),
    "negative modes descending": ("spatial_modes",
                                  lambda n, m, rule=0: list(range(0, m + (rule == 1))) + list(range(-1, -m - 1, -1))),
    "mix sums over the wrong channel axis": ("mix_modes",
                                             lambda xh, r: np.einsum("bixyzt,oixyzt->boxyzt", xh, np.asarray(r))),
    "inverse without 1/N": ("inverse_spectrum",
                            lambda yh, spec: _orig["inverse_spectrum"](yh, spec) * float(spec.npoints)),
    "inverse takes the imaginary part": ("inverse_spectrum",
                                         lambda yh, spec: _orig["inverse_spectrum"](1j * np.asarray(yh), spec)),
    "gelu with tanh approximation": ("gelu", lambda z: 0.5 * np.asarray(z) * (1 + np.tanh(
        0.7978845608 * (np.asarray(z) + 0.044715 * np.asarray(z) ** 3)))),
    "gelu' without the density term": ("gelu_prime", lambda z: _orig["gelu"](z) / np.where(np.asarray(z) == 0, 1, z)),
    "affine with W transposed": ("channel_affine",
                                 lambda x, w, b: _orig["channel_affine"](x, np.asarray(w).T, b)),
    "affine without bias": ("channel_affine", lambda x, w, b: _orig["channel_affine"](x, w, None)),
    "adjoint without conjugating R": ("spectral_conv_bwd", lambda x, r, gy, spec: _orig["spectral_conv_bwd"](
        x, np.conj(r), gy, spec)),
    "mse gradient without the factor 2": ("mse_grad", lambda out, t: 0.5 * _orig["mse_grad"](out, t)),
    "rank-one spectrum forgets the t factor": ("separable_forward_spectrum", lambda fx, fy, fz, ft, spec:
                                               _orig["separable_forward_spectrum"](fx, fy, fz, np.ones_like(ft), spec)),
    "point-sampled inverse drops c_kt": ("inverse_at_points", lambda yh, spec, pts: _orig["inverse_at_points"](
        np.asarray(yh) / O.hermitian_weights(spec.grid[3], O.mode_lists(spec)[3]), spec, pts)),
    "rank-one weight grads use the sum of factors": ("separable_weight_grads", lambda g, x: tuple(
        2 * v for v in _orig["separable_weight_grads"](g, x))),
    "projection without the hidden activation": ("pointwise_mlp2", lambda x, w1, b1, w2, b2:
                                                 O.channel_affine(O.channel_affine(x, w1, b1), w2, b2)),
}


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name, monkeypatch):
    attr, fn = MUTATIONS[name]
    monkeypatch.setattr(O, attr, fn)
    assert _caught(), f"no pin noticed: {name}"
