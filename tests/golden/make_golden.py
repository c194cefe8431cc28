"""Writes tests/golden/block_small.txt from the float64 oracle alone (no GPU code is involved).

The paper prints no worked numerical example of a spectral convolution, so this fixture is not a
citation: it freezes the oracle's output for one small seeded block (forward values and
gradients at fixed positions) so that a later change to the oracle's arithmetic shows up.
Run:  python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import fno_oracle as O  # noqa: E402


def case():
    spec = O.LayerSpec((6, 4, 8, 6), (2, 1, 2, 3), 0)
    rng = np.random.default_rng([2204, 1205])
    lx, ly, lz, lt = [len(k) for k in O.mode_lists(spec)]
    x = rng.standard_normal((2, 3) + spec.grid)
    r = (rng.standard_normal((3, 3, lx, ly, lz, lt)) + 1j * rng.standard_normal((3, 3, lx, ly, lz, lt))) / 3.0
    w = rng.standard_normal((3, 3)) / np.sqrt(3.0)
    b = 0.1 * rng.standard_normal(3)
    target = rng.standard_normal(x.shape)
    return spec, x, r, w, b, target


def values():
    spec, x, r, w, b, target = case()
    out, z, xhat = O.block_fwd(x, r, w, b, spec)
    g = O.block_bwd(x, r, w, b, O.mse_grad(out, target), spec)
    pos = [(0, 0, 0, 0, 0, 0), (1, 2, 5, 3, 7, 5), (0, 1, 2, 1, 3, 4), (1, 0, 4, 2, 6, 1)]
    rows = []
    for p in pos:
        rows.append(("out" + str(p), out[p]))
        rows.append(("z" + str(p), z[p]))
        rows.append(("gx" + str(p), g["gx"][p]))
    rows.append(("xhat_re", xhat[1, 2, 3, 1, 2, 1].real))
    rows.append(("xhat_im", xhat[1, 2, 3, 1, 2, 1].imag))
    rows.append(("gR_re", g["gR"][2, 1, 1, 0, 3, 2].real))
    rows.append(("gR_im", g["gR"][2, 1, 1, 0, 3, 2].imag))
    rows.append(("gR_kt0_re", g["gR"][0, 2, 3, 1, 1, 0].real))
    for o in range(3):
        rows.append((f"gb[{o}]", g["gb"][o]))
        for i in range(3):
            rows.append((f"gW[{o}][{i}]", g["gW"][o, i]))
    rows.append(("loss", O.mse_loss(out, target)))
    return rows


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "block_small.txt")
    with open(path, "w") as f:
        f.write("# written by tests/golden/make_golden.py from oracle/fno_oracle.py; name, value (repr of float64)\n")
        for name, v in values():
            f.write(f"{name}\t{float(v)!r}\n")
    print("wrote", path)
