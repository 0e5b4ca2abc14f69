"""Vectors for the encoder tests: lattice points spoiled in ways that break one membership condition each
(paper Sec. 2.3, conditions (i)-(iii)), so that a missing check in an encoder shows up as a wrong accept."""
import numpy as np


def spoiled_points(pts, rng):
    """pts: int8 [n, 24] points of the ball cut.  Returns an int8 array of vectors most of which are not points:
    one coordinate moved by +-1 or +-2 (parity / Golay word / norm), one sign flipped (sum modulo 8), two
    coordinates swapped (Golay word), one coordinate moved by +-4 (sum modulo 8 and norm), random bytes, and
    extreme values."""
    n = pts.shape[0]
    out = []
    a = pts.astype(np.int16).copy()
    k = rng.integers(0, 24, size=n)
    a[np.arange(n), k] += rng.choice([-2, -1, 1, 2], size=n)
    out.append(a)
    b = pts.astype(np.int16).copy()
    k = rng.integers(0, 24, size=n)
    b[np.arange(n), k] *= -1
    out.append(b)
    c = pts.astype(np.int16).copy()
    i, j = rng.integers(0, 24, size=n), rng.integers(0, 24, size=n)
    c[np.arange(n), i], c[np.arange(n), j] = pts[np.arange(n), j].astype(np.int16), pts[np.arange(n), i].astype(np.int16)
    out.append(c)
    d = pts.astype(np.int16).copy()
    k = rng.integers(0, 24, size=n)
    d[np.arange(n), k] += rng.choice([-4, 4], size=n)
    out.append(d)
    out.append(rng.integers(-128, 128, size=(n, 24)).astype(np.int16))
    out.append(rng.integers(-3, 4, size=(n, 24)).astype(np.int16))
    e = pts.astype(np.int16).copy()
    e[:, 0] = rng.choice([-128, 127, 14, -14, 15, 16], size=n)
    out.append(e)
    out.append(np.zeros((4, 24), dtype=np.int16))
    return np.clip(np.concatenate(out), -128, 127).astype(np.int8)
