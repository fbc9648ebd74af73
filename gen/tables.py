"""Inverse-CDF tables for the noise term of the synthetic logits.

The generator turns 31 random bits k into u = (k + 1/2) / 2^32 in (0, 1/2) and returns the
upper-tail quantile Q(u) of the noise law (sign from a 32nd bit).  Q is tabulated at
k = 0..127 one by one and then at 64 points per octave of k, which resolves the tail
geometrically; between table points the generators interpolate linearly in k.  The table is
built here in double with scipy and rounded once to float32; host and device generators
consume the same bytes.
"""
import numpy as np
from scipy import special, stats

TABLE_LEN = 1666


def _knots() -> np.ndarray:
    ks = list(range(64))
    for sh in range(0, 25):
        ks += [(64 + j) << sh for j in range(64)]
    ks.append(1 << 31)
    return np.array(ks, dtype=np.float64)


def build_table(kind: str, scale: float) -> np.ndarray:
    """kind: 'normal' (N(0,1)) or 'student3' (Student-t, 3 degrees of freedom); values x scale."""
    u = (_knots() + 0.5) / 2.0 ** 32
    if kind == "normal":
        q = -special.ndtri(u)
    elif kind == "student3":
        q = -stats.t.ppf(u, 3)
    else:
        raise ValueError(kind)
    tab = np.zeros(TABLE_LEN, np.float32)
    tab[: q.size] = (scale * q).astype(np.float32)
    tab[q.size:] = tab[q.size - 1]
    assert q.size == TABLE_LEN - 1
    return tab
