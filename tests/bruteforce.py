"""Independent brute-force / definitional checkers used to pin the CPU oracle.

Written from the paper's printed constants and definitions in a different form from the
oracle (explicit tables and exhaustive enumeration instead of closed forms)."""
import itertools

import numpy as np

# Sec. 3.2: the printed 3-bit lattice, in this build's code numbering (sign-magnitude,
# the smallest positive bin repurposed as zero).
LATTICE_W3 = np.array([+1.0, +0.5, +0.25, 0.0, -1.0, -0.5, -0.25, -0.125])
# 4-bit lattice by the same construction (not printed in the paper: this build's reading).
LATTICE_W4 = np.array([2.0 ** -e for e in range(7)] + [0.0] + [-(2.0 ** -e) for e in range(8)])

# Sec. 3.3: the four printed pair sets.
PAIRS = {
    1: [(0, 1), (2, 3), (4, 5), (6, 7)],
    2: [(0, 2), (1, 3), (4, 6), (5, 7)],
    3: [(0, 3), (1, 2), (4, 7), (5, 6)],
    4: [(0, 4), (1, 5), (2, 6), (3, 7)],
}


def lattice(bw):
    return LATTICE_W3 if bw == 3 else LATTICE_W4


def exchange(x, s, signs):
    """Theorem 1 with the printed pair sets: [y_i; y_j] = [[0,-eta],[eta,0]] [x_i; x_j]."""
    y = np.zeros(8)
    for p, (i, j) in enumerate(PAIRS[s]):
        eta = -1.0 if (signs >> p) & 1 else 1.0
        R = np.array([[0.0, -eta], [eta, 0.0]])
        y[i], y[j] = R @ np.array([x[i], x[j]])
    return y


def nearest_code(bw, v):
    L = lattice(bw)
    d = np.abs(v - L)
    best = np.flatnonzero(d == d.min())
    return int(best[np.argmin(np.abs(L[best]))])   # tie -> smaller magnitude


def best_exchange(x, r):
    """Exhaustive search over the 4 x 16 candidates of one micro-block: max <b2, r>."""
    best = (-np.inf, None, None)
    for s, sg in itertools.product((1, 2, 3, 4), range(16)):
        a = float(exchange(x, s, sg) @ r)
        if a > best[0] + 0.0:
            best = (a, s, sg)
    return best


def bases(q):
    """Dense b1, b2 [out, in] from canonical arrays."""
    L = lattice(q["bw"])
    b1 = L[q["codes"]]
    out, inn = b1.shape
    b2 = np.zeros_like(b1)
    for o in range(out):
        for m in range(inn // 8):
            b2[o, 8 * m:8 * m + 8] = exchange(b1[o, 8 * m:8 * m + 8], int(q["pattern"][o, m]) + 1,
                                              int(q["signs"][o, m]))
    return b1, b2


def dequant(q):
    b1, b2 = bases(q)
    c1 = q["c1"].view(np.float16).astype(np.float64)
    c2 = q["c2"].view(np.float16).astype(np.float64)
    return np.repeat(c1, 128, axis=1) * b1 + np.repeat(c2, 128, axis=1) * b2
