"""Arbitrary-precision restatement of the paper's integer maps and of its
sketching-matrix view, used only to pin the C oracle on tiny inputs.

Written from the formulas of Section 3.1 (hash equation), Section 3.2
(forward and idx equations) and Section 4 (sketching matrix: one +-1 per row).
Python ints cannot overflow, and the circular read below follows the
two-piece "p1 . p2" statement of the forward equation rather than the mod
form, so it does not share a formula with the oracle's idx().
"""
import numpy as np

MASK64 = (1 << 64) - 1


def h(coef, P, m, e, x, c):
    Ah, Bh, Ch, Dh = coef[:4]
    return ((Ah * e + Bh * (x & MASK64) + Ch * c + Dh) % P) % m


def g(coef, P, use_sign, e, x, i):
    if not use_sign:
        return 1
    Ag, Bg, Cg, Dg = coef[4:]
    return 2 * (((Ag * e + Bg * (x & MASK64) + Cg * i + Dg) % P) % 2) - 1


def circular_block(M, start, Z):
    """M[start : start+Z] on a circular array, as two pieces when it overflows."""
    m = len(M)
    if start + Z < m:
        return list(M[start:start + Z])
    p1 = list(M[start:m])
    p2 = list(M[0:Z + start - m])
    return p1 + p2


def embedding(coef, P, M, d, Z, use_sign, e, x):
    """E_e(x) = G(x) o (P_0 . P_1 . ... . P_{d/Z-1})."""
    m = len(M)
    prim = []
    for c in range(d // Z):
        prim += circular_block(M, h(coef, P, m, e, x, c), Z)
    return [g(coef, P, use_sign, e, x, i) * prim[i] for i in range(d)]


def position_big_block(coef, P, m, d, Z, e, x, i):
    """Z > d (Section 3.3, Appendix "ROBE-Z"): table e flattened row by row, cut into chunks of Z.
    Element i of token x is entry n = x*d + i; its chunk n // Z is hashed (as the key, chunk number 0)
    and it sits n % Z places into the chunk, circularly."""
    n = (x & MASK64) * d + i
    return (h(coef, P, m, e, n // Z, 0) + n % Z) % m


def position_map(coef, P, m, d, Z, e, x):
    """Array slot of every element of E_e(x): the embedding of the array M[j] = j."""
    return embedding(coef, P, list(range(m)), d, Z, 0, e, x)


def sketch_matrix(coef, P, m, d, Z, use_sign, tokens):
    """Dense S in {0,+-1}^{(len(tokens)*d) x m}; row (t,i) has its single
    non-zero g(e,x,i) at the slot of element i of token t = (e, x)."""
    S = np.zeros((len(tokens) * d, m), dtype=np.float64)
    for t, (e, x) in enumerate(tokens):
        pos = position_map(coef, P, m, d, Z, e, x)
        for i in range(d):
            S[t * d + i, pos[i]] = g(coef, P, use_sign, e, x, i)
    return S
