"""The paper's own matrices, dense, for tiny shapes only (TEST INFRASTRUCTURE).

Section 2 builds the transformation as a product T = C P of a padding matrix P
and a convolution matrix C that acts on the padded, vectorised input; Section 3
gives constructions for both.  They are written here as dense float64 numpy
arrays, following the structure the paper describes (selection rows for P; the
horizontal-slide pattern R repeated along a block diagonal that moves
(n+2p)*s columns per vertical slide for C), so that the C oracle's direct tap
enumeration and sliding-window sum can be pinned to the paper's construction:
C @ P must equal T entry for entry and C @ P @ vec(A) must equal the
convolution.

Readings of garbled passages: P has m*n columns (the printed "(mn)^2" is a
typo; the construction allocates m*n entries); the leading zero block of P is
p padded lines of n+2p entries each, i.e. p*(n+2p) rows, followed by p more
rows for the left border of the first line; every zero block of C has as many
rows as R, floor((n+2p-k)/s) + 1.
"""
from __future__ import annotations

import numpy as np


def padding_matrix(m: int, n: int, p: int) -> np.ndarray:
    """P of Section 2: ((m+2p)(n+2p)) x (mn), one 1 per column.  Input line i
    is an n x n identity block that starts p entries into padded line i + p."""
    W = n + 2 * p
    P = np.zeros(((m + 2 * p) * W, m * n))
    eye = np.eye(n)
    for i in range(m):
        top = W * (i + p) + p
        P[top:top + n, n * i:n * (i + 1)] = eye
    return P


def slide_pattern(K: np.ndarray, n: int, p: int, s: int) -> np.ndarray:
    """R of Section 2: one row per horizontal slide; k segments of n+2p
    columns, segment j holding kernel row j shifted right by s per slide."""
    k = K.shape[0]
    W = n + 2 * p
    slides = (W - k) // s + 1
    R = np.zeros((slides, W * k))
    for i in range(slides):
        for j in range(k):
            R[i, W * j + s * i: W * j + s * i + k] = K[j]
    return R


def convolution_matrix(K: np.ndarray, m: int, n: int, p: int, s: int) -> np.ndarray:
    """C of Section 2: block row v is R preceded by v zero blocks of (n+2p)s
    columns; whatever the vertical slides cannot reach (q lines) stays zero."""
    K = np.asarray(K, dtype=np.float64)
    k = K.shape[0]
    W, H = n + 2 * p, m + 2 * p
    R = slide_pattern(K, n, p, s)
    vslides = (H - k) // s + 1
    q = (H - k) - s * (vslides - 1)
    width = W * s * (vslides - 1) + W * k + W * q
    assert width == W * H                       # C acts on the padded vector
    C = np.zeros((vslides * R.shape[0], width))
    for v in range(vslides):
        C[v * R.shape[0]:(v + 1) * R.shape[0], W * s * v: W * s * v + W * k] = R
    return C


def transformation_matrix(K: np.ndarray, m: int, n: int, p: int, s: int) -> np.ndarray:
    """T = C P, dense: (m_out n_out) x (mn)."""
    return convolution_matrix(K, m, n, p, s) @ padding_matrix(m, n, p)
