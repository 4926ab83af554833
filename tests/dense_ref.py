"""Independent dense constructions used to pin the oracle (pure NumPy / Python loops).

Nothing here calls the oracle or the GPU library.  Everything is written from
the paper's 1-based single-pixel formulas (Section 3, Eq. 1; Theorems 1 and 2
as derived in the supplement's proofs), extended to channels by giving every
tap a C x C block whose current-pixel block is lower triangular.
"""
from __future__ import annotations

import numpy as np


def delta(p, k):
    """Delta(p) = {(i,j): 0 <= p1-i, p2-j < k} minus {p}, 1-based, clipped to i,j >= 1."""
    p1, p2 = p
    out = []
    for i in range(max(1, p1 - k + 1), p1 + 1):
        for j in range(max(1, p2 - k + 1), p2 + 1):
            if (i, j) != (p1, p2):
                out.append((i, j))
    return out


def tap_of(p, q, k):
    """0-based kernel index of W_{(k,k)-p+q}."""
    return (k - p[0] + q[0] - 1, k - p[1] + q[1] - 1)


def masked(w):
    """Kernel with the current-pixel block's strictly upper triangle zeroed."""
    w = np.array(w, dtype=np.float64, copy=True)
    k = w.shape[2]
    w[:, :, k - 1, k - 1] = np.tril(w[:, :, k - 1, k - 1])
    return w


def vec_index(H, W, C, r, c, ch):
    """Row-major pixels, channel innermost (0-based)."""
    return (r * W + c) * C + ch


def dense_M(w, H, W):
    """(C*H*W) x (C*H*W) matrix of the masked convolution, built entry by entry from Eq. 1."""
    w = masked(w)
    C, k = w.shape[0], w.shape[2]
    n = C * H * W
    M = np.zeros((n, n))
    for p1 in range(1, H + 1):
        for p2 in range(1, W + 1):
            for q in delta((p1, p2), k) + [(p1, p2)]:
                a, b = tap_of((p1, p2), q, k)
                for o in range(C):
                    for i in range(C):
                        M[vec_index(H, W, C, p1 - 1, p2 - 1, o),
                          vec_index(H, W, C, q[0] - 1, q[1] - 1, i)] = w[o, i, a, b]
    return M


def to_vec(img):
    """[C,H,W] -> vector in (pixel-major, channel-minor) order."""
    return np.ascontiguousarray(np.transpose(img, (1, 2, 0))).reshape(-1)


def from_vec(vec, C, H, W):
    return np.ascontiguousarray(np.transpose(vec.reshape(H, W, C), (2, 0, 1)))


def gauss_solve(A, b):
    """Plain Gaussian elimination with partial pivoting (the O(n^3) naive baseline of Table 1)."""
    A = np.array(A, dtype=np.float64, copy=True)
    b = np.array(b, dtype=np.float64, copy=True)
    n = A.shape[0]
    for col in range(n):
        piv = col + int(np.argmax(np.abs(A[col:, col])))
        if piv != col:
            A[[col, piv]] = A[[piv, col]]
            b[[col, piv]] = b[[piv, col]]
        for row in range(col + 1, n):
            f = A[row, col] / A[col, col]
            if f != 0.0:
                A[row, col:] -= f * A[col, col:]
                b[row] -= f * b[col]
    x = np.zeros(n)
    for row in range(n - 1, -1, -1):
        x[row] = (b[row] - A[row, row + 1:] @ x[row + 1:]) / A[row, row]
    return x


def dM_dw(H, W, C, k, o, i, a, b):
    """d M / d w[o,i,a,b] as a dense 0/1 matrix."""
    n = C * H * W
    D = np.zeros((n, n))
    for r in range(H):
        for c in range(W):
            rr, cc = r - (k - 1) + a, c - (k - 1) + b
            if rr >= 0 and cc >= 0:
                D[vec_index(H, W, C, r, c, o), vec_index(H, W, C, rr, cc, i)] = 1.0
    return D


def theorem1_jacobian_column(w1, m_h, m_w, p):
    """dx_q/dy_p for all q, single channel with unit current-pixel tap.

    Recursion from the proof of Theorem 1:
      dx_q/dy_p = [q == p] - sum_{r in Delta(q)} W_{(k,k)-q+r} dx_r/dy_p.
    `w1` is the k x k kernel, p is 1-based.  Returns an m_h x m_w array.
    """
    k = w1.shape[0]
    J = np.zeros((m_h + 1, m_w + 1))
    for q1 in range(1, m_h + 1):
        for q2 in range(1, m_w + 1):
            s = 1.0 if (q1, q2) == p else 0.0
            for r in delta((q1, q2), k):
                a, b = tap_of((q1, q2), r, k)
                s -= w1[a, b] * J[r[0], r[1]]
            J[q1, q2] = s
    return J[1:, 1:]


def theorem2_dx_dW(w1, x, tap):
    """dx_q/dW_a for all q, single channel with unit current-pixel tap.

    Recursion at the end of the proof of Theorem 2:
      dx_q/dW_a = -x_{q-(k,k)+a} - sum_{r in Delta(q)} W_{(k,k)-q+r} dx_r/dW_a,
    the first term being absent when q-(k,k)+a falls outside the image.
    `tap` is the 0-based kernel index of a.  Returns an array shaped like x.
    """
    k = w1.shape[0]
    m_h, m_w = x.shape
    D = np.zeros((m_h + 1, m_w + 1))
    for q1 in range(1, m_h + 1):
        for q2 in range(1, m_w + 1):
            s1, s2 = q1 - k + (tap[0] + 1), q2 - k + (tap[1] + 1)   # 1-based q-(k,k)+a
            s = -x[s1 - 1, s2 - 1] if (s1 >= 1 and s2 >= 1) else 0.0
            for r in delta((q1, q2), k):
                a, b = tap_of((q1, q2), r, k)
                s -= w1[a, b] * D[r[0], r[1]]
            D[q1, q2] = s
    return D[1:, 1:]
