"""Oracle (test infrastructure): post-RoPE compression of Q and K.

Section 2 (background): RoPE rotates each row vector q, k by a rotation matrix
H_i that depends on the position i. Section 3 (motivation) and Section 5.1
(design): a common rotation R of the post-RoPE Q_p and K_p leaves the scores
unchanged, (Q_p R)(K_p R)^T = Q_p K_p^T; R comes from the SVD of the matrix that
stacks all rows of Q_p and K_p of a head, X = U Sigma R^T; the rotated vectors
have their components ordered by singular value, and compression by the rate p
deletes the rightmost p * d_h columns of R before rotating. The compressed
Q'_p = Q_p R_p and K'_p = K_p R_p go straight into attention.

Readings where the paper is silent:
  * which pairs RoPE rotates and the frequency schedule are not given. Pairs are
    (2i, 2i+1) as in the cited RoFormer definition; the angles are INPUTS
    (tables cos[pos, i], sin[pos, i], i < d_h / 2), so any schedule can be used.
    `rope_tables` builds the usual theta_i = base^(-2i/d_h).
  * for GQA the paper pairs each query head with its key head; here one R per
    head is computed from that head's own Q_p and K_p rows.
Plain float64, numpy only.
"""
from __future__ import annotations

import numpy as np


def rope_tables(max_pos: int, d_head: int, base: float = 10000.0):
    """cos, sin [max_pos, d_head / 2] for angles pos * base^(-2i / d_head)."""
    i = np.arange(d_head // 2, dtype=np.float64)
    theta = base ** (-2.0 * i / d_head)
    ang = np.arange(max_pos, dtype=np.float64)[:, None] * theta[None, :]
    return np.cos(ang), np.sin(ang)


def rope(x: np.ndarray, pos, cos: np.ndarray, sin: np.ndarray) -> np.ndarray:
    """Rotate the pairs (x[2i], x[2i+1]) of every row t by the angle of position pos[t].

    x [T, d_h]; pos int [T]; cos, sin [max_pos, d_h / 2].
    (y_2i, y_2i+1) = (x_2i c - x_2i+1 s, x_2i s + x_2i+1 c).
    """
    x = np.asarray(x, dtype=np.float64)
    c = np.asarray(cos, dtype=np.float64)[np.asarray(pos)]
    s = np.asarray(sin, dtype=np.float64)[np.asarray(pos)]
    even, odd = x[:, 0::2], x[:, 1::2]
    y = np.empty_like(x)
    y[:, 0::2] = even * c - odd * s
    y[:, 1::2] = even * s + odd * c
    return y


def common_rotation(Qp: np.ndarray, Kp: np.ndarray):
    """R (d_h x d_h, orthogonal) and the singular values of the stacked post-RoPE rows of one head.

    X = [Q_p; K_p] = U Sigma R^T; the columns of R are ordered by descending singular value.
    """
    X = np.concatenate([np.asarray(Qp, dtype=np.float64), np.asarray(Kp, dtype=np.float64)], axis=0)
    _, sigma, Rt = np.linalg.svd(X, full_matrices=False)
    return Rt.T, sigma


def rotate_truncate(Xp: np.ndarray, R: np.ndarray, k: int) -> np.ndarray:
    """X'_p = X_p R_p with R_p = the first k columns of R (the rightmost d_h - k deleted)."""
    return np.asarray(Xp, dtype=np.float64) @ np.asarray(R, dtype=np.float64)[:, :k]
