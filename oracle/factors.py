"""Oracle (test infrastructure): low-rank factors of a projection weight.

Section 2 (low-rank KV compression): the per-head weight W (d x d_h) is
decomposed by SVD into A (d x k) and B (k x d_h), k < d_h, with W ~= A.B; the
latent cache row is x.A and x.A.B approximates x.W.

Reading taken where the paper is silent: the singular values go into A, so
A = U_k diag(sigma_k) and B = V_k^T has orthonormal rows. This matches the
paper's rotation view, where B^T is the rotation matrix R with its rightmost
columns deleted (Section 5.2). The attention output does not depend on how
sigma is split between A and B in exact arithmetic.
"""
from __future__ import annotations

import numpy as np


def truncated_svd_factors(W: np.ndarray, k: int):
    """Return (A, B, sigma): A = U[:, :k] * sigma[:k], B = Vt[:k, :], all float64.

    sigma is the full vector of singular values in descending order.
    """
    W = np.asarray(W, dtype=np.float64)
    d, d_h = W.shape
    if not (1 <= k <= min(d, d_h)):
        raise ValueError(f"kept rank {k} outside [1, {min(d, d_h)}]")
    U, sigma, Vt = np.linalg.svd(W, full_matrices=False)
    A = U[:, :k] * sigma[None, :k]
    B = Vt[:k, :]
    return A, B, sigma
