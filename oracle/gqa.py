"""Oracle (test infrastructure): grouped-query attention on the latent cache.

Section 5.1 (GQA paragraph): in a GQA model several query heads share one key /
value head; the rotation of a key head is computed from the post-RoPE rows of
that key head together with the rows of every query head that attends to it.
Everything else is unchanged: a query head attends to the compressed K' / V'
of its key head exactly as in the multi-head case (Section 5, step 7).

Conventions taken here (the paper gives none): with g query heads per key /
value head, query head hq uses key/value head hq // g (consecutive query heads
form a group, the usual GQA ordering). Latent queries and latent outputs are
ragged by QUERY head: query head hq has width rk[hq // g] in q_lat and
rv[hq // g] in o_lat, heads concatenated in order. The absorbed output
projection has one block M_hq = B_v^{hq // g} . W_o^{hq} per query head.
Plain float64 / Python integers.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np

from . import attention as oa


def kv_head_of(hq: int, g: int) -> int:
    return hq // g


def query_offsets(ranks_kv: Sequence[int], g: int) -> List[int]:
    """Column offset of every query head in a [T, g * sum(ranks_kv)] latent tensor, plus the total."""
    off, run = [], 0
    for h in range(len(ranks_kv)):
        for _ in range(g):
            off.append(run)
            run += int(ranks_kv[h])
    off.append(run)
    return off


def absorb_query(q: np.ndarray, Bk_heads: Sequence[np.ndarray], g: int) -> List[np.ndarray]:
    """q'_hq = q_hq . (B_k^{hq // g})^T: q [T, H_q, d_h] -> list over query heads of [T, rk]."""
    q = np.asarray(q, dtype=np.float64)
    return [q[:, hq, :] @ np.asarray(Bk_heads[hq // g], dtype=np.float64).T for hq in range(q.shape[1])]


def latent_attn_decode(q_lat_heads: Sequence[np.ndarray], K_heads: Sequence[np.ndarray],
                       V_heads: Sequence[np.ndarray], scale: float, g: int) -> List[np.ndarray]:
    """One token: q_lat_heads[hq] is [rk]; K_heads[h] [S, rk], V_heads[h] [S, rv] -> list of [rv] per query head."""
    return [oa.latent_attn_decode(q_lat_heads[hq], K_heads[hq // g], V_heads[hq // g], scale)
            for hq in range(len(q_lat_heads))]


def latent_attn_prefill(Q_lat_heads: Sequence[np.ndarray], K_heads: Sequence[np.ndarray],
                        V_heads: Sequence[np.ndarray], scale: float, causal: bool, g: int) -> List[np.ndarray]:
    return [oa.latent_attn_prefill(Q_lat_heads[hq], K_heads[hq // g], V_heads[hq // g], scale, causal)
            for hq in range(len(Q_lat_heads))]


def fold_output(Bv_heads: Sequence[np.ndarray], W_o: np.ndarray, d_head: int, g: int) -> List[np.ndarray]:
    """M_hq = B_v^{hq // g} . W_o^{hq}; W_o [H_q * d_h, d] -> list over query heads of [rv, d]."""
    W_o = np.asarray(W_o, dtype=np.float64)
    Hq = W_o.shape[0] // d_head
    return [np.asarray(Bv_heads[hq // g], dtype=np.float64) @ W_o[hq * d_head:(hq + 1) * d_head] for hq in range(Hq)]


def common_rotation(Qp_group: Sequence[np.ndarray], Kp: np.ndarray):
    """R of one key head: SVD of the stacked post-RoPE rows of its g query heads and of the key head."""
    X = np.concatenate([np.asarray(a, dtype=np.float64) for a in Qp_group] + [np.asarray(Kp, dtype=np.float64)], axis=0)
    _, sigma, Rt = np.linalg.svd(X, full_matrices=False)
    return Rt.T, sigma
