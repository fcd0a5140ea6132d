"""Oracle (test infrastructure): attention computed directly on latent K/V.

Plain float64 definitions, one head at a time, no tiling, no running softmax,
no splitting of the key range. numpy matrix products are used as steps.

What is computed (Section 2, low-rank KV paragraph and the RoPE-free identity
Q.K^T = E (W_Q B_K^T) K'^T; Section 5 overview, steps 4-7: compressed Q', K',
V' go into attention without decompression):

  K'_h = x . A_k^h            V'_h = x . A_v^h
  q'_h = q_h . (B_k^h)^T
  s_t  = scale * <q'_h, K'_h[t]>
  p    = softmax_t(s)
  o'_h = sum_t p_t V'_h[t]
  y    = sum_h o'_h . (B_v^h . W_o^h)

Readings where the paper is silent: scale defaults to 1/sqrt(d_h) of the
uncompressed head (latent scores approximate the original ones); prefill is
causal, query row i at absolute position pos sees keys t <= pos; the fold of
B_v into W_o is the usual associativity (P V') B_v W_o = (P V') (B_v W_o), the
paper only says V compression follows Palu.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np


def project_latent_kv(x: np.ndarray, A_heads: Sequence[np.ndarray]) -> List[np.ndarray]:
    """Latent rows x.A^h for every head: x [T, d], A^h [d, r_h] -> list of [T, r_h]."""
    x = np.asarray(x, dtype=np.float64)
    return [x @ np.asarray(A, dtype=np.float64) for A in A_heads]


def absorb_query(q: np.ndarray, Bk_heads: Sequence[np.ndarray]) -> List[np.ndarray]:
    """q'_h = q_h . (B_k^h)^T: q [T, H, d_h], B_k^h [rk_h, d_h] -> list of [T, rk_h]."""
    q = np.asarray(q, dtype=np.float64)
    assert q.shape[1] == len(Bk_heads)
    return [q[:, h, :] @ np.asarray(B, dtype=np.float64).T for h, B in enumerate(Bk_heads)]


def softmax_rows(s: np.ndarray) -> np.ndarray:
    """Row softmax with the row maximum subtracted; fully masked rows give zeros."""
    s = np.asarray(s, dtype=np.float64)
    m = np.max(s, axis=-1, keepdims=True)
    m = np.where(np.isfinite(m), m, 0.0)
    e = np.exp(s - m)
    z = np.sum(e, axis=-1, keepdims=True)
    return np.divide(e, z, out=np.zeros_like(e), where=z > 0)


def latent_attn_decode(q_lat: np.ndarray, K_lat: np.ndarray, V_lat: np.ndarray,
                       scale: float, return_probs: bool = False):
    """One query against S latent keys/values of one head.

    q_lat [rk], K_lat [S, rk], V_lat [S, rv] -> o' [rv].  S = 0 gives zeros.
    """
    q_lat = np.asarray(q_lat, dtype=np.float64)
    K_lat = np.asarray(K_lat, dtype=np.float64)
    V_lat = np.asarray(V_lat, dtype=np.float64)
    S = K_lat.shape[0]
    assert V_lat.shape[0] == S and K_lat.shape[1] == q_lat.shape[0]
    if S == 0:
        o = np.zeros(V_lat.shape[1])
        return (o, np.zeros(0)) if return_probs else o
    s = scale * (K_lat @ q_lat)
    p = softmax_rows(s[None, :])[0]
    o = p @ V_lat
    return (o, p) if return_probs else o


def latent_attn_prefill(Q_lat: np.ndarray, K_lat: np.ndarray, V_lat: np.ndarray,
                        scale: float, causal: bool = True) -> np.ndarray:
    """S_q queries against S_kv latent keys/values of one head.

    Q_lat [S_q, rk], K_lat [S_kv, rk], V_lat [S_kv, rv] -> O' [S_q, rv].
    The queries are the last S_q positions of the S_kv-long sequence: query
    row i sits at absolute position S_kv - S_q + i and, when causal, sees keys
    t <= that position.
    """
    Q_lat = np.asarray(Q_lat, dtype=np.float64)
    K_lat = np.asarray(K_lat, dtype=np.float64)
    V_lat = np.asarray(V_lat, dtype=np.float64)
    S_q, S_kv = Q_lat.shape[0], K_lat.shape[0]
    assert S_kv >= S_q
    s = scale * (Q_lat @ K_lat.T)
    if causal:
        pos = (S_kv - S_q) + np.arange(S_q)[:, None]
        t = np.arange(S_kv)[None, :]
        s = np.where(t <= pos, s, -np.inf)
    p = softmax_rows(s)
    return p @ V_lat


def fold_output(Bv_heads: Sequence[np.ndarray], W_o: np.ndarray, d_head: int) -> List[np.ndarray]:
    """M_h = B_v^h . W_o^h, W_o^h = rows h*d_h .. (h+1)*d_h of W_o [H*d_h, d] -> list of [rv_h, d]."""
    W_o = np.asarray(W_o, dtype=np.float64)
    out = []
    for h, B in enumerate(Bv_heads):
        B = np.asarray(B, dtype=np.float64)
        assert B.shape[1] == d_head
        out.append(B @ W_o[h * d_head:(h + 1) * d_head, :])
    return out


def apply_output(o_lat_heads: Sequence[np.ndarray], M_heads: Sequence[np.ndarray]) -> np.ndarray:
    """y = sum_h o'_h . M_h: o'_h [T, rv_h], M_h [rv_h, d] -> [T, d]."""
    y = None
    for o, M in zip(o_lat_heads, M_heads):
        term = np.asarray(o, dtype=np.float64) @ np.asarray(M, dtype=np.float64)
        y = term if y is None else y + term
    return y


def lse_merge(ms: Sequence[float], ls: Sequence[float], accs: Sequence[np.ndarray]) -> np.ndarray:
    """Combine per-chunk softmax states into the output over the union of the chunks.

    Chunk j holds m_j = max score, l_j = sum exp(s - m_j), acc_j = sum exp(s - m_j) V'.
    Result: sum_j acc_j e^{m_j - m} / sum_j l_j e^{m_j - m}, m = max_j m_j.
    (The paper never splits a decode head; this is the definition the split-K
    extension of the library must reproduce.)
    """
    m = max(ms)
    num = None
    den = 0.0
    for mj, lj, aj in zip(ms, ls, accs):
        w = np.exp(mj - m)
        den += lj * w
        num = aj * w if num is None else num + aj * w
    return num / den
