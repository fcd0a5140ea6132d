"""Seeded generators for the five benchmark workloads.

Everything here is input construction: Gaussian draws, orthonormal bases from a
QR of a Gaussian matrix, a planted spectrum, rank draws, and bf16 bit packing.
The method itself (truncated factorisation, latent projection, attention,
scheduling) lives elsewhere; nothing in this file computes any of it.

Shapes follow the 7B-class layer the paper's complexity discussion uses
(d_h = 128, d = 4096, 32 heads; Section 5.1 "compression overhead" paragraph)
and the context lengths of its traces (Table 4), with synthetic values.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

RANK_CHOICES = tuple(range(16, 129, 16))  # kept ranks 16, 32, ..., 128


def make_rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def adaptive_ranks(n_layers: int, n_heads: int, seed: int) -> np.ndarray:
    """Per-(layer, head) kept rank drawn from {16, ..., 128} with P(r) ~ 1/r.

    Returns int32 [n_layers, n_heads]. The skew (many narrow heads, few wide
    ones) is what makes the per-head attention cost uneven.
    """
    vals = np.array(RANK_CHOICES, dtype=np.int64)
    p = 1.0 / vals
    p = p / p.sum()
    g = make_rng(seed)
    return g.choice(vals, size=(n_layers, n_heads), p=p).astype(np.int32)


def random_orthonormal(rows: int, cols: int, g: np.random.Generator) -> np.ndarray:
    """rows x cols matrix (rows >= cols) with orthonormal columns.

    Q factor of a Gaussian matrix, column signs fixed so that diag(R) > 0,
    which makes the draw unique for a seed.
    """
    assert rows >= cols
    a = g.standard_normal((rows, cols))
    q, r = np.linalg.qr(a)
    sgn = np.sign(np.diag(r))
    sgn[sgn == 0] = 1.0
    return q * sgn[None, :]


@dataclass
class PlantedWeight:
    """W = U diag(s) V^T with known factors (U: d x d_h, V: d_h x d_h)."""

    U: np.ndarray
    s: np.ndarray
    V: np.ndarray

    @property
    def W(self) -> np.ndarray:
        return (self.U * self.s[None, :]) @ self.V.T


def planted_weight(d_model: int, d_head: int, decay: float, g: np.random.Generator,
                   exact_rank: Optional[int] = None) -> PlantedWeight:
    """Per-head projection weight with singular values s_i = exp(-i / decay), i = 0..d_h-1.

    With exact_rank = r the spectrum is cut to zero from index r on, so the
    weight has exactly r non-zero singular values.
    """
    U = random_orthonormal(d_model, d_head, g)
    V = random_orthonormal(d_head, d_head, g)
    s = np.exp(-np.arange(d_head, dtype=np.float64) / decay)
    if exact_rank is not None:
        s[exact_rank:] = 0.0
    return PlantedWeight(U=U, s=s, V=V)


def hidden_states(n_tokens: int, d_model: int, g: np.random.Generator) -> np.ndarray:
    """Hidden states x ~ N(0, 1), float64 [n_tokens, d_model]."""
    return g.standard_normal((n_tokens, d_model))


def direct_latent(n_tokens: int, rank: int, decay: float, g: np.random.Generator) -> np.ndarray:
    """Latent rows drawn directly: column i ~ N(0, s_i^2), s_i = exp(-i / decay).

    For x ~ N(0, I) and a weight whose left singular vectors are orthonormal,
    column i of x.(U_r diag(s_r)) is N(0, s_i^2) independently over tokens, so
    this has the value distribution of a projected cache without the
    d_model-sized matrix product.
    """
    s = np.exp(-np.arange(rank, dtype=np.float64) / decay)
    return g.standard_normal((n_tokens, rank)) * s[None, :]


# ----------------------------------------------------------------------------
# bf16 packing (round to nearest, ties to even): plumbing, not arithmetic of
# the method. The oracle consumes the stored bit patterns widened to float64.
# ----------------------------------------------------------------------------

def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = u + np.uint32(0x7FFF) + lsb
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Values of x after a round trip through bf16 storage, as float64."""
    return bf16_bits_to_f64(f64_to_bf16_bits(x)).reshape(np.shape(x))


# ----------------------------------------------------------------------------
# The five workloads
# ----------------------------------------------------------------------------

@dataclass
class Workload:
    name: str
    n_layers: int
    n_heads: int
    d_model: int
    d_head: int
    batch: int
    context: int          # KV length per sequence (decode) or prompt length (prefill)
    kv_dtype: str         # "f32" | "bf16"
    decay: float          # spectrum s_i = exp(-i / decay)
    seed: int
    phase: str            # "decode" | "prefill"
    rank_seed: Optional[int] = None       # adaptive draw; None = explicit ranks
    explicit_ranks: Optional[List[int]] = None
    min_split: int = 1
    granule: int = 64     # tokens per cut of the decode planner (a launch parameter, not part of the method's arithmetic)
    note: str = ""
    _ranks: Optional[np.ndarray] = field(default=None, repr=False)

    def ranks(self) -> np.ndarray:
        """int32 [n_layers, n_heads] kept rank per head (rk = rv = r_h)."""
        if self._ranks is None:
            if self.explicit_ranks is not None:
                r = np.array(self.explicit_ranks, dtype=np.int32)
                r = np.broadcast_to(r, (self.n_layers, self.n_heads)).copy()
            else:
                r = adaptive_ranks(self.n_layers, self.n_heads, self.rank_seed)
            self._ranks = r
        return self._ranks


CONFIGS = {
    # Tiny decode, fp32 storage, full chain from hidden states.
    "c1_tiny_decode_f32": Workload(
        name="c1_tiny_decode_f32", n_layers=1, n_heads=8, d_model=512, d_head=64,
        batch=1, context=512, kv_dtype="f32", decay=8.0, seed=0, phase="decode",
        explicit_ranks=[16, 32, 48, 64, 16, 32, 48, 64]),
    # Llama-2-7B-shaped decode layer, uniform rank 64.
    "c2_uniform_decode": Workload(
        name="c2_uniform_decode", n_layers=1, n_heads=32, d_model=4096, d_head=128,
        batch=8, context=4096, kv_dtype="bf16", decay=32.0, seed=0, phase="decode",
        explicit_ranks=[64] * 32),
    # Adaptive-rank decode, 32 layers.
    "c3_adaptive_decode": Workload(
        name="c3_adaptive_decode", n_layers=32, n_heads=32, d_model=4096, d_head=128,
        batch=16, context=8192, kv_dtype="bf16", decay=32.0, seed=0, phase="decode",
        rank_seed=0, granule=128),
    # Long-context decode, one sequence, split-K over >= 256 chunks per head.
    "c4_long_decode": Workload(
        name="c4_long_decode", n_layers=1, n_heads=32, d_model=4096, d_head=128,
        batch=1, context=131072, kv_dtype="bf16", decay=32.0, seed=1, phase="decode",
        rank_seed=1, min_split=256),
    # Causal prefill plus latent projection.
    "c5_prefill": Workload(
        name="c5_prefill", n_layers=1, n_heads=32, d_model=4096, d_head=128,
        batch=4, context=4096, kv_dtype="bf16", decay=32.0, seed=0, phase="prefill",
        rank_seed=0),
}
