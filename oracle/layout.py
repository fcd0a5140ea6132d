"""Oracle (test infrastructure): offsets of the ragged per-head latent cache.

The paper stores the compressed K' (s x k) and V' per head and per layer in the
KV cache (Section 2) and lets k differ per head (Section 5.2); it does not
give a memory layout. The layout defined here, per layer l and separately for
K' and V':

  unit (b, h) is a dense row-major block [max_seq, r[l, h]];
  blocks of one sequence b are concatenated over h, sequences over b:
      index(b, h, t, i) = b * max_seq * R[l] + off[l, h] + t * r[l, h] + i
      off[l, h]   = max_seq * sum_{h' < h} r[l, h']          (elements)
      off_r[l, h] = sum_{h' < h} r[l, h'],  off_r[l, H] = R[l]
      elems[l]    = max_batch * max_seq * R[l]

so that any token range [t0, t1) of a unit is one contiguous span.
Written with plain Python integers, one loop per index.
"""
from __future__ import annotations

import numpy as np


def layout_tables(ranks, max_batch: int, max_seq: int):
    """ranks: int [L, H] kept ranks of one side (K or V).

    Returns dict(off int64 [L, H], off_r int32 [L, H+1], elems int64 [L]).
    """
    ranks = np.asarray(ranks)
    L, H = ranks.shape
    off = np.zeros((L, H), dtype=np.int64)
    off_r = np.zeros((L, H + 1), dtype=np.int32)
    elems = np.zeros((L,), dtype=np.int64)
    for l in range(L):
        run = 0
        for h in range(H):
            off_r[l, h] = run
            off[l, h] = int(max_seq) * run
            run += int(ranks[l, h])
        off_r[l, H] = run
        elems[l] = int(max_batch) * int(max_seq) * run
    return {"off": off, "off_r": off_r, "elems": elems}


def element_index(tables, ranks, max_seq: int, l: int, b: int, h: int, t: int, i: int) -> int:
    """Flat element index of latent component i of token t of unit (b, h) in layer l."""
    R = int(tables["off_r"][l, -1])
    return b * int(max_seq) * R + int(tables["off"][l, h]) + t * int(ranks[l][h]) + i


def paged_element_index(ranks_layer, page_tokens: int, block_table_row, h: int, t: int, i: int) -> int:
    """Flat element index of latent component i of token t of head h of ONE sequence in a paged buffer.

    Paged storage (the usual block-table scheme of serving systems; the paper's system runs on
    one, Section 6.1, but gives no layout): the buffer of a layer is an array of pages; a page is
    the dense layout above for page_tokens tokens of one sequence, [head][token][component]:
        index = page * page_tokens * R + page_tokens * sum_{h' < h} r[h'] + (t % P) * r[h] + i
    with page = block_table_row[t // P] the physical page of the sequence's logical page t // P.
    In terms of layout_tables this is a layout with max_batch = number of pages, max_seq = P.
    """
    P = int(page_tokens)
    R = sum(int(x) for x in ranks_layer)
    before = sum(int(ranks_layer[hh]) for hh in range(h))
    page = int(block_table_row[t // P])
    return page * P * R + P * before + (t % P) * int(ranks_layer[h]) + i
