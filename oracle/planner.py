"""Oracle (test infrastructure): the work partitioner, step by step, in integers.

Section 5.3 (kernel enhancement for adaptive compression rate):

  decode   every (sequence, head) is one task of cost s_kv * d_sum,
           d_sum = d_qk + d_v + 1; tasks are sorted by cost in descending order
           and given, one at a time, to the worker with the smallest
           accumulated cost.
  prefill  head i uses the row block B_r * d_sum_max / d_sum_i so that every
           Q-block task costs the same, 2 * B_r * s_kv * d_sum; tasks run in
           rounds of N workers; the tasks of an incomplete last round are
           re-split with row block wl / d_sum_i,
           wl = (1/N) * sum_last B_r_i * d_sum_i, and handed one at a time to
           the least-loaded worker. Row blocks are multiples of 16
           (implementation paragraph, Section 6.1).

Readings taken where the paper is silent (all integer, all deterministic):
  * ties: sort by (cost descending, task id ascending); least-loaded ties go
    to the lowest worker id.
  * decode KV-chunk splitting is NOT in the paper (it never splits a decode
    head). Attention over a key range is divisible (partial softmax states
    merge exactly), so the list scheduling is given a per-worker capacity of
    the mean load plus one granule: a task that does not fit is cut at a
    multiple of the granule G and its remainder goes to the next least-loaded
    worker. With split = False and min_split = 1 this is the paper's
    one-task-per-head scheduling, unchanged.
  * prefill cost_mode "paper" uses rows * s_kv * d_sum (the paper's formula
    without the constant 2, no mask); cost_mode "causal" counts only the keys
    a causal query row sees and orders all tasks by descending cost instead of
    rounds. The paper never mentions the mask.
  * the paper's last-round hand-out is "sequentially ... one at a time" with
    no sort; it is done in task order.
  * softmax_cost: the paper's d_sum = d_qk + d_v + 1 charges the softmax one unit
    per score. The parameter replaces that 1 (default 1 = the paper) for kernels
    whose per-score softmax work weighs more than one multiply-add.
"""
from __future__ import annotations

import numpy as np


def _ceil_div(a: int, b: int) -> int:
    return -(-a // b)


def _round_up(a: int, m: int) -> int:
    return _ceil_div(a, m) * m


def lpt_assign(costs, n_workers: int, presorted: bool = False):
    """List scheduling: tasks (sorted by cost desc, id asc unless presorted) each go
    to the worker with the smallest accumulated cost; ties to the lowest id.

    Returns (assignment list of lists of task ids, loads list).
    """
    ids = list(range(len(costs)))
    if not presorted:
        ids.sort(key=lambda i: (-int(costs[i]), i))
    loads = np.zeros(n_workers, dtype=np.int64)
    lists = [[] for _ in range(n_workers)]
    for i in ids:
        w = int(np.argmin(loads))  # first minimum = lowest worker id
        lists[w].append(i)
        loads[w] += int(costs[i])
    return lists, [int(x) for x in loads]


def plan_decode(seq_len, rk, rv, n_workers: int, granule: int = 64, min_split: int = 1,
                split: bool = True, softmax_cost: int = 1, page_tokens: int = 0):
    """Decode plan for one layer.

    seq_len int [B]; rk, rv int [H]. Steps:
      1. unit (b, h) has cost seq_len[b] * d_sum[h], d_sum = rk + rv + 1 (the paper's task cost;
         softmax_cost replaces the "+ 1" when a kernel's softmax work weighs more than one
         multiply-add per score).
      2. every non-empty unit is pre-cut into min(min_split, ceil(S/G)) near-equal chunks whose
         boundaries are multiples of the granule G (min_split = 1: the unit itself).
      3. the chunks are sorted by (cost descending, id ascending) and handed, one at a time, to
         the worker with the smallest accumulated cost (the paper's rule).
      4. extension for divisible work (split = True): a worker is filled up to the mean load
         ceil(total / W). If the chunk does not fit in the room left, the worker takes the number
         of granules nearest to room / (G * d_sum) (ties up, at least one) and the rest of the
         chunk goes to the then least-loaded worker, and so on; no load exceeds
         mean + G * max d_sum. With split = False the room is unlimited and steps 1-3 are exactly
         the paper's scheduling.
      5. paged cache (page_tokens = P > 0, P a multiple of G): a sequence's tokens live in pages
         of P tokens that need not be adjacent in memory, so after step 4 every piece is cut at
         the multiples of P it contains; the parts stay with the piece's worker, in order. The
         schedule itself (steps 1-4) does not depend on P.
    The pieces become tiles, numbered by (unit, t0). Returns a dict of numpy tables:
      tile_b, tile_h, tile_t0, tile_t1 int32 [n_tiles]; tile_cost int64 [n_tiles]
      unit_tile_ptr int32 [B*H + 1]  (tiles of unit u = b*H + h are
                                      unit_tile_ptr[u] .. unit_tile_ptr[u+1]-1)
      worker_ptr int32 [W + 1], worker_tiles int32 [n_tiles] (in hand-out order),
      worker_load int64 [W]
    """
    B, H = len(seq_len), len(rk)
    W, G = int(n_workers), int(granule)
    d_sum = [int(rk[h]) + int(rv[h]) + int(softmax_cost) for h in range(H)]
    total = sum(int(seq_len[b]) * d_sum[h] for b in range(B) for h in range(H))

    chunks = []  # (b, h, t0, t1)
    for b in range(B):
        S = int(seq_len[b])
        for h in range(H):
            if S > 0:
                n = max(1, min(int(min_split), _ceil_div(S, G)))
                size = _round_up(_ceil_div(S, n), G)
                n = _ceil_div(S, size)
                for j in range(n):
                    chunks.append((b, h, j * size, min(S, (j + 1) * size)))
    chunk_cost = [(t1 - t0) * d_sum[h] for (_, h, t0, t1) in chunks]
    order = sorted(range(len(chunks)), key=lambda i: (-chunk_cost[i], i))

    mean = _ceil_div(total, W)
    loads = np.zeros(W, dtype=np.int64)
    pieces = []        # (b, h, t0, t1, worker, hand-out sequence number)
    for i in order:
        b, h, t0, t1 = chunks[i]
        while t0 < t1:
            w = int(np.argmin(loads))          # first minimum = lowest worker id
            take = t1 - t0
            if split:
                room = mean - int(loads[w])
                step = G * d_sum[h]
                fit = max(1, (2 * room + step) // (2 * step)) * G   # nearest granule count, at least one
                take = min(take, fit)
            end = t0 + take
            lo = t0
            while lo < end:                     # one piece per page it touches (all of it when unpaged)
                hi = min(end, (lo // page_tokens + 1) * page_tokens) if page_tokens > 0 else end
                pieces.append((b, h, lo, hi, w, len(pieces)))
                lo = hi
            loads[w] += take * d_sum[h]
            t0 += take

    by_unit = sorted(range(len(pieces)), key=lambda k: (pieces[k][0], pieces[k][1], pieces[k][2]))
    tile_of_piece = {k: tid for tid, k in enumerate(by_unit)}
    unit_tile_ptr = [0] * (B * H + 1)
    for k in by_unit:
        unit_tile_ptr[pieces[k][0] * H + pieces[k][1] + 1] += 1
    for u in range(B * H):
        unit_tile_ptr[u + 1] += unit_tile_ptr[u]
    lists = [[] for _ in range(W)]
    for k, pc in enumerate(pieces):            # pieces are already in hand-out order
        lists[pc[4]].append(tile_of_piece[k])
    worker_ptr = [0]
    worker_tiles = []
    for w in range(W):
        worker_tiles.extend(lists[w])
        worker_ptr.append(len(worker_tiles))
    P = [pieces[k] for k in by_unit]
    return {
        "tile_b": np.array([p[0] for p in P], dtype=np.int32),
        "tile_h": np.array([p[1] for p in P], dtype=np.int32),
        "tile_t0": np.array([p[2] for p in P], dtype=np.int32),
        "tile_t1": np.array([p[3] for p in P], dtype=np.int32),
        "tile_cost": np.array([(p[3] - p[2]) * d_sum[p[1]] for p in P], dtype=np.int64),
        "unit_tile_ptr": np.array(unit_tile_ptr, dtype=np.int32),
        "worker_ptr": np.array(worker_ptr, dtype=np.int32),
        "worker_tiles": np.array(worker_tiles, dtype=np.int32),
        "worker_load": loads.copy(),
    }


def prefill_row_blocks(rk, rv, br_base: int = 64, br_cap: int = 256, softmax_cost: int = 1):
    """B_r per head: round_up_16(ceil(br_base * d_sum_max / d_sum_h)), capped at br_cap."""
    d_sum = [int(a) + int(b) + int(softmax_cost) for a, b in zip(rk, rv)]
    d_max = max(d_sum)
    return [min(int(br_cap), _round_up(_ceil_div(int(br_base) * d_max, ds), 16)) for ds in d_sum]


def _q_block_cost(q0: int, q1: int, q_len: int, kv_len: int, d_sum: int, causal_cost: bool) -> int:
    if not causal_cost:
        return (q1 - q0) * kv_len * d_sum
    # query row i sits at position kv_len - q_len + i and sees that many + 1 keys
    return sum(kv_len - q_len + i + 1 for i in range(q0, q1)) * d_sum


def plan_prefill(q_len, kv_len, rk, rv, n_workers: int, br_base: int = 64, br_cap: int = 256,
                 cost_mode: str = "paper", softmax_cost: int = 1):
    """Prefill plan for one layer.

    q_len, kv_len int [B] (queries are the last q_len positions of kv_len);
    rk, rv int [H]. Returns dict of numpy tables:
      br int32 [H]; task_b, task_h, task_q0, task_q1 int32 [n_tasks]; task_cost int64
      worker_ptr int32 [W+1], worker_tasks int32 [n_tasks], worker_load int64 [W]
    """
    assert cost_mode in ("paper", "causal")
    causal_cost = cost_mode == "causal"
    B, H, W = len(q_len), len(rk), int(n_workers)
    d_sum = [int(rk[h]) + int(rv[h]) + int(softmax_cost) for h in range(H)]
    br = prefill_row_blocks(rk, rv, br_base, br_cap, softmax_cost)

    tasks = []  # (b, h, q0, q1)
    for b in range(B):
        for h in range(H):
            q0 = 0
            while q0 < int(q_len[b]):
                q1 = min(int(q_len[b]), q0 + br[h])
                tasks.append((b, h, q0, q1))
                q0 = q1

    def cost_of(t):
        b, h, q0, q1 = t
        return _q_block_cost(q0, q1, int(q_len[b]), int(kv_len[b]), d_sum[h], causal_cost)

    lists = [[] for _ in range(W)]
    loads = [0] * W
    if causal_cost:
        costs = [cost_of(t) for t in tasks]
        lists, loads = lpt_assign(costs, W)
    else:
        n_tasks = len(tasks)
        n_last = n_tasks % W
        full = n_tasks - n_last
        for i in range(full):
            w = i % W
            lists[w].append(i)
            loads[w] += cost_of(tasks[i])
        if n_last > 0:
            last = tasks[full:]
            wl = _ceil_div(sum((q1 - q0) * d_sum[h] for (_, h, q0, q1) in last), W)
            resplit = []
            for (b, h, q0, q1) in last:
                nb = max(16, (wl // d_sum[h]) // 16 * 16)
                s = q0
                while s < q1:
                    e = min(q1, s + nb)
                    resplit.append((b, h, s, e))
                    s = e
            tasks = tasks[:full] + resplit
            round_loads = np.zeros(W, dtype=np.int64)
            for j, t in enumerate(resplit):
                w = int(np.argmin(round_loads))
                c = cost_of(t)
                lists[w].append(full + j)
                round_loads[w] += c
                loads[w] += c
        costs = [cost_of(t) for t in tasks]

    worker_ptr = [0]
    worker_tasks = []
    for w in range(W):
        worker_tasks.extend(lists[w])
        worker_ptr.append(len(worker_tasks))
    arr = np.array(tasks, dtype=np.int32).reshape(-1, 4)
    return {
        "br": np.array(br, dtype=np.int32),
        "task_b": arr[:, 0].copy(), "task_h": arr[:, 1].copy(),
        "task_q0": arr[:, 2].copy(), "task_q1": arr[:, 3].copy(),
        "task_cost": np.array(costs, dtype=np.int64),
        "worker_ptr": np.array(worker_ptr, dtype=np.int32),
        "worker_tasks": np.array(worker_tasks, dtype=np.int32),
        "worker_load": np.array(loads, dtype=np.int64),
    }
