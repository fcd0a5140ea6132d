"""Pins for the integer oracle: layout bijection, scheduling invariants, list-scheduling
bounds against an exhaustive optimum, the paper's worked decode example, hand-worked
prefill numbers, and Eq. (1) against closed-form geometric tails.
"""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import layout as ol
from oracle import planner as op
from oracle import rank_select as ors
from workloads import generators as gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ layout
def test_layout_is_a_bijection_and_chunks_are_contiguous():
    ranks = np.array([[16, 48, 32], [64, 16, 16]])
    B, S = 2, 5
    tb = ol.layout_tables(ranks, B, S)
    for l in range(2):
        seen = set()
        for b in range(B):
            for h in range(3):
                prev = None
                for t in range(S):
                    for i in range(ranks[l, h]):
                        e = ol.element_index(tb, ranks, S, l, b, h, t, i)
                        assert e not in seen
                        seen.add(e)
                        if prev is not None:
                            assert e == prev + 1      # a unit is one dense run: any [t0,t1) is a span
                        prev = e
        assert seen == set(range(int(tb["elems"][l])))
        assert np.all(np.diff(tb["off"][l]) > 0)
        assert tb["off_r"][l, -1] == ranks[l].sum()
        assert tb["off"][l, -1] + S * ranks[l, -1] == S * ranks[l].sum()


# ------------------------------------------------------------------ decode planner
def _check_decode_invariants(plan, seq_len, rk, rv, W, split=True, G=64):
    B, H = len(seq_len), len(rk)
    n = len(plan["tile_b"])
    d_sum = [int(rk[h] + rv[h] + 1) for h in range(H)]
    # every token of every unit exactly once, tiles of a unit consecutive and ordered
    utp = plan["unit_tile_ptr"]
    assert utp[0] == 0 and utp[-1] == n
    for b in range(B):
        for h in range(H):
            u = b * H + h
            t = 0
            for j in range(utp[u], utp[u + 1]):
                assert (plan["tile_b"][j], plan["tile_h"][j]) == (b, h)
                assert plan["tile_t0"][j] == t and plan["tile_t1"][j] > t
                assert plan["tile_cost"][j] == (plan["tile_t1"][j] - t) * d_sum[h]
                t = plan["tile_t1"][j]
            assert t == seq_len[b]
    # every tile on exactly one worker; loads add up
    assert sorted(plan["worker_tiles"].tolist()) == list(range(n))
    total = sum(int(seq_len[b]) * d_sum[h] for b in range(B) for h in range(H))
    assert int(plan["worker_load"].sum()) == total
    for w in range(W):
        ids = plan["worker_tiles"][plan["worker_ptr"][w]:plan["worker_ptr"][w + 1]]
        assert int(plan["tile_cost"][ids].sum()) == int(plan["worker_load"][w])
        if not split:   # the paper's rule hands a worker its tasks in non-increasing cost order
            assert np.all(np.diff(plan["tile_cost"][ids]) <= 0)
    if n:
        mx = int(plan["worker_load"].max())
        big = int(plan["tile_cost"].max())
        assert mx >= max(math.ceil(total / W), big)
        assert mx <= total / W + big                     # list-scheduling bound
        if split:                                        # capacity: mean load plus one granule
            assert mx <= math.ceil(total / W) + G * max(d_sum)
            assert mx <= total / W + big
            # cuts fall on granule multiples; at most one extra tile per worker
            assert np.all(plan["tile_t0"] % G == 0)


def test_decode_paper_example_from_golden_file():
    spec = {}
    sets = {}
    for line in open(os.path.join(GOLDEN, "decode_schedule_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        if k == "set":
            sets[v[0]] = sorted(int(s[1:]) - 1 for s in v[1:])
        else:
            spec[k] = [int(x) for x in v]
    costs = spec["costs_not_from_paper"]
    W = spec["workers"][0]
    assert len(costs) == spec["tasks"][0] and costs == sorted(costs, reverse=True)
    lists, loads = op.lpt_assign(costs, W)
    assert [sorted(x) for x in lists] == [sets["SM1"], sets["SM2"], sets["SM3"]]
    # the same through the planner proper: one sequence of length 1 per task is not expressible
    # (cost = s_kv * d_sum), so use seven sequences whose lengths are the costs and a single head
    # whose d_sum is 33, with splitting switched off.
    plan = op.plan_decode(costs, [16], [16], W, granule=64, min_split=1, split=False)
    got = [sorted(plan["worker_tiles"][plan["worker_ptr"][w]:plan["worker_ptr"][w + 1]].tolist())
           for w in range(W)]
    assert got == [sets["SM1"], sets["SM2"], sets["SM3"]]
    assert plan["worker_load"].tolist() == [13 * 33, 13 * 33, 12 * 33]


def test_decode_no_split_is_one_task_per_head_sorted_descending():
    seq = [700, 64, 1300]
    rk, rv = [16, 128, 48], [32, 128, 16]
    plan = op.plan_decode(seq, rk, rv, 4, split=False)
    assert len(plan["tile_b"]) == 9 and np.all(np.diff(plan["unit_tile_ptr"]) == 1)
    assert np.array_equal(plan["tile_cost"].reshape(3, 3),
                          np.outer(seq, [49, 257, 65]))
    _check_decode_invariants(plan, seq, rk, rv, 4, split=False)
    # hand-worked: costs sorted 334100 179900 84500 63700 45500 34300 16448 4160 3136
    # first four open workers 0..3; 45500 -> w3 (63700); 34300 -> w2 (84500); 16448 -> w3 (109200);
    # 4160 -> w2 (118800); 3136 -> w2 (122960 < 125648)
    assert plan["worker_load"].tolist() == [334100, 179900, 84500 + 34300 + 4160 + 3136, 63700 + 45500 + 16448]


def _worker_lists(plan, W, key="worker_tiles"):
    return [plan[key][plan["worker_ptr"][w]:plan["worker_ptr"][w + 1]].tolist() for w in range(W)]


def test_decode_split_room_of_half_a_step_rounds_up_hand_worked():
    # Divisible-work extension. One head, rk = rv = 16: d_sum = 33, one granule of 64 tokens costs
    # step = 2112. Sequences of 256 and 64 tokens on W = 2: total = 320 * 33 = 10560, mean = 5280
    # = 2.5 steps. Chunks in descending cost: the 256-token unit (8448), then the 64-token unit (2112).
    #   8448 -> worker 0 (load 0): room 5280 = 2.5 steps, nearest granule count is a tie, ties go UP:
    #           3 granules = 192 tokens stay, load 6336; the other 64 tokens go on
    #        -> worker 1 (load 0): room 2.5 steps, they fit: load 2112
    #   2112 -> worker 1 (2112 < 6336): room 5280 - 2112 = 3168 = 1.5 steps -> 2 granules, fits: load 4224
    # (Ties down would cut the first unit at 128 and send the short unit to worker 0.)
    plan = op.plan_decode([256, 64], [16], [16], 2, granule=64, min_split=1, split=True)
    assert plan["tile_t0"].tolist() == [0, 192, 0] and plan["tile_t1"].tolist() == [192, 256, 64]
    assert plan["tile_b"].tolist() == [0, 0, 1]
    assert plan["tile_cost"].tolist() == [6336, 2112, 2112]
    assert plan["unit_tile_ptr"].tolist() == [0, 2, 3]
    assert _worker_lists(plan, 2) == [[0], [1, 2]]
    assert plan["worker_load"].tolist() == [6336, 4224]
    # a room below half a step still takes one granule: 3 workers, sequences 192 and 64:
    # total 8448, mean 2816 = 1.33 steps. 6336 -> w0 keeps 1 granule (1.33 -> 1), load 2112; the rest (128)
    # -> w1 keeps 1 granule, load 2112; the rest (64) -> w2, load 2112. Then 2112 -> w0 (all equal, lowest
    # id): room 704 = 0.33 steps -> 0 granules, raised to one: load 4224.
    plan = op.plan_decode([192, 64], [16], [16], 3, granule=64, min_split=1, split=True)
    assert plan["tile_t0"].tolist() == [0, 64, 128, 0] and plan["tile_t1"].tolist() == [64, 128, 192, 64]
    assert _worker_lists(plan, 3) == [[0, 3], [1], [2]]
    assert plan["worker_load"].tolist() == [4224, 2112, 2112]


def test_decode_equal_cost_chunks_go_out_lowest_id_first_hand_worked():
    # The paper's rule (no splitting), one head of d_sum 33, W = 2, sequences 64, 64, 64, 128.
    # Costs 2112, 2112, 2112, 4224. Sorted: unit 3, then the three equal ones in id order 0, 1, 2.
    #   unit 3 -> w0 (4224); unit 0 -> w1 (2112); unit 1 -> w1 (2112 < 4224; 4224);
    #   unit 2 -> loads equal, lowest worker: w0 (6336).
    plan = op.plan_decode([64, 64, 64, 128], [16], [16], 2, split=False)
    assert _worker_lists(plan, 2) == [[3, 2], [0, 1]]
    assert plan["worker_load"].tolist() == [6336, 4224]
    # Equal-cost chunks of ONE unit (min_split = 2, splitting on): 256 tokens -> chunks [0,128), [128,256)
    # of cost 4224 each; mean = 4224 = 2 steps. Chunk 0 first -> w0 (room 2 steps: fits), chunk 1 -> w1.
    plan = op.plan_decode([256], [16], [16], 2, granule=64, min_split=2, split=True)
    assert plan["tile_t0"].tolist() == [0, 128] and plan["tile_t1"].tolist() == [128, 256]
    assert _worker_lists(plan, 2) == [[0], [1]]
    # Two heads of equal d_sum (16 + 32 + 1 = 32 + 16 + 1 = 49), one sequence: head 0 goes out first.
    plan = op.plan_decode([128], [16, 32], [32, 16], 2, split=False)
    assert plan["tile_cost"].tolist() == [6272, 6272] and _worker_lists(plan, 2) == [[0], [1]]


def test_decode_softmax_cost_replaces_the_plus_one_hand_worked():
    # d_sum = rk + rv + softmax_cost. Heads A (16 + 16) and B (64 + 64); sequences 400 and 110; W = 2, no split.
    #               softmax_cost 1 (paper): d_sum 33 / 129     softmax_cost 7: d_sum 39 / 135
    #   tile 0 (b0, A)   13200                                   15600
    #   tile 1 (b0, B)   51600                                   54000
    #   tile 2 (b1, A)    3630                                    4290
    #   tile 3 (b1, B)   14190                                   14850
    # paper:  1 -> w0; then 3, 0, 2 all to w1 (14190, 27390, 31020 < 51600)
    # cost 7: 1 -> w0; then 0, 3, 2 all to w1 (15600, 30450, 34740 < 54000): tiles 0 and 3 swap places
    plan = op.plan_decode([400, 110], [16, 64], [16, 64], 2, split=False)
    assert plan["tile_cost"].tolist() == [13200, 51600, 3630, 14190]
    assert _worker_lists(plan, 2) == [[1], [3, 0, 2]] and plan["worker_load"].tolist() == [51600, 31020]
    plan = op.plan_decode([400, 110], [16, 64], [16, 64], 2, split=False, softmax_cost=7)
    assert plan["tile_cost"].tolist() == [15600, 54000, 4290, 14850]
    assert _worker_lists(plan, 2) == [[1], [0, 3, 2]] and plan["worker_load"].tolist() == [54000, 34740]
    # with splitting the granule step scales too: rk = rv = 16, softmax_cost 7 -> d_sum 39, step 2496;
    # sequences 256 and 64 on two workers: mean = 320 * 39 / 2 = 6240 = 2.5 steps -> same cuts as with d_sum 33
    plan = op.plan_decode([256, 64], [16], [16], 2, granule=64, split=True, softmax_cost=7)
    assert plan["tile_t1"].tolist() == [192, 256, 64] and plan["tile_cost"].tolist() == [7488, 2496, 2496]
    assert plan["worker_load"].tolist() == [7488, 4992]


def test_prefill_causal_mode_costs_and_hand_out_order_hand_worked():
    # Causal cost mode: a task costs d_sum * (number of (query row, visible key) pairs); ALL tasks are handed
    # out in descending cost order (ties: lower task id) to the least-loaded worker (ties: lower id).
    # Heads: d_sum 33 (16 + 16 + 1) and 97 (48 + 48 + 1); base row block 16:
    #   B_r = [round_up_16(ceil(16 * 97 / 33) = 48) = 48, 16]. One prompt of 64 tokens.
    # Row i sees i + 1 keys; rows [a, b) see b(b+1)/2 - a(a+1)/2 pairs:
    #   task 0  h0 [0, 48)   1176 pairs * 33 = 38808
    #   task 1  h0 [48, 64)   904 pairs * 33 = 29832
    #   task 2  h1 [0, 16)    136 pairs * 97 = 13192
    #   task 3  h1 [16, 32)   392 pairs * 97 = 38024
    #   task 4  h1 [32, 48)   648 pairs * 97 = 62856
    #   task 5  h1 [48, 64)   904 pairs * 97 = 87688
    # order 5, 4, 0, 3, 1, 2 on W = 2:  5 -> w0 (87688); 4 -> w1 (62856); 0 -> w1 (101664);
    #   3 -> w0 (125712); 1 -> w1 (131496); 2 -> w0 (138904)
    plan = op.plan_prefill([64], [64], [16, 48], [16, 48], 2, br_base=16, br_cap=256, cost_mode="causal")
    assert plan["br"].tolist() == [48, 16]
    assert list(zip(plan["task_h"].tolist(), plan["task_q0"].tolist(), plan["task_q1"].tolist())) == \
        [(0, 0, 48), (0, 48, 64), (1, 0, 16), (1, 16, 32), (1, 32, 48), (1, 48, 64)]
    assert plan["task_cost"].tolist() == [38808, 29832, 13192, 38024, 62856, 87688]
    assert _worker_lists(plan, 2, "worker_tasks") == [[5, 3, 2], [4, 0, 1]]
    assert plan["worker_load"].tolist() == [138904, 131496]
    # the paper's mode on the same input: cost rows * s_kv * d_sum, rounds in task order
    paper = op.plan_prefill([64], [64], [16, 48], [16, 48], 2, br_base=16, br_cap=256, cost_mode="paper")
    assert paper["task_cost"].tolist() == [48 * 64 * 33, 16 * 64 * 33] + [16 * 64 * 97] * 4
    assert _worker_lists(paper, 2, "worker_tasks") == [[0, 2, 4], [1, 3, 5]]
    # chunked prompt: the 32 queries are positions 68..99 of 100 keys, row i sees 69 + i keys.
    # one head (d_sum 33, B_r 16): [0,16) = 16*69 + 120 = 1224 pairs, [16,32) = 16*85 + 120 = 1480 pairs
    plan = op.plan_prefill([32], [100], [16], [16], 2, br_base=16, br_cap=16, cost_mode="causal")
    assert plan["task_cost"].tolist() == [1224 * 33, 1480 * 33]
    assert _worker_lists(plan, 2, "worker_tasks") == [[1], [0]]
    # equal costs (two heads of d_sum 49, one block each): the lower task id goes first, to the lower worker;
    # with softmax_cost 7 both are 55 * 136
    plan = op.plan_prefill([16], [16], [16, 32], [32, 16], 2, br_base=16, br_cap=16, cost_mode="causal")
    assert plan["task_cost"].tolist() == [136 * 49] * 2 and _worker_lists(plan, 2, "worker_tasks") == [[0], [1]]
    plan = op.plan_prefill([16], [16], [16, 32], [32, 16], 2, br_base=16, br_cap=16, cost_mode="causal", softmax_cost=7)
    assert plan["task_cost"].tolist() == [136 * 55] * 2


def test_lpt_tie_breaks():
    lists, loads = op.lpt_assign([5, 5, 5, 5], 3)
    assert lists == [[0, 3], [1], [2]] and loads == [10, 5, 5]


@pytest.mark.parametrize("seed", range(6))
def test_lpt_against_exhaustive_optimum(seed):
    g = gen.make_rng(100 + seed)
    n, W = int(g.integers(4, 9)), int(g.integers(2, 4))
    costs = [int(c) for c in g.integers(1, 40, size=n)]
    _, loads = op.lpt_assign(costs, W)
    best = min(max(sum(c for c, a in zip(costs, assign) if a == w) for w in range(W))
               for assign in itertools.product(range(W), repeat=n))
    assert best <= max(loads) <= (4 / 3 - 1 / (3 * W)) * best + 1e-9      # Graham's bound


@pytest.mark.parametrize("name", ["c2_uniform_decode", "c3_adaptive_decode", "c4_long_decode"])
def test_decode_plan_invariants_on_benchmark_shapes(name):
    wl = gen.CONFIGS[name]
    ranks = wl.ranks()[0]
    seq = [wl.context] * wl.batch
    W = 4096
    plan = op.plan_decode(seq, ranks, ranks, W, granule=64, min_split=wl.min_split)
    _check_decode_invariants(plan, seq, ranks, ranks, W)
    per_unit = np.diff(plan["unit_tile_ptr"])
    assert per_unit.min() >= wl.min_split
    n_chunks = wl.batch * wl.n_heads * wl.min_split
    assert len(plan["tile_b"]) <= n_chunks + W          # every cut fills one worker
    # balance: the busiest worker is within 10 % of the mean on these shapes (one granule of 64
    # tokens of the widest head is 8 % of a 193 KB share)
    assert plan["worker_load"].max() <= 1.10 * plan["worker_load"].mean()


def test_decode_plan_ragged_and_empty_sequences():
    seq = [0, 1, 63, 64, 65, 1000, 0, 4097]
    rk, rv = [16, 112, 64, 32], [48, 16, 64, 128]
    for W, ms, split in [(7, 1, True), (64, 1, True), (5, 3, True), (5, 3, False), (3, 1, False)]:
        plan = op.plan_decode(seq, rk, rv, W, granule=64, min_split=ms, split=split)
        _check_decode_invariants(plan, seq, rk, rv, W, split=split)
    empty = op.plan_decode([0, 0], rk, rv, 4)
    assert len(empty["tile_b"]) == 0 and empty["worker_ptr"].tolist() == [0] * 5


# ------------------------------------------------------------------ prefill planner
def test_prefill_row_blocks_equalise_task_cost():
    # B_r_i = B_r * d_sum_max / d_sum_i (Section 5.3), rounded up to 16 (Section 6.1)
    rk = [16, 32, 64, 128, 48]
    br = op.prefill_row_blocks(rk, rk, br_base=64, br_cap=1 << 20)
    d_sum = [2 * r + 1 for r in rk]
    assert br[3] == 64                                            # the widest head keeps B_r
    assert br[0] == 512 and br[1] == 256 and br[2] == 128         # ceil(64*257/33)=499 -> 512, ...
    for b, ds in zip(br, d_sum):
        assert b % 16 == 0
        assert 64 * 257 <= b * ds < 64 * 257 + 16 * ds            # equal cost up to one 16-row step
    assert op.prefill_row_blocks(rk, rk, 64, 256)[0] == 256       # register cap


def _check_prefill_cover(plan, q_len, H):
    cover = {}
    for b, h, q0, q1 in zip(plan["task_b"], plan["task_h"], plan["task_q0"], plan["task_q1"]):
        assert q1 > q0
        cover.setdefault((int(b), int(h)), []).append((int(q0), int(q1)))
    for b in range(len(q_len)):
        for h in range(H):
            if q_len[b] == 0:
                assert (b, h) not in cover
                continue
            t = 0
            for q0, q1 in sorted(cover[(b, h)]):
                assert q0 == t
                t = q1
            assert t == q_len[b]
    n = len(plan["task_b"])
    assert sorted(plan["worker_tasks"].tolist()) == list(range(n))
    assert int(plan["worker_load"].sum()) == int(plan["task_cost"].sum())


def test_prefill_last_round_hand_worked():
    # Two heads, d_sum = 33 and 97; B_r = [192, 64]  (ceil(64*97/33) = 189 -> 192).
    # One sequence of 256 tokens: head 0 -> rows [0,192), [192,256); head 1 -> four blocks of 64.
    # Six tasks on W = 4 workers: one full round (tasks 0..3), last round = tasks 4, 5
    # (head 1 rows [128,192) and [192,256)).  wl = ceil((64*97 + 64*97) / 4) = 3104;
    # new row block = floor16(3104 / 97 = 32) = 32 -> four tasks of 32 rows, one per worker.
    plan = op.plan_prefill([256], [256], [16, 48], [16, 48], 4, br_base=64, br_cap=256, cost_mode="paper")
    assert plan["br"].tolist() == [192, 64]
    tasks = list(zip(plan["task_h"].tolist(), plan["task_q0"].tolist(), plan["task_q1"].tolist()))
    assert tasks == [(0, 0, 192), (0, 192, 256), (1, 0, 64), (1, 64, 128),
                     (1, 128, 160), (1, 160, 192), (1, 192, 224), (1, 224, 256)]
    assert plan["task_cost"].tolist() == [192 * 256 * 33, 64 * 256 * 33, 64 * 256 * 97, 64 * 256 * 97] + \
        [32 * 256 * 97] * 4
    lists = [plan["worker_tasks"][plan["worker_ptr"][w]:plan["worker_ptr"][w + 1]].tolist() for w in range(4)]
    assert lists == [[0, 4], [1, 5], [2, 6], [3, 7]]
    _check_prefill_cover(plan, [256], 2)


@pytest.mark.parametrize("mode", ["paper", "causal"])
def test_prefill_plan_cover_and_balance(mode):
    wl = gen.CONFIGS["c5_prefill"]
    ranks = wl.ranks()[0]
    q = [wl.context] * wl.batch
    plan = op.plan_prefill(q, q, ranks, ranks, 256, cost_mode=mode)
    _check_prefill_cover(plan, q, wl.n_heads)
    assert np.all(plan["task_q0"] % 16 == 0)
    if mode == "causal":
        # cost = d_sum * sum_{i in block} (i + 1); descending hand-out balances to within 2 %
        j = 17
        h, q0, q1 = plan["task_h"][j], plan["task_q0"][j], plan["task_q1"][j]
        assert plan["task_cost"][j] == (2 * ranks[h] + 1) * (q1 * (q1 + 1) // 2 - q0 * (q0 + 1) // 2)
        assert plan["worker_load"].max() <= 1.02 * plan["worker_load"].mean()


def test_prefill_plan_ragged_lengths():
    plan = op.plan_prefill([0, 5, 130, 17], [0, 9, 130, 4000], [16, 64, 32], [32, 64, 16], 6, cost_mode="paper")
    _check_prefill_cover(plan, [0, 5, 130, 17], 3)
    plan = op.plan_prefill([0, 5, 130, 17], [0, 9, 130, 4000], [16, 64, 32], [32, 64, 16], 6, cost_mode="causal")
    _check_prefill_cover(plan, [0, 5, 130, 17], 3)


# ------------------------------------------------------------------ Eq. (1)
def test_rank_selection_geometric_closed_form():
    # theta_i = e^{-i/c}: tail(j) = (e^{-j/c} - e^{-n/c}) / (1 - e^{-n/c}); invert by hand for each r
    n, c = 128, 32.0
    theta = np.exp(-np.arange(n) / c)
    for r in (0.001, 0.01, 0.05, 0.2, 0.5, 0.9):
        # largest j with tail(j) > r  <=>  e^{-j/c} > r (1 - e^{-n/c}) + e^{-n/c}
        rhs = r * (1 - math.exp(-n / c)) + math.exp(-n / c)
        j_closed = math.ceil(-c * math.log(rhs)) - 1
        j = ors.last_kept_index(theta, r)
        assert j == j_closed
        tail = lambda k: theta[k:].sum() / theta.sum()
        assert tail(j + 1) <= r < tail(j)                   # Eq. (1) itself
        lo, hi = ors.compression_rate_interval(j, n)
        for p in (hi, (lo + hi) / 2):
            assert math.floor((1 - p) * (n - 1) + 1e-12) == j
        assert ors.kept_rank(theta, r) == -(-(j + 1) // 16) * 16
    assert ors.last_kept_index(theta, 0.0) == n - 1         # nothing may be removed
    assert ors.last_kept_index(theta, 1.0) == 0             # keep one dimension at least
    # flat spectrum: removing m of n dimensions removes m/n of the mass
    flat = np.ones(10)
    assert ors.last_kept_index(flat, 0.35) == 6             # dims 7,8,9 removed (0.3 <= 0.35 < 0.4)


def test_paged_plan_is_the_unpaged_plan_cut_at_page_boundaries():
    """Paging must not change the schedule, only cut tiles where a page ends."""
    rk, rv = [16, 64, 32], [32, 64, 16]
    seq = [0, 5, 700, 1300, 256]
    for W, G, P, ms in [(7, 64, 256, 1), (40, 16, 64, 2), (3, 64, 64, 1), (500, 32, 128, 3)]:
        base = op.plan_decode(seq, rk, rv, W, granule=G, min_split=ms)
        paged = op.plan_decode(seq, rk, rv, W, granule=G, min_split=ms, page_tokens=P)
        assert np.array_equal(base["worker_load"], paged["worker_load"])
        # no tile crosses a page boundary, and the tiles still tile every unit exactly
        assert np.all(paged["tile_t0"] // P == (paged["tile_t1"] - 1) // P)
        H = len(rk)
        for b, S in enumerate(seq):
            for h in range(H):
                u = b * H + h
                lo, hi = paged["unit_tile_ptr"][u], paged["unit_tile_ptr"][u + 1]
                cover = sorted(zip(paged["tile_t0"][lo:hi], paged["tile_t1"][lo:hi]))
                assert [c[0] for c in cover] == ([0] + [c[1] for c in cover[:-1]] if cover else [])
                assert (cover[-1][1] if cover else 0) == S
        # merging the parts of a worker's consecutive tiles gives back the unpaged worker lists
        def spans(plan, w):
            out = []
            for t in plan["worker_tiles"][plan["worker_ptr"][w]:plan["worker_ptr"][w + 1]]:
                key = (int(plan["tile_b"][t]), int(plan["tile_h"][t]))
                a, b_ = int(plan["tile_t0"][t]), int(plan["tile_t1"][t])
                if out and out[-1][0] == key and out[-1][2] == a and a % P == 0:
                    out[-1] = (key, out[-1][1], b_)
                else:
                    out.append((key, a, b_))
            return out
        for w in range(W):
            merged, ref = spans(paged, w), spans(base, w)
            # a base piece that itself starts on a page boundary right after the previous one would merge
            # too; compare the covered token sets per unit instead of the span lists in that case
            cov = lambda sp: sorted((k, t) for k, a, b_ in sp for t in range(a, b_, G))
            assert cov(merged) == cov(ref)
    # P = 0 is the unpaged plan itself
    a, b = op.plan_decode(seq, rk, rv, 9), op.plan_decode(seq, rk, rv, 9, page_tokens=0)
    assert all(np.array_equal(a[k], b[k]) for k in a)


def test_paged_element_index_is_a_bijection_onto_the_pages():
    from oracle import layout as ol
    ranks = [16, 48, 32]
    P, n_pages = 8, 5
    table = [3, 0, 4]                      # a sequence of up to 24 tokens
    seen = set()
    for h in range(3):
        for t in range(19):
            for i in range(ranks[h]):
                e = ol.paged_element_index(ranks, P, table, h, t, i)
                assert 0 <= e < n_pages * P * sum(ranks) and e not in seen
                seen.add(e)
                # same element through the dense layout with batch = page, max_seq = P
                tabs = ol.layout_tables([ranks], n_pages, P)
                assert e == ol.element_index(tabs, [ranks], P, 0, table[t // P], h, t % P, i)
    # tokens of one page and head are one contiguous run
    run = [ol.paged_element_index(ranks, P, table, 1, t, i) for t in range(8, 16) for i in range(48)]
    assert run == list(range(run[0], run[0] + 8 * 48))
