"""Pins for the oracle's load-aware router and Algorithm 1 (adaptive chunked prefill).

None of these goes through the oracle's own loop a second time: the figure's stated outcome,
the paper's chunk-cost form, a list-scheduling invariant, special cases that reduce to plain
FIFO chunking, and a second implementation in another style (a heap of ranks, run-length
queues, float ratios replaced by cross-multiplied integers).
"""
import heapq
import json
import os

import numpy as np
import pytest

from oracle.scheduler import adaptive_chunked_prefill, route_request, token_cost
from oracle import build_placement

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_fig4_router_and_batch():
    with open(os.path.join(GOLD, "fig4_router_scheduler.json")) as f:
        g = json.load(f)
    R = g["n_ranks"]
    pending = [0] * R
    for _req, gpu, toks in g["queued"]:
        pending[gpu] += toks
    # the load-aware router sends request 3 away from the GPU that holds request 0
    gpu3 = route_request(pending, g["new_request_tokens"])
    assert gpu3 == g["load_aware_gpu_of_request_3"] != g["round_robin_gpu_of_request_3"]
    assert 3 % R == g["round_robin_gpu_of_request_3"]
    entries = [(req, gpu, 0, toks) for req, gpu, toks in g["queued"]] + [(3, gpu3, 0, 1)]
    take, load, n = adaptive_chunked_prefill(g["budget"], R, entries, min_tokens=(g["budget"] + 1) // 2)
    assert take == g["adaptive_batch_tokens_per_request"] and n == g["budget"]
    assert load == [1, 1, 1]                      # every GPU has one first token to process
    # the naive batch the caption describes (first three tokens of request 0), priced the same way
    naive_load = [sum(token_cost(p) for p in range(g["naive_batch_tokens_per_request"][0])), 0, 0]
    assert max(naive_load) * R / sum(naive_load) == 3.0 and max(load) * R / sum(load) == 1.0


@pytest.mark.parametrize("N,L", [(1, 0), (5, 0), (7, 13), (128, 4096), (1, 99)])
def test_chunk_cost_has_the_papers_form(N, L):
    # a chunk of N tokens after L processed ones: N^2/2 + N L + N/2, i.e. O(N^2 + N L + N)
    assert sum(token_cost(L + j) for j in range(N)) == N * L + N * (N + 1) // 2


def test_single_rank_is_plain_fifo_chunking():
    entries = [(0, 0, 10, 5), (1, 0, 0, 4), (2, 0, 3, 9)]
    take, load, n = adaptive_chunked_prefill(7, 1, entries, min_tokens=7)
    assert take == [5, 2, 0] and n == 7
    assert load == [sum(range(11, 16)) + 1 + 2]
    # with one rank the ratio max/mean is always 1, so the largest candidate wins whatever the floor
    take0, _, n0 = adaptive_chunked_prefill(7, 1, entries, min_tokens=0)
    assert take0 == take and n0 == 7


def test_budget_beyond_everything_schedules_everything():
    entries = [(0, 1, 0, 3), (1, 0, 2, 2), (2, 1, 0, 1)]
    take, load, n = adaptive_chunked_prefill(100, 2, entries, min_tokens=100)
    assert take == [3, 2, 1] and n == 6
    assert load == [3 + 4, (1 + 2 + 3) + 1]


def test_equal_requests_one_per_rank_fill_evenly():
    R, k = 5, 6
    entries = [(r, r, 0, 50) for r in range(R)]
    take, load, n = adaptive_chunked_prefill(R * k, R, entries, min_tokens=R * k)
    assert take == [k] * R and n == R * k and load == [k * (k + 1) // 2] * R


def test_nothing_waiting_gives_an_empty_batch():
    take, load, n = adaptive_chunked_prefill(8, 3, [(0, 1, 5, 0)], min_tokens=4)
    assert take == [0] and n == 0 and load == [0, 0, 0]
    take, load, n = adaptive_chunked_prefill(0, 3, [(0, 1, 5, 2)], min_tokens=0)
    assert take == [0] and n == 0


def test_initial_loads_steer_the_first_tokens():
    # rank 0 is already busy: the first tokens go to rank 1 until it has caught up
    entries = [(0, 0, 0, 10), (1, 1, 0, 10)]
    take, load, n = adaptive_chunked_prefill(3, 2, entries, min_tokens=3, init_load=[5, 0])
    assert take == [0, 3] and load == [5, 6] and n == 3
    take, load, n = adaptive_chunked_prefill(4, 2, entries, min_tokens=4, init_load=[5, 0])
    assert take == [1, 3] and load == [6, 6]


def test_best_batch_stops_before_the_lonely_tail():
    # rank 1 runs dry after 2 tokens; further tokens would all pile onto rank 0
    entries = [(0, 0, 0, 50), (1, 1, 0, 2)]
    take, load, n = adaptive_chunked_prefill(12, 2, entries, min_tokens=2)
    assert take == [2, 2] and load == [3, 3] and n == 4
    # with the floor at the full budget the lonely tail is taken
    take, load, n = adaptive_chunked_prefill(12, 2, entries, min_tokens=12)
    assert take == [10, 2] and n == 12 and load == [55, 3]


def _second_style(budget, R, entries, min_tokens, init_load=None):
    """Independent re-implementation: run-length queues and a heap keyed (load, rank)."""
    queues = [[] for _ in range(R)]
    for e, (_q, rank, done, new) in enumerate(entries):
        if new > 0:
            queues[rank].append([e, done, new])
    load = [0] * R if init_load is None else list(init_load)
    heap = [(load[r], r) for r in range(R) if queues[r]]
    heapq.heapify(heap)
    order = []
    maxes, sums = [], []
    while len(order) < budget and heap:
        _, r = heapq.heappop(heap)
        head = queues[r][0]
        order.append(head[0])
        load[r] += head[1] + 1
        head[1] += 1
        head[2] -= 1
        if head[2] == 0:
            queues[r].pop(0)
        if queues[r]:
            heapq.heappush(heap, (load[r], r))
        maxes.append(max(load))
        sums.append(sum(load))
    if not order:
        return [0] * len(entries), load, 0
    lo = min(min_tokens, len(order))
    best = None
    for i in range(len(order)):
        if i + 1 < lo:
            continue
        if best is None:
            best = i
            continue
        a, b = maxes[i] * sums[best], maxes[best] * sums[i]   # ratio_i vs ratio_best (every sum >= 1)
        if a <= b:
            best = i
    take = [0] * len(entries)
    for e in order[:best + 1]:
        take[e] += 1
    # loads of the chosen prefix, recomputed from the counts alone
    out = [0] * R if init_load is None else list(init_load)
    for e, (_q, rank, done, _new) in enumerate(entries):
        out[rank] += take[e] * done + take[e] * (take[e] + 1) // 2
    return take, out, best + 1


@pytest.mark.parametrize("seed", range(40))
def test_against_a_second_implementation(seed):
    rng = np.random.default_rng(seed)
    R = int(rng.integers(1, 6))
    n = int(rng.integers(0, 9))
    entries = [(i, int(rng.integers(0, R)), int(rng.integers(0, 30)), int(rng.integers(0, 12))) for i in range(n)]
    budget = int(rng.integers(0, 40))
    min_tokens = int(rng.integers(0, budget + 2))
    init = None if seed % 3 else [int(x) for x in rng.integers(0, 20, size=R)]
    got = adaptive_chunked_prefill(budget, R, entries, min_tokens, init)
    want = _second_style(budget, R, entries, min_tokens, init)
    assert got[0] == want[0] and list(got[1]) == list(want[1]) and got[2] == want[2]


@pytest.mark.parametrize("seed", range(20))
def test_list_scheduling_invariant_of_the_full_budget_batch(seed):
    # When rank a took its last token it was the least loaded among the ranks that still had tokens,
    # so a's load before that token cannot exceed the final load of any rank that never ran dry.
    rng = np.random.default_rng(100 + seed)
    R = int(rng.integers(2, 7))
    entries = [(i, int(rng.integers(0, R)), int(rng.integers(0, 200)), int(rng.integers(1, 60))) for i in range(12)]
    budget = int(rng.integers(1, 200))
    take, load, n = adaptive_chunked_prefill(budget, R, entries, min_tokens=budget)
    assert n == min(budget, sum(e[3] for e in entries)) == sum(take)
    last_cost = [0] * R
    left = [0] * R
    took = [0] * R
    for (req, rank, done, new), t in zip(entries, take):
        left[rank] += new - t
        took[rank] += t
        if t:
            last_cost[rank] = done + t          # cost of the last token taken from this entry so far
    # FIFO within a rank: an entry is only touched when the ones before it are exhausted
    for r in range(R):
        seen_partial = False
        for (req, rank, done, new), t in zip(entries, take):
            if rank != r:
                continue
            assert not (seen_partial and t > 0)
            if t < new:
                seen_partial = True
    for a in range(R):
        if not took[a]:
            continue
        for b in range(R):
            if b != a and left[b] > 0:
                assert load[a] - last_cost[a] <= load[b]


def test_router_is_greedy_list_scheduling():
    rng = np.random.default_rng(7)
    R = 5
    pending = [0] * R
    jobs = [int(x) for x in rng.integers(1, 1000, size=200)]
    for j in jobs:
        before = list(pending)
        k = route_request(pending, j)
        assert before[k] == min(before) and k == before.index(min(before))
        assert max(pending) - min(pending) <= max(max(before) - min(before), j)
    assert sum(pending) == sum(jobs)
    assert max(pending) - min(pending) <= max(jobs)
    # same routing as the placement oracle's all-DP, one-head case (the DP-attention special case)
    _, dp, load = build_placement(jobs, [1] * len(jobs), R, 1)
    pending2 = [0] * R
    assert [route_request(pending2, j) for j in jobs] == dp.tolist() and pending2 == load.tolist()


def test_bad_arguments_raise():
    with pytest.raises(ValueError):
        adaptive_chunked_prefill(4, 2, [(0, 2, 0, 1)], 0)
    with pytest.raises(ValueError):
        adaptive_chunked_prefill(4, 0, [], 0)
    with pytest.raises(ValueError):
        route_request([], 1)
