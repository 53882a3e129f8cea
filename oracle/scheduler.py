"""Load-aware router and DP-aware adaptive chunked prefill (oracle side; test infrastructure).

Follows Section 3.1 of the paper, "Fine-grained Load-aware Router":

* Load-Aware DP-Rank Routing: an incoming request goes to the rank whose pending
  DP work, counted in token units, is smallest.  Ties go to the lowest rank.
* Algorithm 1 (DP-aware Adaptive Chunked Prefill): under a global token budget,
  take one token at a time from the head of the schedulable sequence of the
  least-loaded rank that still has one, add the token's cost to that rank's
  load, and remember every batch seen on the way (the candidate set H); return
  the best candidate.

The paper leaves three things open; the readings taken here are:

* cost(t).  The paper prices a chunk of N tokens after L processed ones at
  O(N^2 + N L + N).  A token that has p tokens of its request before it attends
  to p + 1 keys; summing p + 1 over positions L .. L+N-1 gives
  N L + N (N + 1) / 2, which has exactly that form.  So cost(t) = p + 1.
* choose_best_batch(H).  Every candidate is a prefix of the order in which the
  loop took tokens.  Among the prefixes that hold at least ``min_tokens`` tokens
  (or the whole schedule if it is shorter than that), the best is the one with the
  smallest ratio of the largest rank load to the mean rank load (the idle share at
  the synchronisation point); equal ratios go to the larger batch.
* The listed input {W_r} is never used by the printed loop, which starts every
  load at 0.  ``init_load=None`` is that printed start; giving ``init_load`` starts
  the loads at W_r instead (work already committed to the iteration on each rank).

Schedulable tokens are given as queue entries ``(req, rank, n_done, n_new)`` in
arrival order: the request's DP rank, how many of its tokens are already
processed, and how many wait.  S_r is the concatenation, in entry order, of the
waiting tokens of the entries routed to r.
"""
from fractions import Fraction


def token_cost(n_before: int) -> int:
    """Cost of one prefill token that has n_before tokens of its request before it."""
    return int(n_before) + 1


def route_request(pending, work: int) -> int:
    """Pick the rank with the least pending work (ties: lowest), add `work` there, return the rank."""
    if len(pending) < 1:
        raise ValueError("need at least one rank")
    if work < 0:
        raise ValueError("work must be non-negative")
    best = min(range(len(pending)), key=lambda k: (pending[k], k))
    pending[best] += int(work)
    return best


def adaptive_chunked_prefill(budget: int, n_ranks: int, entries, min_tokens: int, init_load=None):
    """Algorithm 1.  Returns (take [n_entries], load [R], n_tokens) of the chosen batch.

    take[e] is the number of leading waiting tokens of entry e that the batch holds.
    """
    R = int(n_ranks)
    if R < 1 or budget < 0 or min_tokens < 0:
        raise ValueError("bad arguments")
    for (_req, rank, n_done, n_new) in entries:
        if not 0 <= rank < R or n_done < 0 or n_new < 0:
            raise ValueError("bad queue entry")
    # S_r as explicit token lists: (entry index, tokens of the request before this one)
    S = {r: [] for r in range(R)}
    for e, (_req, rank, n_done, n_new) in enumerate(entries):
        for j in range(n_new):
            S[rank].append((e, n_done + j))
    L = [0] * R if init_load is None else [int(x) for x in init_load]
    if len(L) != R:
        raise ValueError("init_load must have one entry per rank")
    if any(x < 0 for x in L):
        raise ValueError("a rank's load is work in token units: it cannot be negative")
    B = []                     # tokens in the order taken
    H = []                     # candidates: (size, loads) after every token
    while len(B) < budget and any(S[r] for r in range(R)):
        r_star = min((r for r in range(R) if S[r]), key=lambda r: (L[r], r))
        t = S[r_star].pop(0)
        B.append(t)
        L[r_star] += token_cost(t[1])
        H.append((len(B), list(L)))
    take = [0] * len(entries)
    if not H:
        return take, L, 0
    floor_size = min(int(min_tokens), len(B))
    best = None
    for size, loads in H:
        if size < floor_size:
            continue
        total = sum(loads)
        ratio = Fraction(max(loads) * R, total) if total > 0 else Fraction(1)
        key = (ratio, -size)
        if best is None or key < best[0]:
            best = (key, size, loads)
    _, size, loads = best
    for e, _p in B[:size]:
        take[e] += 1
    return take, loads, size
