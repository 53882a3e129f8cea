"""Head -> rank placement for one decode batch (oracle side).

Follows Section 3.1 of the paper:

* Cyclic placement: KV heads, with their KVCache blocks, go round the ranks
  cyclically and the starting rank rotates.  The paper rotates layer by layer;
  the batches measured here rotate by request index.  Both are the one formula
  ``owner = (h + rot[r] + layer) mod R``.
* Hybrid attention, taken at request granularity: a request is either
  tensor-parallel (its heads spread cyclically) or data-parallel (all of its
  heads on one rank).
* Load-aware DP-rank routing: each incoming request goes to the rank with the
  smallest running load; ties go to the lowest rank; requests arrive in index
  order.  The load unit is KV tokens x KV heads and, as the measured batches
  state it, counts everything placed so far, tensor-parallel shares included.
"""
import numpy as np

MODE_TP = 0
MODE_DP = 1


def build_placement(ctx_len, mode, n_ranks: int, n_kv_heads: int, rot=None, layer: int = 0,
                    rank_load=None):
    """Return (owner [B][H_kv] int32, dp_rank [B] int32, rank_load [R] int64)."""
    B = len(ctx_len)
    R, H = int(n_ranks), int(n_kv_heads)
    if R < 1 or H < 1:
        raise ValueError("need at least one rank and one KV head")
    load = [0] * R if rank_load is None else [int(x) for x in rank_load]
    if len(load) != R:
        raise ValueError("rank_load must have one entry per rank")
    owner = np.empty((B, H), dtype=np.int32)
    dp_rank = np.empty(B, dtype=np.int32)
    for r in range(B):
        L = int(ctx_len[r])
        if L < 1:
            raise ValueError("a decode request holds at least its own token")
        m = int(mode[r])
        if m == MODE_TP:
            start = (r if rot is None else int(rot[r])) + int(layer)
            for h in range(H):
                k = (h + start) % R
                owner[r, h] = k
                load[k] += L
            dp_rank[r] = -1
        elif m == MODE_DP:
            best = 0
            for k in range(1, R):
                if load[k] < load[best]:       # strict: ties keep the lowest rank
                    best = k
            owner[r, :] = best
            dp_rank[r] = best
            load[best] += H * L
        else:
            raise ValueError("mode must be 0 (TP) or 1 (DP)")
    return owner, dp_rank, np.array(load, dtype=np.int64)


def build_placement_hybrid_heads(ctx_len, n_ranks: int, n_kv_heads: int, layer: int = 0, route=None,
                                 rank_load=None, dp_load=None):
    """Hybrid attention as the paper states it (Section 3.1, Fig. 3), at head granularity.

    Every tensor-parallel worker gets the same number of heads, floor(H/R); those
    R*floor(H/R) heads are placed cyclically, the start rotating with the layer
    (Cyclic Placement).  The remaining H mod R heads are replicated and run
    data-parallel: all of a request's leftover heads go to the request's DP rank.
    The DP rank is ``route[r]`` when given, else the rank with the least pending DP
    work in token units (Load-Aware DP-Rank Routing; DP work only, ties to the
    lowest rank, requests in index order).

    Returns (owner [B][H], dp_rank [B] (-1 when no head is left over),
    rank_load [R] total KV tokens x heads, dp_load [R] the DP share of it).
    """
    B = len(ctx_len)
    R, H = int(n_ranks), int(n_kv_heads)
    if R < 1 or H < 1:
        raise ValueError("need at least one rank and one KV head")
    per_rank = H // R
    n_tp = per_rank * R
    n_dp = H - n_tp
    load = [0] * R if rank_load is None else [int(x) for x in rank_load]
    dload = [0] * R if dp_load is None else [int(x) for x in dp_load]
    owner = np.empty((B, H), dtype=np.int32)
    dp_rank = np.empty(B, dtype=np.int32)
    for r in range(B):
        L = int(ctx_len[r])
        if L < 1:
            raise ValueError("a decode request holds at least its own token")
        for h in range(n_tp):
            k = (h + int(layer)) % R
            owner[r, h] = k
            load[k] += L
        if n_dp == 0:
            dp_rank[r] = -1
            continue
        if route is not None:
            best = int(route[r])
            if not 0 <= best < R:
                raise ValueError("route outside [0, R)")
        else:
            best = 0
            for k in range(1, R):
                if dload[k] < dload[best]:
                    best = k
        owner[r, n_tp:] = best
        dp_rank[r] = best
        load[best] += n_dp * L
        dload[best] += n_dp * L
    return owner, dp_rank, np.array(load, dtype=np.int64), np.array(dload, dtype=np.int64)
