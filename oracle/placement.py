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
