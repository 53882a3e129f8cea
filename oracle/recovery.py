"""Recovery planning after a GPU fault (oracle side; test infrastructure).

Follows Section 3.2 of the paper, "Lightning Recovery", as plans (which data moves
where), not as transfers:

* Proactive KVCache Backup: after a fault every surviving GPU keeps the KVCache it
  holds and reloads from the host copy only the part it newly needs.
  ``plan_kv_reload`` is that statement for any pair of placements: a (request, KV
  head) slice is reused when its new owner is its old owner and reloaded by the new
  owner otherwise.
* ``replace_failed_gpu`` builds the placement that moves nothing but the lost data,
  in the way hybrid attention absorbs a lost worker (Section 3.1 with Fig. 5 of
  Section 3.2): slices on surviving GPUs stay; the lost slices of a request become
  data-parallel work on that request's DP rank; a request without a surviving DP rank
  is routed to the GPU with the least pending DP work (ties: lowest id).  It applies
  when the per-worker share of tensor-parallel heads does not grow,
  floor(H/(R-1)) == floor(H/R); otherwise a fresh placement plus ``plan_kv_reload``
  is the plan.
* On-Demand Weight Recovery: FFN weights are cut into shards along the intermediate
  (reduction) dimension, whose order is free, so survivors keep their shards and the
  lost ones are dealt out one at a time to whichever survivor holds the fewest (ties:
  lowest id).  ``plan_ffn_reload`` returns the new owner of every shard.

GPU ids are physical: a placement over R-1 survivors is given in the ids of the
GPUs that survive, so "same owner" means "same device".  Which GPUs live is a mask
over the ids, so a second fault is planned with the first GPU still marked dead.
"""
import numpy as np


def _live(alive):
    live = [g for g, a in enumerate(alive) if a]
    if not live:
        raise ValueError("no GPU survives")
    return live


def plan_kv_reload(ctx_len, old_owner, new_owner, alive):
    """-> (reload [n_gpus], reuse [n_gpus]) in KV tokens x KV heads per GPU, for one layer."""
    old_owner = np.asarray(old_owner)
    new_owner = np.asarray(new_owner)
    if old_owner.shape != new_owner.shape or old_owner.ndim != 2 or old_owner.shape[0] != len(ctx_len):
        raise ValueError("owner maps must both be [n_req][n_kv_heads]")
    n_gpus = len(alive)
    _live(alive)
    reload = [0] * n_gpus
    reuse = [0] * n_gpus
    for r in range(old_owner.shape[0]):
        L = int(ctx_len[r])
        if L < 1:
            raise ValueError("a request holds at least one token")
        for h in range(old_owner.shape[1]):
            a, b = int(old_owner[r, h]), int(new_owner[r, h])
            if not (0 <= a < n_gpus and 0 <= b < n_gpus) or not alive[b]:
                raise ValueError("owner outside the GPUs, or new owner is a dead GPU")
            if a == b:
                reuse[b] += L
            else:
                reload[b] += L
    return np.array(reload, dtype=np.int64), np.array(reuse, dtype=np.int64)


def replace_failed_gpu(ctx_len, old_owner, old_dp_rank, alive, dp_load=None):
    """-> (new_owner [B][H], new_dp_rank [B], dp_load [n_gpus]) moving only the lost slices."""
    old_owner = np.asarray(old_owner)
    B, H = old_owner.shape
    n_gpus = len(alive)
    survivors = _live(alive)
    load = [0] * n_gpus if dp_load is None else [int(x) for x in dp_load]
    new_owner = old_owner.astype(np.int32).copy()
    new_dp = np.asarray(old_dp_rank, dtype=np.int32).copy()
    for r in range(B):
        lost = [h for h in range(H) if not alive[old_owner[r, h]]]
        if not lost:
            continue
        d = int(new_dp[r])
        if d < 0 or not alive[d]:
            d = min(survivors, key=lambda g: (load[g], g))
            new_dp[r] = d
        for h in lost:
            new_owner[r, h] = d
        load[d] += len(lost) * int(ctx_len[r])
    return new_owner, new_dp, np.array(load, dtype=np.int64)


def plan_ffn_reload(shard_owner, alive):
    """-> (new_owner [n_shards], n_load [n_gpus]): survivors keep their shards, lost ones are dealt out."""
    owner = [int(x) for x in shard_owner]
    n_gpus = len(alive)
    survivors = _live(alive)
    if any(not 0 <= g < n_gpus for g in owner):
        raise ValueError("shard owner outside [0, n_gpus)")
    count = [sum(1 for g in owner if g == k) for k in range(n_gpus)]
    n_load = [0] * n_gpus
    new_owner = list(owner)
    for s, g in enumerate(owner):
        if alive[g]:
            continue
        k = min(survivors, key=lambda x: (count[x], x))
        new_owner[s] = k
        count[k] += 1
        n_load[k] += 1
    return np.array(new_owner, dtype=np.int32), np.array(n_load, dtype=np.int32)
