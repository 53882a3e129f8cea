"""Decode attention over a paged KVCache, plain definition in fp64 (oracle side).

One decode step attends a single new query token per request to all of that
request's cached keys (Section 2.1.1 of the paper describes the decode phase
and the KVCache).  For q-head j of request r, with KV head h = j // G:

    s_t = sm_scale * <q[r][j], K[r][h][t]>          t in [0, L_r)
    out = sum_t softmax(s)_t * V[r][h][t]
    lse = ln sum_t exp(s_t)

Stored bits are decoded exactly (bf16, or fp8 e4m3 times the slot's fp32
scale); everything after that is fp64.  Split-K partials and their merge are
written out as well so each library call has its own counterpart, but the
definition above, unsplit and unsharded, is the reference the rest is pinned to.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from .formats import bf16_bits_to_f64, e4m3_bytes_to_f64


def attend(q, K, V, sm_scale: float):
    """q [G][d], K [L][d], V [L][d] in fp64 -> (out [G][d], lse [G])."""
    s = sm_scale * (q @ K.T)
    m = s.max(axis=1, keepdims=True)
    p = np.exp(s - m)
    l = p.sum(axis=1, keepdims=True)
    out = (p @ V) / l
    lse = m[:, 0] + np.log(l[:, 0])
    return out, lse


def gather_pair_kv(kv: dict, pair_index: int, tok_begin: int, tok_end: int):
    """Collect tokens [tok_begin, tok_end) of one pair from the paged pool as fp64 rows."""
    T = kv["page_tokens"]
    first = tok_begin // T
    last = -(-tok_end // T)
    base = int(kv["page_indptr"][pair_index])
    slots = kv["page_ids"][base + first: base + last]
    lo = tok_begin - first * T
    hi = lo + (tok_end - tok_begin)
    d = kv["head_dim"]
    if kv["kv_dtype"] == "fp8":
        ks = kv["k_scale"][slots].astype(np.float64)[:, None, None]
        vs = kv["v_scale"][slots].astype(np.float64)[:, None, None]
        K = (e4m3_bytes_to_f64(kv["k_pool"][slots]) * ks).reshape(-1, d)
        V = (e4m3_bytes_to_f64(kv["v_pool"][slots]) * vs).reshape(-1, d)
    else:
        K = bf16_bits_to_f64(kv["k_pool"][slots]).reshape(-1, d)
        V = bf16_bits_to_f64(kv["v_pool"][slots]).reshape(-1, d)
    return K[lo:hi], V[lo:hi]


def _run(fn, n, workers):
    """Run fn(0..n-1), optionally on `workers` threads (one pair or item each).  While several
    workers run, the BLAS behind numpy is held to one thread apiece so they do not fight."""
    if workers and workers > 1 and n > 1:
        try:
            from threadpoolctl import threadpool_limits
        except ImportError:                      # pragma: no cover
            from contextlib import nullcontext as threadpool_limits
        with threadpool_limits(1), ThreadPoolExecutor(max_workers=workers) as ex:
            return list(ex.map(fn, range(n)))
    return [fn(i) for i in range(n)]


def decode_attention_items(q_bits, kv: dict, items, group: int, sm_scale: float, workers: int = 1):
    """Per work item: attention over the item's token range only, normalised
    within the range.  Returns (part_o [n_items*G][d], part_lse [n_items*G])."""
    d = kv["head_dim"]
    qf = q_bits.reshape(-1, d)
    n = len(items)
    part_o = np.empty((n * group, d), dtype=np.float64)
    part_lse = np.empty(n * group, dtype=np.float64)

    def one(i):
        it = items[i]
        q = bf16_bits_to_f64(qf[it[6]: it[6] + group])
        K, V = gather_pair_kv(kv, int(it[4]), int(it[2]), int(it[3]))
        o, l = attend(q, K, V, sm_scale)
        part_o[it[7]: it[7] + group] = o
        part_lse[it[7]: it[7] + group] = l

    _run(one, n, workers)
    return part_o, part_lse


def merge_lse(part_o, part_lse, chunk_indptr, group: int):
    """Combine a pair's chunk partials: lse = ln sum_c exp(lse_c),
    out = sum_c exp(lse_c - lse) * o_c.  Returns (out [n_pairs*G][d], lse)."""
    n_pairs = len(chunk_indptr) - 1
    d = part_o.shape[1]
    out = np.empty((n_pairs * group, d), dtype=np.float64)
    lse = np.empty(n_pairs * group, dtype=np.float64)
    for p in range(n_pairs):
        c0, c1 = int(chunk_indptr[p]), int(chunk_indptr[p + 1])
        for g in range(group):
            rows = [c * group + g for c in range(c0, c1)]
            lc = part_lse[rows]
            M = lc.max()
            tot = M + np.log(np.exp(lc - M).sum())
            w = np.exp(lc - tot)
            out[p * group + g] = (w[:, None] * part_o[rows]).sum(axis=0)
            lse[p * group + g] = tot
    return out, lse


def decode_attention_pairs(q_bits, kv: dict, pairs, n_q_heads: int, group: int, sm_scale: float,
                           workers: int = 1):
    """Unsplit attention for each (request, KV head) pair of a rank's list.
    Rows [p*G, p*G+G) belong to pair p.  Returns (out, lse) in fp64."""
    d = kv["head_dim"]
    qf = q_bits.reshape(-1, d)
    n = len(pairs)
    out = np.empty((n * group, d), dtype=np.float64)
    lse = np.empty(n * group, dtype=np.float64)

    def one(p):
        r, h, L = int(pairs[p][0]), int(pairs[p][1]), int(pairs[p][2])
        row = r * n_q_heads + h * group
        q = bf16_bits_to_f64(qf[row: row + group])
        K, V = gather_pair_kv(kv, p, 0, L)
        o, l = attend(q, K, V, sm_scale)
        out[p * group: (p + 1) * group] = o
        lse[p * group: (p + 1) * group] = l

    _run(one, n, workers)
    return out, lse


def unsharded_attention(q_bits, kv_all: dict, ctx_len, n_q_heads: int, n_kv_heads: int,
                        sm_scale: float):
    """Attention for every (request, q-head) with no ranks at all.  ``kv_all``
    holds every (request, head) pair in request-major, head-minor order.
    Returns (out [B][H_q][d], lse [B][H_q])."""
    B = len(ctx_len)
    G = n_q_heads // n_kv_heads
    d = kv_all["head_dim"]
    out = np.empty((B, n_q_heads, d), dtype=np.float64)
    lse = np.empty((B, n_q_heads), dtype=np.float64)
    qv = q_bits.reshape(B, n_q_heads, d)
    for r in range(B):
        for h in range(n_kv_heads):
            K, V = gather_pair_kv(kv_all, r * n_kv_heads + h, 0, int(ctx_len[r]))
            q = bf16_bits_to_f64(qv[r, h * G:(h + 1) * G])
            o, l = attend(q, K, V, sm_scale)
            out[r, h * G:(h + 1) * G] = o
            lse[r, h * G:(h + 1) * G] = l
    return out, lse
