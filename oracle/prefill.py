"""Chunked-prefill attention over the paged KVCache, plain definition in fp64 (oracle side).

Section 3.1 of the paper ("Fine-Grained Chunked Prefill") forms prefill batches that hold
chunks of several requests: N new tokens of a request behind L tokens already processed.
The prefill phase (Section 2.1.1) lets every prompt token attend to the tokens up to and
including itself.  So new token i of a chunk (position L + i) of request r, for q-head j with
KV head h = j // G, computes

    s_t = sm_scale * <q[i][j], K[r][h][t]>        t in [0, L + i]
    out = sum_t softmax(s)_t * V[r][h][t]
    lse = ln sum_t exp(s_t)

which is decode attention of that token over the first L + i + 1 cached tokens; the cache
already holds the chunk's own K and V.  Test infrastructure only.

Work list of one rank: (request, KV head) pairs the rank owns whose request has new tokens,
in ascending (request, head); each pair's new tokens are cut into tiles of ``tile_tokens``
query tokens (the last may be shorter), and the keys a tile sees, [0, n_done + q_end), into
split-K chunks of ``kv_chunk_tokens`` keys (0 = one chunk), one item each.  An item's partial
result for a query row is attention over the item's keys that the row may see (none: out = 0,
lse = -inf); the chunk partials of a tile merge exactly as in the decode path.  Q is the ragged
concatenation of the batch's new tokens in request order.  Partial rows: item i owns rows
[i*T, (i+1)*T) with T = tile_tokens*G, token-major and q-head-minor within the tile.  Final
rows: tile k owns rows [k*T, (k+1)*T), so a pair's rows are contiguous from
out_indptr[pair] (only a pair's last tile can be short; the unused rows after it are padding).
"""
import numpy as np

from .attention import attend, gather_pair_kv, _run
from .formats import bf16_bits_to_f64

PREFILL_ITEM_FIELDS = ("pair", "q_begin", "q_end", "n_done", "kv_begin", "kv_end", "q_row", "part_row")
PREFILL_PAIR_FIELDS = ("req", "kv_head", "n_done", "n_new")


def build_prefill_worklist(n_done, n_new, owner, rank: int, n_q_heads: int, tile_tokens: int,
                           kv_chunk_tokens: int = 0):
    """-> (items [n][8] int32, pairs [m][4] int32, sched [n] int32, chunk_indptr [n_tiles+1] int64,
    out_indptr [m+1] int64)."""
    owner = np.asarray(owner)
    B, H = owner.shape
    if n_q_heads % H or tile_tokens < 1 or kv_chunk_tokens < 0:
        raise ValueError("bad head counts, tile size or chunk size")
    G = n_q_heads // H
    T = tile_tokens * G
    q_indptr = [0]
    for r in range(B):
        if n_done[r] < 0 or n_new[r] < 0:
            raise ValueError("negative token count")
        q_indptr.append(q_indptr[-1] + int(n_new[r]))
    items, pairs, chunk_indptr, out_indptr = [], [], [0], [0]
    for r in range(B):
        N, L = int(n_new[r]), int(n_done[r])
        if N == 0:
            continue
        for h in range(H):
            if owner[r, h] != rank:
                continue
            p = len(pairs)
            pairs.append((r, h, L, N))
            for b in range(0, N, tile_tokens):
                e = min(N, b + tile_tokens)
                keys = L + e
                C = kv_chunk_tokens if kv_chunk_tokens else keys
                for k0 in range(0, keys, C):
                    items.append((p, b, e, L, k0, min(keys, k0 + C), (q_indptr[r] + b) * n_q_heads + h * G,
                                  len(items) * T))
                chunk_indptr.append(len(items))
            out_indptr.append((len(chunk_indptr) - 1) * T)
    # longest first: an item streams the keys of its chunk
    order = sorted(range(len(items)), key=lambda i: (-(items[i][5] - items[i][4]), i))
    return (np.array(items, dtype=np.int32).reshape(-1, 8), np.array(pairs, dtype=np.int32).reshape(-1, 4),
            np.array(order, dtype=np.int32), np.array(chunk_indptr, dtype=np.int64),
            np.array(out_indptr, dtype=np.int64))


def choose_prefill_chunk(n_done, n_new, owner, rank: int, n_q_heads: int, tile_tokens: int, max_chunk: int,
                         min_chunk: int, n_slots: int):
    """The split-K chunk of the keys for ``rank``'s batch: four thirds of a slot's fair share of the work.  With T the
    keys that the rank's tiles see, all told, and ``n_slots`` the workgroups the GPU runs at a time, the chunk is
    ceil(4 T / (3 n_slots)) rounded up to a multiple of 32 keys and held within [min_chunk, max_chunk].
    -> (chunk, n_items with it).  Split-K is this build's device, not the paper's: a batch with few long contexts
    (Section 3.1's fine-grained chunked prefill forms such batches when little is waiting) would otherwise run as long as
    its longest tile takes, while a large batch needs no cut at all; an item about as long as a slot's share of the
    whole keeps the longest item from sticking out without cutting finer than that needs."""
    if min_chunk < 32 or min_chunk % 32 or max_chunk < min_chunk or max_chunk % 32:
        raise ValueError("chunk bounds must be multiples of 32, min <= max")
    if n_slots < 1:
        raise ValueError("n_slots < 1")
    uncut = build_prefill_worklist(n_done, n_new, owner, rank, n_q_heads, tile_tokens, 0)[0]
    total = sum(int(it[5]) - int(it[4]) for it in uncut)         # one item per tile: kv_end - kv_begin
    target = -(-4 * total // (3 * int(n_slots)))
    chunk = min(max(-(-target // 32) * 32, min_chunk), max_chunk)
    return chunk, len(build_prefill_worklist(n_done, n_new, owner, rank, n_q_heads, tile_tokens, chunk)[0])


def prefill_attention_items(q_bits, kv: dict, items, pairs, n_q_heads: int, group: int, tile_tokens: int,
                            sm_scale: float):
    """Partial result of every item: rows [i*T, (i+1)*T); rows of tokens a short tile does not have
    stay NaN.  A row that sees none of the item's keys gets out = 0, lse = -inf."""
    d = kv["head_dim"]
    T = tile_tokens * group
    part_o = np.full((len(items) * T, d), np.nan, dtype=np.float64)
    part_lse = np.full(len(items) * T, np.nan, dtype=np.float64)
    qf = q_bits.reshape(-1, d)
    for i in range(len(items)):
        p, b, e, L, k0, k1, q_row, part_row = (int(x) for x in items[i])
        K, V = gather_pair_kv(kv, p, k0, k1)
        for j in range(e - b):
            vis = min(k1, L + b + j + 1) - k0          # keys of this chunk the token may see
            row = part_row + j * group
            if vis <= 0:
                part_o[row:row + group] = 0.0
                part_lse[row:row + group] = -np.inf
                continue
            q = bf16_bits_to_f64(qf[q_row + j * n_q_heads: q_row + j * n_q_heads + group])
            o, l = attend(q, K[:vis], V[:vis], sm_scale)
            part_o[row:row + group] = o
            part_lse[row:row + group] = l
    return part_o, part_lse


def prefill_attention_pairs(q_bits, q_indptr, kv: dict, pairs, n_q_heads: int, group: int, sm_scale: float,
                            workers: int = 1, only_pairs=None, out_indptr=None):
    """Causal attention of every new token of every pair, unsplit.  q_bits [T][H_q][d] bf16 bits,
    q_indptr [B+1].  Returns (out [rows][d], lse [rows]) in fp64; pair p's rows start at
    out_indptr[p], token-major then q-head of the group; padding rows stay NaN."""
    d = kv["head_dim"]
    qv = q_bits.reshape(-1, n_q_heads, d)
    if out_indptr is None:                      # dense rows; pass the work list's out_indptr for its padded rows
        out_indptr = np.zeros(len(pairs) + 1, dtype=np.int64)
        for p in range(len(pairs)):
            out_indptr[p + 1] = out_indptr[p] + int(pairs[p][3]) * group
    out = np.full((int(out_indptr[-1]), d), np.nan, dtype=np.float64)
    lse = np.full(int(out_indptr[-1]), np.nan, dtype=np.float64)
    todo = list(range(len(pairs))) if only_pairs is None else list(only_pairs)

    def one(k):
        p = todo[k]
        r, h, L, N = (int(x) for x in pairs[p])
        K, V = gather_pair_kv(kv, p, 0, L + N)
        for i in range(N):
            q = bf16_bits_to_f64(qv[int(q_indptr[r]) + i, h * group:(h + 1) * group])
            o, l = attend(q, K[:L + i + 1], V[:L + i + 1], sm_scale)
            row = int(out_indptr[p]) + i * group
            out[row:row + group] = o
            lse[row:row + group] = l

    _run(one, len(todo), workers)
    return out, lse


def prefill_attention_row(q_bits, q_indptr, kv: dict, pairs, n_q_heads: int, group: int, sm_scale: float,
                          pair: int, tok: int):
    """One new token of one pair: (out [G][d], lse [G]).  For sampled checks at full size."""
    d = kv["head_dim"]
    r, h, L, N = (int(x) for x in pairs[pair])
    if not 0 <= tok < N:
        raise ValueError("token outside the chunk")
    K, V = gather_pair_kv(kv, pair, 0, L + tok + 1)
    q = bf16_bits_to_f64(q_bits.reshape(-1, n_q_heads, d)[int(q_indptr[r]) + tok, h * group:(h + 1) * group])
    return attend(q, K, V, sm_scale)
