"""One rank's ragged (request, KV head, chunk) work list (oracle side).

The paper's hybrid attention (Section 3.1) leaves each rank with an irregular
set of (request, head) pairs: a cyclic subset of heads for tensor-parallel
requests and every head of the data-parallel requests routed to it.  This list
is that set written down for one kernel launch, with long contexts cut into
chunks of ``chunk_tokens`` (split-K) and a longest-first launch order.

Conventions (they are the interface, so both sides state them):
pairs are numbered in (request, head) ascending order; a pair's chunks are
consecutive items; item i writes partial rows [i*G, i*G+G); the query rows of a
pair start at request*H_q + head*G (consecutive q-heads share a KV head); pair
p's final rows are [p*G, p*G+G); ``sched`` lists item indices by decreasing
token count, equal counts in increasing item index.
"""
import numpy as np

ITEM_FIELDS = ("req", "kv_head", "tok_begin", "tok_end", "pair", "chunk", "q_row", "part_row")
PAIR_FIELDS = ("req", "kv_head", "ctx_len", "n_chunks")


def build_worklist(ctx_len, owner, rank: int, chunk_tokens: int, n_q_heads: int, n_kv_heads: int,
                   page_tokens: int = 16):
    """Return (items [n_items][8] int32, pairs [n_pairs][4] int32, sched int32,
    chunk_indptr int64 [n_pairs+1]) for ``rank``."""
    H = int(n_kv_heads)
    if n_q_heads % H:
        raise ValueError("q heads must be a multiple of KV heads")
    G = n_q_heads // H
    C = int(chunk_tokens)
    if C < 0 or C % page_tokens:
        raise ValueError("chunk must be a whole number of pages")
    items, pairs, indptr = [], [], [0]
    for r in range(len(ctx_len)):
        L = int(ctx_len[r])
        for h in range(H):
            if int(owner[r][h]) != rank:
                continue
            p = len(pairs)
            n_chunks = 1 if C == 0 else -(-L // C)
            pairs.append((r, h, L, n_chunks))
            for c in range(n_chunks):
                begin = 0 if C == 0 else c * C
                end = L if C == 0 else min(L, (c + 1) * C)
                i = len(items)
                items.append((r, h, begin, end, p, c, r * n_q_heads + h * G, i * G))
            indptr.append(len(items))
    items = np.array(items, dtype=np.int32).reshape(-1, 8)
    pairs = np.array(pairs, dtype=np.int32).reshape(-1, 4)
    length = items[:, 3] - items[:, 2]
    sched = sorted(range(len(items)), key=lambda i: (-int(length[i]), i))
    return items, pairs, np.array(sched, dtype=np.int32), np.array(indptr, dtype=np.int64)


def choose_chunk_tokens(ctx_len, owner, rank: int, max_chunk: int, min_chunk: int, n_slots: int,
                        n_kv_heads: int, page_tokens: int = 16):
    """The split-K chunk for ``rank``'s share: four thirds of a slot's fair share of the tokens.  With T the cached
    tokens of the rank's (request, head) pairs, all told, and ``n_slots`` the workgroups the GPU should be running at a
    time, the chunk is ceil(4 T / (3 n_slots)) rounded up to whole pages and held within [min_chunk, max_chunk].
    -> (chunk, n_items).  The chunk is this build's device for long contexts, not the paper's: the ragged share of
    Section 3.1 can be a handful of very long contexts, which would run as long as the longest takes; an item about as
    long as a slot's share of the whole keeps any from sticking out without cutting finer than that needs.  The item
    count is that of ``build_worklist`` with the same chunk."""
    if min_chunk < page_tokens or min_chunk % page_tokens or max_chunk < min_chunk or max_chunk % page_tokens:
        raise ValueError("chunk bounds must be whole pages, min <= max")
    if n_slots < 1:
        raise ValueError("n_slots < 1")
    lens = [int(ctx_len[r]) for r in range(len(ctx_len)) for h in range(n_kv_heads) if int(owner[r][h]) == rank]
    target = -(-4 * sum(lens) // (3 * int(n_slots)))
    C = min(max(-(-target // page_tokens) * page_tokens, int(min_chunk)), int(max_chunk))
    return C, sum(-(-L // C) for L in lens)


def build_worklist_units(ctx_len, owner, rank: int, n_units: int, n_q_heads: int, n_kv_heads: int,
                         page_tokens: int = 16):
    """The same ragged share (Section 3.1) cut for a launch without stragglers: the rank's pairs, in
    (request, head) order, are laid end to end as one stream of KVCache pages, and the stream is cut
    into ``n_units`` runs of equal length (to within one page), one per resident workgroup.  Where a
    run crosses from one pair into the next it is cut there too, so an item is still tokens
    [tok_begin, tok_end) of one pair, and a pair that lies inside one run is a single item.

    With P pages in the stream and U = min(n_units, P) units, unit u holds stream pages
    [floor(u*P/U), floor((u+1)*P/U)).  Items are numbered in stream order, so the items of a unit
    and the items of a pair are both consecutive.  Returns (items [n_items][8], pairs [n_pairs][4],
    unit_indptr int64 [U+1], chunk_indptr int64 [n_pairs+1]); item and pair fields as in
    ``build_worklist`` (chunk = the item's index within its pair, n_chunks = the pair's item count).
    The cut is this build's device, not the paper's.
    """
    H = int(n_kv_heads)
    if n_q_heads % H:
        raise ValueError("q heads must be a multiple of KV heads")
    if n_units < 1:
        raise ValueError("at least one unit")
    G = n_q_heads // H
    T = int(page_tokens)
    mine = [(r, h, int(ctx_len[r])) for r in range(len(ctx_len)) for h in range(H) if int(owner[r][h]) == rank]
    n_pages = [-(-L // T) for (_, _, L) in mine]
    P = sum(n_pages)
    U = min(int(n_units), P)
    cuts = [(u * P) // U for u in range(U + 1)] if U else [0]
    items, pairs, chunk_indptr, unit_indptr = [], [], [0], [0]
    start = 0                      # stream position of the current pair's first page
    u = 0                          # unit that holds the next page to place
    for p, (r, h, L) in enumerate(mine):
        done = 0                   # pages of this pair already placed
        c = 0
        while done < n_pages[p]:
            while start + done >= cuts[u + 1]:          # the stream position has left unit u
                u += 1
                unit_indptr.append(len(items))
            take = min(n_pages[p] - done, cuts[u + 1] - (start + done))
            i = len(items)
            items.append((r, h, done * T, min(L, (done + take) * T), p, c, r * n_q_heads + h * G, i * G))
            done += take
            c += 1
        pairs.append((r, h, L, c))
        chunk_indptr.append(len(items))
        start += n_pages[p]
    while len(unit_indptr) < U + 1:
        unit_indptr.append(len(items))
    return (np.array(items, dtype=np.int32).reshape(-1, 8), np.array(pairs, dtype=np.int32).reshape(-1, 4),
            np.array(unit_indptr, dtype=np.int64), np.array(chunk_indptr, dtype=np.int64))


RECORD_WORDS = 16       # a launch record is 16 int32 words (64 bytes)


def build_launch_records(items, order, chunk_indptr, page_indptr, page_ids, group: int, direct_rows: bool = True,
                         page_tokens: int = 16):
    """A work list written out the way a kernel wants to find it: one 64-byte record per item, in launch
    order, with everything the item's first memory requests depend on already looked up (this build's
    device; the paper describes no kernel).  ``order`` lists item indices in launch order (None: index
    order).  Record k, for item i = order[k], as 16 int32 words:

        0-1   first_page  index into page_ids of the item's first page (int64, low word first):
                          page_indptr[pair] + tok_begin / page_tokens
        2     n_tok       tok_end - tok_begin
        3     q_row       as in the item
        4     row         part_row; or, with ``direct_rows`` and a pair that is this one item,
                          -(pair*group) - 1: the item's rows are the pair's final rows
        5     n_chunks    chunks (items) of the item's pair
        6-13  page_ids[first_page + j] for j = 0..7 (0 beyond the item's last page)
        14    pair
        15    pair_row    first partial row of the pair's first chunk, chunk_indptr[pair] * group (what a
                          kernel that merges a pair itself needs to find the other chunks' rows)

    An item must sit where the merge will look for it: part_row = (chunk_indptr[pair] + chunk) * group.
    """
    n = len(items)
    order = range(n) if order is None else [int(i) for i in order]
    rec = np.zeros((len(order), RECORD_WORDS), dtype=np.int32)
    for k, i in enumerate(order):
        r, h, tb, te, pair, c, q_row, part_row = (int(x) for x in items[i])
        first_page = int(page_indptr[pair]) + tb // page_tokens
        n_pages = -(-(te - tb) // page_tokens)
        rec[k, 0:2] = np.array([first_page], dtype=np.int64).view(np.int32)
        rec[k, 2] = te - tb
        rec[k, 3] = q_row
        c0 = int(chunk_indptr[pair])
        n_chunks = int(chunk_indptr[pair + 1]) - c0
        if not 0 <= c < n_chunks or part_row != (c0 + c) * group:
            raise ValueError("item is not at row (chunk_indptr[pair] + chunk) * group")
        rec[k, 4] = -(pair * group) - 1 if (direct_rows and n_chunks == 1) else part_row
        rec[k, 5] = n_chunks
        rec[k, 14] = pair
        rec[k, 15] = c0 * group
        for j in range(min(8, n_pages)):
            rec[k, 6 + j] = int(page_ids[first_page + j])
    return rec
