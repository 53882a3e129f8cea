"""Pins for the oracle's per-rank work list."""
import numpy as np
import pytest

from oracle import build_placement, build_worklist, choose_chunk_tokens


def _case(seed, B, R, H, frac_dp, lo=1, hi=9000):
    rng = np.random.default_rng(seed)
    ctx = rng.integers(lo, hi, size=B).astype(np.int32)
    mode = (rng.random(B) < frac_dp).astype(np.uint8)
    owner, dp, load = build_placement(ctx, mode, R, H)
    return ctx, owner, load


@pytest.mark.parametrize("chunk", [0, 16, 256, 2048])
def test_items_tile_every_pair_and_sum_to_rank_load(chunk):
    R, H, Hq = 6, 8, 64
    ctx, owner, load = _case(2, 120, R, H, 0.2)
    seen = set()
    for k in range(R):
        items, pairs, sched, indptr = build_worklist(ctx, owner, k, chunk, Hq, H)
        assert int((items[:, 3] - items[:, 2]).sum()) == load[k]
        assert indptr[0] == 0 and indptr[-1] == len(items) and len(indptr) == len(pairs) + 1
        for p, (r, h, L, n_chunks) in enumerate(pairs):
            assert owner[r, h] == k and L == ctx[r]
            assert (r, h) not in seen
            seen.add((r, h))
            its = items[indptr[p]:indptr[p + 1]]
            assert len(its) == n_chunks == (1 if chunk == 0 else -(-L // chunk))
            assert its[0, 2] == 0 and its[-1, 3] == L
            assert (its[1:, 2] == its[:-1, 3]).all()                  # no gap, no overlap
            if chunk:
                assert ((its[:-1, 3] - its[:-1, 2]) == chunk).all()   # all but the last are full
                assert 0 < its[-1, 3] - its[-1, 2] <= chunk
            assert (its[:, 0] == r).all() and (its[:, 1] == h).all() and (its[:, 4] == p).all()
            assert its[:, 5].tolist() == list(range(n_chunks))
            assert (its[:, 6] == r * Hq + h * (Hq // H)).all()
        assert items[:, 7].tolist() == [i * (Hq // H) for i in range(len(items))]
        # pairs ascend in (request, head)
        keys = [(int(a), int(b)) for a, b in pairs[:, :2]]
        assert keys == sorted(keys)
        # sched: a permutation, longest first, equal lengths by index
        assert sorted(sched.tolist()) == list(range(len(items)))
        ln = (items[:, 3] - items[:, 2])[sched]
        assert (ln[1:] <= ln[:-1]).all()
        same = ln[1:] == ln[:-1]
        assert (sched[1:][same] > sched[:-1][same]).all()
    assert len(seen) == len(ctx) * H          # union over ranks covers every (r, h) once


def test_tiny_list_by_hand():
    # 2 ranks, 2 KV heads, 4 q-heads (G=2). r0 TP L=40, r1 DP L=20 -> least load.
    ctx = np.array([40, 20], dtype=np.int32)
    owner, dp, load = build_placement(ctx, [0, 1], 2, 2)
    assert owner.tolist() == [[0, 1], [0, 0]] and load.tolist() == [80, 40]
    items, pairs, sched, indptr = build_worklist(ctx, owner, 0, 16, 4, 2)
    assert pairs.tolist() == [[0, 0, 40, 3], [1, 0, 20, 2], [1, 1, 20, 2]]
    assert items.tolist() == [
        [0, 0, 0, 16, 0, 0, 0, 0], [0, 0, 16, 32, 0, 1, 0, 2], [0, 0, 32, 40, 0, 2, 0, 4],
        [1, 0, 0, 16, 1, 0, 4, 6], [1, 0, 16, 20, 1, 1, 4, 8],
        [1, 1, 0, 16, 2, 0, 6, 10], [1, 1, 16, 20, 2, 1, 6, 12]]
    assert indptr.tolist() == [0, 3, 5, 7]
    assert sched.tolist() == [0, 1, 3, 5, 2, 4, 6]
    items1, pairs1, _, _ = build_worklist(ctx, owner, 1, 0, 4, 2)
    assert pairs1.tolist() == [[0, 1, 40, 1]] and items1.tolist() == [[0, 1, 0, 40, 0, 0, 2, 0]]


def test_rank_with_nothing_gets_an_empty_list():
    ctx = np.array([5], dtype=np.int32)
    owner, _, _ = build_placement(ctx, [1], 3, 2)
    items, pairs, sched, indptr = build_worklist(ctx, owner, 2, 0, 2, 2)
    assert items.shape == (0, 8) and pairs.shape == (0, 4) and len(sched) == 0
    assert indptr.tolist() == [0]


def test_rejects_bad_chunk_and_heads():
    ctx = np.array([5], dtype=np.int32)
    owner = np.zeros((1, 2), dtype=np.int32)
    with pytest.raises(ValueError):
        build_worklist(ctx, owner, 0, 24, 4, 2)
    with pytest.raises(ValueError):
        build_worklist(ctx, owner, 0, 16, 5, 2)


def test_chunk_choice_by_hand():
    # rank 0 holds three pairs of 40, 20 and 20 tokens (the tiny list above): T = 80
    ctx = np.array([40, 20], dtype=np.int32)
    owner, _, _ = build_placement(ctx, [0, 1], 2, 2)
    # chunk 64: 3 items; 48: 3; 32: 2+1+1 = 4; 16: 3+2+2 = 7
    assert choose_chunk_tokens(ctx, owner, 0, 64, 16, 1, 2) == (64, 3)        # ceil(320/3) = 107 -> 112 pages' worth, held to 64
    assert choose_chunk_tokens(ctx, owner, 0, 64, 16, 2, 2) == (64, 3)        # ceil(320/6) = 54 -> 64
    assert choose_chunk_tokens(ctx, owner, 0, 64, 16, 3, 2) == (48, 3)        # ceil(320/9) = 36 -> 48
    assert choose_chunk_tokens(ctx, owner, 0, 64, 16, 4, 2) == (32, 4)        # ceil(320/12) = 27 -> 32
    assert choose_chunk_tokens(ctx, owner, 0, 64, 16, 8, 2) == (16, 7)        # ceil(320/24) = 14 -> 16
    assert choose_chunk_tokens(ctx, owner, 0, 64, 16, 100, 2) == (16, 7)      # never below min_chunk
    assert choose_chunk_tokens(ctx, owner, 0, 64, 32, 100, 2) == (32, 4)
    assert choose_chunk_tokens(ctx, owner, 1, 64, 16, 1, 2) == (64, 1)        # rank 1 holds one pair of 40 tokens: 54 -> 64
    assert choose_chunk_tokens(ctx, owner, 1, 64, 16, 2, 2) == (32, 2)        # ceil(160/6) = 27 -> 32
    for bad in ((64, 24, 1), (64, 16, 0)):
        with pytest.raises(ValueError):
            choose_chunk_tokens(ctx, owner, 0, *bad, 2)


@pytest.mark.parametrize("seed", range(6))
def test_chunk_choice_properties(seed):
    ctx, owner, _ = _case(seed, 40, 3, 4, 0.3, lo=1, hi=30000)
    for rank in range(3):
        whole, _, _, _ = build_worklist(ctx, owner, rank, 0, 8, 4)         # one item per pair: its tokens
        T = int(sum(int(it[3]) - int(it[2]) for it in whole))
        for slots in (1, 7, 50, 256, 10 ** 6):
            C, n = choose_chunk_tokens(ctx, owner, rank, 2048, 256, slots, 4)
            assert 256 <= C <= 2048 and C % 16 == 0
            items, _, _, _ = build_worklist(ctx, owner, rank, C, 8, 4)
            assert n == len(items)                              # the count is the real list's
            share = 4 * T / (3 * slots)
            assert C == 2048 or C >= share                      # four thirds of a slot's share fit in a chunk, unless held to the largest
            assert C == 256 or C - 16 < share                   # and not a page more, unless held to the smallest


# ---- the list cut into equal runs of pages (one per resident workgroup) ---------------------------------
from oracle import build_worklist_units


def test_units_by_hand():
    # Same share as test_tiny_list_by_hand: rank 0 holds (r0,h0) L=40 (3 pages), (r1,h0) and (r1,h1) L=20 (2 pages
    # each): a stream of 7 pages.  Three units: cuts at floor(u*7/3) = 0, 2, 4, 7.
    #   unit 0 = pages 0-1          -> pair 0 tokens [0, 32)
    #   unit 1 = pages 2-3          -> pair 0 [32, 40) and pair 1 [0, 16)
    #   unit 2 = pages 4-6          -> pair 1 [16, 20) and pair 2 [0, 20)
    ctx = np.array([40, 20], dtype=np.int32)
    owner, _, _ = build_placement(ctx, [0, 1], 2, 2)
    items, pairs, unit_indptr, chunk_indptr = build_worklist_units(ctx, owner, 0, 3, 4, 2)
    assert items.tolist() == [
        [0, 0, 0, 32, 0, 0, 0, 0], [0, 0, 32, 40, 0, 1, 0, 2],
        [1, 0, 0, 16, 1, 0, 4, 4], [1, 0, 16, 20, 1, 1, 4, 6],
        [1, 1, 0, 20, 2, 0, 6, 8]]
    assert pairs.tolist() == [[0, 0, 40, 2], [1, 0, 20, 2], [1, 1, 20, 1]]
    assert unit_indptr.tolist() == [0, 1, 3, 5] and chunk_indptr.tolist() == [0, 2, 4, 5]
    # four units: cuts 0, 1, 3, 5, 7 -> [0,16) | [16,40) | pair 1 whole | pair 2 whole
    items, pairs, unit_indptr, chunk_indptr = build_worklist_units(ctx, owner, 0, 4, 4, 2)
    assert [it[2:6] for it in items.tolist()] == [[0, 16, 0, 0], [16, 40, 0, 1], [0, 20, 1, 0], [0, 20, 2, 0]]
    assert unit_indptr.tolist() == [0, 1, 2, 3, 4] and chunk_indptr.tolist() == [0, 2, 3, 4]
    # one unit: every pair is one item; more units than pages: one page per unit
    items, pairs, unit_indptr, _ = build_worklist_units(ctx, owner, 0, 1, 4, 2)
    assert [it[2:4] for it in items.tolist()] == [[0, 40], [0, 20], [0, 20]] and unit_indptr.tolist() == [0, 3]
    items, pairs, unit_indptr, _ = build_worklist_units(ctx, owner, 0, 50, 4, 2)
    assert len(items) == 7 and unit_indptr.tolist() == list(range(8)) and pairs[:, 3].tolist() == [3, 2, 2]
    # a rank with nothing
    items, pairs, unit_indptr, chunk_indptr = build_worklist_units(np.array([5], np.int32), np.zeros((1, 2), np.int32), 1, 4, 2, 2)
    assert items.shape == (0, 8) and pairs.shape == (0, 4) and unit_indptr.tolist() == [0] and chunk_indptr.tolist() == [0]


@pytest.mark.parametrize("n_units", [1, 2, 7, 64, 512, 100000])
def test_units_against_a_page_by_page_partition(n_units):
    """Second style: write out every page of the stream, give page k of P the unit u with
    floor(u*P/U) <= k < floor((u+1)*P/U) (the textbook equal partition of a sequence), and collect runs of
    pages with the same (unit, pair).  Then the invariants the kernels rely on."""
    R, H, Hq = 5, 8, 32
    G = Hq // H
    for seed in range(6):
        ctx, owner, load = _case(40 + seed, 30 + 9 * seed, R, H, 0.3, lo=1, hi=3000 if seed % 2 else 200)
        seen = set()
        for k in range(R):
            items, pairs, unit_indptr, chunk_indptr = build_worklist_units(ctx, owner, k, n_units, Hq, H)
            stream = [(p, j) for p, (r, h, L, _n) in enumerate(pairs) for j in range(-(-int(L) // 16))]
            P = len(stream)
            U = min(n_units, P)
            assert len(unit_indptr) == U + 1 and unit_indptr[0] == 0 and unit_indptr[-1] == len(items)
            cuts = np.array([(u * P) // U for u in range(U + 1)]) if U else np.array([0])
            unit_of_page = np.searchsorted(cuts, np.arange(P), side="right") - 1
            want = []          # (unit, pair, first page, last page + 1)
            for kpage, (p, j) in enumerate(stream):
                u = int(unit_of_page[kpage])
                if want and want[-1][0] == u and want[-1][1] == p:
                    want[-1][3] = j + 1
                else:
                    want.append([u, p, j, j + 1])
            assert len(want) == len(items)
            unit_of_item = np.searchsorted(unit_indptr, np.arange(len(items)), side="right") - 1
            for i, (u, p, a, b) in enumerate(want):
                r, h, L, _n = (int(x) for x in pairs[p])
                assert items[i].tolist()[:5] == [r, h, 16 * a, min(L, 16 * b), p] and unit_of_item[i] == u
            # what the kernels rely on
            assert int((items[:, 3] - items[:, 2]).sum()) == load[k]
            sizes = np.diff(cuts)
            assert U == 0 or (sizes.max() - sizes.min() <= 1 and sizes.min() >= 1)     # equal runs, none empty
            assert chunk_indptr[0] == 0 and chunk_indptr[-1] == len(items)
            for p, (r, h, L, n) in enumerate(pairs):
                its = items[chunk_indptr[p]:chunk_indptr[p + 1]]
                assert len(its) == n >= 1 and its[0, 2] == 0 and its[-1, 3] == L and (its[1:, 2] == its[:-1, 3]).all()
                assert (its[:-1, 3] % 16 == 0).all() and its[:, 5].tolist() == list(range(n))
                assert (its[:, 6] == r * Hq + h * G).all() and owner[r, h] == k
                seen.add((int(r), int(h)))
            assert items[:, 7].tolist() == [i * G for i in range(len(items))]
            assert len(items) <= len(pairs) + max(U - 1, 0)       # a cut adds at most one item
        assert len(seen) == len(ctx) * H


# ---- launch records -------------------------------------------------------------------------------------
from oracle import build_launch_records


def test_launch_records_by_hand():
    # The hand-worked list of test_tiny_list_by_hand (rank 0, chunk 16): pairs (r0,h0) L=40 -> 3 pages at 0..2,
    # (r1,h0) L=20 -> pages 3..4, (r1,h1) L=20 -> pages 5..6 of a 7-entry page table with slots 10, 11, ..., 16.
    ctx = np.array([40, 20], dtype=np.int32)
    owner, _, _ = build_placement(ctx, [0, 1], 2, 2)
    items, pairs, sched, indptr = build_worklist(ctx, owner, 0, 16, 4, 2)
    page_indptr = np.array([0, 3, 5, 7]); page_ids = np.arange(10, 17, dtype=np.int32)
    rec = build_launch_records(items, sched, indptr, page_indptr, page_ids, 2)
    assert sched.tolist() == [0, 1, 3, 5, 2, 4, 6]
    # launch position 2 is item 3 = (r1,h0) tokens [0,16): first page 3 -> slot 13, one page, part row 6
    # (its pair, number 1, has 2 chunks whose partial rows start at row chunk_indptr[1] * G = 3 * 2)
    assert rec[2].tolist() == [3, 0, 16, 4, 6, 2, 13, 0, 0, 0, 0, 0, 0, 0, 1, 6]
    # launch position 4 is item 2 = (r0,h0) tokens [32,40): first page 2 -> slot 12, 8 tokens, part row 4
    # (pair 0: 3 chunks, rows from 0)
    assert rec[4].tolist() == [2, 0, 8, 0, 4, 3, 12, 0, 0, 0, 0, 0, 0, 0, 0, 0]
    # unsplit list, index order: every pair is one item, so every record points at final rows -(p*G) - 1
    items1, pairs1, _, indptr1 = build_worklist(ctx, owner, 0, 0, 4, 2)
    rec1 = build_launch_records(items1, None, indptr1, page_indptr, page_ids, 2)
    assert rec1[:, 4].tolist() == [-1, -3, -5] and rec1[0, 6:14].tolist() == [10, 11, 12, 0, 0, 0, 0, 0]
    assert rec1[:, 5].tolist() == [1, 1, 1] and rec1[:, 14].tolist() == [0, 1, 2] and rec1[:, 15].tolist() == [0, 2, 4]
    assert build_launch_records(items1, None, indptr1, page_indptr, page_ids, 2, direct_rows=False)[:, 4].tolist() == [0, 2, 4]
    # a first page beyond 2^31 entries keeps its high word
    big = build_launch_records(items1[:1], None, indptr1, np.array([2 ** 33 + 5, 2 ** 33 + 8]), {2 ** 33 + 5 + j: 7 + j for j in range(3)}, 2)
    assert big[0, :2].view(np.int64)[0] == 2 ** 33 + 5 and big[0, 6:9].tolist() == [7, 8, 9]


def test_launch_records_invariants():
    """Every record restates its item: the page range it names is the item's, the slots are the page table's,
    the row is the partial row or the pair's final rows, on chunked and equal-run lists."""
    rng = np.random.default_rng(5)
    R, H, Hq = 3, 4, 16
    G = Hq // H
    ctx, owner, load = _case(77, 40, R, H, 0.3, lo=1, hi=700)
    for k in range(R):
        for items, order, indptr in ((lambda t: (t[0], t[2], t[3]))(build_worklist(ctx, owner, k, 64, Hq, H)),
                                     (lambda t: (t[0], None, t[3]))(build_worklist_units(ctx, owner, k, 9, Hq, H))):
            pairs_L = {}
            for it in items:
                pairs_L[int(it[4])] = max(pairs_L.get(int(it[4]), 0), int(it[3]))
            n_pages = [-(-pairs_L[p] // 16) for p in range(len(pairs_L))]
            page_indptr = np.concatenate([[0], np.cumsum(n_pages)])
            page_ids = rng.permutation(int(page_indptr[-1]) + 5)[: int(page_indptr[-1])].astype(np.int32)
            rec = build_launch_records(items, order, indptr, page_indptr, page_ids, G)
            seq = range(len(items)) if order is None else order
            assert len(rec) == len(items)
            for kk, i in enumerate(seq):
                it = items[i]
                fp = int(rec[kk, :2].view(np.int64)[0])
                assert fp == page_indptr[it[4]] + it[2] // 16 and rec[kk, 2] == it[3] - it[2] and rec[kk, 3] == it[6]
                npg = -(-int(rec[kk, 2]) // 16)
                assert fp + npg <= page_indptr[it[4] + 1]
                assert rec[kk, 6:6 + min(8, npg)].tolist() == page_ids[fp: fp + min(8, npg)].tolist()
                assert not rec[kk, 6 + min(8, npg):14].any()
                n_chunks = indptr[it[4] + 1] - indptr[it[4]]
                assert rec[kk, 5] == n_chunks and rec[kk, 14] == it[4] and rec[kk, 15] == indptr[it[4]] * G
                # the rows of the pair's chunks, as the merge reads them, are those the items name
                assert it[7] == rec[kk, 15] + it[5] * G
                single = n_chunks == 1
                assert rec[kk, 4] == (-(int(it[4]) * G) - 1 if single else it[7])
