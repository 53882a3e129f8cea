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
    # rank 0 holds three pairs of 40, 20 and 20 tokens (the tiny list above)
    ctx = np.array([40, 20], dtype=np.int32)
    owner, _, _ = build_placement(ctx, [0, 1], 2, 2)
    # chunk 64: 3 items; 32: 2+1+1 = 4; 16: 3+2+2 = 7
    assert choose_chunk_tokens(ctx, owner, 0, 64, 16, 3, 2) == (64, 3)
    assert choose_chunk_tokens(ctx, owner, 0, 64, 16, 4, 2) == (32, 4)
    assert choose_chunk_tokens(ctx, owner, 0, 64, 16, 5, 2) == (16, 7)
    assert choose_chunk_tokens(ctx, owner, 0, 64, 16, 100, 2) == (16, 7)      # never below min_chunk
    assert choose_chunk_tokens(ctx, owner, 0, 64, 32, 100, 2) == (32, 4)
    assert choose_chunk_tokens(ctx, owner, 0, 48, 16, 4, 2) == (16, 7)        # 48 -> 24 rounds down to one page
    assert choose_chunk_tokens(ctx, owner, 1, 64, 16, 0, 2) == (64, 1)        # nothing asked for: the largest chunk
    with pytest.raises(ValueError):
        choose_chunk_tokens(ctx, owner, 0, 64, 24, 1, 2)


@pytest.mark.parametrize("seed", range(6))
def test_chunk_choice_properties(seed):
    ctx, owner, _ = _case(seed, 40, 3, 4, 0.3, lo=1, hi=30000)
    for rank in range(3):
        for min_items in (0, 1, 50, 256, 10 ** 6):
            C, n = choose_chunk_tokens(ctx, owner, rank, 2048, 256, min_items, 4)
            assert C in (2048, 1024, 512, 256)
            items, _, _, _ = build_worklist(ctx, owner, rank, C, 8, 4)
            assert n == len(items)                              # the count is the real list's
            if C < 2048:                                        # every larger candidate was too short
                bigger, _, _, _ = build_worklist(ctx, owner, rank, 2 * C, 8, 4)
                assert len(bigger) < min_items
            if n < min_items:
                assert C == 256
