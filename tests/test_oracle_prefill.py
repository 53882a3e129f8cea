"""Pins for the oracle's chunked-prefill attention and its work list."""
import math

import numpy as np
import pytest
import torch

from oracle import (bf16_bits_to_f64, build_prefill_worklist, decode_attention_pairs, gather_pair_kv, merge_lse,
                    prefill_attention_items, prefill_attention_pairs, prefill_attention_row)
from workloads import make_kv_pool, make_prefill_q

SCALE = 1.0 / math.sqrt(128.0)


def _setup(seed, n_done, n_new, Hq, Hkv, owner=None, rank=0, tile=8):
    B = len(n_done)
    owner = np.zeros((B, Hkv), dtype=np.int32) if owner is None else np.asarray(owner)
    items, pairs, sched, chunk_indptr, _ = build_prefill_worklist(n_done, n_new, owner, rank, Hq, tile)
    G = Hq // Hkv
    out_indptr = np.concatenate([[0], np.cumsum(pairs[:, 3] * G)]).astype(np.int64) if len(pairs) else np.zeros(1, np.int64)
    ctx = (np.asarray(n_done) + np.asarray(n_new)).astype(np.int32)
    kv = make_kv_pool(seed, pairs[:, :2], ctx, threads=1)
    q_indptr = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int64)
    q = make_prefill_q(seed, int(q_indptr[-1]), Hq, 128)
    return items, pairs, sched, out_indptr, kv, q, q_indptr


def test_dense_causal_softmax_in_torch():
    n_done, n_new, Hq, Hkv = [5, 0, 33], [7, 4, 20], 8, 2
    G = Hq // Hkv
    items, pairs, sched, out_indptr, kv, q, q_indptr = _setup(1, n_done, n_new, Hq, Hkv)
    out, lse = prefill_attention_pairs(q, q_indptr, kv, pairs, Hq, G, SCALE)
    for p, (r, h, L, N) in enumerate(pairs):
        K, V = gather_pair_kv(kv, p, 0, L + N)
        Kt, Vt = torch.from_numpy(K), torch.from_numpy(V)
        Q = torch.from_numpy(bf16_bits_to_f64(q[q_indptr[r]:q_indptr[r] + N, h * G:(h + 1) * G]))   # [N][G][d]
        S = torch.einsum("ngd,td->ngt", Q, Kt) * SCALE
        pos = torch.arange(N)[:, None, None] + L
        S = S.masked_fill(torch.arange(L + N)[None, None, :] > pos, float("-inf"))
        want = torch.einsum("ngt,td->ngd", torch.softmax(S, dim=-1), Vt).reshape(N * G, 128).numpy()
        want_lse = torch.logsumexp(S, dim=-1).reshape(N * G).numpy()
        rows = slice(int(out_indptr[p]), int(out_indptr[p + 1]))
        assert np.abs(out[rows] - want).max() < 1e-12 and np.abs(lse[rows] - want_lse).max() < 1e-12


def test_brute_force_loops():
    n_done, n_new, Hq, Hkv = [3, 0], [2, 3], 4, 2
    G = 2
    items, pairs, sched, out_indptr, kv, q, q_indptr = _setup(2, n_done, n_new, Hq, Hkv)
    out, lse = prefill_attention_pairs(q, q_indptr, kv, pairs, Hq, G, SCALE)
    for p, (r, h, L, N) in enumerate(pairs):
        K, V = gather_pair_kv(kv, p, 0, L + N)
        for i in range(N):
            for g in range(G):
                qv = bf16_bits_to_f64(q[q_indptr[r] + i, h * G + g])
                s = [SCALE * sum(float(qv[c]) * float(K[t][c]) for c in range(128)) for t in range(L + i + 1)]
                m = max(s)
                w = [math.exp(x - m) for x in s]
                tot = sum(w)
                row = int(out_indptr[p]) + i * G + g
                assert abs(lse[row] - (m + math.log(tot))) < 1e-12
                for c in range(0, 128, 17):
                    assert abs(out[row][c] - sum(w[t] * float(V[t][c]) for t in range(L + i + 1)) / tot) < 1e-12


def test_first_token_of_a_fresh_prompt_returns_its_own_value_row():
    items, pairs, sched, out_indptr, kv, q, q_indptr = _setup(3, [0], [4], 4, 1)
    out, lse = prefill_attention_pairs(q, q_indptr, kv, pairs, 4, 4, SCALE)
    K, V = gather_pair_kv(kv, 0, 0, 4)
    for g in range(4):
        assert np.array_equal(out[g], V[0])
        assert abs(lse[g] - SCALE * float(bf16_bits_to_f64(q[0, g]) @ K[0])) < 1e-12


def test_result_does_not_depend_on_how_the_prompt_is_chunked():
    # the same 40-token prompt prefilled in one go, or with 24 tokens already done: tokens 24.. agree
    Hq, Hkv, G = 4, 2, 2
    whole = _setup(4, [0], [40], Hq, Hkv)
    part = _setup(4, [24], [16], Hq, Hkv)
    qw = whole[5]
    out_w, lse_w = prefill_attention_pairs(qw, whole[6], whole[4], whole[1], Hq, G, SCALE)
    out_p, lse_p = prefill_attention_pairs(qw[24:], part[6], part[4], part[1], Hq, G, SCALE)
    for h in range(Hkv):
        a = out_w[int(whole[3][h]) + 24 * G: int(whole[3][h + 1])]
        b = out_p[int(part[3][h]): int(part[3][h + 1])]
        assert np.array_equal(a, b)


def test_one_new_token_is_decode_attention():
    # a chunk of one token behind L processed ones is a decode step over L + 1 cached tokens
    n_done, Hq, Hkv, G = [17, 64, 5], 8, 2, 4
    items, pairs, sched, out_indptr, kv, q, q_indptr = _setup(5, n_done, [1, 1, 1], Hq, Hkv)
    out, lse = prefill_attention_pairs(q, q_indptr, kv, pairs, Hq, G, SCALE)
    dpairs = np.stack([pairs[:, 0], pairs[:, 1], pairs[:, 2] + 1], axis=1)
    out_d, lse_d = decode_attention_pairs(q, kv, dpairs, Hq, G, SCALE)
    assert np.array_equal(out, out_d) and np.array_equal(lse, lse_d)
    o, l = prefill_attention_row(q, q_indptr, kv, pairs, Hq, G, SCALE, pair=3, tok=0)
    assert np.array_equal(o, out[12:16]) and np.array_equal(l, lse[12:16])


def test_worklist_by_hand():
    # 2 requests, 2 KV heads, 4 q-heads (G = 2); rank 1 owns head 1 of request 0 and both heads of request 1
    owner = [[0, 1], [1, 1]]
    items, pairs, sched, chunk_indptr, out_indptr = build_prefill_worklist([40, 0], [5, 3], owner, 1, 4, tile_tokens=4,
                                                                           kv_chunk_tokens=32)
    assert pairs.tolist() == [[0, 1, 40, 5], [1, 0, 0, 3], [1, 1, 0, 3]]
    # tiles: pair 0 -> tokens [0,4) (keys 44: chunks [0,32) [32,44)) and [4,5) (keys 45: [0,32) [32,45)); pairs 1, 2 -> one tile, one chunk
    # (pair, q_begin, q_end, n_done, kv_begin, kv_end, q_row, part_row); T = 4 tokens x 2 = 8 rows per item
    assert items.tolist() == [[0, 0, 4, 40, 0, 32, 0 * 4 + 2, 0], [0, 0, 4, 40, 32, 44, 0 * 4 + 2, 8],
                              [0, 4, 5, 40, 0, 32, 4 * 4 + 2, 16], [0, 4, 5, 40, 32, 45, 4 * 4 + 2, 24],
                              [1, 0, 3, 0, 0, 3, 5 * 4 + 0, 32], [2, 0, 3, 0, 0, 3, 5 * 4 + 2, 40]]
    assert chunk_indptr.tolist() == [0, 2, 4, 5, 6]
    assert out_indptr.tolist() == [0, 16, 24, 32]          # pair 0 has two tiles of 8 rows, the others one
    assert sched.tolist() == [0, 2, 3, 1, 4, 5]            # keys per item: 32, 12, 32, 13, 3, 3
    # no split: one item per tile
    items0, _, sched0, chunk0, out0 = build_prefill_worklist([40, 0], [5, 3], owner, 1, 4, tile_tokens=4)
    assert items0[:, 4:6].tolist() == [[0, 44], [0, 45], [0, 3], [0, 3]] and chunk0.tolist() == [0, 1, 2, 3, 4]
    assert out0.tolist() == out_indptr.tolist() and sched0.tolist() == [1, 0, 2, 3]


@pytest.mark.parametrize("seed", range(10))
def test_worklist_invariants(seed):
    rng = np.random.default_rng(seed)
    B, Hkv, G, R = int(rng.integers(1, 9)), int(rng.integers(1, 5)), int(rng.integers(1, 5)), int(rng.integers(1, 4))
    n_done = rng.integers(0, 100, size=B)
    n_new = rng.integers(0, 40, size=B)
    owner = rng.integers(0, R, size=(B, Hkv))
    tile = int(rng.integers(1, 20))
    chunk = int(rng.integers(0, 4)) * 32
    T = tile * G
    seen = set()
    for k in range(R):
        items, pairs, sched, chunk_indptr, out_indptr = build_prefill_worklist(n_done, n_new, owner, k, Hkv * G, tile, chunk)
        assert sorted(sched.tolist()) == list(range(len(items)))
        keys = [items[i][5] - items[i][4] for i in sched]
        assert keys == sorted(keys, reverse=True)
        assert [it[7] for it in items] == [i * T for i in range(len(items))]
        n_tiles = 0
        for p, (r, h, L, N) in enumerate(pairs):
            assert owner[r, h] == k and N == n_new[r] > 0 and L == n_done[r]
            seen.add((int(r), int(h)))
            assert out_indptr[p] == n_tiles * T
            for b in range(0, N, tile):
                e = min(N, b + tile)
                mine = items[chunk_indptr[n_tiles]:chunk_indptr[n_tiles + 1]]
                assert all(it[0] == p and it[1] == b and it[2] == e and it[3] == L for it in mine)
                assert all(it[6] == (int(n_new[:r].sum()) + b) * Hkv * G + h * G for it in mine)
                # the chunks tile [0, L + e) without gap or overlap, all but the last of full size
                assert mine[0][4] == 0 and mine[-1][5] == L + e
                assert all(a[5] == c[4] for a, c in zip(mine[:-1], mine[1:]))
                assert all(it[5] - it[4] == chunk for it in mine[:-1])
                n_tiles += 1
        assert chunk_indptr[-1] == len(items) and len(chunk_indptr) == n_tiles + 1 and out_indptr[-1] == n_tiles * T
    assert seen == {(r, h) for r in range(B) for h in range(Hkv) if n_new[r] > 0}


@pytest.mark.parametrize("chunk", [32, 64, 96])
def test_chunk_partials_merge_back_to_unsplit(chunk):
    # split-K is exact algebra: merging the items' partials (rows that see none of a chunk included)
    # gives the unsplit result
    n_done, n_new, Hq, Hkv, G, tile = [70, 0, 33], [50, 9, 40], 4, 2, 2, 8
    owner = np.zeros((3, Hkv), dtype=np.int32)
    items, pairs, sched, chunk_indptr, out_indptr = build_prefill_worklist(n_done, n_new, owner, 0, Hq, tile, chunk)
    ctx = (np.asarray(n_done) + np.asarray(n_new)).astype(np.int32)
    kv = make_kv_pool(21, pairs[:, :2], ctx, threads=1)
    q_indptr = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int64)
    q = make_prefill_q(21, int(q_indptr[-1]), Hq, 128)
    part_o, part_lse = prefill_attention_items(q, kv, items, pairs, Hq, G, tile, SCALE)
    assert np.isinf(part_lse[np.isfinite(part_o).all(axis=1)]).any()      # the case of an unseen chunk occurs
    with np.errstate(invalid="ignore"):
        out, lse = merge_lse(part_o, part_lse, chunk_indptr, tile * G)
    want_o, want_l = prefill_attention_pairs(q, q_indptr, kv, pairs, Hq, G, SCALE, out_indptr=out_indptr)
    valid = np.isfinite(want_l)
    assert valid.sum() == int(pairs[:, 3].sum()) * G
    assert np.abs(out[valid] - want_o[valid]).max() < 1e-12 and np.abs(lse[valid] - want_l[valid]).max() < 1e-12


def test_chunk_choice_by_hand_and_on_drawn_batches():
    """choose_prefill_chunk: hand-worked cases for every branch, and on drawn batches the rule restated from a
    token-by-token count of the keys."""
    import oracle
    from oracle import choose_prefill_chunk
    owner = np.zeros((2, 1), dtype=np.int32)
    # one pair, 100 processed + 28 new tokens, tiles of 16: tile 0 sees 116 keys, tile 1 sees 128: T = 244.
    n_done, n_new = [100, 0], [28, 0]
    assert choose_prefill_chunk(n_done, n_new, owner, 0, 2, 16, 256, 32, 2) == (192, 2)     # ceil(4*244/6) = 163 -> 192; 1 + 1 items
    assert choose_prefill_chunk(n_done, n_new, owner, 0, 2, 16, 256, 32, 1) == (256, 2)     # 326 -> 352, held to the largest
    assert choose_prefill_chunk(n_done, n_new, owner, 0, 2, 16, 256, 32, 100) == (32, 8)    # ceil(976/300) = 4 -> 32; 4 + 4 items
    assert choose_prefill_chunk(n_done, n_new, owner, 0, 2, 16, 256, 64, 100) == (64, 4)    # held to the smallest; 2 + 2 items
    assert choose_prefill_chunk(n_done, n_new, owner, 0, 2, 16, 256, 32, 5) == (96, 4)      # ceil(976/15) = 66 -> 96; 2 + 2 items
    assert choose_prefill_chunk(n_done, n_new, owner, 0, 2, 16, 256, 32, 8) == (64, 4)      # ceil(976/24) = 41 -> 64
    # both KV heads of the request on this rank: twice the keys
    both = np.zeros((2, 2), dtype=np.int32)
    assert choose_prefill_chunk(n_done, n_new, both, 0, 4, 16, 256, 32, 4) == (192, 4)
    assert choose_prefill_chunk(n_done, n_new, both, 1, 4, 16, 256, 32, 4) == (32, 0)       # nothing on rank 1: the smallest, no items
    # a last tile of 12 tokens counts its own keys: 3 tiles of 100+16, 100+32, 100+44
    assert choose_prefill_chunk([100], [44], np.zeros((1, 1), dtype=np.int32), 0, 1, 16, 1024, 32, 1) == (544, 3)   # T = 392: 523 -> 544
    for bad in ((100, 32, 1), (64, 128, 1), (64, 16, 1), (64, 32, 0)):
        with pytest.raises(ValueError):
            choose_prefill_chunk(n_done, n_new, owner, 0, 2, 16, *bad)
    rng = np.random.default_rng(21)
    for _ in range(60):
        B, H, R = int(rng.integers(1, 6)), int(rng.integers(1, 4)), int(rng.integers(1, 3))
        n_done = rng.integers(0, 3000, size=B); n_new = rng.integers(0, 200, size=B)
        owner = rng.integers(0, R, size=(B, H)).astype(np.int32)
        tile = int(rng.integers(1, 33)); slots = int(rng.integers(1, 600))
        mx = 32 * int(rng.integers(1, 65)); mn = 32 * int(rng.integers(1, mx // 32 + 1))
        C, n = choose_prefill_chunk(n_done, n_new, owner, 0, 2 * H, tile, mx, mn, slots)
        assert n == len(oracle.build_prefill_worklist(n_done, n_new, owner, 0, 2 * H, tile, C)[0]) and mn <= C <= mx and C % 32 == 0
        # the keys, token by token: the last token of a tile sees what the tile sees
        T = sum(int(n_done[r]) + i + 1 for r in range(B) for h in range(H) if owner[r, h] == 0
                for i in range(int(n_new[r])) if (i + 1) % tile == 0 or i + 1 == int(n_new[r]))
        share = 4 * T / (3 * slots)
        assert C == mx or C >= share                       # long enough for four thirds of a share, unless held to the largest
        assert C == mn or C - 32 < share                   # and not a step longer, unless held to the smallest
