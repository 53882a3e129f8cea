"""Pins for the oracle's chunked-prefill attention and its work list."""
import math

import numpy as np
import pytest
import torch

from oracle import (bf16_bits_to_f64, build_prefill_worklist, decode_attention_pairs, gather_pair_kv,
                    prefill_attention_pairs, prefill_attention_row)
from workloads import make_kv_pool, make_prefill_q

SCALE = 1.0 / math.sqrt(128.0)


def _setup(seed, n_done, n_new, Hq, Hkv, owner=None, rank=0, tile=8):
    B = len(n_done)
    owner = np.zeros((B, Hkv), dtype=np.int32) if owner is None else np.asarray(owner)
    items, pairs, sched, out_indptr = build_prefill_worklist(n_done, n_new, owner, rank, Hq, tile)
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
    # 2 requests, 2 KV heads, 4 q-heads; rank 1 owns head 1 of request 0 and both heads of request 1
    owner = [[0, 1], [1, 1]]
    items, pairs, sched, out_indptr = build_prefill_worklist([10, 0], [5, 3], owner, 1, 4, tile_tokens=4)
    assert pairs.tolist() == [[0, 1, 10, 5], [1, 0, 0, 3], [1, 1, 0, 3]]
    assert out_indptr.tolist() == [0, 10, 16, 22]
    # (req, kv_head, pair, q_begin, q_end, n_done, q_row, out_row); Q rows: request 0 tokens 0..4, request 1 tokens 5..7
    assert items.tolist() == [[0, 1, 0, 0, 4, 10, 0 * 4 + 2, 0], [0, 1, 0, 4, 5, 10, 4 * 4 + 2, 8],
                              [1, 0, 1, 0, 3, 0, 5 * 4 + 0, 10], [1, 1, 2, 0, 3, 0, 5 * 4 + 2, 16]]
    assert sched.tolist() == [1, 0, 2, 3]           # key counts 15, 14, 3, 3


@pytest.mark.parametrize("seed", range(10))
def test_worklist_invariants(seed):
    rng = np.random.default_rng(seed)
    B, Hkv, G, R = int(rng.integers(1, 9)), int(rng.integers(1, 5)), int(rng.integers(1, 5)), int(rng.integers(1, 4))
    n_done = rng.integers(0, 100, size=B)
    n_new = rng.integers(0, 40, size=B)
    owner = rng.integers(0, R, size=(B, Hkv))
    tile = int(rng.integers(1, 20))
    seen = set()
    for k in range(R):
        items, pairs, sched, out_indptr = build_prefill_worklist(n_done, n_new, owner, k, Hkv * G, tile)
        assert sorted(sched.tolist()) == list(range(len(items)))
        keys = [items[i][5] + items[i][4] for i in sched]
        assert keys == sorted(keys, reverse=True)
        for p, (r, h, L, N) in enumerate(pairs):
            assert owner[r, h] == k and N == n_new[r] > 0 and L == n_done[r]
            seen.add((int(r), int(h)))
            mine = [it for it in items if it[2] == p]
            assert [it[3] for it in mine] == list(range(0, N, tile))
            assert all(it[4] == min(N, it[3] + tile) for it in mine)
            assert all(it[7] == out_indptr[p] + it[3] * G for it in mine)
            assert all(it[6] == (int(n_new[:r].sum()) + it[3]) * Hkv * G + h * G for it in mine)
        assert out_indptr[-1] == sum(int(p[3]) for p in pairs) * G
    assert seen == {(r, h) for r in range(B) for h in range(Hkv) if n_new[r] > 0}
