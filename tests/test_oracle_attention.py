"""Pins for the oracle's attention: closed forms, brute force, a library routine,
split/merge consistency and the sharding invariant."""
import math

import numpy as np
import pytest
import torch

import oracle
from oracle import (attend, bf16_bits_to_f64, build_placement, build_worklist,
                    decode_attention_items, decode_attention_pairs, merge_lse, unsharded_attention)
from workloads import make_kv_pool, make_q

SCALE = 1.0 / math.sqrt(128.0)


def test_single_key_returns_its_value_row():
    rng = np.random.default_rng(0)
    q = rng.standard_normal((4, 128)); K = rng.standard_normal((1, 128)); V = rng.standard_normal((1, 128))
    out, lse = attend(q, K, V, SCALE)
    assert np.array_equal(out, np.repeat(V, 4, axis=0))
    assert np.allclose(lse, SCALE * (q @ K[0]), rtol=0, atol=1e-15)


def test_identical_keys_average_the_values():
    rng = np.random.default_rng(1)
    q = rng.standard_normal((3, 128)); k = rng.standard_normal(128); V = rng.standard_normal((37, 128))
    out, lse = attend(q, np.tile(k, (37, 1)), V, SCALE)
    assert np.allclose(out, np.tile(V.mean(axis=0), (3, 1)), atol=1e-14)
    assert np.allclose(lse, SCALE * (q @ k) + math.log(37), atol=1e-13)


def test_zero_query_gives_uniform_weights():
    rng = np.random.default_rng(2)
    K = rng.standard_normal((50, 128)); V = rng.standard_normal((50, 128))
    out, lse = attend(np.zeros((2, 128)), K, V, SCALE)
    assert np.allclose(out, np.tile(V.mean(axis=0), (2, 1)), atol=1e-14)
    assert np.allclose(lse, math.log(50), atol=1e-14)


def test_dominant_key_wins():
    rng = np.random.default_rng(3)
    q = rng.standard_normal((1, 128)); K = rng.standard_normal((20, 128)) * 0.01
    V = rng.standard_normal((20, 128))
    K[7] = q[0] * (60.0 / (SCALE * (q[0] @ q[0])))       # score 60, the rest near 0
    out, lse = attend(q, K, V, SCALE)
    assert np.allclose(out[0], V[7], atol=1e-20 + 20 * math.exp(-59) * np.abs(V).max())
    assert abs(lse[0] - 60.0) < 1e-12


def test_large_scores_do_not_overflow():
    q = np.full((1, 128), 30.0); K = np.full((5, 128), 30.0); V = np.arange(5 * 128, dtype=float).reshape(5, 128)
    out, lse = attend(q, K, V, 1.0)
    assert np.isfinite(out).all() and np.allclose(out[0], V.mean(axis=0))
    assert abs(lse[0] - (30.0 * 30.0 * 128 + math.log(5))) < 1e-9


def test_brute_force_python_loops():
    rng = np.random.default_rng(4)
    G, L, d = 2, 9, 8
    q = rng.standard_normal((G, d)); K = rng.standard_normal((L, d)); V = rng.standard_normal((L, d))
    scale = 0.37
    out, lse = attend(q, K, V, scale)
    for g in range(G):
        s = [scale * sum(q[g][i] * K[t][i] for i in range(d)) for t in range(L)]
        z = sum(math.exp(x) for x in s)
        assert abs(lse[g] - math.log(z)) < 1e-13
        for j in range(d):
            ref = sum(math.exp(s[t]) / z * V[t][j] for t in range(L))
            assert abs(out[g][j] - ref) < 1e-13


def _small_batch(seed=7, B=5, Hq=8, Hkv=2, R=3, kv_dtype="bf16", lens=(1, 17, 33, 100, 250)):
    ctx = np.array(lens[:B], dtype=np.int32)
    q = make_q(seed, B, Hq, 128)
    all_pairs = np.array([(r, h) for r in range(B) for h in range(Hkv)])
    kv_all = make_kv_pool(seed, all_pairs, ctx, kv_dtype=kv_dtype)
    return ctx, q, kv_all


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
def test_unsharded_matches_dense_library_softmax(kv_dtype):
    # gather the pages into dense tensors with torch and use torch.softmax in fp64
    B, Hq, Hkv = 5, 8, 2
    G = Hq // Hkv
    ctx, q, kv = _small_batch(kv_dtype=kv_dtype)
    out, lse = unsharded_attention(q, kv, ctx, Hq, Hkv, SCALE)
    qt = torch.from_numpy(q.view(np.int16)).view(torch.bfloat16).to(torch.float64)
    for r in range(B):
        for h in range(Hkv):
            p = r * Hkv + h
            slots = torch.from_numpy(kv["page_ids"][kv["page_indptr"][p]:kv["page_indptr"][p + 1]].astype(np.int64))
            if kv_dtype == "bf16":
                Kd = torch.from_numpy(kv["k_pool"].view(np.int16)).view(torch.bfloat16)[slots].to(torch.float64)
                Vd = torch.from_numpy(kv["v_pool"].view(np.int16)).view(torch.bfloat16)[slots].to(torch.float64)
            else:
                Kd = torch.from_numpy(kv["k_pool"]).view(torch.float8_e4m3fn)[slots].to(torch.float64) \
                    * torch.from_numpy(kv["k_scale"])[slots].to(torch.float64)[:, None, None]
                Vd = torch.from_numpy(kv["v_pool"]).view(torch.float8_e4m3fn)[slots].to(torch.float64) \
                    * torch.from_numpy(kv["v_scale"])[slots].to(torch.float64)[:, None, None]
            Kd = Kd.reshape(-1, 128)[: ctx[r]]
            Vd = Vd.reshape(-1, 128)[: ctx[r]]
            for g in range(G):
                j = h * G + g                        # consecutive q-heads share a KV head
                s = (Kd @ qt[r, j]) * SCALE
                ref = torch.softmax(s, dim=0) @ Vd
                assert torch.allclose(torch.from_numpy(out[r, j]), ref, rtol=0, atol=1e-13)
                assert abs(lse[r, j] - torch.logsumexp(s, dim=0).item()) < 1e-12
    assert np.isfinite(out).all()       # the NaN-poisoned page tails were never read


def test_gqa_mapping_against_repeat_interleave():
    B, Hq, Hkv = 3, 8, 2
    ctx, q, kv = _small_batch(B=3)
    out, _ = unsharded_attention(q, kv, ctx, Hq, Hkv, SCALE)
    qf = bf16_bits_to_f64(q)
    for r in range(B):
        Ks = np.stack([oracle.gather_pair_kv(kv, r * Hkv + h, 0, int(ctx[r]))[0] for h in range(Hkv)])
        Vs = np.stack([oracle.gather_pair_kv(kv, r * Hkv + h, 0, int(ctx[r]))[1] for h in range(Hkv)])
        Kq = torch.from_numpy(Ks).repeat_interleave(Hq // Hkv, dim=0)      # [Hq][L][d]
        Vq = torch.from_numpy(Vs).repeat_interleave(Hq // Hkv, dim=0)
        s = torch.einsum("hd,hld->hl", torch.from_numpy(qf[r]), Kq) * SCALE
        ref = torch.einsum("hl,hld->hd", torch.softmax(s, dim=-1), Vq)
        assert np.allclose(out[r], ref.numpy(), atol=1e-13)


@pytest.mark.parametrize("chunk", [16, 32, 64, 2048])
def test_chunk_partials_merge_back_to_unsplit(chunk):
    B, Hq, Hkv, R = 5, 8, 2, 3
    G = Hq // Hkv
    ctx, q, _ = _small_batch()
    owner, _, _ = build_placement(ctx, [0, 1, 0, 1, 0], R, Hkv)
    for k in range(R):
        items, pairs, sched, indptr = build_worklist(ctx, owner, k, chunk, Hq, Hkv)
        kv = make_kv_pool(7, pairs[:, :2], ctx)
        po, pl = decode_attention_items(q, kv, items, G, SCALE)
        out, lse = merge_lse(po, pl, indptr, G)
        ref_o, ref_l = decode_attention_pairs(q, kv, pairs, Hq, G, SCALE)
        assert np.allclose(out, ref_o, rtol=0, atol=1e-12)
        assert np.allclose(lse, ref_l, rtol=0, atol=1e-12)


def test_merge_of_one_chunk_is_identity_and_weights_follow_lse():
    po = np.array([[1.0, 2.0], [3.0, 5.0], [7.0, 11.0]])
    pl = np.array([0.0, math.log(3.0), 2.0])
    out, lse = merge_lse(po, pl, np.array([0, 2, 3]), 1)
    # pair 0: weights 1/4 and 3/4; pair 1 passes through
    assert np.allclose(out, [[2.5, 4.25], [7.0, 11.0]], atol=1e-15)
    assert np.allclose(lse, [math.log(4.0), 2.0], atol=1e-15)


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
def test_all_rank_shares_reassemble_unsharded_attention(kv_dtype):
    B, Hq, Hkv, R = 5, 8, 2, 3
    G = Hq // Hkv
    ctx, q, kv_all = _small_batch(kv_dtype=kv_dtype)
    ref_o, ref_l = unsharded_attention(q, kv_all, ctx, Hq, Hkv, SCALE)
    owner, _, load = build_placement(ctx, [0, 1, 0, 0, 1], R, Hkv)
    got_o = np.full_like(ref_o, np.nan); got_l = np.full_like(ref_l, np.nan)
    filled = np.zeros((B, Hq), dtype=int)
    for k in range(R):
        items, pairs, sched, indptr = build_worklist(ctx, owner, k, 32, Hq, Hkv)
        kv = make_kv_pool(7, pairs[:, :2], ctx, kv_dtype=kv_dtype)
        o, l = decode_attention_pairs(q, kv, pairs, Hq, G, SCALE)
        for p, (r, h, L, _n) in enumerate(pairs):
            got_o[r, h * G:(h + 1) * G] = o[p * G:(p + 1) * G]
            got_l[r, h * G:(h + 1) * G] = l[p * G:(p + 1) * G]
            filled[r, h * G:(h + 1) * G] += 1
    assert (filled == 1).all()
    assert np.allclose(got_o, ref_o, rtol=0, atol=1e-12) and np.allclose(got_l, ref_l, rtol=0, atol=1e-12)


def test_threaded_run_equals_serial_run():
    B, Hq, Hkv = 5, 8, 2
    ctx, q, kv = _small_batch()
    pairs = np.array([(r, h, ctx[r], 1) for r in range(B) for h in range(Hkv)], dtype=np.int32)
    a = decode_attention_pairs(q, kv, pairs, Hq, 4, SCALE, workers=1)
    b = decode_attention_pairs(q, kv, pairs, Hq, 4, SCALE, workers=4)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
