"""Pins for the oracle's placement (cyclic, hybrid, least-load routing)."""
import itertools
import json
import os

import numpy as np
import pytest

from oracle import build_placement

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _gold(name):
    with open(os.path.join(GOLD, name)) as f:
        return json.load(f)


def _naive_heads_per_rank(H, R):
    """Contiguous split of H heads over R ranks, the larger shares first."""
    return [len(x) for x in np.array_split(np.arange(H), R)]


def test_fig2_cyclic_capacity_gain():
    g = _gold("fig2_cyclic_4heads_tp3.json")
    H, R = g["n_kv_heads"], g["n_ranks"]
    naive = _naive_heads_per_rank(H, R)
    assert max(naive) == g["naive_worst_rank_heads_per_layer"]
    per_rank = np.zeros(R, dtype=np.int64)
    for layer in range(R):
        owner, dp, load = build_placement([1], [0], R, H, rot=[0], layer=layer)
        per_rank += np.bincount(owner[0], minlength=R)
        assert np.array_equal(load, np.bincount(owner[0], minlength=R))
    assert per_rank.tolist() == [g["cyclic_heads_per_rank_over_n_ranks_layers"]] * R
    # memory is capped by the fullest rank: naive fills max(naive) per layer everywhere
    gain = (max(naive) * R) / per_rank.max()
    assert gain == g["capacity_gain"]


def test_sec2_naive_8_on_7_and_what_cyclic_does_to_it():
    g = _gold("sec2_8heads_7gpus.json")
    H, R = g["n_kv_heads"], g["n_ranks"]
    naive = _naive_heads_per_rank(H, R)
    assert (max(naive), min(naive)) == (g["max_heads_on_a_rank"], g["min_heads_on_a_rank"])
    assert sum(1 for x in naive if x == 2) == g["ranks_with_two_heads"]
    # one cyclic step has the same 2-vs-1 skew; seven rotations even it out exactly
    owner, _, _ = build_placement([1], [0], R, H, rot=[0])
    one = np.bincount(owner[0], minlength=R)
    assert (one.max(), one.min()) == (2, 1)
    _, _, load = build_placement([1] * R, [0] * R, R, H)       # rot = request index
    assert load.tolist() == [H] * R


def test_hand_worked_hybrid_example():
    g = _gold("hand_hybrid_3ranks.json")
    owner, dp, load = build_placement(g["ctx_len"], g["mode"], g["n_ranks"], g["n_kv_heads"])
    assert owner.tolist() == g["owner"]
    assert dp.tolist() == g["dp_rank"]
    assert load.tolist() == g["rank_load"]


@pytest.mark.parametrize("H,R", [(8, 8), (8, 4), (8, 2), (4, 4), (32, 8)])
def test_rank_count_dividing_heads_is_uniform_tp(H, R):
    # Section 3.1: with 8 heads on 8 workers hybrid attention is plain TP-8
    rng = np.random.default_rng(1)
    ctx = rng.integers(1, 100, size=9)
    owner, dp, load = build_placement(ctx, np.zeros(9, np.uint8), R, H)
    for r in range(9):
        assert np.bincount(owner[r], minlength=R).tolist() == [H // R] * R
    assert (dp == -1).all()
    assert load.tolist() == [int(ctx.sum()) * (H // R)] * R


def test_dp_attention_special_case_single_head():
    # one replicated head, every request data-parallel: plain least-loaded routing
    ctx = [5, 3, 9, 1, 1, 4]
    owner, dp, load = build_placement(ctx, [1] * 6, 3, 1)
    # by hand: 5->r0 [5,0,0]; 3->r1 [5,3,0]; 9->r2 [5,3,9]; 1->r1 [5,4,9]; 1->r1 [5,5,9]; 4->r0
    assert dp.tolist() == [0, 1, 2, 1, 1, 0]
    assert owner[:, 0].tolist() == dp.tolist()
    assert load.tolist() == [9, 5, 9]


def _brute(ctx, mode, R, H, rot, layer):
    """Second implementation in another style: sets of (r, h) per rank."""
    held = {k: set() for k in range(R)}
    def weight(k):
        return sum(ctx[r] for (r, _h) in held[k])
    for r in range(len(ctx)):
        if mode[r] == 0:
            for h in range(H):
                held[(h + rot[r] + layer) % R].add((r, h))
        else:
            loads = [weight(k) for k in range(R)]
            k = loads.index(min(loads))
            held[k] |= {(r, h) for h in range(H)}
    return held


def test_brute_force_enumeration_tiny():
    checked = 0
    for R in range(1, 5):
        for H in range(1, 6):
            for B in range(1, 4):
                for mode in itertools.product([0, 1], repeat=B):
                    for ctx in ([1] * B, [3, 1, 2][:B], [2, 2, 5][:B]):
                        rot = [(7 * r + 1) % 5 for r in range(B)]
                        for layer in (0, 2):
                            owner, dp, load = build_placement(ctx, mode, R, H, rot=rot, layer=layer)
                            held = _brute(ctx, mode, R, H, rot, layer)
                            for k in range(R):
                                got = {(r, h) for r in range(B) for h in range(H) if owner[r, h] == k}
                                assert got == held[k]
                                assert load[k] == sum(ctx[r] for (r, _h) in held[k])
                            checked += 1
    assert checked > 1000


def test_every_head_has_exactly_one_owner_in_range():
    rng = np.random.default_rng(5)
    for R in (3, 5, 6, 7):
        ctx = rng.integers(1, 5000, size=200)
        mode = (rng.random(200) < 0.3).astype(np.uint8)
        owner, dp, load = build_placement(ctx, mode, R, 8)
        assert owner.shape == (200, 8) and owner.min() >= 0 and owner.max() < R
        assert load.sum() == 8 * int(ctx.sum())
        for r in range(200):
            if mode[r]:
                assert (owner[r] == dp[r]).all() and 0 <= dp[r] < R
            else:
                assert dp[r] == -1
                assert owner[r].tolist() == [(h + r) % R for h in range(8)]


def test_list_scheduling_invariant_after_every_dp_assignment():
    # greedy least-load = online makespan list scheduling: a step cannot widen the
    # spread beyond max(previous spread, the job just placed)
    rng = np.random.default_rng(9)
    R, H = 5, 8
    ctx = rng.integers(1, 20000, size=150)
    mode = (rng.random(150) < 0.6).astype(np.uint8)
    prev = np.zeros(R, dtype=np.int64)
    for n in range(1, 151):
        owner, dp, load = build_placement(ctx[:n], mode[:n], R, H)
        if mode[n - 1]:
            spread_before = prev.max() - prev.min()
            assert load.max() - load.min() <= max(spread_before, H * int(ctx[n - 1]))
            assert prev[dp[n - 1]] == prev.min()
            assert dp[n - 1] == int(np.argmin(prev))       # lowest rank among ties
        prev = load


def test_equal_length_all_tp_balance():
    R, H, L = 7, 8, 100
    for B in range(1, 30):
        _, _, load = build_placement([L] * B, [0] * B, R, H)
        assert load.max() - load.min() <= L
        if B % R == 0:
            assert load.max() == load.min()


def test_ragged_all_tp_base_load_is_shared():
    # every rank holds floor(H/R) heads of every request; only the H mod R extra heads differ
    rng = np.random.default_rng(3)
    R, H = 7, 8
    ctx = rng.integers(64, 512, size=16)
    owner, _, load = build_placement(ctx, [0] * 16, R, H)
    extra = np.zeros(R, dtype=np.int64)
    for r in range(16):
        extra[(0 + r) % R] += ctx[r]          # head 7 lands where head 0 did: (7 + r) % 7 == r % 7
    assert (load - (H // R) * ctx.sum()).tolist() == extra.tolist()


def test_incoming_rank_load_is_continued():
    o1, d1, l1 = build_placement([4, 6], [1, 1], 3, 2, rank_load=[5, 0, 7])
    assert d1.tolist() == [1, 0] and l1.tolist() == [17, 8, 7]


def test_negative_rotation_wraps_like_mathematical_mod():
    owner, _, _ = build_placement([1], [0], 5, 3, rot=[-2])
    assert owner[0].tolist() == [3, 4, 0]


def test_rejects_bad_input():
    with pytest.raises(ValueError):
        build_placement([0], [0], 3, 2)
    with pytest.raises(ValueError):
        build_placement([1], [2], 3, 2)
    with pytest.raises(ValueError):
        build_placement([1], [0], 0, 2)
