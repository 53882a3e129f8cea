"""Pins for the oracle's head-level hybrid placement (the paper's literal statement)."""
import itertools
import json
import os

import numpy as np
import pytest

from oracle import build_placement, build_placement_hybrid_heads

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_fig3_units_per_gpu():
    with open(os.path.join(GOLD, "fig3_hybrid_4heads_tp3.json")) as f:
        g = json.load(f)
    H, R = g["n_kv_heads"], g["n_ranks"]
    L = 10
    # as routed in the figure
    owner, dp, load, dload = build_placement_hybrid_heads([L] * 3, R, H, route=g["route"])
    assert owner.tolist() == g["hybrid_owner_layer0"] and dp.tolist() == g["route"]
    assert (load // L).tolist() == g["hybrid_units_per_rank_equal_lengths"]
    assert (dload // L).tolist() == [1, 1, 1]
    # the load-aware router reaches the same routing by itself for equal lengths
    owner2, dp2, load2, _ = build_placement_hybrid_heads([L] * 3, R, H)
    assert owner2.tolist() == owner.tolist() and dp2.tolist() == dp.tolist()
    # naive non-uniform TP: contiguous split of 4 heads over 3 GPUs, every request on every GPU
    naive = [len(x) for x in np.array_split(np.arange(H), R)]
    assert naive == g["naive_heads_per_rank"]
    assert [n * 3 for n in naive] == g["naive_units_per_rank_equal_lengths"]
    # idle time removed: the slowest GPU does 4 units instead of 6
    assert max(g["naive_units_per_rank_equal_lengths"]) / (load.max() // L) == 1.5


def test_eight_heads_on_seven_workers_as_in_the_text():
    # Section 3.1: seven TP workers get one head each, the eighth head is replicated and run DP
    rng = np.random.default_rng(0)
    ctx = rng.integers(1, 4000, size=50)
    owner, dp, load, dload = build_placement_hybrid_heads(ctx, 7, 8)
    for r in range(50):
        assert owner[r, :7].tolist() == list(range(7))          # layer 0: head h on worker h
        assert owner[r, 7] == dp[r] and 0 <= dp[r] < 7
    assert (load - dload).tolist() == [int(ctx.sum())] * 7        # the TP part is perfectly even
    assert dload.sum() == ctx.sum()
    # and with eight workers it is plain TP-8: nothing left over
    owner8, dp8, load8, dload8 = build_placement_hybrid_heads(ctx, 8, 8)
    assert (dp8 == -1).all() and dload8.sum() == 0 and load8.tolist() == [int(ctx.sum())] * 8
    assert owner8[0].tolist() == list(range(8))


def test_layer_rotation_moves_the_tp_heads_cyclically():
    owner, _, _, _ = build_placement_hybrid_heads([5], 3, 7, layer=0)
    owner1, _, _, _ = build_placement_hybrid_heads([5], 3, 7, layer=1)
    assert owner[0, :6].tolist() == [0, 1, 2, 0, 1, 2] and owner1[0, :6].tolist() == [1, 2, 0, 1, 2, 0]
    for layer in range(6):
        o, _, load, _ = build_placement_hybrid_heads([5], 3, 7, layer=layer, route=[0])
        assert np.bincount(o[0, :6], minlength=3).tolist() == [2, 2, 2]


def test_single_replicated_head_is_dp_attention():
    # the DP-attention design for MLA models: one head, duplicated on all GPUs, requests spread by load
    ctx = [5, 3, 9, 1, 1, 4]
    owner, dp, load, dload = build_placement_hybrid_heads(ctx, 3, 1)
    assert dp.tolist() == [0, 1, 2, 1, 1, 0] and owner[:, 0].tolist() == dp.tolist()
    assert load.tolist() == dload.tolist() == [9, 5, 9]
    # same routing as the request-level builder with every request DP
    _, dp_b, load_b = build_placement(ctx, [1] * 6, 3, 1)
    assert dp_b.tolist() == dp.tolist() and load_b.tolist() == load.tolist()


def test_router_looks_at_dp_work_only():
    # incoming total load is lopsided, DP load is not: the router must ignore the former
    owner, dp, load, dload = build_placement_hybrid_heads([7], 3, 4, rank_load=[100, 0, 0], dp_load=[0, 5, 5])
    assert dp.tolist() == [0] and dload.tolist() == [7, 5, 5] and load.tolist() == [114, 7, 7]


def test_list_scheduling_invariant_on_dp_load():
    rng = np.random.default_rng(4)
    R, H = 5, 8          # 5 TP heads, 3 left over
    ctx = rng.integers(1, 30000, size=200)
    prev = np.zeros(R, dtype=np.int64)
    for n in range(1, 201):
        _, dp, _, dload = build_placement_hybrid_heads(ctx[:n], R, H)
        assert dp[n - 1] == int(np.argmin(prev))
        assert dload.max() - dload.min() <= max(prev.max() - prev.min(), 3 * int(ctx[n - 1]))
        prev = dload


def _brute(ctx, R, H, layer, route):
    held = {k: [] for k in range(R)}
    dp_held = {k: [] for k in range(R)}
    n_tp = (H // R) * R
    for r, L in enumerate(ctx):
        for h in range(n_tp):
            held[(h + layer) % R].append((r, h))
        if n_tp < H:
            if route is None:
                sums = [sum(ctx[rr] for rr, _ in dp_held[k]) for k in range(R)]
                k = sums.index(min(sums))
            else:
                k = route[r]
            for h in range(n_tp, H):
                held[k].append((r, h)); dp_held[k].append((r, h))
    return held


def test_brute_force_enumeration_tiny():
    n = 0
    for R in range(1, 5):
        for H in range(1, 7):
            for ctx in ([1], [3, 1], [2, 2, 5], [4, 1, 1, 1]):
                for layer in (0, 1, 5):
                    for route in (None, [(2 * r + 1) % R for r in range(len(ctx))]):
                        owner, dp, load, dload = build_placement_hybrid_heads(ctx, R, H, layer=layer, route=route)
                        held = _brute(ctx, R, H, layer, route)
                        for k in range(R):
                            got = sorted((r, h) for r in range(len(ctx)) for h in range(H) if owner[r, h] == k)
                            assert got == sorted(held[k])
                            assert load[k] == sum(ctx[r] for r, _ in held[k])
                        n += 1
    assert n > 500


def test_rejects_bad_input():
    with pytest.raises(ValueError):
        build_placement_hybrid_heads([0], 3, 4)
    with pytest.raises(ValueError):
        build_placement_hybrid_heads([1], 3, 4, route=[3])
    with pytest.raises(ValueError):
        build_placement_hybrid_heads([1], 0, 4)
