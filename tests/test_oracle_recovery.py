"""Pins for the oracle's recovery planner (Section 3.2 of the paper)."""
import json
import os

import numpy as np
import pytest

from oracle import build_placement_hybrid_heads
from oracle.recovery import plan_ffn_reload, plan_kv_reload, replace_failed_gpu

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _mask(n, *dead):
    return [g not in dead for g in range(n)]


def _fig5():
    with open(os.path.join(GOLD, "fig5_on_demand_recovery.json")) as f:
        return json.load(f)


def test_fig5_ffn_shards():
    g = _fig5()
    new_owner, n_load = plan_ffn_reload(g["shard_owner_tp4"], _mask(g["n_gpus"], g["failed"]))
    assert n_load.tolist() == g["on_demand_shards_loaded_per_gpu"]
    assert np.bincount(new_owner, minlength=4).tolist() == g["on_demand_shards_held_per_gpu"]
    # nobody's own shard moved, only the lost ones found a new home
    for s, (a, b) in enumerate(zip(g["shard_owner_tp4"], new_owner)):
        assert (a == b) != (s in g["lost_shards"])
    # the naive fallback the figure contrasts: contiguous TP3 re-shard, every GPU loads what it lacks
    S, R1 = g["n_ffn_shards"], g["n_gpus"] - 1
    naive = [0] * g["n_gpus"]
    for k in range(R1):
        need = set(range(k * S // R1, (k + 1) * S // R1))
        have = {s for s, o in enumerate(g["shard_owner_tp4"]) if o == k}
        naive[k] = len(need - have)
    assert naive == g["naive_contiguous_tp3_shards_loaded_per_gpu"]
    assert set(range(8, 12)) - {8} == set(g["lost_shards"])          # the last GPU loads FFN 9, 10, 11
    assert n_load.sum() == 3 < sum(naive) == 6 and n_load.max() == 1 < max(naive) == 3


def test_fig5_kv_only_the_lost_head_moves_and_spreads_over_the_survivors():
    g = _fig5()
    B, H, L = 9, g["n_kv_heads"], 100
    ctx = [L] * B
    old_owner = np.tile(np.array(g["head_owner_tp4"]), (B, 1))
    new_owner, new_dp, dload = replace_failed_gpu(ctx, old_owner, [-1] * B, _mask(g["n_gpus"], g["failed"]))
    assert (new_owner[:, :3] == old_owner[:, :3]).all()               # heads 0..2 stay where they are
    assert new_owner[:, g["lost_head"]].tolist() == [0, 1, 2] * 3     # head 3 becomes DP work, request by request
    reload, reuse = plan_kv_reload(ctx, old_owner, new_owner, _mask(g["n_gpus"], g["failed"]))
    assert reload.tolist() == [3 * L, 3 * L, 3 * L, 0] and reuse.tolist() == [B * L] * 3 + [0]
    assert dload.tolist() == reload.tolist()


def test_eight_to_seven_lost_head_is_evenly_reloaded():
    # 8 KV heads on 8 GPUs, one fails: 64 equal requests reload the lost head on 7 survivors, 9 or 10 each
    B, L = 64, 512
    old_owner = np.tile(np.arange(8), (B, 1))
    for failed in (0, 3, 7):
        new_owner, new_dp, _ = replace_failed_gpu([L] * B, old_owner, [-1] * B, _mask(8, failed))
        reload, reuse = plan_kv_reload([L] * B, old_owner, new_owner, _mask(8, failed))
        live = [g for g in range(8) if g != failed]
        assert reload[failed] == 0 and reload.sum() == B * L
        assert sorted(set((reload[live] // L).tolist())) == [9, 10]
        assert reuse[live].tolist() == [B * L] * 7


def test_failing_the_last_gpu_equals_a_fresh_hybrid_placement():
    # survivors 0..6 keep heads 0..6; head 7 is the replicated head of hybrid attention on 7 workers
    rng = np.random.default_rng(3)
    ctx = rng.integers(1, 5000, size=40)
    old_owner, _, _, _ = build_placement_hybrid_heads(ctx, 8, 8)           # plain TP-8
    new_owner, new_dp, dload = replace_failed_gpu(ctx, old_owner, [-1] * 40, _mask(8, 7))
    fresh_owner, fresh_dp, _, fresh_dload = build_placement_hybrid_heads(ctx, 7, 8)
    assert new_owner.tolist() == fresh_owner.tolist() and new_dp.tolist() == fresh_dp.tolist()
    assert dload[:7].tolist() == fresh_dload.tolist()
    # failing another GPU: a fresh placement renumbers the workers and moves far more than was lost
    survivors = [g for g in range(8) if g != 2]
    fresh_phys = np.array(survivors)[fresh_owner]
    reload_fresh, _ = plan_kv_reload(ctx, old_owner, fresh_phys, _mask(8, 2))
    keep_owner, _, _ = replace_failed_gpu(ctx, old_owner, [-1] * 40, _mask(8, 2))
    reload_keep, _ = plan_kv_reload(ctx, old_owner, keep_owner, _mask(8, 2))
    # heads 0, 1 stay; heads 2..6 slide from GPUs 2..6 to GPUs 3..7; head 7 stays only where it is routed to GPU 7
    assert reload_fresh.sum() == 5 * ctx.sum() + ctx[fresh_phys[:, 7] != 7].sum()
    assert reload_keep.sum() == ctx.sum() < reload_fresh.sum()


def test_second_failure_keeps_dp_ranks_and_reroutes_orphans():
    # 8 heads on 7 GPUs (hybrid: 7 TP heads + 1 DP head), GPU 4 fails
    rng = np.random.default_rng(9)
    ctx = rng.integers(1, 3000, size=30)
    old_owner, old_dp, _, old_dload = build_placement_hybrid_heads(ctx, 7, 8)
    new_owner, new_dp, dload = replace_failed_gpu(ctx, old_owner, old_dp, _mask(7, 4), dp_load=old_dload * (np.arange(7) != 4))
    for r in range(30):
        if old_dp[r] != 4:
            assert new_dp[r] == old_dp[r]
            assert new_owner[r].tolist() == [h if h != 4 else old_dp[r] for h in range(7)] + [old_dp[r]]
        else:                                  # both its TP head 4 and its DP head were on the failed GPU
            assert new_dp[r] != 4 and new_owner[r, 4] == new_owner[r, 7] == new_dp[r]
    reload, reuse = plan_kv_reload(ctx, old_owner, new_owner, _mask(7, 4))
    lost = int(ctx.sum()) + int(ctx[old_dp == 4].sum())
    assert reload.sum() == lost and reload[4] == 0 and reuse[4] == 0
    assert reload.sum() + reuse.sum() == 8 * ctx.sum()
    assert (new_owner != 4).all()


@pytest.mark.parametrize("seed", range(25))
def test_kv_diff_by_sets(seed):
    rng = np.random.default_rng(50 + seed)
    n, B, H = int(rng.integers(2, 7)), int(rng.integers(0, 8)), int(rng.integers(1, 6))
    failed = int(rng.integers(0, n))
    live = [g for g in range(n) if g != failed]
    ctx = rng.integers(1, 100, size=B)
    old = rng.integers(0, n, size=(B, H))
    new = np.array(live)[rng.integers(0, n - 1, size=(B, H))] if B else np.zeros((0, H), dtype=int)
    reload, reuse = plan_kv_reload(ctx, old, new, _mask(n, failed))
    held_before = {g: {(r, h) for r in range(B) for h in range(H) if old[r, h] == g} for g in range(n)}
    held_after = {g: {(r, h) for r in range(B) for h in range(H) if new[r, h] == g} for g in range(n)}
    for g in range(n):
        assert reuse[g] == sum(int(ctx[r]) for r, _ in held_after[g] & held_before[g])
        assert reload[g] == sum(int(ctx[r]) for r, _ in held_after[g] - held_before[g])


@pytest.mark.parametrize("S,R", [(56, 8), (12, 4), (30, 6), (13, 5), (7, 3), (100, 7)])
def test_ffn_deal_is_minimal_and_even(S, R):
    owner = [s * R // S for s in range(S)]                       # contiguous shards, as even as S allows
    for failed in range(R):
        new_owner, n_load = plan_ffn_reload(owner, _mask(R, failed))
        lost = owner.count(failed)
        assert n_load.sum() == lost and n_load[failed] == 0      # exactly the lost shards cross PCIe
        held = np.bincount(new_owner, minlength=R)
        live = [g for g in range(R) if g != failed]
        assert held[failed] == 0 and held[live].max() - held[live].min() <= 1
        assert all(a == b for a, b in zip(owner, new_owner) if a != failed)
    if S % R == 0 and (S // R) % (R - 1) == 0:
        assert set(n_load[[g for g in range(R) if g != failed]].tolist()) == {S // R // (R - 1)}


def test_bad_arguments_raise():
    with pytest.raises(ValueError):
        plan_kv_reload([5], [[0]], [[1]], [True, False])   # new owner is the dead GPU
    with pytest.raises(ValueError):
        plan_ffn_reload([0, 1, 5], [True, False, True])
    with pytest.raises(ValueError):
        replace_failed_gpu([5], np.array([[0]]), [-1], [False])


def test_two_faults_one_after_the_other_never_route_to_the_first_dead_gpu():
    ctx = [10] * 12
    owner8 = np.tile(np.arange(8), (12, 1))
    o7, d7, l7 = replace_failed_gpu(ctx, owner8, [-1] * 12, _mask(8, 5))
    o6, d6, l6 = replace_failed_gpu(ctx, o7, d7, _mask(8, 5, 1), dp_load=l7)
    assert set(np.unique(o6)) == {0, 2, 3, 4, 6, 7}
    reload, reuse = plan_kv_reload(ctx, o7, o6, _mask(8, 5, 1))
    assert reload[[1, 5]].tolist() == [0, 0] and reload.sum() == int((o7 == 1).sum()) * 10
    # both at once gives a valid plan as well: everything on the two dead GPUs is reloaded, nothing else
    o6b, _, _ = replace_failed_gpu(ctx, owner8, [-1] * 12, _mask(8, 5, 1))
    reload_b, reuse_b = plan_kv_reload(ctx, owner8, o6b, _mask(8, 5, 1))
    assert reload_b.sum() == 2 * 120 and reuse_b.sum() == 6 * 120
