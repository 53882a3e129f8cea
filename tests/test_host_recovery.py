"""The C++ recovery planner against the oracle, value for value (no GPU needed)."""
import json
import os

import numpy as np
import pytest

import oracle
import paper_2511_14116_amd as fs
from oracle.recovery import plan_ffn_reload, plan_kv_reload, replace_failed_gpu

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _mask(n, *dead):
    return [g not in dead for g in range(n)]


@pytest.fixture(scope="module", autouse=True)
def _lib():
    if not os.path.exists(fs.library_path()):
        from paper_2511_14116_amd.build import build
        build(verbose=False)
    return fs.load_library()


def test_fig5_through_the_library():
    with open(os.path.join(GOLD, "fig5_on_demand_recovery.json")) as f:
        g = json.load(f)
    new_owner, n_load = fs.fs_plan_ffn_reload(g["shard_owner_tp4"], _mask(g["n_gpus"], g["failed"]))
    assert n_load.tolist() == g["on_demand_shards_loaded_per_gpu"]
    assert np.bincount(new_owner, minlength=4).tolist() == g["on_demand_shards_held_per_gpu"]
    B, L = 9, 100
    old_owner = np.tile(np.array(g["head_owner_tp4"], dtype=np.int32), (B, 1))
    new_owner, new_dp, dload = fs.fs_replace_failed_gpu([L] * B, old_owner, [-1] * B, _mask(g["n_gpus"], g["failed"]))
    assert (new_owner[:, :3] == old_owner[:, :3]).all() and new_owner[:, 3].tolist() == [0, 1, 2] * 3
    reload, reuse = fs.fs_plan_kv_reload([L] * B, old_owner, new_owner, _mask(g["n_gpus"], g["failed"]))
    assert reload.tolist() == [300, 300, 300, 0] and reuse.tolist() == [900, 900, 900, 0]


@pytest.mark.parametrize("seed", range(40))
def test_planner_matches_oracle(seed):
    rng = np.random.default_rng(2000 + seed)
    n = int(rng.integers(2, 9))
    alive = rng.integers(0, 2, size=n).astype(bool)
    alive[int(rng.integers(0, n))] = True
    B, H = int(rng.integers(0, 30)), int(rng.integers(1, 9))
    ctx = rng.integers(1, 9000, size=B).astype(np.int32)
    old = rng.integers(0, n, size=(B, H)).astype(np.int32)
    old_dp = rng.integers(-1, n, size=B).astype(np.int32)
    dload = rng.integers(0, 50000, size=n)
    want = replace_failed_gpu(ctx, old, old_dp, alive, dload)
    got = fs.fs_replace_failed_gpu(ctx, old, old_dp, alive, dload)
    for a, b in zip(got, want):
        assert np.array_equal(a, b)
    w_reload, w_reuse = plan_kv_reload(ctx, old, want[0], alive)
    g_reload, g_reuse = fs.fs_plan_kv_reload(ctx, old, got[0], alive)
    assert np.array_equal(g_reload, w_reload) and np.array_equal(g_reuse, w_reuse)
    S = int(rng.integers(0, 80))
    shard_owner = rng.integers(0, n, size=S).astype(np.int32)
    w_new, w_load = plan_ffn_reload(shard_owner, alive)
    g_new, g_load = fs.fs_plan_ffn_reload(shard_owner, alive)
    assert np.array_equal(g_new, w_new) and np.array_equal(g_load, w_load)


def test_70b_shape_eight_to_seven_to_six():
    # the measured 70B-shaped batch: 8 KV heads, 512 requests; TP-8, then one GPU lost, then another
    from workloads import make_requests
    w = make_requests(2)
    ctx = w["ctx_len"]
    B = len(ctx)
    shape = fs.FsShape(B, 64, 8, 128, 16, 8)
    owner8, dp8, load8, dload8 = fs.fs_build_placement_hybrid_heads(shape, ctx, layer=0)
    assert (dp8 == -1).all()
    owner7, dp7, dload7 = fs.fs_replace_failed_gpu(ctx, owner8, dp8, _mask(8, 5))
    reload7, reuse7 = fs.fs_plan_kv_reload(ctx, owner8, owner7, _mask(8, 5))
    live = [g for g in range(8) if g != 5]
    assert reload7.sum() == ctx.sum() and reload7[5] == 0
    assert reload7[live].max() - reload7[live].min() <= ctx.max()          # the lost head spreads evenly
    assert (reuse7[live] == ctx.sum()).all()
    owner6, dp6, dload6 = fs.fs_replace_failed_gpu(ctx, owner7, dp7, _mask(8, 5, 1), dload7)
    reload6, reuse6 = fs.fs_plan_kv_reload(ctx, owner7, owner6, _mask(8, 5, 1))
    live = [g for g in range(8) if g not in (5, 1)]
    assert set(np.unique(owner6)) <= set(live)
    assert reload6.sum() == (owner7 == 1).astype(np.int64).sum(axis=1) @ ctx.astype(np.int64)
    # every rank's share after both faults still feeds the work-list builder unchanged (ids are physical: 8 slots)
    total = 0
    for g in live:
        items, pairs, sched, indptr = fs.fs_build_worklist(shape, ctx, owner6, g, 2048)
        total += int((items["tok_end"] - items["tok_begin"]).sum())
    assert total == 8 * int(ctx.astype(np.int64).sum())


def test_errors():
    with pytest.raises(fs.FsError):
        fs.fs_plan_kv_reload([5], [[0]], [[1]], [1, 0])
    with pytest.raises(fs.FsError):
        fs.fs_plan_ffn_reload([0, 1, 5], [1, 0, 1])
    with pytest.raises(fs.FsError):
        fs.fs_replace_failed_gpu([5], [[0]], [-1], [0])
    with pytest.raises(fs.FsError):
        fs.fs_replace_failed_gpu([0], [[0]], [-1], [0, 1])
