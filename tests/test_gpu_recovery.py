"""GPU end-to-end check of the recovery plans (Section 3.2 of the paper, Fig. 5): after a GPU fault
the survivors' new shares, run through the kernels, still give every (request, q-head) exactly once
and equal to unsharded attention, and what the plan says is reloaded plus what is kept is what each
survivor then holds.

Bar: maps and lists bit-exact against the oracle; fp32 outputs within 2e-3 abs + 1e-2 rel of the
fp64 oracle; LSE within 1e-3.  Every input is seeded and synthetic.
"""
import os
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2511_14116_amd as fs
from paper_2511_14116_amd.device import DeviceShare
from workloads import make_requests, make_q, make_kv_pool

pytestmark = pytest.mark.gpu

ABS_TOL, REL_TOL, LSE_TOL = 2e-3, 1e-2, 1e-3


def say(msg):
    print(f"[recovery] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", autouse=True)
def _lib():
    if not os.path.exists(fs.library_path()):
        raise RuntimeError("libfailsafe.so is not built: GPU tests never fall back to anything else")
    fs.load_library()


def check(out, lse, ref_o, ref_l, what):
    out = np.asarray(out, dtype=np.float64); lse = np.asarray(lse, dtype=np.float64)
    assert np.isfinite(out).all() and np.isfinite(lse).all(), f"{what}: non-finite or missing output"
    err = np.abs(out - ref_o)
    worst = float((err / (ABS_TOL + REL_TOL * np.abs(ref_o))).max())
    lerr = float(np.abs(lse - ref_l).max())
    say(f"{what}: max err/tol {worst:.3f}, lse err {lerr:.2e}")
    assert worst <= 1.0, f"{what}: output outside 2e-3 + 1e-2*|ref| (worst ratio {worst})"
    assert lerr <= LSE_TOL, f"{what}: lse off by {lerr}"


def run_all_gpus(w, q, owner, alive, chunk, persistent):
    """Every live GPU's share of ``owner`` through the library and the kernels; rows scattered back to
    [B][H_q].  A dead GPU must own nothing.  -> (out, lse, times each (request, q-head) was written,
    KV tokens x heads each GPU holds)."""
    n_gpus = len(alive)
    B, Hq, Hkv, G = w["n_req"], w["n_q_heads"], w["n_kv_heads"], w["group"]
    sh = fs.FsShape(B, Hq, Hkv, 128, 16, n_gpus)
    full_o = np.full((B, Hq, 128), np.nan); full_l = np.full((B, Hq), np.nan)
    written = np.zeros((B, Hq), dtype=np.int64)
    held = np.zeros(n_gpus, dtype=np.int64)
    for k in range(n_gpus):
        items, pairs, sched, indptr = fs.fs_build_worklist(sh, w["ctx_len"], owner, k, chunk)
        oi, op, osch, oind = oracle.build_worklist(w["ctx_len"], owner, k, chunk, Hq, Hkv)
        assert items.view(np.int32).reshape(-1, 8).tobytes() == oi.tobytes() and sched.tobytes() == osch.tobytes()
        assert indptr.tobytes() == oind.tobytes()
        if not alive[k]:
            assert len(items) == 0 and len(pairs) == 0, f"dead GPU {k} still owns work"
            continue
        if len(items) == 0:
            continue
        held[k] = int(op[:, 2].sum())
        kv = make_kv_pool(w["seed"], op[:, :2], w["ctx_len"])
        ds = DeviceShare(sh, q, kv, w["sm_scale"])
        ds.set_worklist(items, pairs, sched, indptr)
        ds.run(persistent=persistent)
        torch.cuda.synchronize()
        out, lse = ds.out.cpu().numpy(), ds.lse.cpu().numpy()
        for p, (r, h, L, _n) in enumerate(op):
            full_o[r, h * G:(h + 1) * G] = out[p * G:(p + 1) * G]
            full_l[r, h * G:(h + 1) * G] = lse[p * G:(p + 1) * G]
            written[r, h * G:(h + 1) * G] += 1
    return full_o, full_l, written, held


def test_two_faults_in_a_row_every_survivor_on_the_gpu():
    """TP-8 with 8 KV heads loses GPU 3, then GPU 6.  After each fault: fs_replace_failed_gpu moves only
    the lost slices (they become data-parallel work of the survivors), fs_plan_kv_reload prices the move,
    every survivor's list runs through the kernels, and the gathered rows equal unsharded attention."""
    w = make_requests(1, n_req=28, max_len=1800)
    B, Hq, Hkv, G = w["n_req"], w["n_q_heads"], w["n_kv_heads"], w["group"]
    n_gpus = 8
    q = make_q(w["seed"], B, Hq, 128)
    ctx = w["ctx_len"]
    sh8 = fs.FsShape(B, Hq, Hkv, 128, 16, n_gpus)
    # before any fault: the paper's head-level placement on 8 workers is uniform TP (one head each)
    owner, dp, load, dload = fs.fs_build_placement_hybrid_heads(sh8, ctx, layer=2)
    ref = oracle.build_placement_hybrid_heads(ctx, n_gpus, Hkv, layer=2)
    for a, b in zip((owner, dp, load, dload), ref):
        assert a.tobytes() == b.tobytes()
    assert (dp == -1).all()

    all_pairs = np.array([(r, h) for r in range(B) for h in range(Hkv)])
    kv_all = make_kv_pool(w["seed"], all_pairs, ctx)
    un_o, un_l = oracle.unsharded_attention(q, kv_all, ctx, Hq, Hkv, w["sm_scale"])

    alive = np.ones(n_gpus, dtype=bool)
    full_o, full_l, written, held = run_all_gpus(w, q, owner, alive, 256, persistent=False)
    assert (written == 1).all() and held.tolist() == load.tolist()
    check(full_o, full_l, un_o, un_l, "before the fault, 8 GPUs gathered vs unsharded")

    for fault, dead in enumerate((3, 6)):
        say(f"fault {fault}: GPU {dead} dies")
        lost_tokens = int(sum(int(ctx[r]) for r in range(B) for h in range(Hkv) if owner[r, h] == dead))
        alive[dead] = False
        new_owner, new_dp, new_dload = fs.fs_replace_failed_gpu(ctx, owner, dp, alive, dload)
        want = oracle.replace_failed_gpu(ctx, owner, dp, alive, dload)
        for a, b in zip((new_owner, new_dp, new_dload), want):
            assert np.array_equal(a, b)
        reload, reuse = fs.fs_plan_kv_reload(ctx, owner, new_owner, alive)
        w_reload, w_reuse = oracle.plan_kv_reload(ctx, owner, new_owner, alive)
        assert np.array_equal(reload, w_reload) and np.array_equal(reuse, w_reuse)
        # only the dead GPU's slices move, and they are spread over the survivors (a request's lost slices go to one
        # GPU, so the survivors' reloads differ by a few requests' slices at most)
        assert int(reload.sum()) == lost_tokens and reload[dead] == 0 and reuse[dead] == 0
        live_reload = reload[alive]
        assert live_reload.max() - live_reload.min() <= int(ctx.max()) * Hkv
        for persistent in (False, True):
            full_o, full_l, written, held = run_all_gpus(w, q, new_owner, alive, 256, persistent)
            assert (written == 1).all(), "a (request, q-head) is missing or computed twice"
            assert np.array_equal(held, reload + reuse), "reload + reuse is not what the survivors hold"
            check(full_o, full_l, un_o, un_l,
                  f"after fault {fault} ({int(alive.sum())} survivors, persistent={persistent}) gathered vs unsharded")
        owner, dp, dload = new_owner, new_dp, new_dload


def test_fresh_placement_after_a_fault_and_its_reload_diff():
    """Where the tensor-parallel share per worker grows (8 heads: 4 survivors of 5 hold two heads each),
    the plan is a fresh head-level placement on the survivors plus the diff.  The survivors' shares of the
    fresh placement run through the kernels and gather to unsharded attention; reload + reuse is what each
    holds."""
    w = make_requests(1, n_req=18, max_len=1500)
    B, Hq, Hkv, G = w["n_req"], w["n_q_heads"], w["n_kv_heads"], w["group"]
    q = make_q(w["seed"], B, Hq, 128)
    ctx = w["ctx_len"]
    n_gpus, dead = 5, 1
    old_owner, old_dp, _, _ = fs.fs_build_placement_hybrid_heads(fs.FsShape(B, Hq, Hkv, 128, 16, n_gpus), ctx, layer=0)
    alive = np.ones(n_gpus, dtype=bool); alive[dead] = False
    live = np.flatnonzero(alive)
    # fresh placement over the 4 survivors, in logical ranks, then renamed to the physical GPU ids
    lo_owner, lo_dp, lo_load, _ = fs.fs_build_placement_hybrid_heads(fs.FsShape(B, Hq, Hkv, 128, 16, len(live)), ctx, layer=0)
    ref = oracle.build_placement_hybrid_heads(ctx, len(live), Hkv, layer=0)
    assert lo_owner.tobytes() == ref[0].tobytes() and lo_load.tobytes() == ref[2].tobytes()
    new_owner = live[lo_owner].astype(np.int32)
    reload, reuse = fs.fs_plan_kv_reload(ctx, old_owner, new_owner, alive)
    w_reload, w_reuse = oracle.plan_kv_reload(ctx, old_owner, new_owner, alive)
    assert np.array_equal(reload, w_reload) and np.array_equal(reuse, w_reuse)
    all_pairs = np.array([(r, h) for r in range(B) for h in range(Hkv)])
    kv_all = make_kv_pool(w["seed"], all_pairs, ctx)
    un_o, un_l = oracle.unsharded_attention(q, kv_all, ctx, Hq, Hkv, w["sm_scale"])
    full_o, full_l, written, held = run_all_gpus(w, q, new_owner, alive, 128, persistent=False)
    assert (written == 1).all()
    assert np.array_equal(held, reload + reuse) and np.array_equal(held[live], lo_load)
    check(full_o, full_l, un_o, un_l, "fresh placement on 4 of 5 GPUs gathered vs unsharded")
