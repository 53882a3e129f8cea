"""GPU parity of the sweep over a list cut into equal runs of pages (fs_build_worklist_units +
fs_decode_attention_units, through the C ABI) against the CPU oracle.

Bar: lists bit-exact; fp32 outputs within 2e-3 abs + 1e-2 rel of the fp64 oracle, LSE within 1e-3.  The cuts
differ from the chunked list's, so against the other sweeps the results agree to rounding, not bit for bit;
two launches on the same list must agree bit for bit.  Every input is seeded and synthetic.
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

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import test_gpu_parity as TD      # noqa: E402  (helper: check_merge_in_sweep)

pytestmark = pytest.mark.gpu

ABS_TOL, REL_TOL, LSE_TOL = 2e-3, 1e-2, 1e-3


def say(msg):
    print(f"[units] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", autouse=True)
def _lib():
    if not os.path.exists(fs.library_path()):
        raise RuntimeError("libfailsafe.so is not built: GPU tests never fall back to anything else")
    fs.load_library()


def check(out, lse, ref_o, ref_l, what):
    out = np.asarray(out, dtype=np.float64); lse = np.asarray(lse, dtype=np.float64)
    assert np.isfinite(out).all() and np.isfinite(lse).all(), f"{what}: non-finite output"
    err = np.abs(out - ref_o)
    worst = float((err / (ABS_TOL + REL_TOL * np.abs(ref_o))).max()) if err.size else 0.0
    lerr = float(np.abs(lse - ref_l).max()) if lse.size else 0.0
    say(f"{what}: max err/tol {worst:.3f}, lse err {lerr:.2e}")
    assert worst <= 1.0, f"{what}: output outside 2e-3 + 1e-2*|ref| (worst ratio {worst})"
    assert lerr <= LSE_TOL, f"{what}: lse off by {lerr}"


def run_units(w, q, rank, n_units, owner, o_owner=None):
    """Build rank's list with the library, compare it with the oracle's byte for byte, run the kernels."""
    sh = fs.FsShape(w["n_req"], w["n_q_heads"], w["n_kv_heads"], 128, 16, w["n_ranks"])
    items, pairs, unit_indptr, chunk_indptr = fs.fs_build_worklist_units(sh, w["ctx_len"], owner, rank, n_units)
    oi, op, ou, oc = oracle.build_worklist_units(w["ctx_len"], owner if o_owner is None else o_owner, rank, n_units,
                                                 w["n_q_heads"], w["n_kv_heads"])
    assert items.view(np.int32).reshape(-1, 8).tobytes() == oi.tobytes() and unit_indptr.tobytes() == ou.tobytes()
    assert chunk_indptr.tobytes() == oc.tobytes() and pairs.view(np.int32).reshape(-1, 4).tobytes() == op.tobytes()
    kv = make_kv_pool(w["seed"], op[:, :2] if len(op) else np.zeros((0, 2)), w["ctx_len"], kv_dtype=w["kv_dtype"])
    ds = DeviceShare(sh, q, kv, w["sm_scale"])
    ds.set_worklist_units(items, pairs, unit_indptr, chunk_indptr)
    # from launch records first (item order, one workgroup per unit), then from the items: the same bits
    rec = fs.fs_build_launch_records(sh, items, None, chunk_indptr, kv["page_indptr"], kv["page_ids"])
    want = oracle.build_launch_records(oi, None, oc, kv["page_indptr"], kv["page_ids"], w["n_q_heads"] // w["n_kv_heads"])
    assert rec.view(np.int32).reshape(-1, 16).tobytes() == want.tobytes()
    if len(items):
        ds.set_records(rec)
        ds.run_records(units=True)
        torch.cuda.synchronize()
        from_records = [ds.out.clone(), ds.lse.clone(), ds.part_o.clone(), ds.part_lse.clone()]
        # and with the split pairs merged inside the sweep (pair counters handed over): the same final bits
        TD.check_merge_in_sweep(ds, from_records[:2], True, f"units={n_units} rank {rank}")
        for a, b in zip(from_records[2:], (ds.part_o, ds.part_lse)):
            assert (torch.isnan(a) == torch.isnan(b)).all() and torch.equal(torch.nan_to_num(a), torch.nan_to_num(b)), \
                "merging inside the sweep changed the partial rows"
        for t in (ds.part_o, ds.part_lse, ds.out, ds.lse):
            t.fill_(float("nan"))
    ds.run_units()
    torch.cuda.synchronize()
    if len(items):
        for a, b in zip(from_records, (ds.out, ds.lse, ds.part_o, ds.part_lse)):
            assert torch.equal(a, b, ) or (torch.isnan(a) == torch.isnan(b)).all() and torch.equal(torch.nan_to_num(a), torch.nan_to_num(b)), \
                "the records call and the items call differ"
    return ds, kv, op, oi, chunk_indptr


def partial_rows_of_split_pairs(ds, chunk_indptr):
    counts = np.diff(chunk_indptr)
    return torch.from_numpy(np.repeat(np.repeat(counts > 1, counts), ds.group)).to(ds.device)


@pytest.mark.parametrize("n_units", [1, 3, 20, 512, 100000])
def test_small_batches_every_rank(n_units):
    """Tiny and ragged batches with every relation of units to pages (one unit for everything, fewer units than
    pairs, a page per unit): every rank's share against the oracle, the items' partial rows against the
    oracle's per-item attention, the rows of all ranks gathered against unsharded attention."""
    for cfg_id, kw in ((0, {}), (1, dict(n_req=40, max_len=2500))):
        w = make_requests(cfg_id, **kw)
        B, Hq, Hkv, G = w["n_req"], w["n_q_heads"], w["n_kv_heads"], w["group"]
        q = make_q(w["seed"], B, Hq, 128)
        sh = fs.FsShape(B, Hq, Hkv, 128, 16, w["n_ranks"])
        owner, _, _ = fs.fs_build_placement(sh, w["ctx_len"], w["mode"])
        full_o = np.full((B, Hq, 128), np.nan); full_l = np.full((B, Hq), np.nan)
        for k in range(w["n_ranks"]):
            ds, kv, op, oi, chunk_indptr = run_units(w, q, k, n_units, owner)
            if len(op) == 0:
                continue
            ref_o, ref_l = oracle.decode_attention_pairs(q, kv, op, Hq, G, w["sm_scale"], workers=8)
            out, lse = ds.out.cpu().numpy(), ds.lse.cpu().numpy()
            check(out, lse, ref_o, ref_l, f"cfg{cfg_id} units={n_units} rank {k} ({len(oi)} items, {len(op)} pairs)")
            split = partial_rows_of_split_pairs(ds, chunk_indptr)
            if split.any():
                po, pl = oracle.decode_attention_items(q, kv, oi, G, w["sm_scale"], workers=8)
                m = split.cpu().numpy()
                check(ds.part_o.cpu().numpy()[m], ds.part_lse.cpu().numpy()[m], po[m], pl[m], f"cfg{cfg_id} units={n_units} rank {k} partial rows")
            assert torch.isnan(ds.part_lse[~split]).all(), "a pair that is one item wrote partial rows"
            for p, (r, h, L, _n) in enumerate(op):
                full_o[r, h * G:(h + 1) * G] = out[p * G:(p + 1) * G]
                full_l[r, h * G:(h + 1) * G] = lse[p * G:(p + 1) * G]
        all_pairs = np.array([(r, h) for r in range(B) for h in range(Hkv)])
        kv_all = make_kv_pool(w["seed"], all_pairs, w["ctx_len"])
        un_o, un_l = oracle.unsharded_attention(q, kv_all, w["ctx_len"], Hq, Hkv, w["sm_scale"])
        check(full_o, full_l, un_o, un_l, f"cfg{cfg_id} units={n_units}: all ranks gathered vs unsharded")


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (8, 4), (12, 4), (64, 8), (32, 2)])
def test_group_sizes_and_ragged_lengths(Hq, Hkv, kv_dtype):
    lens = [1, 2, 15, 16, 17, 31, 33, 47, 48, 64, 65, 127, 128, 129, 255, 257, 300, 511, 513, 700, 1000, 1025]
    w = make_requests(0, n_req=len(lens))
    w.update(n_q_heads=Hq, n_kv_heads=Hkv, group=Hq // Hkv, n_ranks=2, ctx_len=np.array(lens, dtype=np.int32), kv_dtype=kv_dtype)
    q = make_q(w["seed"] + 3, len(lens), Hq, 128)
    sh = fs.FsShape(len(lens), Hq, Hkv, 128, 16, 2)
    owner, _, _ = fs.fs_build_placement(sh, w["ctx_len"], w["mode"])
    for n_units in (5, 64):
        ds, kv, op, oi, chunk_indptr = run_units(w, q, 1, n_units, owner)
        ref_o, ref_l = oracle.decode_attention_pairs(q, kv, op, Hq, Hq // Hkv, w["sm_scale"], workers=8)
        check(ds.out.cpu().numpy(), ds.lse.cpu().numpy(), ref_o, ref_l, f"{kv_dtype} G={Hq // Hkv} units={n_units}")


def _full(cfg_id, rank, kv_dtype=None, **req_kw):
    w = make_requests(cfg_id, **req_kw)
    if kv_dtype:
        w["kv_dtype"] = kv_dtype
    q = make_q(w["seed"], w["n_req"], w["n_q_heads"], 128)
    sh = fs.FsShape(w["n_req"], w["n_q_heads"], w["n_kv_heads"], 128, 16, w["n_ranks"])
    owner, _, _ = fs.fs_build_placement(sh, w["ctx_len"], w["mode"])
    o_owner, _, _ = oracle.build_placement(w["ctx_len"], w["mode"], w["n_ranks"], w["n_kv_heads"])
    n_units = 2 * torch.cuda.get_device_properties(0).multi_processor_count       # what bench.py --units 0 launches
    what = f"cfg{cfg_id}{' ' + str(req_kw) if req_kw else ''}{' held as ' + kv_dtype if kv_dtype else ''} rank {rank}, {n_units} units"
    say(f"{what}: generating pool")
    ds, kv, op, oi, chunk_indptr = run_units(w, q, rank, n_units, owner, o_owner)
    say(f"{what}: {len(op)} pairs, {len(oi)} items, {ds.kv_bytes / 1e6:.1f} MB of K+V")
    ref_o, ref_l = oracle.decode_attention_pairs(q, kv, op, w["n_q_heads"], w["group"], w["sm_scale"],
                                                 workers=min(16, len(os.sched_getaffinity(0))))
    check(ds.out.cpu().numpy(), ds.lse.cpu().numpy(), ref_o, ref_l, f"{what}, all {len(op)} pairs")
    first = [t.clone() for t in (ds.out, ds.lse)]
    for rep in range(3):                       # same list, same bits
        ds.out.fill_(float("nan")); ds.lse.fill_(float("nan")); ds.part_o.fill_(float("nan"))
        ds.run_units()
        torch.cuda.synchronize()
        assert torch.equal(ds.out, first[0]) and torch.equal(ds.lse, first[1]), f"{what}: launch {rep} differs from the first"


def test_config1_full_size_every_pair():
    _full(1, 0)


def test_config2_full_size_every_pair():
    _full(2, 0)


def test_config4_fp8_full_size_every_pair():
    _full(4, 0)


def test_config2_held_as_fp8_full_size_every_pair():
    _full(2, 0, kv_dtype="fp8")


@pytest.mark.parametrize("rank", range(5))
@pytest.mark.parametrize("variant", ["seeded", "forced_tail"])
def test_config3_every_rank_every_pair(variant, rank):
    _full(3, rank, **(dict(force_first_len=131072) if variant == "forced_tail" else {}))
