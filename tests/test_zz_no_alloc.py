"""The entry point that allocates nothing (fs_decode_attention_fused_static: counters and partial rows in a
fixed array inside the library) against fs_decode_attention_fused with caller-held buffers, through the C ABI.

Two calls in a row on one GPU share the library's array: a long split list first (persistent sweep, thousands
of partial rows), then a smaller one (one workgroup per item, fewer rows), nothing cleared by the caller in
between.  Same kernels and the same order of sums, so the bar is the same bits; the second list is also held
against the CPU oracle (2e-3 abs + 1e-2 rel, LSE within 1e-3).  Every input is seeded and synthetic.
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


def say(msg):
    print(f"[no-alloc] {msg}", flush=True)
    sys.stdout.flush()


def _share(cfg_id, n_req, max_len, chunk, rank=0):
    w = make_requests(cfg_id, n_req=n_req, max_len=max_len)
    sh = fs.FsShape(w["n_req"], w["n_q_heads"], w["n_kv_heads"], 128, 16, w["n_ranks"])
    q = make_q(w["seed"], w["n_req"], w["n_q_heads"], 128)
    owner, _, _ = fs.fs_build_placement(sh, w["ctx_len"], w["mode"])
    items, pairs, sched, indptr = fs.fs_build_worklist(sh, w["ctx_len"], owner, rank, chunk)
    kv = make_kv_pool(w["seed"], np.stack([pairs["req"], pairs["kv_head"]], axis=1), w["ctx_len"], kv_dtype=w["kv_dtype"])
    ds = DeviceShare(sh, q, kv, w["sm_scale"])
    ds.set_worklist(items, pairs, sched, indptr)
    return w, q, kv, pairs, ds


def _static(ds):
    fs.fs_decode_attention_fused_static(ds.shape, ds.view, ds.items, ds.sched, ds.n_items, ds.chunk_indptr, ds.n_pairs,
                                        ds.out, ds.lse, torch.cuda.current_stream().cuda_stream)


def test_static_scratch_entry_point_two_calls_in_a_row():
    if not os.path.exists(fs.library_path()):
        raise RuntimeError("libfailsafe.so is not built: GPU tests never fall back to anything else")
    fs.load_library()
    # first call: a long list (persistent sweep from 1024 items on), most pairs split
    w1, q1, kv1, pairs1, big = _share(1, n_req=200, max_len=4000, chunk=128)
    # second call: a smaller list (one workgroup per item), some pairs split, some not
    w2, q2, kv2, pairs2, small = _share(1, n_req=24, max_len=900, chunk=256, rank=1)
    say(f"first list {big.n_items} items / {big.n_pairs} pairs, second {small.n_items} items / {small.n_pairs} pairs")
    assert big.n_items >= 1024 and big.n_items * big.group <= 32768 and big.n_items > big.n_pairs
    assert small.n_items < 1024 and small.n_pairs < small.n_items < big.n_items

    want = []
    for ds in (big, small):
        ds.run_fused(persistent=True)             # caller-held partial rows and counters
        torch.cuda.synchronize()
        want.append((ds.out.clone(), ds.lse.clone()))
        ds.out.fill_(float("nan")); ds.lse.fill_(float("nan"))
    torch.cuda.synchronize()

    _static(big)                                  # two calls in a row on the library's one array
    _static(small)
    torch.cuda.synchronize()
    for name, ds, (o, l) in (("first", big, want[0]), ("second", small, want[1])):
        assert torch.equal(ds.out, o) and torch.equal(ds.lse, l), f"{name} call differs from fs_decode_attention_fused"

    pr = pairs2.view(np.int32).reshape(-1, 4)
    ref_o, ref_l = oracle.decode_attention_pairs(q2, kv2, pr, w2["n_q_heads"], w2["group"], w2["sm_scale"], workers=8)
    out = small.out.cpu().numpy().astype(np.float64); lse = small.lse.cpu().numpy().astype(np.float64)
    assert (np.abs(out - ref_o) <= 2e-3 + 1e-2 * np.abs(ref_o)).all() and (np.abs(lse - ref_l) <= 1e-3).all()

    # once more in the other order, and the long list again after the short one left its rows behind
    for ds in (small, big, small):
        ds.out.fill_(float("nan")); ds.lse.fill_(float("nan"))
    _static(small)
    _static(big)
    torch.cuda.synchronize()
    assert torch.equal(small.out, want[1][0]) and torch.equal(big.out, want[0][0]) and torch.equal(big.lse, want[0][1])

    # a split list beyond the array's 32768 partial rows is refused before anything is launched
    with pytest.raises(fs.FsError) as e:
        fs.fs_decode_attention_fused_static(big.shape, big.view, big.items, big.sched, 32768 // big.group + 1,
                                            big.chunk_indptr, 5, big.out, big.lse, torch.cuda.current_stream().cuda_stream)
    assert e.value.status == fs.FS_ECAPACITY and "32768" in str(e.value)
    torch.cuda.synchronize()


def test_static_scratch_entry_point_with_an_fp8_cache():
    """The same entry point over fp8 K/V (one workgroup per item; the partial rows of split pairs in the library's
    array): two calls in a row, the second smaller, the bits of fs_decode_attention_fused, and the oracle's values."""
    fs.load_library()
    w1, q1, kv1, pairs1, big = _share(4, n_req=120, max_len=2048, chunk=256)
    w2, q2, kv2, pairs2, small = _share(4, n_req=30, max_len=700, chunk=128, rank=2)
    assert w1["kv_dtype"] == "fp8" and big.n_items > big.n_pairs and small.n_pairs < small.n_items < big.n_items
    say(f"fp8: first list {big.n_items} items / {big.n_pairs} pairs, second {small.n_items} items / {small.n_pairs} pairs")
    want = []
    for ds in (big, small):
        ds.run_fused(persistent=True)
        torch.cuda.synchronize()
        want.append((ds.out.clone(), ds.lse.clone()))
        ds.out.fill_(float("nan")); ds.lse.fill_(float("nan"))
    _static(big)
    _static(small)
    torch.cuda.synchronize()
    for name, ds, (o, l) in (("first", big, want[0]), ("second", small, want[1])):
        assert torch.equal(ds.out, o) and torch.equal(ds.lse, l), f"{name} call differs from fs_decode_attention_fused"
    pr = pairs2.view(np.int32).reshape(-1, 4)
    ref_o, ref_l = oracle.decode_attention_pairs(q2, kv2, pr, w2["n_q_heads"], w2["group"], w2["sm_scale"], workers=8)
    out = small.out.cpu().numpy().astype(np.float64); lse = small.lse.cpu().numpy().astype(np.float64)
    assert (np.abs(out - ref_o) <= 2e-3 + 1e-2 * np.abs(ref_o)).all() and (np.abs(lse - ref_l) <= 1e-3).all()
