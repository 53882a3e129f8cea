"""The C++ host builders against the oracle, bit for bit (no GPU needed)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
import paper_2511_14116_amd as fs
from workloads import CONFIGS, make_requests

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _lib():
    if not os.path.exists(fs.library_path()):
        from paper_2511_14116_amd.build import build
        build(verbose=False)
    return fs.load_library()


def _shape(B, Hq, Hkv, R, d=128, page=16):
    return fs.FsShape(B, Hq, Hkv, d, page, R)


def _items_as_rows(items):
    return items.view(np.int32).reshape(-1, 8)


def test_library_exports_every_declared_symbol():
    with open(os.path.join(ROOT, "include", "failsafe.h")) as f:
        header = f.read()
    declared = set(re.findall(r"FS_API[^;(]*?\b(fs_[a-z_0-9]+)\s*\(", header))
    assert {"fs_build_placement", "fs_build_placement_hybrid_heads", "fs_build_worklist", "fs_choose_chunk_tokens", "fs_decode_attention",
            "fs_decode_attention_persistent", "fs_decode_attention_fused", "fs_decode_attention_units", "fs_build_worklist_units", "fs_build_launch_records", "fs_decode_attention_records", "fs_pack_kv_slots", "fs_merge_lse", "fs_build_prefill_worklist", "fs_prefill_attention", "fs_prefill_attention_fused", "fs_choose_prefill_chunk",
            "fs_route_request", "fs_route_requests", "fs_schedule_prefill", "fs_plan_kv_reload", "fs_replace_failed_gpu", "fs_plan_ffn_reload", "fs_kv_elem_offset", "fs_stream_read_probe", "fs_set_option", "fs_get_option", "fs_last_error",
            "fs_abi_version"} <= declared
    lib = C.CDLL(fs.library_path())
    for name in declared:
        assert hasattr(lib, name), name
    assert fs.fs_abi_version() == 4


def test_struct_sizes_match_the_header():
    assert C.sizeof(fs.FsShape) == 24 and fs.ITEM_DTYPE.itemsize == 32 and fs.PAIR_DTYPE.itemsize == 16
    assert C.sizeof(fs.FsKvView) == 96


@pytest.mark.parametrize("cfg_id", sorted(CONFIGS))
def test_configs_bit_exact(cfg_id):
    w = make_requests(cfg_id)
    sh = _shape(w["n_req"], w["n_q_heads"], w["n_kv_heads"], w["n_ranks"])
    owner, dp, load = fs.fs_build_placement(sh, w["ctx_len"], w["mode"])
    o_owner, o_dp, o_load = oracle.build_placement(w["ctx_len"], w["mode"], w["n_ranks"], w["n_kv_heads"])
    assert owner.tobytes() == o_owner.tobytes()
    assert dp.tobytes() == o_dp.tobytes() and load.tobytes() == o_load.tobytes()
    ranks = range(w["n_ranks"]) if cfg_id in (0, 3) else [0]
    for k in ranks:
        for chunk in sorted({w["chunk_tokens"], 0, 2048}):
            items, pairs, sched, indptr = fs.fs_build_worklist(sh, w["ctx_len"], owner, k, chunk)
            oi, op, osch, oind = oracle.build_worklist(w["ctx_len"], o_owner, k, chunk,
                                                       w["n_q_heads"], w["n_kv_heads"])
            assert _items_as_rows(items).tobytes() == oi.tobytes()
            assert pairs.view(np.int32).reshape(-1, 4).tobytes() == op.tobytes()
            assert sched.tobytes() == osch.tobytes() and indptr.tobytes() == oind.tobytes()


def test_random_small_cases_bit_exact():
    rng = np.random.default_rng(11)
    for _ in range(300):
        R = int(rng.integers(1, 9)); H = int(rng.integers(1, 9)); G = int(rng.integers(1, 5))
        B = int(rng.integers(0, 12))
        ctx = rng.integers(1, 400, size=B).astype(np.int32)
        mode = (rng.random(B) < 0.4).astype(np.uint8)
        rot = rng.integers(-20, 20, size=B).astype(np.int32) if rng.random() < 0.5 else None
        layer = int(rng.integers(0, 5))
        init = rng.integers(0, 1000, size=R)
        sh = _shape(B, H * G, H, R)
        owner, dp, load = fs.fs_build_placement(sh, ctx, mode, rot=rot, layer=layer, rank_load=init)
        oo, od, ol = oracle.build_placement(ctx, mode, R, H, rot=rot, layer=layer, rank_load=init)
        assert owner.tobytes() == oo.tobytes() and dp.tobytes() == od.tobytes() and load.tobytes() == ol.tobytes()
        k = int(rng.integers(0, R)); chunk = int(rng.choice([0, 16, 32, 128]))
        items, pairs, sched, indptr = fs.fs_build_worklist(sh, ctx, owner, k, chunk)
        oi, op, osch, oind = oracle.build_worklist(ctx, oo, k, chunk, H * G, H)
        assert _items_as_rows(items).tobytes() == oi.tobytes()
        assert pairs.view(np.int32).reshape(-1, 4).tobytes() == op.tobytes()
        assert sched.tobytes() == osch.tobytes() and indptr.tobytes() == oind.tobytes()


def _units_equal(got, want):
    items, pairs, unit_indptr, chunk_indptr = got
    oi, op, ou, oc = want
    return (_items_as_rows(items).tobytes() == oi.tobytes() and pairs.view(np.int32).reshape(-1, 4).tobytes() == op.tobytes()
            and unit_indptr.tobytes() == ou.tobytes() and chunk_indptr.tobytes() == oc.tobytes())


def test_units_list_bit_exact_configs_and_random():
    """fs_build_worklist_units against the oracle's cut, byte for byte: the five batches at full size and drawn
    small cases with every relation of units to pages (one unit, fewer than pairs, more than pages)."""
    for cfg_id in range(5):
        w = make_requests(cfg_id)
        sh = _shape(w["n_req"], w["n_q_heads"], w["n_kv_heads"], w["n_ranks"])
        owner, _, _ = fs.fs_build_placement(sh, w["ctx_len"], w["mode"])
        for k in (range(w["n_ranks"]) if cfg_id in (0, 3) else [0]):
            for n_units in (1, 37, 512, 10 ** 7):
                assert _units_equal(fs.fs_build_worklist_units(sh, w["ctx_len"], owner, k, n_units),
                                    oracle.build_worklist_units(w["ctx_len"], owner, k, n_units, w["n_q_heads"], w["n_kv_heads"]))
    rng = np.random.default_rng(12)
    for _ in range(400):
        R = int(rng.integers(1, 6)); H = int(rng.integers(1, 9)); G = int(rng.integers(1, 5)); B = int(rng.integers(0, 12))
        ctx = rng.integers(1, int(rng.choice([20, 400, 5000])), size=B).astype(np.int32)
        owner = rng.integers(0, R, size=(B, H)).astype(np.int32)
        k = int(rng.integers(0, R)); n_units = int(rng.choice([1, 2, 3, 5, 8, 64, 1000]))
        sh = _shape(B, H * G, H, R)
        assert _units_equal(fs.fs_build_worklist_units(sh, ctx, owner, k, n_units),
                            oracle.build_worklist_units(ctx, owner, k, n_units, H * G, H))
    # errors: no units, a short array
    sh = _shape(2, 4, 2, 2)
    ctx = np.array([40, 20], dtype=np.int32); owner = np.zeros((2, 2), dtype=np.int32)
    with pytest.raises(fs.FsError) as e:
        fs.fs_build_worklist_units(sh, ctx, owner, 0, 0)
    assert e.value.status == fs.FS_EINVAL
    lib = fs.load_library()
    ni, npairs, nu = C.c_int64(0), C.c_int64(0), C.c_int64(0)
    items = np.empty(3, dtype=fs.ITEM_DTYPE); pairs = np.empty(4, dtype=fs.PAIR_DTYPE)
    ui = np.empty(5, dtype=np.int64); ci = np.empty(5, dtype=np.int64)
    i32p = C.POINTER(C.c_int32)
    st = lib.fs_build_worklist_units(C.byref(sh), ctx.ctypes.data_as(i32p), owner.ctypes.data_as(i32p), 0, 4,
                                     items.ctypes.data, 3, pairs.ctypes.data, 4, ui.ctypes.data, 4, ci.ctypes.data,
                                     C.byref(ni), C.byref(npairs), C.byref(nu))
    assert st == fs.FS_ECAPACITY and (ni.value, npairs.value, nu.value) == (7, 4, 4)   # 10 pages in 4 runs of 2-3: three of the cuts fall inside a pair


def test_launch_records_bit_exact_and_errors():
    """fs_build_launch_records against the oracle's records, byte for byte, for chunked lists in launch order and
    equal-run lists in item order; malformed inputs are refused."""
    rng = np.random.default_rng(13)
    assert fs.RECORD_DTYPE.itemsize == 64
    for case in range(120):
        R = int(rng.integers(1, 5)); H = int(rng.integers(1, 9)); G = int(rng.integers(1, 5)); B = int(rng.integers(1, 12))
        ctx = rng.integers(1, int(rng.choice([20, 400, 3000])), size=B).astype(np.int32)
        owner = rng.integers(0, R, size=(B, H)).astype(np.int32)
        k = int(rng.integers(0, R))
        sh = _shape(B, H * G, H, R)
        if case % 2:
            items, pairs, order, ci = fs.fs_build_worklist(sh, ctx, owner, k, int(rng.choice([0, 16, 64, 256])))
        else:
            items, pairs, _u, ci = fs.fs_build_worklist_units(sh, ctx, owner, k, int(rng.choice([1, 3, 9, 200])))
            order = None
        n_pages = -(-pairs["ctx_len"].astype(np.int64) // 16)
        page_indptr = np.concatenate([[0], np.cumsum(n_pages)]).astype(np.int64)
        total = int(page_indptr[-1])
        page_ids = rng.permutation(total + 3)[:total].astype(np.int32)
        for direct in (True, False):
            rec = fs.fs_build_launch_records(sh, items, order, ci, page_indptr, page_ids, direct_rows=direct)
            want = oracle.build_launch_records(_items_as_rows(items), order, ci, page_indptr, page_ids, G, direct_rows=direct)
            assert rec.view(np.int32).reshape(-1, 16).tobytes() == want.tobytes()
    # errors: an order entry out of range, a page table too short for the item
    sh = _shape(2, 4, 2, 1)
    ctx = np.array([40, 20], dtype=np.int32); owner = np.zeros((2, 2), dtype=np.int32)
    items, pairs, sched, ci = fs.fs_build_worklist(sh, ctx, owner, 0, 16)
    page_indptr = np.array([0, 3, 6, 8, 10], dtype=np.int64); page_ids = np.arange(10, dtype=np.int32)
    fs.fs_build_launch_records(sh, items, sched, ci, page_indptr, page_ids)
    bad_order = sched.copy(); bad_order[0] = len(items)
    for args in ((bad_order, page_indptr, page_ids), (sched, page_indptr - np.array([0, 1, 1, 1, 1]), page_ids), (sched, page_indptr, page_ids[:9])):
        with pytest.raises(fs.FsError) as e:
            fs.fs_build_launch_records(sh, items, args[0], ci, args[1], args[2])
        assert e.value.status == fs.FS_EINVAL
    # an item that does not sit at row (chunk_indptr[pair] + chunk) * G, where the merge would look for it
    moved = items.copy(); moved["part_row"][1] += 2
    wrong_chunk = items.copy(); wrong_chunk["chunk"][0] = 3
    for bad in (moved, wrong_chunk):
        with pytest.raises(fs.FsError) as e:
            fs.fs_build_launch_records(sh, bad, sched, ci, page_indptr, page_ids)
        assert e.value.status == fs.FS_EINVAL
        with pytest.raises(ValueError):
            oracle.build_launch_records(_items_as_rows(bad), sched, ci, page_indptr, page_ids, 2)


def test_sched_sort_fallback_path_matches():
    # few items with very different lengths take the comparison sort instead of the counting sort
    ctx = np.array([100000, 7, 100000, 50000], dtype=np.int32)
    sh = _shape(4, 2, 2, 1)
    owner, _, _ = fs.fs_build_placement(sh, ctx, np.zeros(4, np.uint8))
    items, pairs, sched, indptr = fs.fs_build_worklist(sh, ctx, owner, 0, 0)
    _, _, osch, _ = oracle.build_worklist(ctx, owner, 0, 0, 2, 2)
    assert sched.tolist() == osch.tolist() == [0, 1, 4, 5, 6, 7, 2, 3]


def test_error_statuses():
    sh = _shape(1, 4, 2, 3)
    with pytest.raises(fs.FsError) as e:
        fs.fs_build_placement(sh, [0], [0])
    assert e.value.status == fs.FS_EINVAL and "ctx_len" in str(e.value)
    with pytest.raises(fs.FsError) as e:
        fs.fs_build_placement(sh, [5], [3])
    assert e.value.status == fs.FS_EINVAL
    with pytest.raises(fs.FsError):
        fs.fs_build_placement(_shape(1, 4, 2, 0), [5], [0])
    owner = np.zeros((1, 2), np.int32)
    with pytest.raises(fs.FsError) as e:
        fs.fs_build_worklist(sh, [5], owner, 3, 0)
    assert e.value.status == fs.FS_EINVAL
    with pytest.raises(fs.FsError) as e:
        fs.fs_build_worklist(sh, [5], owner, 0, 24)
    assert e.value.status == fs.FS_EINVAL
    with pytest.raises(fs.FsError) as e:
        fs.fs_build_worklist(sh, [5], np.full((1, 2), 7, np.int32), 0, 0)
    assert e.value.status == fs.FS_EINVAL
    # capacity: arrays too small -> FS_ECAPACITY
    small = (np.empty(1, fs.ITEM_DTYPE), np.empty(1, fs.PAIR_DTYPE), np.empty(1, np.int32), np.empty(2, np.int64))
    with pytest.raises(fs.FsError) as e:
        fs.fs_build_worklist(sh, [5], owner, 0, 0, out=small)
    assert e.value.status == fs.FS_ECAPACITY and "2 items" in str(e.value)
    with pytest.raises(fs.FsError):
        fs.fs_set_option("waves_per_group", 3)
    with pytest.raises(fs.FsError):
        fs.fs_set_option("no_such_knob", 1)
    assert fs.fs_get_option("no_such_knob") == -1 and fs.fs_get_option("waves_per_group") in (1, 2, 4)


def test_device_entry_points_validate_before_touching_the_gpu():
    sh = _shape(1, 4, 2, 3)
    kv = fs.FsKvView()
    fs.fs_decode_attention(sh, kv, None, None, 0, None, None)            # empty list: no-op
    fs.fs_merge_lse(None, None, None, 0, 2, 128, None, None)             # no pairs: no-op
    with pytest.raises(fs.FsError) as e:
        fs.fs_decode_attention(sh, kv, None, None, 3, None, None)
    assert e.value.status == fs.FS_EINVAL
    with pytest.raises(fs.FsError) as e:
        fs.fs_decode_attention(_shape(1, 4, 2, 3, d=64), kv, None, None, 3, None, None)
    assert e.value.status == fs.FS_EUNSUPPORTED
    with pytest.raises(fs.FsError) as e:
        fs.fs_decode_attention(_shape(1, 34, 2, 3), kv, None, None, 3, None, None)
    assert e.value.status == fs.FS_EINVAL
    # the persistent form of the sweep checks the same things, plus its counters and the K/V type
    fs.fs_decode_attention_persistent(sh, kv, None, None, 0, None, None, None)       # empty list: no-op
    with pytest.raises(fs.FsError) as e:
        fs.fs_decode_attention_persistent(sh, kv, None, None, 3, None, None, None)
    assert e.value.status == fs.FS_EINVAL
    with pytest.raises(fs.FsError) as e:
        fs.fs_decode_attention_persistent(_shape(1, 4, 2, 3, d=64), kv, None, None, 3, None, None, None)
    assert e.value.status == fs.FS_EUNSUPPORTED
    kv8 = fs.FsKvView(kv_dtype=fs.FS_KV_FP8_E4M3)                   # fp8 K/V is served by every form: the NULL pointers are what is wrong
    with pytest.raises(fs.FsError) as e:
        fs.fs_decode_attention_persistent(sh, kv8, None, None, 3, None, None, None)
    assert e.value.status == fs.FS_EINVAL
    # the fused call: the same checks, and the pair count must fit the list
    fs.fs_decode_attention_fused(sh, kv, None, None, 0, None, 0, None, None, None, None, None)   # empty list: no-op
    for n_items, n_pairs in ((3, 4), (3, -1), (3, 0), (3, 2)):          # too many pairs, negative, none, NULL pointers
        with pytest.raises(fs.FsError) as e:
            fs.fs_decode_attention_fused(sh, kv, None, None, n_items, None, n_pairs, None, None, None, None, None)
        assert e.value.status == fs.FS_EINVAL
    with pytest.raises(fs.FsError) as e:
        fs.fs_decode_attention_fused(_shape(1, 4, 2, 3, d=64), kv, None, None, 3, None, 3, None, None, None, None, None)
    assert e.value.status == fs.FS_EUNSUPPORTED
    fs.fs_decode_attention_units(sh, kv, None, 0, None, 0, None, 0, None, None, None, None)          # empty list: no-op
    for n_items, n_units, n_pairs in ((3, 4, 3), (3, 2, 4), (3, 0, 2), (3, 2, 2)):        # counts that cannot be; NULL pointers
        with pytest.raises(fs.FsError) as e:
            fs.fs_decode_attention_units(sh, kv, None, n_items, None, n_units, None, n_pairs, None, None, None, None)
        assert e.value.status == fs.FS_EINVAL
    with pytest.raises(fs.FsError) as e:
        fs.fs_decode_attention_units(sh, kv8, None, 3, None, 2, None, 2, None, None, None, None)
    assert e.value.status == fs.FS_EINVAL
    fs.fs_decode_attention_records(sh, kv, None, 0, None, 0, None, 0, None, None, None, None, None)  # empty list: no-op
    for n_items, n_units, n_pairs in ((3, 0, 4), (3, 0, 0), (3, 0, 2)):
        with pytest.raises(fs.FsError) as e:
            fs.fs_decode_attention_records(sh, kv, None, n_items, None, n_units, None, n_pairs, None, None, None, None)
        assert e.value.status == fs.FS_EINVAL
    with pytest.raises(fs.FsError) as e:     # pair counters for a sweep that merges nothing
        fs.fs_decode_attention_records(sh, kv, None, 3, None, 0, None, 0, None, None, None, None, pair_counters_dev=64)
    assert e.value.status == fs.FS_EINVAL
    with pytest.raises(fs.FsError) as e:     # claim counters with equal runs: those are not claimed
        fs.fs_decode_attention_records(sh, kv, None, 3, 64, 2, 64, 2, None, None, None, None, claim_dev=64)
    assert e.value.status == fs.FS_EINVAL and "claim_dev" in str(e.value)
    with pytest.raises(fs.FsError) as e:     # claim counters not 8-byte aligned
        fs.fs_decode_attention_records(sh, kv, None, 3, None, 0, 64, 2, None, None, None, None, claim_dev=68)
    assert e.value.status == fs.FS_EINVAL and "claim_dev" in str(e.value)
    fs.fs_pack_kv_slots(None, 4096, None, 4096, 0, fs.FS_KV_BF16, False)                            # no slots: no-op
    for args in ((None, 4096, None, 4096, 3, fs.FS_KV_BF16), (64, 4096, 8192, 100, 3, fs.FS_KV_BF16), (64, 4096, 8192, 4096, 3, 9)):
        with pytest.raises(fs.FsError) as e:
            fs.fs_pack_kv_slots(*args, False)
        assert e.value.status == fs.FS_EINVAL
    # prefill: empty list is a no-op; a tile beyond the kernel's is refused before any launch
    fs.fs_prefill_attention(sh, kv, None, None, 0, 1, None, None)
    with pytest.raises(fs.FsError) as e:
        fs.fs_prefill_attention(sh, kv, None, None, 1, 10 ** 6, None, None)
    assert e.value.status == fs.FS_EINVAL
    # a softmax scale that is not positive, or an unknown statement about V, is refused before any launch
    import torch
    dummy = torch.zeros(64, dtype=torch.uint8).data_ptr()      # any non-NULL, 16-byte aligned address: nothing is launched
    for field, value in (("sm_scale", 0.0), ("sm_scale", -0.1), ("v_range", 7)):
        bad = fs.FsKvView(q=dummy, k_pool=dummy, v_pool=dummy, k_slot_stride=4096, v_slot_stride=4096, page_indptr=dummy,
                          page_ids=dummy, kv_dtype=fs.FS_KV_BF16, sm_scale=0.1)
        setattr(bad, field, value)
        with pytest.raises(fs.FsError) as e:
            fs.fs_prefill_attention(sh, bad, dummy, None, 1, 1, dummy, dummy)
        assert e.value.status == fs.FS_EINVAL and field in str(e.value)
    fs.fs_prefill_attention_fused(sh, kv, None, None, 0, 1, None, 0, None, None, None, None, None)     # empty list: no-op
    for n_items, n_tiles in ((3, 4), (3, 0), (3, 2)):
        with pytest.raises(fs.FsError) as e:
            fs.fs_prefill_attention_fused(sh, kv, None, None, n_items, 1, None, n_tiles, None, None, None, None, None)
        assert e.value.status == fs.FS_EINVAL
    with pytest.raises(fs.FsError) as e:
        fs.fs_merge_lse(None, None, None, 4, 2, 64, None, None)
    assert e.value.status == fs.FS_EUNSUPPORTED
    with pytest.raises(fs.FsError) as e:
        fs.fs_merge_lse(None, None, None, 4, 2, 128, None, None)
    assert e.value.status == fs.FS_EINVAL


def test_slot_orders_are_permutations_with_the_documented_formulas():
    for is_v in (False, True):
        src = fs.slot_permutation(fs.FS_KV_BF16, is_v)
        assert sorted(src.tolist()) == list(range(2048))
    # K: 16-byte pieces (8 consecutive d of one token); lanes (d/8 % 4, tok) of a 64-lane load are contiguous
    assert fs.fs_kv_elem_offset(fs.FS_KV_BF16, 0, 0, 0) == 0
    assert fs.fs_kv_elem_offset(fs.FS_KV_BF16, 0, 1, 0) == 8
    assert fs.fs_kv_elem_offset(fs.FS_KV_BF16, 0, 0, 8) == 128
    assert fs.fs_kv_elem_offset(fs.FS_KV_BF16, 0, 0, 32) == 512
    assert fs.fs_kv_elem_offset(fs.FS_KV_BF16, 0, 15, 127) == 2047
    # V: 4 consecutive tokens of one d sit together
    assert [fs.fs_kv_elem_offset(fs.FS_KV_BF16, 1, t, 0) for t in range(5)] == [0, 1, 2, 3, 128]
    assert fs.fs_kv_elem_offset(fs.FS_KV_BF16, 1, 0, 16) == 4
    assert fs.fs_kv_elem_offset(fs.FS_KV_BF16, 1, 0, 1) == 8
    assert fs.fs_kv_elem_offset(fs.FS_KV_BF16, 1, 0, 32) == 512
    # fp8, K and V alike: 16-byte pieces (16 consecutive d of one token); lanes (d/16 % 4, tok) of a 64-lane load are
    # contiguous, the two halves of d a kilobyte apart
    for is_v in (0, 1):
        assert sorted(fs.slot_permutation(fs.FS_KV_FP8_E4M3, bool(is_v)).tolist()) == list(range(2048))
        assert [fs.fs_kv_elem_offset(fs.FS_KV_FP8_E4M3, is_v, 0, d) for d in (0, 1, 15, 16, 63, 64, 127)] == [0, 1, 15, 256, 783, 1024, 1807]
        assert [fs.fs_kv_elem_offset(fs.FS_KV_FP8_E4M3, is_v, t, 0) for t in (1, 2, 15)] == [16, 32, 240]
        assert fs.fs_kv_elem_offset(fs.FS_KV_FP8_E4M3, is_v, 15, 127) == 2047
    assert fs.fs_kv_elem_offset(fs.FS_KV_BF16, 0, 16, 0) == -1 and fs.fs_kv_elem_offset(7, 0, 0, 0) == -1
    x = np.arange(2 * 2048, dtype=np.uint16).reshape(2, 16, 128)
    y = fs.pack_slots(x, fs.FS_KV_BF16, False)
    assert y[1].reshape(-1)[8] == 2048 + 1 * 128 + 0


def test_bound_calls_fill_caller_arrays_like_the_plain_calls():
    w = make_requests(1)
    sh = _shape(w["n_req"], w["n_q_heads"], w["n_kv_heads"], w["n_ranks"])
    ctx = np.ascontiguousarray(w["ctx_len"], dtype=np.int32)
    mode = np.ascontiguousarray(w["mode"], dtype=np.uint8)
    owner = np.empty((w["n_req"], w["n_kv_heads"]), np.int32); dp = np.empty(w["n_req"], np.int32)
    load = np.zeros(w["n_ranks"], np.int64)
    place = fs.bind_build_placement(sh, ctx, mode, owner, dp, load)
    place()
    o2, d2, l2 = fs.fs_build_placement(sh, ctx, mode)
    assert owner.tobytes() == o2.tobytes() and dp.tobytes() == d2.tobytes() and load.tobytes() == l2.tobytes()
    load.fill(0); place()                       # reusable
    assert load.tobytes() == l2.tobytes()
    items, pairs, sched, indptr = fs.fs_build_worklist(sh, ctx, owner, 2, 512)
    bufs = (np.empty(len(items) + 5, fs.ITEM_DTYPE), np.empty(len(pairs), fs.PAIR_DTYPE),
            np.empty(len(items) + 5, np.int32), np.empty(len(pairs) + 1, np.int64))
    wl = fs.bind_build_worklist(sh, ctx, owner, 2, 512, *bufs)
    wl()
    assert (wl.n_items.value, wl.n_pairs.value) == (len(items), len(pairs))
    assert bufs[0][:len(items)].tobytes() == items.tobytes() and bufs[2][:len(items)].tobytes() == sched.tobytes()
    assert bufs[3].tobytes() == indptr.tobytes()
    with pytest.raises(TypeError):
        fs.bind_build_placement(sh, ctx.astype(np.int64), mode, owner, dp, load)


def test_hybrid_heads_bit_exact_random_and_configs():
    rng = np.random.default_rng(21)
    for trial in range(300):
        R = int(rng.integers(1, 9)); H = int(rng.integers(1, 12)); B = int(rng.integers(0, 14))
        ctx = rng.integers(1, 5000, size=B).astype(np.int32)
        layer = int(rng.integers(-3, 40))
        route = rng.integers(0, R, size=B).astype(np.int32) if rng.random() < 0.4 else None
        init = rng.integers(0, 1000, size=R); dinit = rng.integers(0, 1000, size=R)
        sh = _shape(B, H, H, R)
        got = fs.fs_build_placement_hybrid_heads(sh, ctx, layer=layer, route=route, rank_load=init, dp_load=dinit)
        ref = oracle.build_placement_hybrid_heads(ctx, R, H, layer=layer, route=route, rank_load=init, dp_load=dinit)
        for a, b in zip(got, ref):
            assert a.tobytes() == b.tobytes()
    for cfg_id in (1, 2, 3):
        w = make_requests(cfg_id)
        sh = _shape(w["n_req"], w["n_q_heads"], w["n_kv_heads"], w["n_ranks"])
        for layer in (0, 1, 5):
            got = fs.fs_build_placement_hybrid_heads(sh, w["ctx_len"], layer=layer)
            ref = oracle.build_placement_hybrid_heads(w["ctx_len"], w["n_ranks"], w["n_kv_heads"], layer=layer)
            for a, b in zip(got, ref):
                assert a.tobytes() == b.tobytes()
            # the map feeds the ordinary work-list builder
            items, pairs, sched, indptr = fs.fs_build_worklist(sh, w["ctx_len"], got[0], 0, w["chunk_tokens"])
            oi, op, osch, oind = oracle.build_worklist(w["ctx_len"], ref[0], 0, w["chunk_tokens"], w["n_q_heads"], w["n_kv_heads"])
            assert _items_as_rows(items).tobytes() == oi.tobytes() and sched.tobytes() == osch.tobytes()
    with pytest.raises(fs.FsError) as e:
        fs.fs_build_placement_hybrid_heads(_shape(1, 4, 4, 3), [5], route=[3])
    assert e.value.status == fs.FS_EINVAL
    with pytest.raises(fs.FsError):
        fs.fs_build_placement_hybrid_heads(_shape(1, 4, 4, 3), [0])


def test_chunk_choice_matches_oracle():
    rng = np.random.default_rng(11)
    for case in range(40):
        B, H, R = int(rng.integers(1, 30)), int(rng.integers(1, 5)), int(rng.integers(1, 5))
        ctx = rng.integers(1, 40000, size=B).astype(np.int32)
        owner = rng.integers(0, R, size=(B, H)).astype(np.int32)
        sh = _shape(B, 2 * H, H, R)
        for rank in range(R):
            for max_c, min_c, want in ((2048, 256, 256), (4096, 16, 37), (512, 512, 10 ** 5), (2048, 48, 1), (48, 16, 9)):      # want: slots
                got = fs.fs_choose_chunk_tokens(sh, ctx, owner, rank, max_c, min_c, want)
                assert got == oracle.choose_chunk_tokens(ctx, owner, rank, max_c, min_c, want, H)
                items, _, _, _ = fs.fs_build_worklist(sh, ctx, owner, rank, got[0])
                assert len(items) == got[1]
    sh = _shape(2, 4, 2, 2)
    ctx, owner = np.array([5, 9], dtype=np.int32), np.zeros((2, 2), dtype=np.int32)
    for bad in ((64, 24, 1), (16, 32, 1), (64, 8, 1), (64, 16, 0)):
        with pytest.raises(fs.FsError):
            fs.fs_choose_chunk_tokens(sh, ctx, owner, 0, *bad)
    with pytest.raises(fs.FsError):
        fs.fs_choose_chunk_tokens(sh, ctx, owner, 2, 64, 16, 1)
    with pytest.raises(fs.FsError):
        fs.fs_choose_chunk_tokens(sh, np.array([5, 0], dtype=np.int32), owner, 0, 64, 16, 1)
