"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bar: placement maps and work lists bit-exact; fp32 outputs within 2e-3 abs + 1e-2 rel of the
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
    print(f"[parity] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", autouse=True)
def _lib():
    if not os.path.exists(fs.library_path()):
        raise RuntimeError("libfailsafe.so is not built: GPU tests never fall back to anything else")
    fs.load_library()
    yield
    fs.fs_set_option("waves_per_group", 4)
    fs.fs_set_option("prefetch_pages", 2)


def check(out, lse, ref_o, ref_l, what):
    out = np.asarray(out, dtype=np.float64); lse = np.asarray(lse, dtype=np.float64)
    assert np.isfinite(out).all() and np.isfinite(lse).all(), f"{what}: non-finite output"
    err = np.abs(out - ref_o)
    tol = ABS_TOL + REL_TOL * np.abs(ref_o)
    worst = float((err / tol).max()) if err.size else 0.0
    lerr = float(np.abs(lse - ref_l).max()) if lse.size else 0.0
    say(f"{what}: max err/tol {worst:.3f}, max |err| {float(err.max()) if err.size else 0:.2e}, lse err {lerr:.2e}")
    assert worst <= 1.0, f"{what}: output outside 2e-3 + 1e-2*|ref| (worst ratio {worst})"
    assert lerr <= LSE_TOL, f"{what}: lse off by {lerr}"


def shape_of(w):
    return fs.FsShape(w["n_req"], w["n_q_heads"], w["n_kv_heads"], w["head_dim"], w["page_tokens"], w["n_ranks"])


def run_rank(w, q, rank, chunk, owner, interleave=True, use_sched=True, pairs_subset=None, scales_by_page=True,
             kv_edit=None):
    """Build rank's list with the library, run the kernels, return everything needed to compare.  ``kv_edit(kv)``
    may rewrite the cache (in place) before it goes to the device; the oracle reads the same arrays."""
    sh = shape_of(w)
    items, pairs, sched, indptr = fs.fs_build_worklist(sh, w["ctx_len"], owner, rank, chunk)
    kv = make_kv_pool(w["seed"], np.stack([pairs["req"], pairs["kv_head"]], axis=1) if len(pairs) else np.zeros((0, 2)),
                      w["ctx_len"], kv_dtype=w["kv_dtype"])
    if kv_edit is not None:
        kv_edit(kv)
    ds = DeviceShare(sh, q, kv, w["sm_scale"], interleave_kv=interleave, scales_by_page=scales_by_page)
    ds.set_worklist(items, pairs, sched, indptr)
    ds.run(use_sched=use_sched)
    torch.cuda.synchronize()
    return ds, kv, items, pairs, sched, indptr


def pairs_rows(pairs):
    return pairs.view(np.int32).reshape(-1, 4)


def items_rows(items):
    return items.view(np.int32).reshape(-1, 8)


# ------------------------------------------------------------------------------------------------
def test_config0_every_rank_and_reassembly():
    """Tiny all-TP batch, R=7: each rank's share against the oracle, then all shares gathered by
    head against unsharded attention for every (request, q-head)."""
    w = make_requests(0)
    q = make_q(w["seed"], w["n_req"], w["n_q_heads"], 128)
    sh = shape_of(w)
    owner, dp, load = fs.fs_build_placement(sh, w["ctx_len"], w["mode"])
    o_owner, o_dp, o_load = oracle.build_placement(w["ctx_len"], w["mode"], w["n_ranks"], w["n_kv_heads"])
    assert owner.tobytes() == o_owner.tobytes() and load.tobytes() == o_load.tobytes()
    G = w["group"]
    B, Hq = w["n_req"], w["n_q_heads"]
    full_o = np.full((B, Hq, 128), np.nan); full_l = np.full((B, Hq), np.nan)
    for k in range(w["n_ranks"]):
        say(f"config 0 rank {k}")
        ds, kv, items, pairs, sched, indptr = run_rank(w, q, k, w["chunk_tokens"], owner)
        oi, op, osch, oind = oracle.build_worklist(w["ctx_len"], o_owner, k, w["chunk_tokens"], Hq, w["n_kv_heads"])
        assert items_rows(items).tobytes() == oi.tobytes() and sched.tobytes() == osch.tobytes()
        ref_o, ref_l = oracle.decode_attention_pairs(q, kv, op, Hq, G, w["sm_scale"])
        out, lse = ds.out.cpu().numpy(), ds.lse.cpu().numpy()
        check(out, lse, ref_o, ref_l, f"cfg0 rank {k}")
        for p, (r, h, L, _n) in enumerate(op):
            full_o[r, h * G:(h + 1) * G] = out[p * G:(p + 1) * G]
            full_l[r, h * G:(h + 1) * G] = lse[p * G:(p + 1) * G]
    all_pairs = np.array([(r, h) for r in range(B) for h in range(w["n_kv_heads"])])
    kv_all = make_kv_pool(w["seed"], all_pairs, w["ctx_len"])
    un_o, un_l = oracle.unsharded_attention(q, kv_all, w["ctx_len"], Hq, w["n_kv_heads"], w["sm_scale"])
    check(full_o, full_l, un_o, un_l, "cfg0 all ranks gathered vs unsharded")


@pytest.mark.parametrize("waves", [1, 2, 4])
@pytest.mark.parametrize("prefetch", [1, 2, 3])
def test_launch_shapes_on_ragged_lengths(waves, prefetch):
    """Every wavefront count and prefetch depth on lengths that hit all loop phases: fewer pages
    than wavefronts, exact multiples, one token, ragged tails."""
    fs.fs_set_option("waves_per_group", waves)
    fs.fs_set_option("prefetch_pages", prefetch)
    lens = [1, 2, 15, 16, 17, 31, 32, 33, 47, 48, 64, 65, 95, 96, 97, 127, 128, 129, 160, 161, 255, 256,
            257, 300, 511, 512, 513, 700, 1000, 1023, 1024, 1025]
    w = make_requests(0, n_req=len(lens))
    w["ctx_len"] = np.array(lens, dtype=np.int32)
    w["n_ranks"] = 3
    q = make_q(w["seed"] + 1, w["n_req"], w["n_q_heads"], 128)
    sh = shape_of(w)
    owner, _, _ = fs.fs_build_placement(sh, w["ctx_len"], w["mode"])
    for chunk in (0, 256):
        say(f"ragged waves={waves} prefetch={prefetch} chunk={chunk}")
        ds, kv, items, pairs, sched, indptr = run_rank(w, q, 1, chunk, owner)
        ref_o, ref_l = oracle.decode_attention_pairs(q, kv, pairs_rows(pairs), w["n_q_heads"], w["group"], w["sm_scale"])
        check(ds.out.cpu().numpy(), ds.lse.cpu().numpy(), ref_o, ref_l, f"ragged w{waves} p{prefetch} c{chunk}")
    fs.fs_set_option("waves_per_group", 4)
    fs.fs_set_option("prefetch_pages", 2)


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (8, 4), (12, 4), (32, 8), (64, 8), (32, 2)])
def test_group_sizes(Hq, Hkv):
    """G = 1, 2, 3, 4, 8, 16 q-heads per KV head."""
    rng = np.random.default_rng(Hq * 100 + Hkv)
    B = 6
    w = make_requests(1, n_req=B)
    w.update(n_q_heads=Hq, n_kv_heads=Hkv, group=Hq // Hkv, n_ranks=3,
             ctx_len=rng.integers(1, 900, size=B).astype(np.int32), mode=np.array([0, 1, 0, 1, 0, 0], np.uint8))
    q = make_q(w["seed"] + 2, B, Hq, 128)
    sh = shape_of(w)
    owner, _, _ = fs.fs_build_placement(sh, w["ctx_len"], w["mode"])
    for k in range(3):
        say(f"group Hq={Hq} Hkv={Hkv} rank {k}")
        ds, kv, items, pairs, sched, indptr = run_rank(w, q, k, 128, owner)
        if len(pairs) == 0:
            continue
        ref_o, ref_l = oracle.decode_attention_pairs(q, kv, pairs_rows(pairs), Hq, Hq // Hkv, w["sm_scale"])
        check(ds.out.cpu().numpy(), ds.lse.cpu().numpy(), ref_o, ref_l, f"G={Hq // Hkv} rank {k}")


def test_partials_and_merge_separately():
    """fs_decode_attention's per-item partials and fs_merge_lse, each against its own oracle twin."""
    w = make_requests(1, n_req=12, max_len=3000)
    q = make_q(w["seed"], 12, w["n_q_heads"], 128)
    sh = shape_of(w)
    owner, _, _ = fs.fs_build_placement(sh, w["ctx_len"], w["mode"])
    ds, kv, items, pairs, sched, indptr = run_rank(w, q, 0, 256, owner)
    G = w["group"]
    po, pl = oracle.decode_attention_items(q, kv, items_rows(items), G, w["sm_scale"])
    check(ds.part_o.cpu().numpy(), ds.part_lse.cpu().numpy(), po, pl, "partials, chunk 256")
    # merge alone, on the oracle's own partials rounded to fp32 (so only the merge is under test)
    po32 = torch.from_numpy(po.astype(np.float32)).cuda(); pl32 = torch.from_numpy(pl.astype(np.float32)).cuda()
    out = torch.empty((len(pairs) * G, 128), dtype=torch.float32, device="cuda"); lse = torch.empty(len(pairs) * G, dtype=torch.float32, device="cuda")
    fs.fs_merge_lse(po32, pl32, ds.chunk_indptr, len(pairs), G, 128, out, lse, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    mo, ml = oracle.merge_lse(po32.cpu().numpy().astype(np.float64), pl32.cpu().numpy().astype(np.float64), indptr, G)
    check(out.cpu().numpy(), lse.cpu().numpy(), mo, ml, "merge alone")


def test_merge_with_widely_spread_lse():
    """Chunks whose lse differ by hundreds: weights underflow to zero without NaN."""
    rng = np.random.default_rng(5)
    G, n_pairs = 4, 9
    counts = [1, 2, 3, 5, 8, 1, 17, 64, 2]
    indptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    n_items = int(indptr[-1])
    po = rng.standard_normal((n_items * G, 128)).astype(np.float32)
    pl = (rng.standard_normal(n_items * G) * 60).astype(np.float32)
    out = torch.empty((n_pairs * G, 128), dtype=torch.float32, device="cuda"); lse = torch.empty(n_pairs * G, dtype=torch.float32, device="cuda")
    fs.fs_merge_lse(torch.from_numpy(po).cuda(), torch.from_numpy(pl).cuda(), torch.from_numpy(indptr).cuda(),
                    n_pairs, G, 128, out, lse, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    mo, ml = oracle.merge_lse(po.astype(np.float64), pl.astype(np.float64), indptr, G)
    check(out.cpu().numpy(), lse.cpu().numpy(), mo, ml, "merge, spread lse")


@pytest.mark.parametrize("G,n_pairs", [(8, 1100), (4, 2100), (128, 70), (6, 1500)])
def test_merge_of_many_rows(G, n_pairs):
    """More rows than the chip holds wavefronts: groups that are a multiple of four go four rows to a
    wavefront (the others one), with pairs of one chunk, of a few, and of more than 64."""
    rng = np.random.default_rng(600 + G)
    counts = rng.choice([1, 1, 1, 2, 3, 7], size=n_pairs)
    counts[rng.integers(0, n_pairs, size=3)] = [65, 70, 130]
    indptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    n_items = int(indptr[-1])
    assert n_pairs * G > 8192
    po = rng.standard_normal((n_items * G, 128)).astype(np.float32)
    pl = (rng.standard_normal(n_items * G) * 6).astype(np.float32)
    out = torch.empty((n_pairs * G, 128), dtype=torch.float32, device="cuda"); lse = torch.empty(n_pairs * G, dtype=torch.float32, device="cuda")
    fs.fs_merge_lse(torch.from_numpy(po).cuda(), torch.from_numpy(pl).cuda(), torch.from_numpy(indptr).cuda(),
                    n_pairs, G, 128, out, lse, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    mo, ml = oracle.merge_lse(po.astype(np.float64), pl.astype(np.float64), indptr, G)
    check(out.cpu().numpy(), lse.cpu().numpy(), mo, ml, f"merge, many rows, G={G}")


def test_single_key_closed_form_and_layout_variants():
    """L = 1: out is the V row exactly (weight 1.0 is exact in bf16) and lse is the score; the same
    share gives the same bits with K/V interleaved or in two pools, scheduled or in index order."""
    w = make_requests(0, n_req=8)
    w["ctx_len"] = np.array([1, 1, 1, 16, 17, 1, 300, 1], dtype=np.int32)
    q = make_q(w["seed"], 8, w["n_q_heads"], 128)
    sh = shape_of(w)
    w["n_ranks"] = 1; sh.n_ranks = 1
    owner, _, _ = fs.fs_build_placement(sh, w["ctx_len"], w["mode"])
    ds, kv, items, pairs, sched, indptr = run_rank(w, q, 0, 0, owner)
    out = ds.out.cpu().numpy(); lse = ds.lse.cpu().numpy()
    G = w["group"]
    for p, (r, h, L, _n) in enumerate(pairs_rows(pairs)):
        if L != 1:
            continue
        K, V = oracle.gather_pair_kv(kv, p, 0, 1)
        for g in range(G):
            assert np.array_equal(out[p * G + g].astype(np.float64), V[0]), "single key must return its V row"
            s = w["sm_scale"] * float(oracle.bf16_bits_to_f64(q[r, h * G + g]) @ K[0])
            assert abs(lse[p * G + g] - s) < 1e-5 * max(1.0, abs(s))
    ds2, *_ = run_rank(w, q, 0, 0, owner, interleave=False, use_sched=False)
    assert torch.equal(ds.out, ds2.out) and torch.equal(ds.lse, ds2.lse)


def test_unused_slots_and_page_tails_are_never_read():
    """The generator poisons spare slots and the tail of each last page with NaN patterns; a finite
    result on lengths with every tail size proves they were not used."""
    lens = list(range(1, 34))
    w = make_requests(0, n_req=len(lens))
    w["ctx_len"] = np.array(lens, dtype=np.int32); w["n_ranks"] = 2
    q = make_q(w["seed"], len(lens), w["n_q_heads"], 128)
    sh = shape_of(w)
    owner, _, _ = fs.fs_build_placement(sh, w["ctx_len"], w["mode"])
    ds, kv, items, pairs, sched, indptr = run_rank(w, q, 0, 16, owner)
    ref_o, ref_l = oracle.decode_attention_pairs(q, kv, pairs_rows(pairs), w["n_q_heads"], w["group"], w["sm_scale"])
    check(ds.out.cpu().numpy(), ds.lse.cpu().numpy(), ref_o, ref_l, "poisoned tails, chunk 16")


def test_large_scores_stay_finite():
    """Scores of several tens in magnitude (softmax scale 1.0, near one-hot weights): the running-max rescale
    keeps everything finite and the stated bar holds unchanged.  In the log2 domain such a score is ~130, where
    an fp32 ulp is 1.5e-5, so a weight is off by ~1e-5 relative and the lse by ~1e-5 absolute."""
    w = make_requests(0, n_req=4)
    w["ctx_len"] = np.array([200, 77, 1024, 33], dtype=np.int32); w["n_ranks"] = 1
    w["sm_scale"] = 1.0
    q = make_q(w["seed"], 4, w["n_q_heads"], 128)
    sh = shape_of(w)
    owner, _, _ = fs.fs_build_placement(sh, w["ctx_len"], w["mode"])
    for chunk in (128, 0):
        ds, kv, items, pairs, sched, indptr = run_rank(w, q, 0, chunk, owner)
        ref_o, ref_l = oracle.decode_attention_pairs(q, kv, pairs_rows(pairs), w["n_q_heads"], w["group"], 1.0)
        assert np.abs(ref_l).max() > 30.0            # the case is what it says it is
        check(ds.out.cpu().numpy(), ds.lse.cpu().numpy(), ref_o, ref_l, f"large scores, chunk {chunk}")


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
def test_device_slot_packing_matches_the_layout_definition(kv_dtype):
    """fs_pack_kv_slots on the device against the gather that fs_kv_elem_offset defines (applied on the host),
    byte for byte, into separate pools and into the two halves of an interleaved pool."""
    from paper_2511_14116_amd.layout import pack_slots
    rng = np.random.default_rng(3)
    code = fs.FS_KV_BF16 if kv_dtype == "bf16" else fs.FS_KV_FP8_E4M3
    n_slots, elt = 37, (np.uint16 if kv_dtype == "bf16" else np.uint8)
    slot_bytes = 2048 * np.dtype(elt).itemsize
    stream = torch.cuda.current_stream().cuda_stream
    for is_v in (False, True):
        host = rng.integers(0, np.iinfo(elt).max, size=(n_slots, 16, 128), dtype=elt)
        want = pack_slots(host, code, is_v).reshape(n_slots, -1)
        src = torch.from_numpy(host.view(np.int16 if kv_dtype == "bf16" else np.uint8)).cuda()
        dst = torch.zeros((n_slots, 2048), dtype=src.dtype, device="cuda")
        fs.fs_pack_kv_slots(src, slot_bytes, dst, slot_bytes, n_slots, code, is_v, stream)
        both = torch.zeros((n_slots, 2, 2048), dtype=src.dtype, device="cuda")
        fs.fs_pack_kv_slots(src, slot_bytes, both.data_ptr() + (slot_bytes if is_v else 0), 2 * slot_bytes, n_slots, code, is_v, stream)
        torch.cuda.synchronize()
        assert dst.cpu().numpy().view(elt).tobytes() == want.tobytes()
        half = both[:, 1 if is_v else 0].cpu().numpy().view(elt)
        assert half.tobytes() == want.tobytes() and not both[:, 0 if is_v else 1].any()
    with pytest.raises(fs.FsError) as e:          # in place is refused
        fs.fs_pack_kv_slots(src, slot_bytes, src, slot_bytes, n_slots, code, False, stream)
    assert e.value.status == fs.FS_EINVAL


def test_empty_rank_is_a_no_op():
    w = make_requests(0, n_req=1)
    w["ctx_len"] = np.array([40], dtype=np.int32); w["mode"] = np.array([1], np.uint8)
    q = make_q(w["seed"], 1, w["n_q_heads"], 128)
    sh = shape_of(w)
    owner, dp, _ = fs.fs_build_placement(sh, w["ctx_len"], w["mode"])
    empty = [k for k in range(w["n_ranks"]) if k != dp[0]][0]
    ds, kv, items, pairs, sched, indptr = run_rank(w, q, empty, 0, owner)
    assert ds.n_items == 0 and ds.n_pairs == 0 and ds.out.numel() == 0


# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("G,Hkv", [(1, 8), (2, 4), (3, 2), (4, 2), (6, 2), (8, 1), (12, 1), (16, 1)])
def test_fp8_small(G, Hkv):
    """fp8 K/V, every group size class up to 16, ragged lengths, split and not."""
    B = 10
    w = make_requests(4, n_req=B)
    w.update(n_q_heads=G * Hkv, n_kv_heads=Hkv, group=G, n_ranks=3,
             ctx_len=np.array([1, 7, 16, 17, 100, 129, 512, 777, 1500, 2048], dtype=np.int32))
    q = make_q(w["seed"], B, G * Hkv, 128)
    sh = shape_of(w)
    owner, _, _ = fs.fs_build_placement(sh, w["ctx_len"], w["mode"])
    for k in range(3):
        for chunk in (0, 512):
            what = f"fp8 G={G} rank {k} chunk {chunk}"
            say(what)
            ds, kv, items, pairs, sched, indptr = run_rank(w, q, k, chunk, owner)
            ref_o, ref_l = oracle.decode_attention_pairs(q, kv, pairs_rows(pairs), G * Hkv, G, w["sm_scale"])
            check(ds.out.cpu().numpy(), ds.lse.cpu().numpy(), ref_o, ref_l, what)
            # the scales gathered by slot instead of read in page-table order: the same numbers, the same bits
            ds2, *_ = run_rank(w, q, k, chunk, owner, scales_by_page=False)
            assert ds.page_scales is not None and ds2.page_scales is None
            assert torch.equal(ds.out, ds2.out) and torch.equal(ds.lse, ds2.lse)
            check_records(ds, kv, items, sched, indptr, what)


def test_fp8_every_byte_pattern():
    """A cache that holds every e4m3 bit pattern but the two NaNs - subnormals, both zeros, the largest values - in K
    and in V, under every lane and byte position of the kernel's loads (K is converted to bf16 by an instruction that
    takes a scale, V's bytes pass through an fp8 product on their way into the second one: both must be exact)."""
    G, Hkv, B = 4, 2, 6
    w = make_requests(4, n_req=B)
    w.update(n_q_heads=G * Hkv, n_kv_heads=Hkv, group=G, n_ranks=1,
             ctx_len=np.array([16, 33, 254, 508, 509, 1024], dtype=np.int32))
    q = make_q(w["seed"], B, G * Hkv, 128)
    owner, _, _ = fs.fs_build_placement(shape_of(w), w["ctx_len"], w["mode"])
    patterns = np.array([b for b in range(256) if b & 0x7F != 0x7F], dtype=np.uint8)      # 254 of them

    def every_pattern(kv):
        rng = np.random.default_rng(5)
        for pool, scale, s in ((kv["k_pool"], kv["k_scale"], 1.0 / 2048), (kv["v_pool"], kv["v_scale"], 1.0 / 64)):
            live = pool != np.uint8(0x7F)                      # the unread tails keep their NaN bytes
            n_slots, T, D = pool.shape
            # element (slot, t, d) takes pattern (7 slot + 3 t + d) mod 254, so a token row runs through 128 patterns
            # in a row and every pattern meets every byte position; one slot in four is shuffled instead
            idx = (7 * np.arange(n_slots)[:, None, None] + 3 * np.arange(T)[None, :, None] + np.arange(D)[None, None, :]) % 254
            vals = patterns[idx]
            for sl in range(0, n_slots, 4):
                vals[sl] = patterns[rng.integers(0, 254, size=(T, D))]
            pool[live] = vals[live]
            scale[~np.isnan(scale)] = np.float32(s)
    for chunk in (0, 256):
        what = f"fp8 every byte pattern, chunk {chunk}"
        say(what)
        ds, kv, items, pairs, sched, indptr = run_rank(w, q, 0, chunk, owner, kv_edit=every_pattern)
        assert set(np.unique(kv["v_pool"])) >= set(patterns.tolist()) and set(np.unique(kv["k_pool"])) >= set(patterns.tolist())
        ref_o, ref_l = oracle.decode_attention_pairs(q, kv, pairs_rows(pairs), G * Hkv, G, w["sm_scale"])
        check(ds.out.cpu().numpy(), ds.lse.cpu().numpy(), ref_o, ref_l, what)


@pytest.mark.parametrize("cfg_id", [1, 4, "4 with groups of 4"])
def test_repeated_launches_agree_bit_for_bit(cfg_id):
    """The kernels have no atomics on data and a fixed order of sums: launches on the same inputs must leave
    the same bits (partials and merged rows), whichever form of the sweep runs.  A difference means a race."""
    grouped = cfg_id == "4 with groups of 4"           # fp8 K/V under a group of q-heads
    w = make_requests(4 if grouped else cfg_id, n_req=96)
    if grouped:
        w.update(n_q_heads=32, n_kv_heads=8, group=4)
    q = make_q(w["seed"], 96, w["n_q_heads"], 128)
    owner, _, _ = fs.fs_build_placement(shape_of(w), w["ctx_len"], w["mode"])
    ds, kv, items, pairs, sched, indptr = run_rank(w, q, 0, 512, owner)
    first = [t.clone() for t in (ds.part_o, ds.part_lse, ds.out, ds.lse)]
    forms = [False] * 3 + [True] * 3
    for rep, persistent in enumerate(forms):
        for t in (ds.part_o, ds.part_lse, ds.out, ds.lse):
            t.fill_(float("nan"))
        ds.run(persistent=persistent)
        torch.cuda.synchronize()
        for name, a, b in zip(("part_o", "part_lse", "out", "lse"), first, (ds.part_o, ds.part_lse, ds.out, ds.lse)):
            assert torch.equal(a, b), f"launch {rep} (persistent={persistent}): {name} differs from the first launch"


def check_records(ds, kv, items, sched, indptr, what):
    """fs_decode_attention_records (one workgroup per record, launch order) on the share that ``ds`` has just run
    from items: the library's records equal the oracle's byte for byte, and the call leaves the same final rows."""
    G = ds.group
    rec = fs.fs_build_launch_records(ds.shape, items, sched, indptr, kv["page_indptr"], kv["page_ids"])
    want = oracle.build_launch_records(items_rows(items), sched, indptr, kv["page_indptr"], kv["page_ids"], G)
    assert rec.view(np.int32).reshape(-1, 16).tobytes() == want.tobytes(), f"{what}: launch records differ from the oracle's"
    ref = [ds.out.clone(), ds.lse.clone()]
    ds.set_records(rec)
    for t in (ds.part_o, ds.part_lse, ds.out, ds.lse):
        t.fill_(float("nan"))
    for claim in (False, True):          # one workgroup per record; resident workgroups claiming the records
        for t in (ds.part_o, ds.part_lse, ds.out, ds.lse):
            t.fill_(float("nan"))
        ds.run_records(claim=claim)
        torch.cuda.synchronize()
        assert torch.equal(ds.out, ref[0]) and torch.equal(ds.lse, ref[1]), f"{what}: the records call (claim={claim}) leaves other final rows"
        assert not claim or ds.claim.cpu().tolist() == [0, 0], f"{what}: the claim counters are not back at zero"
    check_merge_in_sweep(ds, ref, False, what)
    check_merge_in_sweep(ds, ref, False, what, claim=True)


def check_merge_in_sweep(ds, ref, units, what, claim=False):
    """The same call with pair counters: split pairs are merged by the workgroup that writes their last partial rows,
    no merge kernel runs.  Twice in a row (the counters must be back at zero), same bits as ``ref`` = [out, lse].
    claim: resident workgroups that claim the records instead of one workgroup per record."""
    what = f"{what} (claim={claim})"
    for rep in range(2):
        for t in (ds.part_o, ds.part_lse, ds.out, ds.lse):
            t.fill_(float("nan"))
        ds.run_records(units=units, merge_in_sweep=True, claim=claim)
        torch.cuda.synchronize()
        bad = (~((ds.out == ref[0]).all(dim=1) & (ds.lse == ref[1]))).nonzero().flatten().cpu().numpy()
        assert len(bad) == 0, (f"{what}: merge inside the sweep (units={units}, call {rep}) leaves other final rows: {len(bad)} rows, "
                               f"first {int(bad[0])} (pair {int(bad[0]) // ds.group}), lse {float(ds.lse[int(bad[0])])} vs {float(ref[1][int(bad[0])])}")
        assert int(ds.pair_counters.abs().sum()) == 0, f"{what}: the pair counters are not back at zero after call {rep}"
        assert not claim or ds.claim.cpu().tolist() == [0, 0], f"{what}: the claim counters are not back at zero after call {rep}"


def check_fused(ds, indptr, what):
    """fs_decode_attention_fused on the share that ``ds`` has just run the two-call way: the same final bits,
    the same partial rows for split pairs, no partial row written for a pair that is one item."""
    want = [t.clone() for t in (ds.part_o, ds.part_lse, ds.out, ds.lse)]
    G = ds.group
    counts = np.diff(indptr)
    split_rows = torch.from_numpy(np.repeat(np.repeat(counts > 1, counts), G)).to(ds.device)   # per partial row
    forms = (False, True) if ds.kv_dtype == fs.FS_KV_BF16 else (False,)
    for persistent in forms:
        for t in (ds.part_o, ds.part_lse, ds.out, ds.lse):
            t.fill_(float("nan"))
        ds.run_fused(persistent=persistent)
        torch.cuda.synchronize()
        assert torch.equal(ds.out, want[2]) and torch.equal(ds.lse, want[3]), f"{what}: fused call (persistent={persistent}) leaves other final rows"
        assert torch.equal(ds.part_o[split_rows], want[0][split_rows]) and torch.equal(ds.part_lse[split_rows], want[1][split_rows])
        assert torch.isnan(ds.part_lse[~split_rows]).all() and torch.isnan(ds.part_o[~split_rows]).all(), \
            f"{what}: the fused call wrote partial rows of an unsplit pair"
        if persistent:
            assert ds.claim.cpu().tolist() == [0, 0]


# ------------------------------------------------------------------------------------------------
def _full_config(cfg_id, rank, kv_dtype=None, builders_chunk=False, **req_kw):
    """A config at its full size in the launch shape the benchmark times: every pair of the share against
    the oracle (threaded over pairs), and for bf16 the persistent form of the sweep bit for bit against one
    workgroup per item.  builders_chunk: the chunk the benchmark takes for a large share instead of the config's own
    (items of half a resident workgroup's share of the rank's tokens with bf16 K/V, where resident workgroups claim the
    launch records; of 8/9 of it with fp8, one workgroup per record)."""
    w = make_requests(cfg_id, **req_kw)
    if kv_dtype:
        w["kv_dtype"] = kv_dtype
    q = make_q(w["seed"], w["n_req"], w["n_q_heads"], 128)
    sh = shape_of(w)
    owner, dp, load = fs.fs_build_placement(sh, w["ctx_len"], w["mode"])
    o_owner, _, o_load = oracle.build_placement(w["ctx_len"], w["mode"], w["n_ranks"], w["n_kv_heads"])
    assert owner.tobytes() == o_owner.tobytes() and load.tobytes() == o_load.tobytes()
    chunk = w["chunk_tokens"]
    if w.get("chunk_adaptive"):           # the builder's choice, as bench.py makes it: an item per compute unit
        n_cu = torch.cuda.get_device_properties(0).multi_processor_count
        chunk, n_chosen = fs.fs_choose_chunk_tokens(sh, w["ctx_len"], owner, rank, w["chunk_tokens"], 256, n_cu)
        assert (chunk, n_chosen) == oracle.choose_chunk_tokens(w["ctx_len"], o_owner, rank, w["chunk_tokens"], 256, n_cu,
                                                               w["n_kv_heads"])
    if builders_chunk:
        n_cu = torch.cuda.get_device_properties(0).multi_processor_count
        slots = 16 * n_cu // 3 if w["kv_dtype"] == "bf16" else 3 * n_cu
        chunk, n_chosen = fs.fs_choose_chunk_tokens(sh, w["ctx_len"], owner, rank, 32768, 256, slots)
        assert (chunk, n_chosen) == oracle.choose_chunk_tokens(w["ctx_len"], o_owner, rank, 32768, 256, slots, w["n_kv_heads"])
    what = f"cfg{cfg_id}{' ' + str(req_kw) if req_kw else ''}{' as ' + kv_dtype if kv_dtype else ''} rank {rank}"
    say(f"{what}: generating pool (chunk {chunk})")
    ds, kv, items, pairs, sched, indptr = run_rank(w, q, rank, chunk, owner)
    oi, op, osch, oind = oracle.build_worklist(w["ctx_len"], o_owner, rank, chunk, w["n_q_heads"], w["n_kv_heads"])
    assert items_rows(items).tobytes() == oi.tobytes() and sched.tobytes() == osch.tobytes() and indptr.tobytes() == oind.tobytes()
    assert pairs_rows(pairs).tobytes() == op.tobytes()
    say(f"{what}: {len(pairs)} pairs, {len(items)} items (longest pair {int(op[:, 3].max()) if len(op) else 0} chunks), "
        f"{ds.kv_bytes / 1e6:.1f} MB of K+V")
    if len(items) == 0:
        return ds
    G = w["group"]
    workers = min(16, len(os.sched_getaffinity(0)))
    ref_o, ref_l = oracle.decode_attention_pairs(q, kv, op, w["n_q_heads"], G, w["sm_scale"], workers=workers)
    check(ds.out.cpu().numpy(), ds.lse.cpu().numpy(), ref_o, ref_l, f"{what}, all {len(op)} pairs")
    if w["kv_dtype"] == "bf16":
        first = [t.clone() for t in (ds.part_o, ds.part_lse, ds.out, ds.lse)]
        for t in (ds.part_o, ds.part_lse, ds.out, ds.lse):
            t.fill_(float("nan"))
        for _ in range(2):                # back to back on one pair of counters that nobody clears
            ds.decode_persistent()
        ds.merge()
        torch.cuda.synchronize()
        for name, a, b in zip(("part_o", "part_lse", "out", "lse"), first, (ds.part_o, ds.part_lse, ds.out, ds.lse)):
            assert torch.equal(a, b), f"{what}: persistent sweep leaves other bits in {name}"
        assert ds.claim.cpu().tolist() == [0, 0]
    check_fused(ds, indptr, what)
    check_records(ds, kv, items, sched, indptr, what)
    return ds


def test_config1_full_size_every_pair():
    _full_config(1, 0)


def test_config2_full_size_every_pair():
    _full_config(2, 0)


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
def test_config2_full_size_on_the_builders_chunk_every_pair(kv_dtype):
    """The 70B-shaped batch as the benchmark launches it by default: the builder's chunk, launch records (claimed by
    resident workgroups and one workgroup per record), split pairs merged inside the sweep; and the same batch held
    as fp8."""
    _full_config(2, 0, kv_dtype=None if kv_dtype == "bf16" else kv_dtype, builders_chunk=True)


@pytest.mark.parametrize("rank", range(5))
@pytest.mark.parametrize("variant", ["seeded", "forced_tail"])
def test_config3_every_rank_every_pair(variant, rank):
    """The skewed long-context batch (Section 3.1 names it as the case where stragglers return), R = 5: the
    config's own seeded draw and the variant whose request 0 has 131072 tokens, every rank's share in turn,
    both forms of the sweep."""
    _full_config(3, rank, **(dict(force_first_len=131072) if variant == "forced_tail" else {}))


def test_config4_fp8_full_size_every_pair():
    _full_config(4, 0)


# ------------------------------------------------------------------------------------------------
def test_hip_graph_replays_match_eager():
    """The benchmark replays the step's GPU side as a HIP graph.  Captured once, replayed several
    times with eager work and synchronisation in between, every replay must reproduce the eager
    result bit for bit (the kernels are deterministic)."""
    w = make_requests(1, n_req=24, max_len=2500)
    q = make_q(w["seed"], 24, w["n_q_heads"], 128)
    sh = shape_of(w)
    owner, _, _ = fs.fs_build_placement(sh, w["ctx_len"], w["mode"])
    ds, kv, items, pairs, sched, indptr = run_rank(w, q, 0, 256, owner)
    eager_o, eager_l = ds.out.clone(), ds.lse.clone()
    cap = torch.cuda.Stream()
    dec = fs.bind_decode_attention(sh, ds.view, ds.items, ds.sched, ds.n_items, ds.part_o, ds.part_lse, cap.cuda_stream)
    mrg = fs.bind_merge_lse(ds.part_o, ds.part_lse, ds.chunk_indptr, ds.n_pairs, ds.group, 128, ds.out, ds.lse, cap.cuda_stream)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=cap):
        dec()
        mrg()
    for rep in range(4):
        ds.out.fill_(float("nan")); ds.lse.fill_(float("nan")); ds.part_o.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(ds.out, eager_o) and torch.equal(ds.lse, eager_l), f"replay {rep} differs"
        ds.run()                       # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(ds.out, eager_o)
    ref_o, ref_l = oracle.decode_attention_pairs(q, kv, pairs_rows(pairs), w["n_q_heads"], w["group"], w["sm_scale"])
    check(ds.out.cpu().numpy(), ds.lse.cpu().numpy(), ref_o, ref_l, "graph replay vs oracle")


@pytest.mark.parametrize("claiming", [False, True])
def test_hip_graph_replays_of_the_sweep_that_merges(claiming):
    """fs_decode_attention_records with pair counters (split pairs merged inside the sweep) captured as a HIP
    graph: the counters go back to zero inside every launch, so replays need nothing cleared between them; every
    replay, with eager launches of the same call and of the two-call form in between, gives the eager bits.
    claiming: resident workgroups that claim the records, whose two counters go back to zero the same way."""
    w = make_requests(1, n_req=24, max_len=2500)
    q = make_q(w["seed"], 24, w["n_q_heads"], 128)
    sh = shape_of(w)
    owner, _, _ = fs.fs_build_placement(sh, w["ctx_len"], w["mode"])
    ds, kv, items, pairs, sched, indptr = run_rank(w, q, 0, 256, owner)
    eager_o, eager_l = ds.out.clone(), ds.lse.clone()
    assert ds.n_items > ds.n_pairs
    ds.set_records(fs.fs_build_launch_records(sh, items, sched, indptr, kv["page_indptr"], kv["page_ids"]))
    counters = torch.zeros(ds.n_pairs, dtype=torch.int32, device=ds.device)
    claim = torch.zeros(2, dtype=torch.int32, device=ds.device) if claiming else None
    cap = torch.cuda.Stream()
    call = fs.bind_decode_attention_records(sh, ds.view, ds.records, ds.n_items, None, 0, ds.chunk_indptr, ds.n_pairs,
                                            ds.part_o, ds.part_lse, ds.out, ds.lse, counters, claim, cap.cuda_stream)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=cap):
        call()
    for rep in range(4):
        ds.out.fill_(float("nan")); ds.lse.fill_(float("nan")); ds.part_o.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(ds.out, eager_o) and torch.equal(ds.lse, eager_l), f"replay {rep} differs"
        assert int(counters.abs().sum()) == 0, f"replay {rep} left a pair counter standing"
        assert claim is None or claim.cpu().tolist() == [0, 0], f"replay {rep} left a claim counter standing"
        ds.run()                       # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(ds.out, eager_o)


def test_head_level_hybrid_every_rank_and_reassembly():
    """The paper's literal hybrid attention (Section 3.1): 8 KV heads on 7 workers, one head each
    tensor-parallel (rotated by layer), the eighth replicated and routed by least pending DP load.
    Every rank's share against the oracle, then gathered against unsharded attention."""
    w = make_requests(1, n_req=20, max_len=1200)
    B, Hq, Hkv, R, G = w["n_req"], w["n_q_heads"], w["n_kv_heads"], 7, w["group"]
    w["n_ranks"] = R
    q = make_q(w["seed"], B, Hq, 128)
    sh = shape_of(w)
    layer = 3
    owner, dp, load, dload = fs.fs_build_placement_hybrid_heads(sh, w["ctx_len"], layer=layer)
    ref = oracle.build_placement_hybrid_heads(w["ctx_len"], R, Hkv, layer=layer)
    for a, b in zip((owner, dp, load, dload), ref):
        assert a.tobytes() == b.tobytes()
    full_o = np.full((B, Hq, 128), np.nan); full_l = np.full((B, Hq), np.nan)
    for k in range(R):
        say(f"head-level hybrid rank {k}")
        ds, kv, items, pairs, sched, indptr = run_rank(w, q, k, 256, owner)
        pr = pairs_rows(pairs)
        assert int(pr[:, 2].sum()) == load[k]
        ref_o, ref_l = oracle.decode_attention_pairs(q, kv, pr, Hq, G, w["sm_scale"])
        out, lse = ds.out.cpu().numpy(), ds.lse.cpu().numpy()
        check(out, lse, ref_o, ref_l, f"head-level rank {k}")
        for p, (r, h, L, _n) in enumerate(pr):
            full_o[r, h * G:(h + 1) * G] = out[p * G:(p + 1) * G]
            full_l[r, h * G:(h + 1) * G] = lse[p * G:(p + 1) * G]
    all_pairs = np.array([(r, h) for r in range(B) for h in range(Hkv)])
    kv_all = make_kv_pool(w["seed"], all_pairs, w["ctx_len"])
    un_o, un_l = oracle.unsharded_attention(q, kv_all, w["ctx_len"], Hq, Hkv, w["sm_scale"])
    check(full_o, full_l, un_o, un_l, "head-level hybrid, all ranks gathered vs unsharded")


def test_persistent_sweep_small_batches_against_oracle():
    """The persistent form of the sweep: every rank of the tiny batch and a ragged split-K batch,
    element by element against the oracle, and bit for bit against the one-workgroup-per-item form
    (same wavefront split, same page order, same merge)."""
    say("persistent sweep, small batches")
    for cfg_id, kw, chunk in ((0, {}, 0), (0, {}, 64), (1, dict(n_req=48, max_len=3000), 256)):
        w = make_requests(cfg_id, **kw)
        q = make_q(w["seed"], w["n_req"], w["n_q_heads"], 128)
        owner, dp, load = fs.fs_build_placement(shape_of(w), w["ctx_len"], w["mode"])
        for rank in range(w["n_ranks"]):
            ds, kv, items, pairs, sched, indptr = run_rank(w, q, rank, chunk, owner)
            if len(items) == 0:
                continue
            ref_part_o, ref_part_l = ds.part_o.clone(), ds.part_lse.clone()
            ds.part_o.fill_(float("nan")); ds.part_lse.fill_(float("nan"))
            ds.out.fill_(float("nan")); ds.lse.fill_(float("nan"))
            ds.decode_persistent()
            ds.merge()
            torch.cuda.synchronize()
            assert torch.equal(ds.part_o, ref_part_o) and torch.equal(ds.part_lse, ref_part_l)
            ref_o, ref_l = oracle.decode_attention_pairs(q, kv, pairs_rows(pairs), w["n_q_heads"], w["group"], w["sm_scale"])
            check(ds.out.cpu().numpy(), ds.lse.cpu().numpy(), ref_o, ref_l,
                  f"persistent cfg{cfg_id} chunk={chunk} rank {rank} ({len(items)} items)")
            # every launch leaves its two counters at zero, so a second launch on the same pair, with
            # nothing cleared in between, gives the same bits
            assert ds.claim.cpu().tolist() == [0, 0]
            ds.part_o.fill_(float("nan")); ds.part_lse.fill_(float("nan"))
            ds.decode_persistent()
            torch.cuda.synchronize()
            assert torch.equal(ds.part_o, ref_part_o) and torch.equal(ds.part_lse, ref_part_l)
            assert ds.claim.cpu().tolist() == [0, 0]


@pytest.mark.parametrize("seed", range(8))
def test_persistent_sweep_random_lists_match_the_plain_sweep(seed):
    """Random shares with many small items (lists several times longer than the resident workgroups, every
    group size, ragged chunks): the persistent sweep leaves the same bits as one workgroup per item, its
    counters at zero, and the merged rows of every pair within tolerance of the oracle."""
    rng = np.random.default_rng(1000 + seed)
    Hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.choice([1, 2, 4, 8, 16]))
    R = int(rng.integers(1, 4))
    B = int(rng.integers(20, 100))
    chunk = int(rng.choice([16, 32, 48, 128]))
    if seed % 2:                          # every other case: one rank, small chunks -> thousands of items
        R, chunk, B = 1, int(rng.choice([16, 32])), max(B, 60)
    ctx = rng.integers(1, 500, size=B).astype(np.int32)
    mode = (rng.random(B) < 0.3).astype(np.uint8)
    sh = fs.FsShape(B, Hkv * G, Hkv, 128, 16, R)
    owner, dp, load = fs.fs_build_placement(sh, ctx, mode)
    rank = int(rng.integers(0, R))
    items, pairs, sched, indptr = fs.fs_build_worklist(sh, ctx, owner, rank, chunk)
    say(f"random persistent seed {seed}: B={B} Hkv={Hkv} G={G} R={R} chunk={chunk} -> {len(items)} items")
    if len(items) == 0:
        pytest.skip("empty share")
    q = make_q(77 + seed, B, Hkv * G, 128)
    kv = make_kv_pool(77 + seed, np.stack([pairs["req"], pairs["kv_head"]], axis=1), ctx)
    ds = DeviceShare(sh, q, kv, 1.0 / np.sqrt(128.0))
    ds.set_worklist(items, pairs, sched, indptr)
    ds.run()
    torch.cuda.synchronize()
    ref_part_o, ref_part_l = ds.part_o.clone(), ds.part_lse.clone()
    ref_out, ref_lse = ds.out.clone(), ds.lse.clone()
    for use_sched in (True, False):
        ds.part_o.fill_(float("nan")); ds.part_lse.fill_(float("nan"))
        ds.out.fill_(float("nan")); ds.lse.fill_(float("nan"))
        ds.run(use_sched=use_sched, persistent=True)
        torch.cuda.synchronize()
        assert torch.equal(ds.part_o, ref_part_o) and torch.equal(ds.part_lse, ref_part_l)
        assert torch.equal(ds.out, ref_out) and torch.equal(ds.lse, ref_lse)
        assert ds.claim.cpu().tolist() == [0, 0]
    pr = pairs_rows(pairs)
    ref_o, ref_l = oracle.decode_attention_pairs(q, kv, pr, Hkv * G, G, 1.0 / np.sqrt(128.0), workers=8)
    check(ds.out.cpu().numpy(), ds.lse.cpu().numpy(), ref_o, ref_l, f"random persistent seed {seed}, all {len(pr)} pairs")
    check_fused(ds, indptr, f"random persistent seed {seed}")


@pytest.mark.parametrize("cfg_id,kw,chunk", [(0, {}, 0), (0, {}, 64), (1, dict(n_req=40, max_len=2500), 512),
                                             (4, dict(n_req=30), 0), (4, dict(n_req=30), 1024)])
def test_fused_call_small_batches(cfg_id, kw, chunk):
    """The one-call form on lists with no split pair (no merge is launched and no partial buffer is needed),
    with some, and with fp8 K/V: element by element against the oracle and bit for bit against the two calls."""
    w = make_requests(cfg_id, **kw)
    q = make_q(w["seed"], w["n_req"], w["n_q_heads"], 128)
    owner, _, _ = fs.fs_build_placement(shape_of(w), w["ctx_len"], w["mode"])
    for rank in (0, w["n_ranks"] - 1):
        ds, kv, items, pairs, sched, indptr = run_rank(w, q, rank, chunk, owner)
        if len(items) == 0:
            continue
        say(f"fused cfg{cfg_id} chunk {chunk} rank {rank}: {len(items)} items, {len(pairs)} pairs")
        check_fused(ds, indptr, f"fused cfg{cfg_id} chunk {chunk} rank {rank}")
        check_records(ds, kv, items, sched, indptr, f"records cfg{cfg_id} chunk {chunk} rank {rank}")
        ref_o, ref_l = oracle.decode_attention_pairs(q, kv, pairs_rows(pairs), w["n_q_heads"], w["group"], w["sm_scale"])
        check(ds.out.cpu().numpy(), ds.lse.cpu().numpy(), ref_o, ref_l, f"fused cfg{cfg_id} chunk {chunk} rank {rank}")
        if len(items) == len(pairs):      # nothing is split: the call takes no partial buffers at all
            ds.out.fill_(float("nan")); ds.lse.fill_(float("nan"))
            fs.fs_decode_attention_fused(ds.shape, ds.view, ds.items, ds.sched, ds.n_items, ds.chunk_indptr, ds.n_pairs,
                                         None, None, None, ds.out, ds.lse, torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            check(ds.out.cpu().numpy(), ds.lse.cpu().numpy(), ref_o, ref_l, f"fused, no partial buffers, cfg{cfg_id} rank {rank}")
