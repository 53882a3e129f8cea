"""GPU parity of chunked-prefill attention (through the C ABI) against the CPU oracle.

Bar: tile lists bit-exact; fp32 outputs within 2e-3 abs + 1e-2 rel of the fp64 oracle; LSE
within 1e-3.  Every input is seeded and synthetic.
"""
import math
import os
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2511_14116_amd as fs
from paper_2511_14116_amd.device import DeviceShare
from workloads import make_kv_pool, make_prefill_q, make_prefill_queue

pytestmark = pytest.mark.gpu

ABS_TOL, REL_TOL, LSE_TOL = 2e-3, 1e-2, 1e-3
SCALE = 1.0 / math.sqrt(128.0)
DEFAULT_WAVES, DEFAULT_CT = 4, 2


def say(msg):
    print(f"[prefill] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", autouse=True)
def _lib():
    if not os.path.exists(fs.library_path()):
        raise RuntimeError("libfailsafe.so is not built: GPU tests never fall back to anything else")
    fs.load_library()
    global DEFAULT_WAVES, DEFAULT_CT
    DEFAULT_WAVES, DEFAULT_CT = fs.fs_get_option("prefill_waves"), fs.fs_get_option("prefill_col_tiles")
    yield
    fs.fs_set_option("prefill_waves", DEFAULT_WAVES)
    fs.fs_set_option("prefill_col_tiles", DEFAULT_CT)


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


def run_share(seed, n_done, n_new, Hq, Hkv, owner, rank, R, tile=None, use_sched=True, interleave=True, chunk=0,
              kv_edit=None, v_range=fs.FS_V_FP16_RANGE, kv_dtype="bf16", scales_by_page=True):
    """``v_range``: what the call is told about V.  The generator draws N(0,1) values, which convert to fp16
    exactly, so the statement FS_V_FP16_RANGE is true unless ``kv_edit`` plants something else."""
    n_done = np.asarray(n_done, dtype=np.int32); n_new = np.asarray(n_new, dtype=np.int32)
    B = len(n_done)
    G = Hq // Hkv
    sh = fs.FsShape(B, Hq, Hkv, 128, 16, R)
    tile = fs.fs_prefill_tile_tokens(G) if tile is None else tile
    items, pairs, sched, chunk_indptr, out_indptr = fs.fs_build_prefill_worklist(sh, n_done, n_new, owner, rank, tile, chunk)
    w_items, w_pairs, w_sched, w_chunks, w_indptr = oracle.build_prefill_worklist(n_done, n_new, owner, rank, Hq, tile, chunk)
    assert items.view(np.int32).reshape(-1, 8).tobytes() == w_items.tobytes()
    assert sched.tobytes() == w_sched.tobytes() and out_indptr.tobytes() == w_indptr.tobytes()
    assert chunk_indptr.tobytes() == w_chunks.tobytes()
    ctx = (n_done + n_new).astype(np.int32)
    kv = make_kv_pool(seed, w_pairs[:, :2], ctx, kv_dtype=kv_dtype)
    if kv_edit is not None:
        kv_edit(kv)
    q_indptr = np.concatenate([[0], np.cumsum(n_new)]).astype(np.int64)
    q = make_prefill_q(seed, int(q_indptr[-1]), Hq, 128)
    ds = DeviceShare(sh, q, kv, SCALE, interleave_kv=interleave, v_range=v_range, scales_by_page=scales_by_page)
    ds.set_prefill_worklist(items, sched, chunk_indptr, tile, out_indptr)
    ds.prefill(use_sched=use_sched)
    torch.cuda.synchronize()
    ds.w_items, ds.tile = w_items, tile
    if len(items):
        check_one_call_form(ds, chunk_indptr, use_sched)
    return ds, kv, q, q_indptr, w_pairs, out_indptr


def check_one_call_form(ds, chunk_indptr, use_sched=True):
    """fs_prefill_attention_fused on the list that ``ds`` has just run the two-call way: the same final bits, the
    same partial rows for split tiles, none written for a tile that is one chunk."""
    want = [t.clone() for t in (ds.prefill_part_o, ds.prefill_part_lse, ds.prefill_out, ds.prefill_lse)]
    counts = np.diff(chunk_indptr)
    split_rows = torch.from_numpy(np.repeat(np.repeat(counts > 1, counts), ds.prefill_tile_rows)).to(ds.device)
    for t in (ds.prefill_part_o, ds.prefill_part_lse, ds.prefill_out, ds.prefill_lse):
        t.fill_(float("nan"))
    ds.prefill_fused(use_sched=use_sched)
    torch.cuda.synchronize()
    bad = (~((ds.prefill_out == want[2]).all(dim=1) & (ds.prefill_lse == want[3]))).nonzero().flatten().cpu().numpy()
    if len(bad):
        T = ds.prefill_tile_rows
        r = int(bad[0])
        raise AssertionError(f"the one-call form leaves other final rows: {len(bad)} rows, first {r} (tile {r // T} of "
                             f"{counts[r // T]} chunks, row {r % T} of {T}); lse {float(ds.prefill_lse[r])} vs "
                             f"{float(want[3][r])}; out[:4] {ds.prefill_out[r, :4].tolist()} vs {want[2][r, :4].tolist()}; "
                             f"tiles hit {sorted(set((bad // T).tolist()))[:12]}")
    assert torch.equal(ds.prefill_part_lse[split_rows], want[1][split_rows]) and torch.equal(ds.prefill_part_o[split_rows], want[0][split_rows])
    assert torch.isnan(ds.prefill_part_lse[~split_rows]).all(), "the one-call form wrote partial rows of an unsplit tile"
    ds.prefill(use_sched=use_sched)            # leave the buffers as the two calls leave them (callers look at partial rows)
    torch.cuda.synchronize()


def compare_all(ds, kv, q, q_indptr, pairs, Hq, G, what, out_indptr):
    """Final rows (after the split-K merge) against the unsplit oracle; padding rows must be finite."""
    ref_o, ref_l = oracle.prefill_attention_pairs(q, q_indptr, kv, pairs, Hq, G, SCALE, workers=8, out_indptr=out_indptr)
    out, lse = ds.prefill_out.cpu().numpy(), ds.prefill_lse.cpu().numpy()
    assert np.isfinite(out).all() and np.isfinite(lse).all(), f"{what}: non-finite output (padding rows included)"
    valid = np.isfinite(ref_l)
    assert valid.sum() == int(pairs[:, 3].sum()) * G if len(pairs) else valid.sum() == 0
    check(out[valid], lse[valid], ref_o[valid], ref_l[valid], what)


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (8, 4), (12, 4), (32, 8), (64, 8), (32, 2), (10, 2)])
def test_group_sizes_ragged_chunks(Hq, Hkv, kv_dtype):
    say(f"group sizes Hq={Hq} Hkv={Hkv} {kv_dtype}")
    rng = np.random.default_rng(Hq * 100 + Hkv)
    n_done = [0, 37, 160, 0, 511, 16]
    n_new = [45, 1, 70, 0, 33, 129]
    owner = rng.integers(0, 2, size=(6, Hkv)).astype(np.int32)
    for rank in range(2):
        # fp8: rank 0 with V stated to fit fp16, rank 1 without a statement (V in bf16, weights as hi + lo)
        v_range = fs.FS_V_ANY if (kv_dtype == "fp8" and rank == 1) else fs.FS_V_FP16_RANGE
        ds, kv, q, q_indptr, pairs, oi = run_share(40 + Hq + Hkv, n_done, n_new, Hq, Hkv, owner, rank, 2,
                                                   chunk=(0, 64)[rank], kv_dtype=kv_dtype, v_range=v_range)
        compare_all(ds, kv, q, q_indptr, pairs, Hq, Hq // Hkv, f"Hq={Hq} Hkv={Hkv} {kv_dtype} rank {rank}", oi)


@pytest.mark.parametrize("v_range", [fs.FS_V_FP16_RANGE, fs.FS_V_ANY])
def test_fp8_cache_with_every_byte_pattern(v_range):
    """An fp8 cache that holds all 254 non-NaN e4m3 patterns in K and V under every lane and byte position of the
    kernel's loads (K converted to bf16 by an instruction that takes a scale, V's bytes through an fp8 product with
    the selection matrix), scales by slot and in page-table order, split-K and not."""
    Hq, Hkv = 8, 2
    n_done = [0, 100, 509, 16]
    n_new = [33, 17, 70, 254]
    owner = np.zeros((4, Hkv), dtype=np.int32)
    patterns = np.array([b for b in range(256) if b & 0x7F != 0x7F], dtype=np.uint8)

    def every_pattern(kv):
        rng = np.random.default_rng(6)
        for pool, scale, sc in ((kv["k_pool"], kv["k_scale"], 1.0 / 2048), (kv["v_pool"], kv["v_scale"], 1.0 / 64)):
            live = pool != np.uint8(0x7F)
            n_slots, T, D = pool.shape
            idx = (7 * np.arange(n_slots)[:, None, None] + 3 * np.arange(T)[None, :, None] + np.arange(D)[None, None, :]) % 254
            vals = patterns[idx]
            for sl in range(0, n_slots, 4):
                vals[sl] = patterns[rng.integers(0, 254, size=(T, D))]
            pool[live] = vals[live]
            ok = ~np.isnan(scale)
            scale[ok] = (np.float32(sc) * (1.0 + 0.5 * rng.random(int(ok.sum())))).astype(np.float32)   # a scale of its own per slot
    for chunk in (0, 64):
        what = f"prefill, fp8 cache with every byte pattern, v_range {v_range}, chunk {chunk}"
        say(what)
        ds, kv, q, q_indptr, pairs, oi = run_share(77, n_done, n_new, Hq, Hkv, owner, 0, 1, chunk=chunk, kv_dtype="fp8",
                                                   kv_edit=every_pattern, v_range=v_range)
        assert set(np.unique(kv["v_pool"])) >= set(patterns.tolist()) and set(np.unique(kv["k_pool"])) >= set(patterns.tolist())
        compare_all(ds, kv, q, q_indptr, pairs, Hq, Hq // Hkv, what, oi)
        # the scales gathered by slot instead of read in page-table order: the same numbers, the same bits
        ds2, *_ = run_share(77, n_done, n_new, Hq, Hkv, owner, 0, 1, chunk=chunk, kv_dtype="fp8", kv_edit=every_pattern,
                            v_range=v_range, scales_by_page=False)
        assert ds.page_scales is not None and ds2.page_scales is None
        assert torch.equal(ds.prefill_out, ds2.prefill_out) and torch.equal(ds.prefill_lse, ds2.prefill_lse)


@pytest.mark.parametrize("waves,ct", [(4, 1), (4, 2), (4, 4), (8, 1), (8, 2)])
def test_launch_shapes(waves, ct):
    say(f"launch shape waves={waves} ct={ct}")
    fs.fs_set_option("prefill_waves", waves)
    fs.fs_set_option("prefill_col_tiles", ct)
    try:
        n_done = [0, 100, 1000, 31]
        n_new = [97, 64, 200, 3]
        owner = np.zeros((4, 2), dtype=np.int32)
        for chunk in (0, 32, 256):
            ds, kv, q, q_indptr, pairs, oi = run_share(7, n_done, n_new, 16, 2, owner, 0, 1, use_sched=(waves == 4), chunk=chunk)
            compare_all(ds, kv, q, q_indptr, pairs, 16, 8, f"waves={waves} ct={ct} chunk={chunk}", oi)
        # a tile smaller than the kernel's natural one
        ds, kv, q, q_indptr, pairs, oi = run_share(8, n_done, n_new, 16, 2, owner, 0, 1, tile=3, chunk=96)
        compare_all(ds, kv, q, q_indptr, pairs, 16, 8, f"waves={waves} ct={ct} tile=3", oi)
        # the same shape over an fp8 cache, with and without a statement about V
        for v_range in (fs.FS_V_FP16_RANGE, fs.FS_V_ANY):
            ds, kv, q, q_indptr, pairs, oi = run_share(9, n_done, n_new, 16, 2, owner, 0, 1, chunk=256, kv_dtype="fp8", v_range=v_range)
            compare_all(ds, kv, q, q_indptr, pairs, 16, 8, f"waves={waves} ct={ct} fp8 v_range={v_range}", oi)
    finally:
        fs.fs_set_option("prefill_waves", DEFAULT_WAVES)
        fs.fs_set_option("prefill_col_tiles", DEFAULT_CT)


def test_first_token_closed_form_and_one_token_chunks():
    say("closed forms")
    owner = np.zeros((3, 1), dtype=np.int32)
    ds, kv, q, q_indptr, pairs, out_indptr = run_share(9, [0, 0, 300], [1, 20, 1], 4, 1, owner, 0, 1)
    out = ds.prefill_out.cpu().numpy()
    for p in (0, 1):        # the first token of a fresh prompt sees only itself: out is its own V row, exactly
        _, V = oracle.gather_pair_kv(kv, p, 0, 1)
        for g in range(4):
            assert np.array_equal(out[int(out_indptr[p]) + g].astype(np.float64), V[0])
    compare_all(ds, kv, q, q_indptr, pairs, 4, 4, "one-token chunks", out_indptr)


@pytest.mark.parametrize("waves,ct", [(8, 1), (4, 2)])
def test_wide_value_path(waves, ct):
    """The bf16 hi + lo form of the second product (v_range = FS_V_ANY): same bar, and the first token
    of a prompt still returns its own V row exactly."""
    say(f"wide V path waves={waves} ct={ct}")
    fs.fs_set_option("prefill_waves", waves)
    fs.fs_set_option("prefill_col_tiles", ct)
    try:
        n_done, n_new = [0, 100, 1000, 31, 0], [97, 64, 200, 3, 1]
        owner = np.zeros((5, 2), dtype=np.int32)
        for chunk in (0, 256):
            ds, kv, q, q_indptr, pairs, oi = run_share(21, n_done, n_new, 16, 2, owner, 0, 1, chunk=chunk, v_range=fs.FS_V_ANY)
            compare_all(ds, kv, q, q_indptr, pairs, 16, 8, f"wide V, waves={waves} ct={ct} chunk={chunk}", oi)
        out = ds.prefill_out.cpu().numpy()
        for p in range(len(pairs)):
            if pairs[p, 2] == 0:                    # a fresh prompt: its first token sees only itself
                _, V = oracle.gather_pair_kv(kv, p, 0, 1)
                for g in range(8):
                    assert np.array_equal(out[int(oi[p]) + g].astype(np.float64), V[0])
    finally:
        fs.fs_set_option("prefill_waves", DEFAULT_WAVES)
        fs.fs_set_option("prefill_col_tiles", DEFAULT_CT)


def test_value_range_of_the_second_product():
    """V values at and beyond the edges of fp16's range.  With no statement about V (FS_V_ANY) magnitudes of 1e5
    and 1e-6 count in full; with FS_V_FP16_RANGE the values at the very edges of the stated range (65504 and
    2^-14) are exact.  Both against the oracle as it stands.  A caller whose statement is false gets finite
    rows (the header says how such values enter); nothing more is claimed for that case."""
    say("V range")

    def planter(big, neg_big, tiny):
        def edit(kv):
            for p in range(len(kv["page_indptr"]) - 1):
                slot = int(kv["page_ids"][int(kv["page_indptr"][p])])       # first page of the pair: token 0 always exists
                kv["v_pool"][slot, 0, 3] = big
                kv["v_pool"][slot, 0, 64] = neg_big
                kv["v_pool"][slot, 0, 127] = tiny
        return edit

    beyond = planter(0x47C3, 0xC7C3, 0x3586)         # bf16 bits of 99840, -99840, 9.98e-7
    edge = planter(0x477F, 0xC77F, 0x3880)           # 65280 (the largest bf16 below 65504), -65280, 2^-14
    n_done, n_new = [0, 40, 7], [33, 20, 1]
    owner = np.zeros((3, 2), dtype=np.int32)
    Hq, G = 8, 4
    for name, edit, v_range, compare in (("beyond fp16, no statement", beyond, fs.FS_V_ANY, True),
                                         ("edges of fp16, stated", edge, fs.FS_V_FP16_RANGE, True),
                                         ("beyond fp16, false statement", beyond, fs.FS_V_FP16_RANGE, False)):
        ds, kv, q, q_indptr, pairs, oi = run_share(23, n_done, n_new, Hq, 2, owner, 0, 1, chunk=32, kv_edit=edit,
                                                   v_range=v_range)
        out, lse = ds.prefill_out.cpu().numpy(), ds.prefill_lse.cpu().numpy()
        assert np.isfinite(out).all() and np.isfinite(lse).all(), name
        if not compare:
            continue
        got_o, got_l, ref_o, ref_l = [], [], [], []
        qf = oracle.bf16_bits_to_f64(q.reshape(-1, Hq, 128))
        for p in range(len(pairs)):
            r, h, L, N = (int(x) for x in pairs[p])
            for tok in range(N):
                K, V = oracle.gather_pair_kv(kv, p, 0, L + tok + 1)
                if v_range == fs.FS_V_ANY:
                    assert abs(V[0, 3]) > 65504 and abs(V[0, 64]) > 65504 and 0 < abs(V[0, 127]) < 2.0 ** -14
                o, l = oracle.attend(qf[int(q_indptr[r]) + tok, h * G:(h + 1) * G], K, V, SCALE)
                row = int(oi[p]) + tok * G
                got_o.append(out[row:row + G]); got_l.append(lse[row:row + G]); ref_o.append(o); ref_l.append(l)
        check(np.concatenate(got_o), np.concatenate(got_l), np.concatenate(ref_o), np.concatenate(ref_l), f"V {name}")


def test_chunked_prefill_feeds_from_the_scheduler():
    """Router -> Algorithm 1 -> head-level hybrid placement -> tile list -> kernel, every rank in turn."""
    say("scheduler-formed batch, every rank")
    R, Hq, Hkv, budget = 3, 16, 4, 600
    queue = make_prefill_queue(5, 10, median=300, sigma=0.8, cap=2000)
    prompt, n_done = queue["prompt_len"], queue["n_done"]
    pending = np.zeros(R, dtype=np.int64)
    entries = np.zeros(len(prompt), dtype=fs.PREFILL_ENTRY_DTYPE)
    for i in range(len(prompt)):
        rank = fs.fs_route_request(pending, int(prompt[i] - n_done[i]))
        entries[i] = (i, rank, int(n_done[i]), int(prompt[i] - n_done[i]))
    take, load, n_tok = fs.fs_schedule_prefill(R, budget, budget // 2, entries)
    assert n_tok > 0
    ctx = np.maximum(n_done + take, 1).astype(np.int32)
    sh = fs.FsShape(len(prompt), Hq, Hkv, 128, 16, R)
    owner, dp, _, _ = fs.fs_build_placement_hybrid_heads(sh, ctx, layer=1, route=entries["rank"])
    rows = 0
    for rank in range(R):
        ds, kv, q, q_indptr, pairs, out_indptr = run_share(11, n_done, take, Hq, Hkv, owner, rank, R, chunk=128)
        compare_all(ds, kv, q, q_indptr, pairs, Hq, Hq // Hkv, f"scheduled batch rank {rank}", out_indptr)
        rows += int(pairs[:, 3].sum()) * (Hq // Hkv) if len(pairs) else 0
    assert rows == int(take.sum()) * Hq        # every (token, q-head) of the batch is computed exactly once


def test_hip_graph_replays_match_eager():
    """The prefill benchmark replays upload, attention and merge as one HIP graph.  Captured once and
    replayed several times with eager work and synchronisation in between, every replay must leave the
    bits of the eager launch (the kernels are deterministic), from the list the upload brought."""
    say("prefill: graph replays")
    rng = np.random.default_rng(91)
    Hq, Hkv, R = 32, 8, 2
    n_done, n_new = [0, 200, 1030, 48], [150, 40, 90, 700]
    owner = rng.integers(0, R, size=(4, Hkv)).astype(np.int32)
    ds, kv, q, q_indptr, pairs, oi = run_share(77, n_done, n_new, Hq, Hkv, owner, 1, R, chunk=256)
    eager_o, eager_l = ds.prefill_out.clone(), ds.prefill_lse.clone()
    host_items = ds.prefill_items.cpu().pin_memory()
    cap = torch.cuda.Stream()
    sp = cap.cuda_stream
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=cap):
        ds.prefill_items.copy_(host_items, non_blocking=True)
        fs.fs_prefill_attention(ds.shape, ds.view, ds.prefill_items, ds.prefill_sched, ds.n_prefill_items,
                                ds.prefill_tile_tokens, ds.prefill_part_o, ds.prefill_part_lse, sp)
        fs.fs_merge_lse(ds.prefill_part_o, ds.prefill_part_lse, ds.prefill_chunk_indptr, ds.n_prefill_tiles,
                        ds.prefill_tile_rows, 128, ds.prefill_out, ds.prefill_lse, sp)
    for rep in range(4):
        ds.prefill_out.fill_(float("nan")); ds.prefill_lse.fill_(float("nan")); ds.prefill_part_o.fill_(float("nan"))
        ds.prefill_items.zero_()                   # the replayed upload has to bring the list back
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(ds.prefill_out, eager_o) and torch.equal(ds.prefill_lse, eager_l), f"replay {rep} differs"
        ds.prefill()                               # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(ds.prefill_out, eager_o)
    compare_all(ds, kv, q, q_indptr, pairs, Hq, Hq // Hkv, "graph replay vs oracle", oi)


@pytest.mark.parametrize("waves,ct,wide,kv_dtype", [(8, 1, 0, "bf16"), (4, 2, 0, "bf16"), (8, 1, 1, "bf16"), (8, 1, 0, "fp8"),
                                                   (8, 1, 1, "fp8"), (4, 1, 0, "fp8")])
def test_repeated_launches_agree_bit_for_bit(waves, ct, wide, kv_dtype):
    """Launches on the same inputs must leave the same bits in every launch shape (fixed order of sums, no
    atomics on data): a difference means a race between the workgroup's stages, or a matrix-core result read
    before the instruction that writes it has finished (the running reference maximum then comes out of
    whatever the registers held, which moves the rounding of a whole row)."""
    say(f"prefill: repeated launches, waves={waves} ct={ct} wide={wide} {kv_dtype}")
    fs.fs_set_option("prefill_waves", waves); fs.fs_set_option("prefill_col_tiles", ct)
    try:
        rng = np.random.default_rng(92)
        Hq, Hkv, R = 64, 8, 2
        n_done, n_new = [0, 300, 2100, 16], [260, 70, 130, 900]
        owner = rng.integers(0, R, size=(4, Hkv)).astype(np.int32)
        ds, kv, q, q_indptr, pairs, oi = run_share(78, n_done, n_new, Hq, Hkv, owner, 0, R, chunk=512, kv_dtype=kv_dtype,
                                                   v_range=fs.FS_V_ANY if wide else fs.FS_V_FP16_RANGE)
        first = [t.clone() for t in (ds.prefill_part_o, ds.prefill_part_lse, ds.prefill_out, ds.prefill_lse)]
        for rep in range(5):
            for t in (ds.prefill_part_o, ds.prefill_part_lse, ds.prefill_out, ds.prefill_lse):
                t.fill_(float("nan"))
            ds.prefill()
            torch.cuda.synchronize()
            for name, a, b in zip(("part_o", "part_lse", "out", "lse"), first,
                                  (ds.prefill_part_o, ds.prefill_part_lse, ds.prefill_out, ds.prefill_lse)):
                assert torch.equal(a, b), f"launch {rep}: {name} differs from the first launch"
    finally:
        fs.fs_set_option("prefill_waves", 8); fs.fs_set_option("prefill_col_tiles", 1)


@pytest.mark.parametrize("waves,ct", [(8, 1), (4, 1), (4, 2)])
def test_scores_that_jump_far_above_the_reference_maximum(waves, ct):
    """The kernel keeps a row's reference maximum lazily (it follows the running maximum only when that gets
    2^8 ahead).  Keys 96..127 of every pair are 32 times larger than the rest, so their scores lie tens of
    powers of two above everything seen before them: the reference must move there, or the weights overflow."""
    say(f"prefill: score jump, waves={waves} ct={ct}")
    fs.fs_set_option("prefill_waves", waves); fs.fs_set_option("prefill_col_tiles", ct)
    try:
        def louder_keys(kv):
            for p in range(len(kv["page_indptr"]) - 1):
                first = int(kv["page_indptr"][p])
                slots = kv["page_ids"][first + 6:first + 8]
                kv["k_pool"][slots] += np.uint16(5 << 7)          # bf16 exponent + 5
        owner = np.zeros((3, 2), dtype=np.int32)
        for chunk in (0, 64):
            ds, kv, q, q_indptr, pairs, oi = run_share(321, [200, 128, 90], [40, 3, 70], 16, 2, owner, 0, 1, chunk=chunk,
                                                       kv_edit=louder_keys)
            compare_all(ds, kv, q, q_indptr, pairs, 16, 8, f"score jump {waves}x{ct} chunk={chunk}", oi)
    finally:
        fs.fs_set_option("prefill_waves", 8); fs.fs_set_option("prefill_col_tiles", 1)


def test_unused_tails_and_spare_slots_are_never_used():
    say("poisoned tails")
    # contexts that end mid-page and mid-pair: the poisoned tail of the last page must not leak
    owner = np.zeros((4, 2), dtype=np.int32)
    for chunk in (0, 32):
        ds, kv, q, q_indptr, pairs, oi = run_share(13, [1, 17, 30, 47], [14, 16, 19, 2], 8, 2, owner, 0, 1, chunk=chunk)
        compare_all(ds, kv, q, q_indptr, pairs, 8, 4, f"tails chunk={chunk}", oi)


def test_partials_item_by_item():
    say("partials")
    # every item's partial rows against the oracle's, rows that see none of a chunk included
    n_done, n_new, Hq, Hkv = [70, 0, 33], [50, 9, 40], 8, 2
    owner = np.zeros((3, Hkv), dtype=np.int32)
    ds, kv, q, q_indptr, pairs, oi = run_share(17, n_done, n_new, Hq, Hkv, owner, 0, 1, tile=8, chunk=64)
    ref_o, ref_l = oracle.prefill_attention_items(q, kv, ds.w_items, pairs, Hq, 4, 8, SCALE)
    part_o, part_l = ds.prefill_part_o.cpu().numpy().astype(np.float64), ds.prefill_part_lse.cpu().numpy().astype(np.float64)
    unseen = np.isneginf(ref_l)
    assert unseen.any() and np.array_equal(np.isneginf(part_l), unseen)
    assert (part_o[unseen] == 0).all()
    pad = np.isnan(ref_l)                       # rows a short last tile does not have: written as zeros
    assert (part_o[pad] == 0).all() and (part_l[pad] == 0).all()
    seen = ~unseen & ~pad
    check(part_o[seen], part_l[seen], ref_o[seen], ref_l[seen], "partials")


def test_empty_share_and_bad_arguments():
    say("empty share, errors")
    sh = fs.FsShape(2, 8, 2, 128, 16, 2)
    owner = np.zeros((2, 2), dtype=np.int32)
    items, pairs, sched, chunk_indptr, out_indptr = fs.fs_build_prefill_worklist(sh, [5, 6], [3, 4], owner, 1, 4)
    assert len(items) == 0
    dummy = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    kvv = fs.FsKvView(q=dummy.data_ptr(), k_pool=dummy.data_ptr(), v_pool=dummy.data_ptr(), k_slot_stride=4096,
                      v_slot_stride=4096, k_scale=None, v_scale=None, page_indptr=dummy.data_ptr(),
                      page_ids=dummy.data_ptr(), kv_dtype=fs.FS_KV_BF16, sm_scale=SCALE)
    fs.fs_prefill_attention(sh, kvv, None, None, 0, 4, dummy, dummy)          # no-op
    with pytest.raises(fs.FsError):
        fs.fs_prefill_attention(sh, kvv, dummy, None, 1, 10 ** 6, dummy, dummy)   # tile beyond the kernel's
    kvv.kv_dtype = fs.FS_KV_FP8_E4M3
    with pytest.raises(fs.FsError):
        fs.fs_prefill_attention(sh, kvv, dummy, None, 1, 4, dummy, dummy)


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
def test_bench_batch_full_size_sampled(kv_dtype):
    """The batch `bench.py --path prefill` times, in its launch configuration: sampled (pair, token)
    rows against the oracle, one by one, plus finiteness of every row."""
    say(f"bench batch, sampled rows, {kv_dtype}")
    import bench_prefill
    w = bench_prefill.prefill_workload(fs)
    shape, G, pairs, items = w["shape"], w["G"], w["pairs"], w["items"]
    assert w["tile"] == fs.fs_prefill_tile_tokens(G) and w["kv_chunk"] == 2272      # what the chunk choice gives on this batch (ceil(4 * 863803 / (3 * 512)) = 2250 -> 2272)
    ctx = (w["n_done"] + w["n_new"]).astype(np.int32)
    kv = make_kv_pool(w["seed"], np.stack([pairs["req"], pairs["kv_head"]], axis=1), ctx, kv_dtype=kv_dtype)
    q_indptr = np.concatenate([[0], np.cumsum(w["n_new"])]).astype(np.int64)
    q = make_prefill_q(w["seed"], int(q_indptr[-1]), shape.n_q_heads, 128)
    ds = DeviceShare(shape, q, kv, SCALE, v_range=fs.FS_V_FP16_RANGE)
    ds.set_prefill_worklist(items, w["sched"], w["chunk_indptr"], w["tile"], w["out_indptr"])
    ds.prefill()
    torch.cuda.synchronize()
    check_one_call_form(ds, w["chunk_indptr"])
    out, lse = ds.prefill_out.cpu().numpy(), ds.prefill_lse.cpu().numpy()
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    pr = np.stack([pairs[n] for n in oracle.PREFILL_PAIR_FIELDS], axis=1)
    rng = np.random.default_rng(3)
    longest = int(np.argmax(pr[:, 2] + pr[:, 3]))
    samples = [(longest, int(pr[longest, 3]) - 1), (longest, 0), (0, 0)]
    samples += [(int(p), int(rng.integers(0, pr[p, 3]))) for p in rng.integers(0, len(pr), size=40)]
    got_o, got_l, ref_o, ref_l = [], [], [], []
    for p, tok in samples:
        o, l = oracle.prefill_attention_row(q, q_indptr, kv, pr, shape.n_q_heads, G, SCALE, p, tok)
        row = int(w["out_indptr"][p]) + tok * G
        got_o.append(out[row:row + G]); got_l.append(lse[row:row + G]); ref_o.append(o); ref_l.append(l)
    check(np.concatenate(got_o), np.concatenate(got_l), np.concatenate(ref_o), np.concatenate(ref_l),
          f"bench batch ({kv_dtype}), {len(samples)} sampled rows")
