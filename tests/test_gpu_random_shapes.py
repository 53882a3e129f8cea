"""Randomised parity: both attention paths on drawn shapes (groups, heads, ranks, lengths with 0/1/ragged
tails, split-K chunks, launch order, pool layout, tile sizes, the wide second product) against the oracle,
and the persistent decode sweep against the plain one bit for bit.  Seeded; every case is small."""
import os
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2511_14116_amd as fs
from workloads import make_requests, make_q

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import test_gpu_parity as TD      # noqa: E402  (helpers: run_rank, check, shape_of, pairs_rows)
import test_gpu_prefill as TP     # noqa: E402  (helpers: run_share, compare_all)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _lib():
    if not os.path.exists(fs.library_path()):
        raise RuntimeError("libfailsafe.so is not built: GPU tests never fall back to anything else")
    fs.load_library()
    yield
    _defaults()


@pytest.fixture(autouse=True)
def _options_back_to_defaults():
    yield
    _defaults()


def _defaults():
    for key, value in (("prefill_waves", 8), ("prefill_col_tiles", 1), ("waves_per_group", 4),
                       ("prefetch_pages", 2)):
        fs.fs_set_option(key, value)


@pytest.mark.parametrize("seed", range(4))
def test_prefill_on_drawn_shapes(seed):
    rng = np.random.default_rng(8100 + seed)
    rng_kv = np.random.default_rng(8150 + seed)      # the cache's type: a stream of its own, so the cases stay as drawn
    for case in range(25):
        Hkv = int(rng.choice([1, 2, 4, 8])); G = int(rng.choice([1, 2, 3, 4, 5, 8, 16])); Hq = Hkv * G
        R = int(rng.integers(1, 4)); B = int(rng.integers(1, 6))
        n_done = (rng.integers(0, 700, size=B) * (rng.random(B) < 0.7)).astype(np.int32)
        n_new = rng.choice([0, 1, 2, 15, 16, 17, 31, 33, 64, 100, 257], size=B).astype(np.int32)
        if n_new.sum() == 0:
            n_new[0] = 5
        owner = rng.integers(0, R, size=(B, Hkv)).astype(np.int32)
        chunk = int(rng.choice([0, 32, 64, 256, 1024]))
        tile = int(rng.integers(1, fs.fs_prefill_tile_tokens(G) + 1)) if rng.random() < 0.3 else None
        wide = int(rng.random() < 0.25)
        kv_dtype = "fp8" if rng_kv.random() < 0.4 else "bf16"
        what = f"prefill seed {seed} case {case}: {kv_dtype} Hkv={Hkv} G={G} R={R} n_done={n_done.tolist()} n_new={n_new.tolist()} chunk={chunk} tile={tile} wide={wide}"
        TP.say(what)
        ds, kv, q, q_indptr, pairs, oi = TP.run_share(9000 + 100 * seed + case, n_done, n_new, Hq, Hkv, owner,
                                                      int(rng.integers(0, R)), R, tile=tile, chunk=chunk,
                                                      use_sched=bool(rng.random() < 0.8), interleave=bool(rng.random() < 0.7),
                                                      v_range=fs.FS_V_ANY if wide else fs.FS_V_FP16_RANGE, kv_dtype=kv_dtype)
        if len(pairs):
            TP.compare_all(ds, kv, q, q_indptr, pairs, Hq, G, what, oi)


@pytest.mark.parametrize("seed", range(4))
def test_decode_on_drawn_shapes(seed):
    rng = np.random.default_rng(8200 + seed)
    for case in range(25):
        cfg = int(rng.choice([1, 1, 3, 4]))
        n_req = int(rng.integers(1, 40))
        w = make_requests(cfg, seed=7000 + 100 * seed + case, n_req=n_req, max_len=int(rng.choice([40, 300, 3000])))
        Hkv = int(rng.choice([1, 2, 8])); G = int(rng.choice([1, 2, 3, 4, 6, 8, 16]))
        w.update(n_q_heads=G * Hkv, n_kv_heads=Hkv, group=G, n_ranks=int(rng.integers(1, 8)))
        q = make_q(w["seed"], n_req, G * Hkv, 128)
        owner, _, _ = fs.fs_build_placement(TD.shape_of(w), w["ctx_len"], w["mode"])
        rank, chunk = int(rng.integers(0, w["n_ranks"])), int(rng.choice([0, 16, 64, 512, 2048]))
        what = f"decode seed {seed} case {case}: cfg {cfg} B={n_req} Hkv={Hkv} G={G} R={w['n_ranks']} rank {rank} chunk {chunk}"
        TD.say(what)
        ds, kv, items, pairs, sched, indptr = TD.run_rank(w, q, rank, chunk, owner, interleave=bool(rng.random() < 0.7),
                                                          use_sched=bool(rng.random() < 0.8))
        if not len(pairs):
            continue
        ref_o, ref_l = oracle.decode_attention_pairs(q, kv, TD.pairs_rows(pairs), G * Hkv, G, w["sm_scale"])
        TD.check(ds.out.cpu().numpy(), ds.lse.cpu().numpy(), ref_o, ref_l, what)
        # from launch records, with the merge as a kernel and inside the sweep: the same bits
        TD.check_records(ds, kv, items, sched, indptr, what)
        plain = ds.out.clone()
        ds.run(persistent=True)
        torch.cuda.synchronize()
        assert torch.equal(plain, ds.out), f"{what}: the persistent sweep differs from the plain one"


@pytest.mark.parametrize("seed", range(2))
def test_drawn_launch_shapes(seed):
    """The same draws under drawn launch shapes of both kernels (wavefronts per item, pages prefetched, prefill
    wavefronts x column tiles): every shape against the oracle; the persistent sweep matches the plain one bit
    for bit where the plain one splits an item over four wavefronts as it does."""
    rng = np.random.default_rng(8300 + seed)
    try:
        for case in range(25):
            pw, pc = [(8, 1), (8, 2), (4, 1), (4, 2), (4, 4)][int(rng.integers(0, 5))]
            fs.fs_set_option("prefill_waves", pw); fs.fs_set_option("prefill_col_tiles", pc)
            wide = bool(rng.random() < 0.25)
            fs.fs_set_option("waves_per_group", int(rng.choice([1, 2, 4]))); fs.fs_set_option("prefetch_pages", int(rng.integers(1, 4)))
            Hkv = int(rng.choice([1, 2, 8])); G = int(rng.choice([1, 2, 4, 8, 16])); Hq = Hkv * G
            R = int(rng.integers(1, 4)); B = int(rng.integers(1, 5))
            n_done = (rng.integers(0, 600, size=B) * (rng.random(B) < 0.7)).astype(np.int32)
            n_new = rng.choice([1, 16, 17, 33, 100, 257], size=B).astype(np.int32)
            owner = rng.integers(0, R, size=(B, Hkv)).astype(np.int32)
            chunk = int(rng.choice([0, 64, 256]))
            what = f"shapes seed {seed} case {case}: prefill {pw}x{pc} Hkv={Hkv} G={G} n_done={n_done.tolist()} n_new={n_new.tolist()} chunk={chunk}"
            TP.say(what)
            ds, kv, q, q_indptr, pairs, oi = TP.run_share(9500 + 100 * seed + case, n_done, n_new, Hq, Hkv, owner,
                                                          int(rng.integers(0, R)), R, chunk=chunk,
                                                          v_range=fs.FS_V_ANY if wide else fs.FS_V_FP16_RANGE)
            if len(pairs):
                TP.compare_all(ds, kv, q, q_indptr, pairs, Hq, G, what, oi)
            n_req = int(rng.integers(1, 30))
            w = make_requests(1, seed=7700 + 100 * seed + case, n_req=n_req, max_len=int(rng.choice([300, 3000])))
            w.update(n_q_heads=Hq, n_kv_heads=Hkv, group=G, n_ranks=int(rng.integers(1, 6)))
            qd = make_q(w["seed"], n_req, Hq, 128)
            owner_d, _, _ = fs.fs_build_placement(TD.shape_of(w), w["ctx_len"], w["mode"])
            what = f"shapes seed {seed} case {case}: decode waves {fs.fs_get_option('waves_per_group')} prefetch {fs.fs_get_option('prefetch_pages')} B={n_req} Hkv={Hkv} G={G}"
            dd, kvd, items, prs, sched, indptr = TD.run_rank(w, qd, 0, int(rng.choice([0, 64, 512])), owner_d)
            if not len(prs):
                continue
            ref_o, ref_l = oracle.decode_attention_pairs(qd, kvd, TD.pairs_rows(prs), Hq, G, w["sm_scale"])
            TD.check(dd.out.cpu().numpy(), dd.lse.cpu().numpy(), ref_o, ref_l, what)
            if fs.fs_get_option("waves_per_group") == 4:
                plain = dd.out.clone()
                dd.run(persistent=True)
                torch.cuda.synchronize()
                assert torch.equal(plain, dd.out), f"{what}: the persistent sweep differs from the plain one"
    finally:
        _defaults()
